"""Helpers for callers of the binding (tests, smoke, bench): move a generated workload to
the device and drive the C-ABI library through the ctypes binding.  No arithmetic of the
method lives here."""
from __future__ import annotations

from typing import Dict, Optional

import numpy as np
import torch

from paper_2603_30033_amd import binding as ta
from paper_2603_30033_amd import workloads as wl

W_KEYS = ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")


def torch_dtype(dtype: str):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[dtype]


def to_device(a: np.ndarray, dtype: str) -> torch.Tensor:
    """Host fp32 array (already rounded to the storage type) -> contiguous device tensor."""
    return torch.from_numpy(np.ascontiguousarray(a)).to(torch_dtype(dtype)).cuda().contiguous()


def to_host(t: torch.Tensor) -> np.ndarray:
    return t.detach().to(torch.float32).cpu().numpy()


class Layer:
    """A context plus device copies of one workload's weights."""

    def __init__(self, w: wl.Workload, inp: Optional[Dict[str, np.ndarray]], max_positions: Optional[int] = None,
                 save_for_backward: bool = False, device_weights: Optional[Dict[str, torch.Tensor]] = None):
        """Weights come from the host arrays `inp`, or are the device tensors `device_weights` (e.g. what a
        conversion entry point wrote)."""
        self.w = w
        rt1, rt2, rt3 = w.ranks_post()
        if max_positions is None:
            max_positions = max(w.pos0 + w.N, w.kv_len, 1)
        self.ctx = ta.tucker_attn_create(
            d_model=w.d_model, n_heads=w.n_heads, d_head=w.d_head, r1=w.r1, r2=w.r2, r3=w.r3,
            rt1=rt1, rt2=rt2, rt3=rt3, causal=w.causal, rope_base=w.rope_base, dtype=w.dtype,
            max_positions=max_positions, shared_kv=w.shared_kv, save_for_backward=save_for_backward)
        # with a shared key-value projection the library never reads the value basis: it gets none
        if device_weights is not None:
            self.weights = {k: device_weights[k] for k in W_KEYS if not (w.shared_kv and k == "Ut3")}
        else:
            self.weights = {k: to_device(inp[k], w.dtype) for k in W_KEYS if not (w.shared_kv and k == "Ut3")}
        self._ws = None

    def close(self):
        if self.ctx is not None:
            ta.tucker_attn_destroy(self.ctx)
            self.ctx = None

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def freeze_weights(self) -> None:
        """Prepare the operand-layout copies of the weights once; later calls skip that step."""
        self._prepared = torch.empty(max(ta.tucker_attn_prepared_weights_bytes(self.ctx), 256), dtype=torch.uint8,
                                     device="cuda")
        ta.tucker_attn_prepare_weights(self.ctx, self.weights, self._prepared)

    def workspace(self, nbytes: int) -> torch.Tensor:
        if self._ws is None or self._ws.numel() < nbytes:
            self._ws = torch.empty(max(nbytes, 256), dtype=torch.uint8, device="cuda")
        return self._ws

    def forward(self, X: torch.Tensor, pos0: int = 0, Kc=None, Vc=None, Y=None) -> torch.Tensor:
        B, N = X.shape[0], X.shape[1]
        if Y is None:
            Y = torch.empty_like(X)
        ws = self.workspace(ta.tucker_attn_workspace_bytes(self.ctx, B, N))
        ta.tucker_attn_forward(self.ctx, self.weights, X, Y, pos0, Kc, Vc, ws)
        return Y

    def backward(self, X: torch.Tensor, dY: torch.Tensor, pos0: int = 0, forward_state: bool = False):
        """Returns (dX, dict of fp32 weight gradients).  forward_state: reuse what the forward call just
        before left in the shared workspace (needs a layer made with save_for_backward)."""
        B, N = X.shape[0], X.shape[1]
        dX = torch.empty_like(X)
        grads = {"d" + k: torch.empty(self.weights[k].shape, dtype=torch.float32, device="cuda") for k in self.weights}
        ws = self.workspace(ta.tucker_attn_backward_workspace_bytes(self.ctx, B, N))
        ta.tucker_attn_backward(self.ctx, self.weights, X, dY, dX, grads, pos0, ws, forward_state=forward_state)
        return dX, grads

    def decode(self, x: torch.Tensor, Kc: torch.Tensor, Vc: Optional[torch.Tensor], kv_len, y=None) -> torch.Tensor:
        if y is None:
            y = torch.empty_like(x)
        ws = self.workspace(ta.tucker_attn_decode_workspace_bytes(self.ctx, x.shape[0]))
        ta.tucker_attn_decode(self.ctx, self.weights, x, y, Kc, Vc, [int(v) for v in kv_len], ws)
        return y


# ---- weight front-ends ---------------------------------------------------------------------------

def _empty_weights(shapes: Dict[str, tuple], like: torch.Tensor) -> Dict[str, torch.Tensor]:
    return {k: torch.empty(shape, dtype=like.dtype, device="cuda") for k, shape in shapes.items()}


def from_gqa(WQ, WK, WV, WO, n_heads: int, n_groups: int) -> Dict[str, torch.Tensor]:
    """Device tensors of classic GQA weights -> device tensors of the equivalent Tucker weights."""
    d, n = WQ.shape
    g = WK.shape[1]
    out = _empty_weights(dict(C=(n_heads, n, g), U1=(n_heads, n_heads), U2=(d, n), U3=(d, g), Ct=(n_heads, n, g),
                              Ut1=(n_heads, n_heads), Ut2=(d, n), Ut3=(d, g)), WQ)
    ta.tucker_convert_from_gqa(WQ, WK, WV, WO, n_heads, n_groups, out)
    return out


def from_mla(WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, n_heads: int) -> Dict[str, torch.Tensor]:
    d, dcq = WDQ.shape
    dck, n = WUK.shape
    shapes = dict(C=(n_heads, dcq, dck), U1=(n_heads, n_heads), U2=(d, dcq), U3=(d, dck), Ct=(n_heads, n, dck),
                  Ut1=(n_heads, n_heads), Ut2=(d, n))
    if WDV is not None:
        shapes["Ut3"] = (d, dck)
    out = _empty_weights(shapes, WDQ)
    ta.tucker_convert_from_mla(WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, n_heads, out)
    return out


def from_mha_hosvd(WQ, WK, WV, WO, n_heads: int, ranks, ranks_t, shared_kv: bool = False,
                   want_singular_values: bool = False):
    """Returns (device Tucker weights, singular values or None); the iteration report of the call is kept
    in `from_mha_hosvd.last_info`."""
    d, n = WQ.shape
    (r1, r2, r3), (t1, t2, t3) = ranks, ranks_t
    shapes = dict(C=(r1, r2, r3), U1=(n_heads, r1), U2=(d, r2), U3=(d, r3), Ct=(t1, t2, t3), Ut1=(n_heads, t1),
                  Ut2=(d, t2))
    if not shared_kv:
        shapes["Ut3"] = (d, t3)
    out = _empty_weights(shapes, WQ)
    ws = torch.empty(max(ta.tucker_convert_hosvd_workspace_bytes(d, n_heads, n // n_heads), 256), dtype=torch.uint8,
                     device="cuda")
    _, sv, from_mha_hosvd.last_info = ta.tucker_convert_from_mha_hosvd(
        WQ, WK, WV, WO, n_heads, ranks, ranks_t, shared_kv, out, ws, want_singular_values=want_singular_values)
    return out, sv
