"""Thin ctypes binding of libtucker_attn.so: argument marshalling only.

Same names as the C ABI (include/tucker_attn.h).  PyTorch supplies device memory and the
HIP stream; every step of the forward and backward passes runs in the library's kernels.  There is no
fallback: if the shared library is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Tuple

_HERE = os.path.dirname(os.path.abspath(__file__))
# TUCKER_ATTN_LIB names another build of the same library (comparing two builds in one session)
LIB_PATH = os.environ.get("TUCKER_ATTN_LIB") or os.path.join(_HERE, "libtucker_attn.so")

TUCKER_ATTN_F32 = 0
TUCKER_ATTN_BF16 = 1

EXPORTED = [
    "tucker_attn_create", "tucker_attn_destroy", "tucker_attn_parameter_count", "tucker_attn_cache_bytes",
    "tucker_attn_workspace_bytes",
    "tucker_attn_decode_workspace_bytes", "tucker_attn_forward", "tucker_attn_decode", "tucker_attn_decode_static",
    "tucker_attn_backward_workspace_bytes", "tucker_attn_backward",
    "tucker_attn_prepared_weights_bytes", "tucker_attn_prepare_weights", "tucker_attn_release_weights",
    "tucker_attn_profile_enable", "tucker_attn_profile_read", "tucker_attn_measure_mfma_ceiling",
    "tucker_attn_status_string",
]
EXPORTED_CONVERT = [
    "tucker_convert_from_gqa", "tucker_convert_from_mla", "tucker_convert_hosvd_workspace_bytes",
    "tucker_convert_from_mha_hosvd",
]


class TuckerAttnError(RuntimeError):
    pass


class tucker_attn_config(C.Structure):
    _fields_ = [("d_model", C.c_int32), ("n_heads", C.c_int32), ("d_head", C.c_int32),
                ("r1", C.c_int32), ("r2", C.c_int32), ("r3", C.c_int32),
                ("rt1", C.c_int32), ("rt2", C.c_int32), ("rt3", C.c_int32),
                ("causal", C.c_int32), ("use_rope", C.c_int32), ("rope_base", C.c_float),
                ("dtype", C.c_int32), ("max_positions", C.c_int32), ("shared_kv", C.c_int32),
                ("save_for_backward", C.c_int32)]


class tucker_attn_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")]


GRAD_KEYS = ("dC", "dU1", "dU2", "dU3", "dCt", "dUt1", "dUt2", "dUt3")


class tucker_attn_grads(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in GRAD_KEYS]


WEIGHT_KEYS = ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")


class tucker_convert_weights_out(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in WEIGHT_KEYS]


class tucker_convert_hosvd_info(C.Structure):
    _fields_ = [("sweeps", C.c_int32 * 6), ("jacobi_launches", C.c_int64), ("jacobi_ms", C.c_double),
                ("jacobi_bytes", C.c_double)]


_lib = None


def load_library() -> C.CDLL:
    """Load the shared library (once).  Raises if it has not been built."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise TuckerAttnError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2603_30033_amd.build` "
            "(there is no CPU fallback)")
    lib = C.CDLL(LIB_PATH)
    ctx_p = C.c_void_p
    lib.tucker_attn_create.argtypes = [C.POINTER(tucker_attn_config), C.POINTER(ctx_p)]
    lib.tucker_attn_create.restype = C.c_int
    lib.tucker_attn_destroy.argtypes = [ctx_p]
    lib.tucker_attn_destroy.restype = None
    lib.tucker_attn_parameter_count.argtypes = [C.POINTER(tucker_attn_config)]
    lib.tucker_attn_parameter_count.restype = C.c_size_t
    lib.tucker_attn_cache_bytes.argtypes = [ctx_p, C.c_int32, C.c_int32]
    lib.tucker_attn_cache_bytes.restype = C.c_size_t
    lib.tucker_attn_workspace_bytes.argtypes = [ctx_p, C.c_int32, C.c_int32]
    lib.tucker_attn_workspace_bytes.restype = C.c_size_t
    lib.tucker_attn_decode_workspace_bytes.argtypes = [ctx_p, C.c_int32]
    lib.tucker_attn_decode_workspace_bytes.restype = C.c_size_t
    lib.tucker_attn_forward.argtypes = [ctx_p, C.POINTER(tucker_attn_weights), C.c_void_p, C.c_void_p,
                                        C.c_int32, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_int32,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tucker_attn_forward.restype = C.c_int
    lib.tucker_attn_decode.argtypes = [ctx_p, C.POINTER(tucker_attn_weights), C.c_void_p, C.c_void_p,
                                       C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                       C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tucker_attn_decode.restype = C.c_int
    lib.tucker_attn_decode_static.argtypes = [ctx_p, C.POINTER(tucker_attn_weights), C.c_void_p, C.c_void_p,
                                              C.c_void_p, C.c_void_p, C.c_int32, C.POINTER(C.c_int32), C.c_int32,
                                              C.c_void_p]
    lib.tucker_attn_decode_static.restype = C.c_int
    lib.tucker_attn_backward_workspace_bytes.argtypes = [ctx_p, C.c_int32, C.c_int32]
    lib.tucker_attn_backward_workspace_bytes.restype = C.c_size_t
    lib.tucker_attn_backward.argtypes = [ctx_p, C.POINTER(tucker_attn_weights), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.POINTER(tucker_attn_grads), C.c_int32, C.c_int32, C.c_int32, C.c_int32,
                                         C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tucker_attn_backward.restype = C.c_int
    lib.tucker_attn_prepared_weights_bytes.argtypes = [ctx_p]
    lib.tucker_attn_prepared_weights_bytes.restype = C.c_size_t
    lib.tucker_attn_prepare_weights.argtypes = [ctx_p, C.POINTER(tucker_attn_weights), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tucker_attn_prepare_weights.restype = C.c_int
    lib.tucker_attn_release_weights.argtypes = [ctx_p]
    lib.tucker_attn_release_weights.restype = C.c_int
    lib.tucker_attn_profile_enable.argtypes = [ctx_p, C.c_int32]
    lib.tucker_attn_profile_enable.restype = C.c_int
    lib.tucker_attn_profile_read.argtypes = [ctx_p, C.POINTER(C.c_char_p), C.POINTER(C.c_float), C.c_int32]
    lib.tucker_attn_profile_read.restype = C.c_int
    lib.tucker_attn_measure_mfma_ceiling.argtypes = [C.c_int32, C.c_int32, C.POINTER(C.c_float)]
    lib.tucker_attn_measure_mfma_ceiling.restype = C.c_int
    lib.tucker_attn_status_string.argtypes = [C.c_int]
    lib.tucker_attn_status_string.restype = C.c_char_p
    out_p = C.POINTER(tucker_convert_weights_out)
    lib.tucker_convert_from_gqa.argtypes = [C.c_int32] * 5 + [C.c_void_p] * 4 + [out_p, C.c_void_p]
    lib.tucker_convert_from_gqa.restype = C.c_int
    lib.tucker_convert_from_mla.argtypes = [C.c_int32] * 6 + [C.c_void_p] * 7 + [out_p, C.c_void_p]
    lib.tucker_convert_from_mla.restype = C.c_int
    lib.tucker_convert_hosvd_workspace_bytes.argtypes = [C.c_int32] * 3
    lib.tucker_convert_hosvd_workspace_bytes.restype = C.c_size_t
    lib.tucker_convert_from_mha_hosvd.argtypes = [C.c_int32] * 4 + [C.c_void_p] * 4 + [C.c_int32] * 7 + [
        out_p, C.POINTER(C.c_double), C.POINTER(tucker_convert_hosvd_info), C.c_void_p, C.c_size_t, C.c_void_p]
    lib.tucker_convert_from_mha_hosvd.restype = C.c_int
    _lib = lib
    return lib


def tucker_attn_status_string(status: int) -> str:
    return load_library().tucker_attn_status_string(int(status)).decode()


def _check(status: int, what: str) -> None:
    if status != 0:
        raise TuckerAttnError(f"{what}: status {status} ({tucker_attn_status_string(status)})")


def _ptr(t) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream_ptr(stream) -> Optional[int]:
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return s.cuda_stream or None


def tucker_attn_create(*, d_model, n_heads, d_head, r1, r2, r3, rt1=None, rt2=None, rt3=None, causal=True,
                       rope_base=None, dtype="bf16", max_positions=1, shared_kv=False,
                       save_for_backward=False) -> int:
    """Returns an opaque context handle (int).  Needs a current HIP device when rope_base is set."""
    cfg = tucker_attn_config(d_model, n_heads, d_head, r1, r2, r3, rt1 or r1, rt2 or r2, rt3 or r3,
                             int(bool(causal)), int(rope_base is not None), float(rope_base or 0.0),
                             {"f32": TUCKER_ATTN_F32, "bf16": TUCKER_ATTN_BF16}[dtype], int(max_positions),
                             int(bool(shared_kv)), int(bool(save_for_backward)))
    ctx = C.c_void_p()
    _check(load_library().tucker_attn_create(C.byref(cfg), C.byref(ctx)), "tucker_attn_create")
    return ctx.value


def tucker_attn_destroy(ctx: int) -> None:
    load_library().tucker_attn_destroy(ctx)


def tucker_attn_parameter_count(*, d_model, n_heads, r1, r2, r3, rt1=None, rt2=None, rt3=None, shared_kv=False) -> int:
    cfg = tucker_attn_config(d_model, n_heads, 1, r1, r2, r3, rt1 or r1, rt2 or r2, rt3 or r3, 0, 0, 0.0, TUCKER_ATTN_BF16,
                             1, int(bool(shared_kv)), 0)
    return int(load_library().tucker_attn_parameter_count(C.byref(cfg)))


def tucker_attn_cache_bytes(ctx: int, B: int, Lmax: int) -> int:
    return int(load_library().tucker_attn_cache_bytes(ctx, B, Lmax))


def tucker_attn_workspace_bytes(ctx: int, B: int, N: int) -> int:
    return int(load_library().tucker_attn_workspace_bytes(ctx, B, N))


def tucker_attn_decode_workspace_bytes(ctx: int, B: int) -> int:
    return int(load_library().tucker_attn_decode_workspace_bytes(ctx, B))


def _weights_struct(w: Dict[str, "object"]) -> tucker_attn_weights:
    return tucker_attn_weights(*[_ptr(w.get(k)) for k in ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")])


def tucker_attn_forward(ctx: int, weights: Dict, X, Y, pos0: int = 0, Kcache_out=None, Vcache_out=None,
                        workspace=None, stream=None, check: bool = True) -> int:
    """X, Y: contiguous device tensors [B, N, d]; weights: dict of contiguous device tensors;
    workspace: device uint8 tensor of at least tucker_attn_workspace_bytes bytes."""
    B, N = int(X.shape[0]), int(X.shape[1])
    Lmax = int(Kcache_out.shape[1]) if Kcache_out is not None else 0
    ws = _weights_struct(weights)
    st = load_library().tucker_attn_forward(ctx, C.byref(ws), X.data_ptr(), Y.data_ptr(), B, N, int(pos0),
                                            _ptr(Kcache_out), _ptr(Vcache_out), Lmax,
                                            _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                            _stream_ptr(stream))
    if check:
        _check(st, "tucker_attn_forward")
    return st


def tucker_attn_decode(ctx: int, weights: Dict, x, y, Kcache, Vcache, kv_len: List[int], workspace=None,
                       stream=None, check: bool = True) -> int:
    """x, y: [B, d]; Kcache/Vcache: [B, Lmax, r3]/[B, Lmax, rt3] (updated in place; with a shared
    key-value projection Vcache is None and Kcache is the one cache of unrotated latent rows);
    kv_len: host ints, cache length including the new token."""
    B = int(x.shape[0])
    Lmax = int(Kcache.shape[1])
    lens = (C.c_int32 * B)(*[int(v) for v in kv_len])
    ws = _weights_struct(weights)
    st = load_library().tucker_attn_decode(ctx, C.byref(ws), x.data_ptr(), y.data_ptr(), Kcache.data_ptr(),
                                           _ptr(Vcache), Lmax, lens, B,
                                           _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                           _stream_ptr(stream))
    if check:
        _check(st, "tucker_attn_decode")
    return st


def tucker_attn_decode_static(ctx: int, weights: Dict, x, y, Kcache, Vcache, kv_len: List[int], stream=None,
                              check: bool = True) -> int:
    """tucker_attn_decode on the library's own static scratch array (no workspace, no allocation)."""
    B = int(x.shape[0])
    Lmax = int(Kcache.shape[1])
    lens = (C.c_int32 * B)(*[int(v) for v in kv_len])
    ws = _weights_struct(weights)
    st = load_library().tucker_attn_decode_static(ctx, C.byref(ws), x.data_ptr(), y.data_ptr(), Kcache.data_ptr(),
                                                  _ptr(Vcache), Lmax, lens, B, _stream_ptr(stream))
    if check:
        _check(st, "tucker_attn_decode_static")
    return st


def tucker_attn_backward_workspace_bytes(ctx: int, B: int, N: int) -> int:
    return int(load_library().tucker_attn_backward_workspace_bytes(ctx, B, N))


def tucker_attn_backward(ctx: int, weights: Dict, X, dY, dX, grads: Dict, pos0: int = 0, workspace=None,
                         stream=None, check: bool = True, forward_state: bool = False) -> int:
    """X, dY, dX: contiguous device tensors [B, N, d] of the storage type; grads: dict of contiguous fp32
    device tensors keyed dC, dU1, dU2, dU3, dCt, dUt1, dUt2 and (unless the latent is shared) dUt3,
    shaped like the weights; all are overwritten.  forward_state: the workspace is the one the
    forward call of a save_for_backward context just used with the same inputs."""
    B, N = int(X.shape[0]), int(X.shape[1])
    ws = _weights_struct(weights)
    gs = tucker_attn_grads(*[_ptr(grads.get(k)) for k in GRAD_KEYS])
    st = load_library().tucker_attn_backward(ctx, C.byref(ws), X.data_ptr(), dY.data_ptr(), dX.data_ptr(),
                                             C.byref(gs), B, N, int(pos0), int(bool(forward_state)),
                                             _ptr(workspace), 0 if workspace is None else workspace.numel(),
                                             _stream_ptr(stream))
    if check:
        _check(st, "tucker_attn_backward")
    return st


def tucker_attn_prepared_weights_bytes(ctx: int) -> int:
    return int(load_library().tucker_attn_prepared_weights_bytes(ctx))


def tucker_attn_prepare_weights(ctx: int, weights: Dict, prepared, stream=None, check: bool = True) -> int:
    """prepared: device uint8 tensor of at least tucker_attn_prepared_weights_bytes bytes; the caller keeps it
    (and the weight tensors) alive until tucker_attn_release_weights."""
    ws = _weights_struct(weights)
    st = load_library().tucker_attn_prepare_weights(ctx, C.byref(ws), _ptr(prepared),
                                                    0 if prepared is None else prepared.numel(), _stream_ptr(stream))
    if check:
        _check(st, "tucker_attn_prepare_weights")
    return st


def tucker_attn_release_weights(ctx: int) -> None:
    _check(load_library().tucker_attn_release_weights(ctx), "tucker_attn_release_weights")


def tucker_attn_profile_enable(ctx: int, on: bool) -> None:
    _check(load_library().tucker_attn_profile_enable(ctx, int(bool(on))), "tucker_attn_profile_enable")


def tucker_attn_profile_read(ctx: int) -> List[Tuple[str, float]]:
    names = (C.c_char_p * 41)()
    ms = (C.c_float * 41)()
    n = load_library().tucker_attn_profile_read(ctx, names, ms, 41)
    if n < 0:
        _check(n, "tucker_attn_profile_read")
    return [(names[i].decode(), float(ms[i])) for i in range(n)]


def tucker_attn_measure_mfma_ceiling(from_lds: bool, iters: int = 20000) -> float:
    """TFLOP/s of a bf16 MFMA loop on the current device (operands in registers, or one re-read from LDS)."""
    out = C.c_float()
    _check(load_library().tucker_attn_measure_mfma_ceiling(int(bool(from_lds)), int(iters), C.byref(out)),
           "tucker_attn_measure_mfma_ceiling")
    return float(out.value)


# ---- weight front-ends (include/tucker_convert.h) ------------------------------------------------

def _dtype_code(t) -> int:
    import torch
    if t.dtype == torch.float32:
        return TUCKER_ATTN_F32
    if t.dtype == torch.bfloat16:
        return TUCKER_ATTN_BF16
    raise TuckerAttnError(f"unsupported storage type {t.dtype}")


def _out_struct(out: Dict) -> tucker_convert_weights_out:
    return tucker_convert_weights_out(*[_ptr(out.get(k)) for k in WEIGHT_KEYS])


def tucker_convert_from_gqa(WQ, WK, WV, WO, n_heads: int, n_groups: int, out: Dict, stream=None,
                            check: bool = True) -> int:
    """out: dict of preallocated device tensors C, U1, U2, U3, Ct, Ut1, Ut2, Ut3."""
    d, n = WQ.shape
    st = load_library().tucker_convert_from_gqa(_dtype_code(WQ), d, n_heads, n // n_heads, n_groups, _ptr(WQ), _ptr(WK),
                                                _ptr(WV), _ptr(WO), C.byref(_out_struct(out)), _stream_ptr(stream))
    if check:
        _check(st, "tucker_convert_from_gqa")
    return st


def tucker_convert_from_mla(WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, n_heads: int, out: Dict, stream=None,
                            check: bool = True) -> int:
    d, dcq = WDQ.shape
    dck, n = WUK.shape
    st = load_library().tucker_convert_from_mla(_dtype_code(WDQ), d, n_heads, n // n_heads, dcq, dck, _ptr(WDQ), _ptr(WUQ),
                                                _ptr(WDKV), _ptr(WUK), _ptr(WDV), _ptr(WUV), _ptr(WO),
                                                C.byref(_out_struct(out)), _stream_ptr(stream))
    if check:
        _check(st, "tucker_convert_from_mla")
    return st


def tucker_convert_hosvd_workspace_bytes(d: int, n_heads: int, d_head: int) -> int:
    return int(load_library().tucker_convert_hosvd_workspace_bytes(d, n_heads, d_head))


def tucker_convert_from_mha_hosvd(WQ, WK, WV, WO, n_heads: int, ranks, ranks_t, shared_kv: bool, out: Dict,
                                  workspace, want_singular_values: bool = False, stream=None, check: bool = True):
    """Returns (status, singular values as a list of 2*(nH+2d) floats or None, info dict)."""
    d, n = WQ.shape
    sv = (C.c_double * (2 * (n_heads + 2 * d)))() if want_singular_values else None
    info = tucker_convert_hosvd_info()
    st = load_library().tucker_convert_from_mha_hosvd(
        _dtype_code(WQ), d, n_heads, n // n_heads, _ptr(WQ), _ptr(WK), _ptr(WV), _ptr(WO), *[int(r) for r in ranks],
        *[int(r) for r in ranks_t], int(bool(shared_kv)), C.byref(_out_struct(out)), sv, C.byref(info), _ptr(workspace),
        workspace.numel() * workspace.element_size() if workspace is not None else 0, _stream_ptr(stream))
    if check:
        _check(st, "tucker_convert_from_mha_hosvd")
    return st, (list(sv) if sv is not None else None), dict(
        sweeps=list(info.sweeps), jacobi_launches=int(info.jacobi_launches), jacobi_ms=float(info.jacobi_ms),
        jacobi_bytes=float(info.jacobi_bytes))
