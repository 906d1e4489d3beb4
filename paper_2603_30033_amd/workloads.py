"""Seeded synthetic inputs for the Tucker-attention forward pass.

This module only draws random numbers and shapes them; it holds none of the
method's arithmetic (no projection, no softmax, no rotation).  The CPU oracle
and the HIP library are both fed the arrays it returns, so neither side ever
sees a value produced by the other.

Shapes follow the paper's problem statement (Definition "Tucker Attention":
core C[r1,r2,r3], U1[nH,r1], U2[d,r2], U3[d,r3] and the tilde set for the
post-softmax tensor); the first five named workloads take the model shapes of the
paper's hyper-parameter table (GPT-2 small, ViT-B/16) and an N=4096 LLaMA-like
layer; two more take rank shapes the paper itself trains ([8,128,64] on GPT-2,
[32,128,128] on its LLaMA3-1B layer).  The paper's datasets are not used: attention-forward cost does not
depend on the data, so Gaussian tokens stand in for them.

Value recipes
  "fan_in"      every tensor i.i.d. N(0,1) times 1/sqrt(fan_in), fan_in = size
                of the index the tensor is contracted over in the forward pass
                (U2,U3,Ut3: d; Ut2: rt2; U1,Ut1: r1; C: r2; Ct: rt3; X: 1).
  "orthonormal" factor matrices have orthonormal columns (Q of a QR of a
                Gaussian matrix, signs fixed so diag(R) > 0); cores are
                N(0, 1/r2) resp. N(0, 1/rt2); X is N(0,1), optionally followed
                by a per-token LayerNorm (zero mean, unit variance, no affine).
Draw order (one numpy default_rng(seed) stream): X, C, U1, U2, U3, Ct, Ut1,
Ut2, Ut3, then any decode-only tensors.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, Optional

import numpy as np


@dataclass(frozen=True)
class Workload:
    name: str
    B: int
    N: int                      # prefill: tokens per sequence; decode: 1
    d_model: int
    n_heads: int
    d_head: int
    r1: int
    r2: int
    r3: int
    dtype: str                  # "f32" | "bf16": storage type of X, weights, caches, Y
    causal: bool
    rope_base: Optional[float]  # None = no latent RoPE
    seed: int
    recipe: str                 # "fan_in" | "orthonormal"
    layernorm_x: bool = False
    mode: str = "prefill"       # "prefill" | "decode"
    kv_len: int = 0             # decode: cache length INCLUDING the new token
    rt1: int = 0                # post-softmax ranks; 0 = tie to r1, r2, r3
    rt2: int = 0
    rt3: int = 0
    pos0: int = 0
    shared_kv: bool = False     # shared key-value down-projection: value basis = key basis, one cache

    def ranks_post(self):
        return (self.rt1 or self.r1, self.rt2 or self.r2, self.rt3 or self.r3)


WORKLOADS: Dict[str, Workload] = {
    # config 1: tiny causal, fp32
    "tiny_f32": Workload("tiny_f32", B=1, N=128, d_model=256, n_heads=4, d_head=64,
                         r1=2, r2=32, r3=32, dtype="f32", causal=True, rope_base=1e4,
                         seed=0, recipe="fan_in"),
    # config 2: GPT-2-small-shaped causal layer, bf16
    "gpt2_small": Workload("gpt2_small", B=8, N=1024, d_model=768, n_heads=12, d_head=64,
                           r1=4, r2=64, r3=64, dtype="bf16", causal=True, rope_base=1e4,
                           seed=1, recipe="orthonormal", layernorm_x=True),
    # config 3: ViT-B-shaped non-causal layer, bf16, no RoPE
    "vit_b": Workload("vit_b", B=256, N=197, d_model=768, n_heads=12, d_head=64,
                      r1=4, r2=48, r3=48, dtype="bf16", causal=False, rope_base=None,
                      seed=2, recipe="orthonormal"),
    # config 4: LLaMA-7B-shaped causal layer, bf16, N=4096
    "llama7b_n4096": Workload("llama7b_n4096", B=2, N=4096, d_model=4096, n_heads=32, d_head=128,
                              r1=8, r2=128, r3=128, dtype="bf16", causal=True, rope_base=1e4,
                              seed=3, recipe="orthonormal"),
    # config 5: long-context decode against a latent KV cache, bf16
    "decode_32k": Workload("decode_32k", B=16, N=1, d_model=4096, n_heads=32, d_head=128,
                           r1=8, r2=128, r3=128, dtype="bf16", causal=True, rope_base=1e4,
                           seed=4, recipe="orthonormal", mode="decode", kv_len=32768),
    # shared key-value down-projection (Section "KV Caching"): configs 4 and 5 with one latent
    "llama7b_n4096_shared_kv": Workload("llama7b_n4096_shared_kv", B=2, N=4096, d_model=4096, n_heads=32,
                                        d_head=128, r1=8, r2=128, r3=128, dtype="bf16", causal=True,
                                        rope_base=1e4, seed=7, recipe="orthonormal", shared_kv=True),
    "decode_32k_shared_kv": Workload("decode_32k_shared_kv", B=16, N=1, d_model=4096, n_heads=32, d_head=128,
                                     r1=8, r2=128, r3=128, dtype="bf16", causal=True, rope_base=1e4,
                                     seed=8, recipe="orthonormal", mode="decode", kv_len=32768, shared_kv=True),
    # the paper's own rank shapes (tables of Section "Experiments"): unequal query and key ranks on
    # the GPT-2 layer, and its LLaMA3-1B layer with r1 = nH and RoPE base 5e5
    "gpt2_r8_128_64": Workload("gpt2_r8_128_64", B=8, N=1024, d_model=768, n_heads=12, d_head=64,
                               r1=8, r2=128, r3=64, dtype="bf16", causal=True, rope_base=1e4,
                               seed=5, recipe="orthonormal", layernorm_x=True),
    "llama1b_r32_128_128": Workload("llama1b_r32_128_128", B=4, N=2048, d_model=2048, n_heads=32, d_head=64,
                                    r1=32, r2=128, r3=128, dtype="bf16", causal=True, rope_base=5e5,
                                    seed=6, recipe="orthonormal"),
}


def scaled(w: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (smaller B/N for oracle-sized cases)."""
    return replace(w, **kw)


# ---------------------------------------------------------------------------------------
# bf16 storage rounding (round-to-nearest-even on the top 16 bits of an fp32 word)
# ---------------------------------------------------------------------------------------

def bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 array holding the bf16 encoding (RNE)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_storage(x: np.ndarray, dtype: str) -> np.ndarray:
    """The fp32 value the storage type actually holds (identity for f32)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    if dtype == "f32":
        return x
    if dtype == "bf16":
        return bf16_bits_to_f32(bf16_bits(x)).reshape(x.shape)
    raise ValueError(dtype)


# ---------------------------------------------------------------------------------------
# generators
# ---------------------------------------------------------------------------------------

def _orthonormal(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    g = rng.standard_normal((rows, cols))
    q, r = np.linalg.qr(g)
    q = q * np.sign(np.diag(r))[None, :]
    return q.astype(np.float32)


def _normal(rng, shape, std):
    return (rng.standard_normal(shape) * std).astype(np.float32)


def make_classic_weights(d: int, n_heads: int, d_head: int, seed: int, dtype: str, kv_width: Optional[int] = None,
                         decay: float = 0.5) -> Dict[str, np.ndarray]:
    """Seeded stand-ins for trained MHA / GQA projection matrices: WQ [d, nH dH], WK, WV [d, kv_width]
    (default nH dH), WO [nH dH, d].  Each is an orthonormal basis of the model dimension with a power-law
    weighting j^-decay times a Gaussian mixing matrix, so that the mode unfoldings of the stacked per-head
    products have decaying spectra (as trained layers do) instead of a flat one.  fp32 arrays already
    rounded to the storage type."""
    rng = np.random.default_rng(seed)
    n = n_heads * d_head
    g = n if kv_width is None else kv_width
    s = np.power(1.0 + np.arange(d), -decay)

    def one(cols):
        basis = _orthonormal(rng, d, d).astype(np.float64)
        return (basis * s) @ rng.standard_normal((d, cols)) / np.sqrt(np.sum(s * s))

    out = dict(WQ=one(n), WK=one(g), WV=one(g), WO=one(n).T.copy())
    return {k: round_to_storage(v.astype(np.float32), dtype) for k, v in out.items()}


def make_inputs(w: Workload) -> Dict[str, np.ndarray]:
    """All tensors of one workload, fp32 arrays already rounded to the storage dtype.

    Keys: X [B,N,d]; C [r1,r2,r3]; U1 [nH,r1]; U2 [d,r2]; U3 [d,r3];
          Ct [rt1,rt2,rt3]; Ut1 [nH,rt1]; Ut2 [d,rt2]; Ut3 [d,rt3].
    Decode workloads add: Kcache, Vcache [B,kv_len,r3/rt3] (row kv_len-1 zero, to be
    written by the decode step itself) and kv_len [B] int32; X is then [B,1,d].  With
    shared_kv, Ut3 is a copy of U3 and the decode cache is the single Lcache [B,kv_len,r3].
    """
    rng = np.random.default_rng(w.seed)
    d, nH = w.d_model, w.n_heads
    r1, r2, r3 = w.r1, w.r2, w.r3
    rt1, rt2, rt3 = w.ranks_post()
    if rt1 > nH or r1 > nH:
        if w.recipe == "orthonormal":
            raise ValueError("orthonormal head factors need r1 <= n_heads")

    x = rng.standard_normal((w.B, w.N, d)).astype(np.float32)
    if w.layernorm_x:
        mu = x.mean(axis=-1, keepdims=True)
        sd = x.std(axis=-1, keepdims=True)
        x = ((x - mu) / sd).astype(np.float32)

    if w.recipe == "fan_in":
        C = _normal(rng, (r1, r2, r3), 1.0 / np.sqrt(r2))
        U1 = _normal(rng, (nH, r1), 1.0 / np.sqrt(r1))
        U2 = _normal(rng, (d, r2), 1.0 / np.sqrt(d))
        U3 = _normal(rng, (d, r3), 1.0 / np.sqrt(d))
        Ct = _normal(rng, (rt1, rt2, rt3), 1.0 / np.sqrt(rt3))
        Ut1 = _normal(rng, (nH, rt1), 1.0 / np.sqrt(rt1))
        Ut2 = _normal(rng, (d, rt2), 1.0 / np.sqrt(rt2))
        Ut3 = _normal(rng, (d, rt3), 1.0 / np.sqrt(d))
    elif w.recipe == "orthonormal":
        C = _normal(rng, (r1, r2, r3), 1.0 / np.sqrt(r2))
        U1 = _orthonormal(rng, nH, r1)
        U2 = _orthonormal(rng, d, r2)
        U3 = _orthonormal(rng, d, r3)
        Ct = _normal(rng, (rt1, rt2, rt3), 1.0 / np.sqrt(rt2))
        Ut1 = _orthonormal(rng, nH, rt1)
        Ut2 = _orthonormal(rng, d, rt2)
        Ut3 = _orthonormal(rng, d, rt3)
    else:
        raise ValueError(w.recipe)

    if w.shared_kv:
        # the value basis is the key basis (it is still drawn, so that the stream of random numbers
        # of a workload does not depend on this switch)
        if rt3 != r3:
            raise ValueError("shared key-value projection needs rt3 == r3")
        Ut3 = U3.copy()
    out = dict(X=x, C=C, U1=U1, U2=U2, U3=U3, Ct=Ct, Ut1=Ut1, Ut2=Ut2, Ut3=Ut3)

    if w.mode == "decode":
        # The cached rows stand for rotated keys / values of earlier N(0,1) tokens seen
        # through orthonormal U3 / Ut3: such rows are themselves i.i.d. N(0,1) (an
        # orthonormal projection and a rotation both preserve the distribution), so they
        # are drawn directly at width r3 instead of projecting B*kv_len*d token values.
        L = w.kv_len
        kc = np.empty((w.B, L, r3), dtype=np.float32)
        vc = np.empty((w.B, L, rt3), dtype=np.float32)
        for b in range(w.B):
            kc[b] = rng.standard_normal((L, r3), dtype=np.float32)
            vc[b] = rng.standard_normal((L, rt3), dtype=np.float32)
        kc[:, L - 1, :] = 0.0
        vc[:, L - 1, :] = 0.0
        if w.shared_kv:
            out["Lcache"] = kc                  # one cache: the unrotated latent rows
        else:
            out["Kcache"] = kc
            out["Vcache"] = vc
        out["kv_len"] = np.full((w.B,), L, dtype=np.int32)

    for k, v in out.items():
        if v.dtype == np.float32:
            out[k] = round_to_storage(v, w.dtype)
    return out


def weights_of(inp: Dict[str, np.ndarray]) -> Dict[str, np.ndarray]:
    return {k: inp[k] for k in ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")}
