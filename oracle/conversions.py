"""CPU oracle for the conversions of classic attention weights into Tucker-attention weights
(TEST INFRASTRUCTURE ONLY; the product path may not import it).

Three front-ends onto the one layer of Definition "Tucker Attention":

  * MHA / GQA / MQA: the exact representation with a selector core (appendix "Tucker
    Representations of MQA, GQA, and MLA": the lemma on D_i = A_i B_i^T and the theorem on the
    ranks (nH, d, nG dH) of grouped-query attention).
  * MLA: the exact representation with the down-projections as mode-2 / mode-3 bases and the
    products of the up-projections as core slices (theorem on the ranks (nH, dcQ, dcK) of MLA;
    Section "Simplified RoPE for MLA": with latent RoPE switched on in the layer, this core IS
    the fused query matrix of the coupled-RoPE form, the rotation acting in the key latent).
  * MHA -> Tucker by a truncated higher-order SVD of the stacked per-head products
    W_i = WQ_i WK_i^T and W~_i = (WV_i WO_i)^T (appendix "Converting pretrained MHA parameters
    to approximate attention parameters").  Written from the definition: the dense tensors are
    formed, each mode is unfolded, the leading left singular vectors of every unfolding are the
    factor, the core is the tensor contracted with the transposed factors.

Readings where the paper is silent:
  * the query matrix of the coupled-RoPE equation is printed with the value up-projection in
    the place where dimensions and the preceding MLA theorem require the transposed key
    up-projection; the core slice is WUQ_i WUK_i^T.
  * singular vectors are unique up to sign; both sides make the entry of largest magnitude of
    every factor column positive (ties: the first such entry).  Columns are ordered by
    decreasing singular value.
  * "sharing U3" for a shared key-value latent: the mode-3 factor of the pre-softmax tensor is
    also used as the mode-3 factor of the post-softmax tensor, whose core is the contraction
    with that factor.

All arithmetic in fp64.
"""
from __future__ import annotations

from typing import Dict, Optional, Sequence

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# ---------------------------------------------------------------------------------------------
# exact representations
# ---------------------------------------------------------------------------------------------

def selector_core(n_heads: int, d_head: int, n_groups: int) -> np.ndarray:
    """C[i, (i,l), (g(i),l)] = 1, zero elsewhere; g(i) = i // (nH/nG).  Shape [nH, nH dH, nG dH]."""
    if n_heads % n_groups:
        raise ValueError("heads must divide evenly into groups")
    per = n_heads // n_groups
    C = np.zeros((n_heads, n_heads * d_head, n_groups * d_head), dtype=F64)
    for i in range(n_heads):
        for l in range(d_head):
            C[i, i * d_head + l, (i // per) * d_head + l] = 1.0
    return C


def gqa_to_tucker(WQ, WK, WV, WO, n_heads: int, n_groups: int) -> Dict[str, np.ndarray]:
    """Grouped-query attention (nG = nH: MHA, nG = 1: MQA) as Tucker attention.

    WQ [d, nH dH], WK, WV [d, nG dH], WO [nH dH, d].  Ranks (nH, nH dH, nG dH) for both tensors.
    """
    WQ, WK, WV, WO = _f64(WQ), _f64(WK), _f64(WV), _f64(WO)
    d_head = WQ.shape[1] // n_heads
    core = selector_core(n_heads, d_head, n_groups)
    eye = np.eye(n_heads, dtype=F64)
    return dict(C=core, U1=eye, U2=WQ.copy(), U3=WK.copy(),
                Ct=core.copy(), Ut1=eye.copy(), Ut2=WO.T.copy(), Ut3=WV.copy())


def mla_to_tucker(WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, n_heads: int) -> Dict[str, np.ndarray]:
    """Multi-head latent attention as Tucker attention.

    WDQ [d, dcQ], WUQ [dcQ, nH dH], WDKV [d, dcK], WUK [dcK, nH dH], WDV [d, dcK] or None
    (None: the value latent is the key latent, no Ut3 is returned and the layer runs with a
    shared key-value latent), WUV [dcK, nH dH], WO [nH dH, d].
    Pre-softmax ranks (nH, dcQ, dcK); post-softmax ranks (nH, nH dH, dcK).
    """
    WDQ, WUQ, WDKV, WUK, WUV, WO = (_f64(a) for a in (WDQ, WUQ, WDKV, WUK, WUV, WO))
    n = WUQ.shape[1]
    d_head = n // n_heads
    dck = WDKV.shape[1]
    C = np.zeros((n_heads, WDQ.shape[1], dck), dtype=F64)
    Ct = np.zeros((n_heads, n, dck), dtype=F64)
    for i in range(n_heads):
        sl = slice(i * d_head, (i + 1) * d_head)
        C[i] = WUQ[:, sl] @ WUK[:, sl].T                        # fused query-key core slice
        Ct[i, sl, :] = WUV[:, sl].T                              # head i reads only its own rows of WO
    eye = np.eye(n_heads, dtype=F64)
    out = dict(C=C, U1=eye, U2=WDQ.copy(), U3=WDKV.copy(), Ct=Ct, Ut1=eye.copy(), Ut2=WO.T.copy())
    if WDV is not None:
        out["Ut3"] = _f64(WDV).copy()
    return out


# ---------------------------------------------------------------------------------------------
# truncated higher-order SVD
# ---------------------------------------------------------------------------------------------

def unfold(T: np.ndarray, mode: int) -> np.ndarray:
    """Mode-k unfolding: rows indexed by mode k, columns by the other two modes."""
    return np.moveaxis(T, mode, 0).reshape(T.shape[mode], -1)


def fix_signs(U: np.ndarray) -> np.ndarray:
    """Make the entry of largest magnitude of every column positive (first one on ties)."""
    U = U.copy()
    for k in range(U.shape[1]):
        j = int(np.argmax(np.abs(U[:, k])))
        if U[j, k] < 0:
            U[:, k] = -U[:, k]
    return U


def leading_left_singular_vectors(M: np.ndarray, r: int):
    """The r left singular vectors of M with the largest singular values, and all singular values."""
    U, s, _ = np.linalg.svd(M, full_matrices=False)
    return fix_signs(U[:, :r]), s


def hosvd(T: np.ndarray, ranks: Sequence[int], U3: Optional[np.ndarray] = None):
    """Truncated higher-order SVD of a 3-way tensor: T ~ C x1 U1 x2 U2 x3 U3.

    With U3 given, that matrix is used as the mode-3 factor instead of the singular vectors.
    Returns (C, U1, U2, U3, [singular values of the three unfoldings])."""
    T = _f64(T)
    r1, r2, r3 = ranks
    U1, s1 = leading_left_singular_vectors(unfold(T, 0), r1)
    U2, s2 = leading_left_singular_vectors(unfold(T, 1), r2)
    if U3 is None:
        U3, s3 = leading_left_singular_vectors(unfold(T, 2), r3)
    else:
        U3, s3 = _f64(U3), None
    C = np.einsum("ijk,ia,jb,kc->abc", T, U1, U2, U3, optimize=True)
    return C, U1, U2, U3, (s1, s2, s3)


def attention_tensors(WQ, WK, WV, WO, n_heads: int):
    """W[i] = WQ_i WK_i^T and W~[i] = (WV_i WO_i)^T (output index first), both [nH, d, d]."""
    WQ, WK, WV, WO = _f64(WQ), _f64(WK), _f64(WV), _f64(WO)
    d_head = WQ.shape[1] // n_heads
    hs = lambda i: slice(i * d_head, (i + 1) * d_head)
    W = np.stack([WQ[:, hs(i)] @ WK[:, hs(i)].T for i in range(n_heads)])
    Wt = np.stack([(WV[:, hs(i)] @ WO[hs(i), :]).T for i in range(n_heads)])
    return W, Wt


def mha_to_tucker_hosvd(WQ, WK, WV, WO, n_heads: int, ranks: Sequence[int], ranks_t: Sequence[int],
                        shared_kv: bool = False) -> Dict[str, np.ndarray]:
    """MHA weights (WQ, WK, WV [d, nH dH], WO [nH dH, d]) to Tucker weights of the given ranks."""
    W, Wt = attention_tensors(WQ, WK, WV, WO, n_heads)
    C, U1, U2, U3, _ = hosvd(W, ranks)
    if shared_kv:
        if ranks_t[2] != ranks[2]:
            raise ValueError("a shared latent needs equal key and value ranks")
        Ct, Ut1, Ut2, _, _ = hosvd(Wt, ranks_t, U3=U3)
        return dict(C=C, U1=U1, U2=U2, U3=U3, Ct=Ct, Ut1=Ut1, Ut2=Ut2)
    Ct, Ut1, Ut2, Ut3, _ = hosvd(Wt, ranks_t)
    return dict(C=C, U1=U1, U2=U2, U3=U3, Ct=Ct, Ut1=Ut1, Ut2=Ut2, Ut3=Ut3)
