"""CPU oracle for the Tucker-attention forward pass (TEST INFRASTRUCTURE ONLY).

A plain, slow, fp64 numpy implementation of what the layer computes, written
from the paper's definitions.  It exists so that tests can grade the HIP library
against it; nothing on the product path may import, call or fall back to it, and
it shares no code with the HIP path.

Two forms of the same result are given and must agree with each other:

  dense_definition_forward   the result exactly as the paper defines it
                             (Section "Tensor attention reformulation":
                             H1 = softmax(W x2 X x3 X / sqrt(dH)),
                             H2 = W~ x3 X, output_jk = sum_{i,l} H1_ijl H2_ikl,
                             with W, W~ given by the Tucker representation of
                             Definition "Tucker Attention").  Tiny shapes only:
                             it materialises the nH x d x d tensors.
  per_head_forward           per-head weights WQ_i = U2 G_i, WK = U3, WV = U~3,
                             WO_i built from the cores and factors, followed by
                             textbook attention with a full N x N score matrix
                             and a max-subtracted row softmax (the MHA head
                             formula of the same section, summed over heads).
                             This is the form the GPU is graded against.

Both are exact reformulations of one another (linear algebra only), so every
function here is pinned by tests against closed forms, brute force and the
special cases the paper proves (MHA, GQA/MQA, MLA); none is "parity unpinned".

Readings of the paper taken here (it is silent or inconsistent on these):
  * softmax scale is 1/sqrt(d_head), d_head a free parameter (the paper keeps
    dH = d/nH in the scale although the contraction runs over r3);
  * causal mask: key n is visible to query m iff n <= m in absolute positions;
  * RoPE matrix (the paper defers to RoFormer, Eq. 15): 2x2 rotations on adjacent
    channel pairs (2j, 2j+1), theta_j = base**(-2j/r), angle = position*theta_j,
    row-vector form x' = x R(p):  x'_{2j}   = x_{2j} cos - x_{2j+1} sin,
                                  x'_{2j+1} = x_{2j} sin + x_{2j+1} cos;
  * latent RoPE (Definition "Latent RoPE for Tucker Attention") rotates the
    per-head query AFTER the core, in the r3-wide key space, and the shared key;
    values and the r2 space are never rotated;
  * the KV-caching formula prints the post-softmax core inside the softmax and
    stops at "x3 V": read as the pre-softmax core inside, and the nH x r~3 result
    still goes through the post-softmax core and U~2 as in the definition;
  * the decoded token is the last row of the cache: cache length L includes it,
    its position is L-1 and it attends rows 0..L-1;
  * the cache stores rotated keys and unrotated values;
  * a batch is B independent sequences, positions start at pos0 in each.
"""
from __future__ import annotations

import math
from typing import Dict, Optional, Sequence

import numpy as np

F64 = np.float64


def _f64(a):
    return np.asarray(a, dtype=F64)


# ---------------------------------------------------------------------------------------
# Rotary embedding in the latent key space (Section "Rotary Position Embedding")
# ---------------------------------------------------------------------------------------

def rope_frequencies(r: int, base: float) -> np.ndarray:
    """theta_j = base**(-2j/r), j = 0 .. r/2-1."""
    if r % 2:
        raise ValueError("RoPE needs an even width")
    j = np.arange(r // 2, dtype=F64)
    return np.power(F64(base), -2.0 * j / F64(r))


def rope_matrix(p: int, r: int, base: float) -> np.ndarray:
    """Dense r x r matrix R(p, r) acting on ROW vectors: x' = x @ R."""
    ang = F64(p) * rope_frequencies(r, base)
    R = np.zeros((r, r), dtype=F64)
    for j in range(r // 2):
        c, s = math.cos(ang[j]), math.sin(ang[j])
        R[2 * j, 2 * j] = c
        R[2 * j + 1, 2 * j] = -s
        R[2 * j, 2 * j + 1] = s
        R[2 * j + 1, 2 * j + 1] = c
    return R


def rope_rotate(x: np.ndarray, positions: np.ndarray, base: float) -> np.ndarray:
    """Rotate each row x[..., t, :] by its position: pairwise form of x @ R(p)."""
    x = _f64(x)
    r = x.shape[-1]
    ang = _f64(positions)[:, None] * rope_frequencies(r, base)[None, :]      # [T, r/2]
    c, s = np.cos(ang), np.sin(ang)
    even, odd = x[..., 0::2], x[..., 1::2]
    out = np.empty_like(x)
    out[..., 0::2] = even * c - odd * s
    out[..., 1::2] = even * s + odd * c
    return out


# ---------------------------------------------------------------------------------------
# Tucker representation (Definition "Tucker Attention")
# ---------------------------------------------------------------------------------------

def tucker_tensor(C, U1, U2, U3) -> np.ndarray:
    """W[i,j,k] = sum_{a,b,c} C[a,b,c] U1[i,a] U2[j,b] U3[k,c]  (C x1 U1 x2 U2 x3 U3)."""
    return np.einsum("abc,ia,jb,kc->ijk", _f64(C), _f64(U1), _f64(U2), _f64(U3), optimize=True)


def head_mixed_core(C, U1) -> np.ndarray:
    """G[i] = sum_a U1[i,a] C[a,:,:]  (C x1 U1), shape [nH, r2, r3]."""
    return np.einsum("ia,abc->ibc", _f64(U1), _f64(C))


def softmax_rows(S: np.ndarray) -> np.ndarray:
    """Row-wise softmax with max subtraction; -inf entries get weight 0."""
    m = np.max(S, axis=-1, keepdims=True)
    E = np.exp(S - m)
    return E / np.sum(E, axis=-1, keepdims=True)


def _visible(q_pos: np.ndarray, k_pos: np.ndarray, causal: bool) -> np.ndarray:
    if not causal:
        return np.ones((q_pos.size, k_pos.size), dtype=bool)
    return k_pos[None, :] <= q_pos[:, None]


# ---------------------------------------------------------------------------------------
# Form 1: the dense definition (tiny shapes)
# ---------------------------------------------------------------------------------------

def dense_definition_forward(X, wts: Dict[str, np.ndarray], d_head: int, causal: bool,
                             rope_base: Optional[float] = None, pos0: int = 0) -> np.ndarray:
    """Y[b] from H1/H2 and the head-and-sequence contraction, one sequence at a time.

    Without RoPE the pre-softmax scores are X W_i X^T with the materialised W.  With
    latent RoPE the bilinear form depends on the two positions, so each score is
    evaluated literally as  (X_m U2 G_i) R(m) R(n)^T (X_n U3)^T  with dense rotation
    matrices (Definition "Latent RoPE for Tucker Attention").
    """
    X = _f64(X)
    B, N, d = X.shape
    U2, U3 = _f64(wts["U2"]), _f64(wts["U3"])
    Wt = tucker_tensor(wts["Ct"], wts["Ut1"], wts["Ut2"], wts["Ut3"])     # [nH, d(out), d(value)]
    nH = Wt.shape[0]
    scale = 1.0 / math.sqrt(d_head)
    pos = pos0 + np.arange(N)
    vis = _visible(pos, pos, causal)
    Y = np.zeros((B, N, d), dtype=F64)
    if rope_base is None:
        W = tucker_tensor(wts["C"], wts["U1"], wts["U2"], wts["U3"])      # [nH, d(query), d(key)]
    else:
        G = head_mixed_core(wts["C"], wts["U1"])
        r3 = U3.shape[1]
        Rs = [rope_matrix(int(p), r3, rope_base) for p in pos]
    for b in range(B):
        x = X[b]
        H2 = np.einsum("ikv,lv->ikl", Wt, x)                               # [nH, d, N]
        for i in range(nH):
            if rope_base is None:
                S = x @ W[i] @ x.T
            else:
                qh = x @ U2 @ G[i]                                          # [N, r3]
                kk = x @ U3                                                 # [N, r3]
                S = np.empty((N, N), dtype=F64)
                for m in range(N):
                    for n in range(N):
                        S[m, n] = qh[m] @ Rs[m] @ Rs[n].T @ kk[n]
            S = np.where(vis, S * scale, -np.inf)
            H1 = softmax_rows(S)                                            # [N(j), N(l)]
            Y[b] += np.einsum("jl,kl->jk", H1, H2[i])
    return Y


# ---------------------------------------------------------------------------------------
# Form 2: per-head weights + textbook attention (all sizes)
# ---------------------------------------------------------------------------------------

def per_head_weights(wts: Dict[str, np.ndarray]):
    """WQ[i] = U2 G_i  [nH,d,r3];  WK = U3;  WV = U~3;  WO[i][c,k] = sum_b G~_i[b,c] U~2[k,b]."""
    G = head_mixed_core(wts["C"], wts["U1"])                               # [nH, r2, r3]
    Gt = head_mixed_core(wts["Ct"], wts["Ut1"])                            # [nH, rt2, rt3]
    WQ = np.einsum("jb,ibc->ijc", _f64(wts["U2"]), G)
    WO = np.einsum("ibc,kb->ick", Gt, _f64(wts["Ut2"]))
    return WQ, _f64(wts["U3"]), _f64(wts["Ut3"]), WO


def latent_kv(X, wts, rope_base: Optional[float], pos0: int = 0):
    """What the cache stores for each sequence: rotated keys X U3 R(pos) and values X U~3."""
    X = _f64(X)
    B, N, _ = X.shape
    K = X @ _f64(wts["U3"])
    V = X @ _f64(wts["Ut3"])
    if rope_base is not None:
        K = rope_rotate(K, pos0 + np.arange(N), rope_base)
    return K, V


def per_head_forward(X, wts: Dict[str, np.ndarray], d_head: int, causal: bool,
                     rope_base: Optional[float] = None, pos0: int = 0,
                     rows: Optional[Sequence[int]] = None,
                     batches: Optional[Sequence[int]] = None) -> np.ndarray:
    """Y[b, rows, :] via per-head textbook attention.

    rows / batches select which query tokens / sequences are evaluated (all by default);
    every selected row still attends the whole sequence, so a sampled row equals the same
    row of the full result.
    """
    X = _f64(X)
    B, N, d = X.shape
    WQ, WK, WV, WO = per_head_weights(wts)
    nH = WQ.shape[0]
    rows = np.arange(N) if rows is None else np.asarray(rows, dtype=np.int64)
    batches = range(B) if batches is None else batches
    scale = 1.0 / math.sqrt(d_head)
    k_pos = pos0 + np.arange(N)
    q_pos = pos0 + rows
    vis = _visible(q_pos, k_pos, causal)
    Y = np.zeros((len(batches), rows.size, d), dtype=F64)
    for bi, b in enumerate(batches):
        x = X[b]
        K = x @ WK
        V = x @ WV
        if rope_base is not None:
            K = rope_rotate(K, k_pos, rope_base)
        for i in range(nH):
            Q = x[rows] @ WQ[i]
            if rope_base is not None:
                Q = rope_rotate(Q, q_pos, rope_base)
            S = np.where(vis, (Q @ K.T) * scale, -np.inf)
            P = softmax_rows(S)
            Y[bi] += (P @ V) @ WO[i]
    return Y


def decode_step(x, Kcache, Vcache, kv_len, wts: Dict[str, np.ndarray], d_head: int,
                rope_base: Optional[float] = None):
    """One generated token per sequence against a latent KV cache (Section "KV Caching").

    x [B,d]; Kcache/Vcache [B,Lmax,r3]/[B,Lmax,rt3]; kv_len[b] = cache length INCLUDING
    the new token.  Row kv_len[b]-1 of the caches is (over)written from x[b] (rotated key,
    plain value); the query sits at position kv_len[b]-1 and attends rows 0..kv_len[b]-1.
    Returns (y [B,d], Kcache_new, Vcache_new) as fp64 copies.
    """
    x = _f64(x)
    Kc = _f64(Kcache).copy()
    Vc = _f64(Vcache).copy()
    WQ, WK, WV, WO = per_head_weights(wts)
    nH = WQ.shape[0]
    B, d = x.shape
    scale = 1.0 / math.sqrt(d_head)
    y = np.zeros((B, d), dtype=F64)
    for b in range(B):
        L = int(kv_len[b])
        p = np.array([L - 1])
        k_new = x[b:b + 1] @ WK
        if rope_base is not None:
            k_new = rope_rotate(k_new, p, rope_base)
        Kc[b, L - 1] = k_new[0]
        Vc[b, L - 1] = (x[b:b + 1] @ WV)[0]
        K, V = Kc[b, :L], Vc[b, :L]
        for i in range(nH):
            q = x[b:b + 1] @ WQ[i]
            if rope_base is not None:
                q = rope_rotate(q, p, rope_base)
            P = softmax_rows((q @ K.T) * scale)
            y[b] += ((P @ V) @ WO[i])[0]
    return y, Kc, Vc


def decode_step_shared_kv(x, Lcache, kv_len, wts: Dict[str, np.ndarray], d_head: int,
                          rope_base: Optional[float] = None):
    """Decode with the shared key-value down-projection of Section "KV Caching": keys and values
    are both the latent L = X U3, so ONE cache of N*r3 numbers is kept.  Because latent RoPE
    rotates keys but never values, the cache holds the UNROTATED latent; the key of row n is its
    rotation to position n, formed when the row is read.  The value basis of wts is not used.

    x [B,d]; Lcache [B,Lmax,r3]; kv_len[b] includes the new token, whose latent is written to
    row kv_len[b]-1.  Returns (y [B,d], Lcache_new) as fp64 copies.
    """
    x = _f64(x)
    Lc = _f64(Lcache).copy()
    WQ, WK, _, WO = per_head_weights(wts)
    nH = WQ.shape[0]
    B, d = x.shape
    scale = 1.0 / math.sqrt(d_head)
    y = np.zeros((B, d), dtype=F64)
    for b in range(B):
        L = int(kv_len[b])
        Lc[b, L - 1] = (x[b:b + 1] @ WK)[0]
        V = Lc[b, :L]
        K = V if rope_base is None else rope_rotate(V, np.arange(L), rope_base)
        p = np.array([L - 1])
        for i in range(nH):
            q = x[b:b + 1] @ WQ[i]
            if rope_base is not None:
                q = rope_rotate(q, p, rope_base)
            P = softmax_rows((q @ K.T) * scale)
            y[b] += ((P @ V) @ WO[i])[0]
    return y, Lc


def relative_l2(a, b) -> float:
    """||a - b||_2 / ||b||_2 over all elements (b is the reference)."""
    a, b = _f64(a), _f64(b)
    return float(np.linalg.norm((a - b).ravel()) / np.linalg.norm(b.ravel()))


def relative_l2_rows(a, b, floor=None):
    """Per-row version of relative_l2: ||a[r] - b[r]||_2 / max(||b[r]||_2, floor) for every vector r
    along the last axis.  `floor` (default: a hundredth of the root-mean-square row norm of b) keeps a
    reference row that is zero or tiny from turning rounding noise into a large ratio."""
    a, b = _f64(a), _f64(b)
    num = np.linalg.norm(a - b, axis=-1)
    den = np.linalg.norm(b, axis=-1)
    if floor is None:
        floor = 0.01 * math.sqrt(float(np.mean(den ** 2))) if den.size else 0.0
    return num / np.maximum(np.maximum(den, floor), np.finfo(F64).tiny)
