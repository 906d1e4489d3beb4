"""CPU oracle for the gradients of the Tucker-attention layer (TEST INFRASTRUCTURE ONLY).

The paper trains the layer (its timing tables carry a backward column next to the forward
one) but prints no gradient formulas: the backward pass is the derivative of the forward pass
of Definition "Tucker Attention" with latent RoPE, and has a plain definition.  This file
writes that derivative out by the chain rule, one sequence and one head at a time, with full
N x N score matrices in fp64:

    loss = sum(dY * Y(X, C, U1, U2, U3, C~, U~1, U~2, U~3))

and returns d loss / d (each argument).  Nothing here is blocked, fused or recomputed in
tiles; the product path may not import it.

Steps of the forward pass, in the notation of `tucker_oracle.per_head_forward`:
    Ql = X U2                 Kl = X U3              Vl = X U~3  (Vl = Kl with a shared latent)
    Qh_i = Ql G_i             G_i = sum_a U1[i,a] C[a]
    Q_i = rope(Qh_i)          K = rope(Kl)           (rotation by position, row vectors)
    P_i = softmax(mask(Q_i K^T / sqrt(dH)))
    O_i = P_i Vl              Z = sum_i O_i G~_i^T   G~_i = sum_a U~1[i,a] C~[a]
    Y = Z U~2^T
Each is differentiated in reverse order below.  The rotation is orthogonal, so its
derivative is the rotation by the negated angle.

With a shared key-value latent (Section "KV Caching") the value basis is the key basis: the
gradient of U3 collects the key path and the value path, and no gradient of U~3 exists.

Pins (tests/test_oracle_backward_pins.py): central finite differences of the independently
pinned forward oracle for every returned array, directional derivatives at larger sizes,
linearity in dY, the tied-weights identity for the shared latent, and the closed form of a
one-token sequence (softmax of one score is constant, so the layer is linear in X).
"""
from __future__ import annotations

import math
from typing import Dict, Optional

import numpy as np

from .tucker_oracle import _f64, _visible, head_mixed_core, rope_rotate, softmax_rows

F64 = np.float64


def _unrotate(x: np.ndarray, positions: np.ndarray, base: Optional[float]) -> np.ndarray:
    """Derivative of rope_rotate with respect to its input, applied to a cotangent: the
    transpose of an orthogonal block rotation is the rotation by the negated angle."""
    if base is None:
        return x
    return rope_rotate(x, -_f64(positions), base)


def backward(X, dY, wts: Dict[str, np.ndarray], d_head: int, causal: bool,
             rope_base: Optional[float] = None, pos0: int = 0,
             shared_kv: bool = False, return_mixed: bool = False) -> Dict[str, np.ndarray]:
    """Gradients of sum(dY * Y) for X [B,N,d] and every weight array.

    Returns a dict with keys dX, dC, dU1, dU2, dU3, dCt, dUt1, dUt2 and, unless the latent is
    shared, dUt3.  All fp64.  return_mixed adds dG and dGt, the gradients of the head-mixed cores
    G_i = sum_a U1[i,a] C[a] and G~_i, from which dC, dU1, dCt, dUt1 are contracted.
    """
    X, dY = _f64(X), _f64(dY)
    B, N, d = X.shape
    C, U1, U2, U3 = (_f64(wts[k]) for k in ("C", "U1", "U2", "U3"))
    Ct, Ut1, Ut2 = (_f64(wts[k]) for k in ("Ct", "Ut1", "Ut2"))
    Ut3 = U3 if shared_kv else _f64(wts["Ut3"])
    G = head_mixed_core(C, U1)                                   # [nH, r2, r3]
    Gt = head_mixed_core(Ct, Ut1)                                # [nH, rt2, rt3]
    nH = G.shape[0]
    scale = 1.0 / math.sqrt(d_head)
    pos = pos0 + np.arange(N)
    vis = _visible(pos, pos, causal)

    dX = np.zeros_like(X)
    dG, dGt = np.zeros_like(G), np.zeros_like(Gt)
    dU2, dU3, dUt2, dUt3 = np.zeros_like(U2), np.zeros_like(U3), np.zeros_like(Ut2), np.zeros_like(Ut3)

    for b in range(B):
        x = X[b]
        Ql, Kl, Vl = x @ U2, x @ U3, x @ Ut3
        K = Kl if rope_base is None else rope_rotate(Kl, pos, rope_base)

        # forward once more, keeping what the derivative needs
        P, O = [], []
        Z = np.zeros((N, Gt.shape[1]), dtype=F64)
        for i in range(nH):
            Qh = Ql @ G[i]
            Q = Qh if rope_base is None else rope_rotate(Qh, pos, rope_base)
            S = np.where(vis, (Q @ K.T) * scale, -np.inf)
            P.append(softmax_rows(S))
            O.append(P[i] @ Vl)
            Z += O[i] @ Gt[i].T

        # Y = Z U~2^T
        dZ = dY[b] @ Ut2                                          # [N, rt2]
        dUt2 += dY[b].T @ Z
        dQl = np.zeros_like(Ql)
        dK = np.zeros_like(K)
        dVl = np.zeros_like(Vl)
        for i in range(nH):
            # Z = sum_i O_i G~_i^T
            dO = dZ @ Gt[i]                                       # [N, rt3]
            dGt[i] += dZ.T @ O[i]
            # O_i = P_i Vl
            dP = dO @ Vl.T
            dVl += P[i].T @ dO
            # P_i = softmax(S_i): dS = P * (dP - rowsum(dP * P)); masked entries have P = 0
            dS = P[i] * (dP - np.sum(dP * P[i], axis=1, keepdims=True))
            # S_i = scale * Q_i K^T
            Qh = Ql @ G[i]
            Q = Qh if rope_base is None else rope_rotate(Qh, pos, rope_base)
            dQ = scale * (dS @ K)
            dK += scale * (dS.T @ Q)
            # Q_i = rope(Qh_i),  Qh_i = Ql G_i
            dQh = _unrotate(dQ, pos, rope_base)
            dQl += dQh @ G[i].T
            dG[i] += Ql.T @ dQh
        dKl = _unrotate(dK, pos, rope_base)
        # Ql = x U2, Kl = x U3, Vl = x U~3
        dX[b] = dQl @ U2.T + dKl @ U3.T + dVl @ Ut3.T
        dU2 += x.T @ dQl
        dU3 += x.T @ dKl
        if shared_kv:
            dU3 += x.T @ dVl
        else:
            dUt3 += x.T @ dVl

    # G_i = sum_a U1[i,a] C[a]  and the same for the post-softmax core
    out = {
        "dX": dX,
        "dC": np.einsum("ia,ibc->abc", U1, dG),
        "dU1": np.einsum("ibc,abc->ia", dG, C),
        "dU2": dU2,
        "dU3": dU3,
        "dCt": np.einsum("ia,ibc->abc", Ut1, dGt),
        "dUt1": np.einsum("ibc,abc->ia", dGt, Ct),
        "dUt2": dUt2,
    }
    if not shared_kv:
        out["dUt3"] = dUt3
    if return_mixed:
        out["dG"], out["dGt"] = dG, dGt
    return out


def head_factor_cancellation(dG, C) -> float:
    """How much the head-factor gradient dU1[i,a] = sum_bc dG[i,b,c] C[a,b,c] cancels: the norm of the sums
    of absolute terms over the norm of the sums themselves (1 = no cancellation).  A relative perturbation
    eps of the terms moves the result by up to eps times this factor, relative to its own size."""
    dG, C = _f64(dG), _f64(C)
    val = np.einsum("ibc,abc->ia", dG, C)
    mag = np.einsum("ibc,abc->ia", np.abs(dG), np.abs(C))
    return float(np.linalg.norm(mag) / np.linalg.norm(val))
