"""Brute-force MHA / GQA / MLA references (TEST INFRASTRUCTURE ONLY).

Written separately from tucker_oracle (own softmax, explicit per-head loops, no
shared helper) so that the special cases the paper proves -- MHA, GQA/MQA and
MLA are Tucker attention with particular cores and factors (Section "MQA, GQA
and MLA are special cases", Lemma/Theorems of the appendix "Tucker
Representations of MQA, GQA, and MLA") -- pin the oracle against something other
than itself.  fp64, tiny inputs.
"""
from __future__ import annotations

import math

import numpy as np
from scipy.special import softmax as _scipy_softmax


def _attend(Q, K, V, d_head, causal):
    N = Q.shape[0]
    S = (Q @ K.T) / math.sqrt(d_head)
    if causal:
        for m in range(N):
            S[m, m + 1:] = -np.inf
    return _scipy_softmax(S, axis=1) @ V


def mha_reference(X, WQ, WK, WV, WO, n_heads, causal=False):
    """MHA(X) = sum_i softmax(X WQ_i (X WK_i)^T / sqrt(dH)) X WV_i WO_i  (the head formula).

    X [N,d]; WQ, WK, WV [d, nH*dH] with head i in columns i*dH..(i+1)*dH-1; WO [nH*dH, d]
    with head i in the matching rows.
    """
    X = np.asarray(X, dtype=np.float64)
    dH = WQ.shape[1] // n_heads
    Y = np.zeros((X.shape[0], WO.shape[1]))
    for i in range(n_heads):
        sl = slice(i * dH, (i + 1) * dH)
        head = _attend(X @ WQ[:, sl], X @ WK[:, sl], X @ WV[:, sl], dH, causal)
        Y += head @ WO[sl, :]
    return Y


def gqa_reference(X, WQ, WKg, WVg, WO, n_heads, n_groups, causal=False):
    """GQA: query head i uses KV head g(i) = i // (nH / nG).  WKg, WVg [d, nG*dH]."""
    X = np.asarray(X, dtype=np.float64)
    dH = WQ.shape[1] // n_heads
    per = n_heads // n_groups
    Y = np.zeros((X.shape[0], WO.shape[1]))
    for i in range(n_heads):
        g = i // per
        q = slice(i * dH, (i + 1) * dH)
        kv = slice(g * dH, (g + 1) * dH)
        head = _attend(X @ WQ[:, q], X @ WKg[:, kv], X @ WVg[:, kv], dH, causal)
        Y += head @ WO[q, :]
    return Y


def mla_reference(X, WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, n_heads, causal=False):
    """MLA without positional encoding.

    Queries  X WDQ WUQ_i        (WDQ [d,dcQ], WUQ [dcQ, nH*dH]),
    keys     X WDKV WUK_i       (WDKV [d,dcK], WUK [dcK, nH*dH]),
    values   X WDV WUV_i        (WDV [d,dcK] -- pass WDKV for the shared-KV variant --
                                 WUV [dcK, nH*dH]),
    output   full-rank WO [nH*dH, d].
    """
    X = np.asarray(X, dtype=np.float64)
    dH = WUQ.shape[1] // n_heads
    cq = X @ WDQ
    ckv = X @ WDKV
    cv = X @ WDV
    Y = np.zeros((X.shape[0], WO.shape[1]))
    for i in range(n_heads):
        sl = slice(i * dH, (i + 1) * dH)
        head = _attend(cq @ WUQ[:, sl], ckv @ WUK[:, sl], cv @ WUV[:, sl], dH, causal)
        Y += head @ WO[sl, :]
    return Y


def bilinear_attention_reference(X, W, Wt, d_head, causal=False):
    """Attention with arbitrary per-head d x d forms, element by element.

    Y[j,k] = sum_i sum_l softmax_l( x_j W_i x_l^T / sqrt(dH) ) * (Wt_i x_l)[k],
    W, Wt [nH,d,d], Wt_i maps a value-side token to the output (output index first).
    Pure Python loops: only for very small N, d.
    """
    X = np.asarray(X, dtype=np.float64)
    N, d = X.shape
    nH = W.shape[0]
    Y = np.zeros((N, d))
    for i in range(nH):
        for j in range(N):
            last = j if causal else N - 1
            s = [float(X[j] @ W[i] @ X[l]) / math.sqrt(d_head) for l in range(last + 1)]
            mx = max(s)
            e = [math.exp(v - mx) for v in s]
            z = sum(e)
            for l in range(last + 1):
                Y[j] += (e[l] / z) * (Wt[i] @ X[l])
    return Y
