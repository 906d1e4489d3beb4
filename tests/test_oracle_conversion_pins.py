"""Pins for the conversion oracle (classic attention weights -> Tucker weights).  The exact
representations are checked against brute-force MHA / GQA / MLA written separately; the truncated
higher-order SVD against planted decompositions, closed forms and the error bounds of the
decomposition.  All CPU, fp64, small."""
import math

import numpy as np
import pytest

from oracle import classic_attention as ca
from oracle import conversions as cv
from oracle import tucker_oracle as orc

RNG = np.random.default_rng


def close(a, b, tol=1e-10):
    assert np.max(np.abs(np.asarray(a) - np.asarray(b))) <= tol * max(1.0, float(np.max(np.abs(b))))


def mha_weights(rng, d, nH, dH):
    n = nH * dH
    return (rng.standard_normal((d, n)), rng.standard_normal((d, n)), rng.standard_normal((d, n)),
            rng.standard_normal((n, d)))


def orthonormal(rng, m, r):
    q, _ = np.linalg.qr(rng.standard_normal((m, r)))
    return q


# ---- exact representations -----------------------------------------------------------------------

@pytest.mark.parametrize("nG", [4, 2, 1])
def test_gqa_front_end_reproduces_grouped_query_attention(nG):
    rng = RNG(41)
    d, nH, dH, N = 10, 4, 3, 7
    WQ, WO = rng.standard_normal((d, nH * dH)), rng.standard_normal((nH * dH, d))
    WK, WV = rng.standard_normal((d, nG * dH)), rng.standard_normal((d, nG * dH))
    X = rng.standard_normal((1, N, d))
    w = cv.gqa_to_tucker(WQ, WK, WV, WO, nH, nG)
    assert w["C"].shape == (nH, nH * dH, nG * dH) and w["Ut2"].shape == (d, nH * dH)
    close(orc.per_head_forward(X, w, dH, True)[0], ca.gqa_reference(X[0], WQ, WK, WV, WO, nH, nG, causal=True))
    # the Tucker tensors are the stacked per-head products themselves
    per = nH // nG
    W = orc.tucker_tensor(w["C"], w["U1"], w["U2"], w["U3"])
    Wt = orc.tucker_tensor(w["Ct"], w["Ut1"], w["Ut2"], w["Ut3"])
    for i in range(nH):
        q, g = slice(i * dH, (i + 1) * dH), slice((i // per) * dH, (i // per + 1) * dH)
        close(W[i], WQ[:, q] @ WK[:, g].T)
        close(Wt[i], (WV[:, g] @ WO[q, :]).T)


@pytest.mark.parametrize("shared", [False, True])
def test_mla_front_end_reproduces_latent_attention(shared):
    rng = RNG(42)
    d, nH, dH, N, dcq, dck = 9, 3, 4, 6, 5, 4
    WDQ, WUQ = rng.standard_normal((d, dcq)), rng.standard_normal((dcq, nH * dH))
    WDKV, WUK = rng.standard_normal((d, dck)), rng.standard_normal((dck, nH * dH))
    WDV = None if shared else rng.standard_normal((d, dck))
    WUV, WO = rng.standard_normal((dck, nH * dH)), rng.standard_normal((nH * dH, d))
    X = rng.standard_normal((1, N, d))
    w = cv.mla_to_tucker(WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, nH)
    assert ("Ut3" in w) == (not shared)
    full = dict(w, Ut3=w["U3"]) if shared else w
    ref = ca.mla_reference(X[0], WDQ, WUQ, WDKV, WUK, WDKV if shared else WDV, WUV, WO, nH, causal=True)
    close(orc.per_head_forward(X, full, dH, True)[0], ref)


def test_mla_front_end_with_latent_rope_is_the_coupled_rope_form():
    # scores written out from the coupled-RoPE equation with dense rotation matrices, token pair by
    # token pair: x_m WDQ (WUQ_i WUK_i^T) R(m) R(n)^T WDKV^T x_n
    rng = RNG(43)
    d, nH, dH, N, dcq, dck, base = 6, 2, 3, 5, 4, 4, 30.0
    WDQ, WUQ = rng.standard_normal((d, dcq)), rng.standard_normal((dcq, nH * dH))
    WDKV, WUK = rng.standard_normal((d, dck)), rng.standard_normal((dck, nH * dH))
    WUV, WO = rng.standard_normal((dck, nH * dH)), rng.standard_normal((nH * dH, d))
    X = rng.standard_normal((1, N, d))
    w = cv.mla_to_tucker(WDQ, WUQ, WDKV, WUK, None, WUV, WO, nH)
    got = orc.per_head_forward(X, dict(w, Ut3=w["U3"]), dH, True, rope_base=base)[0]
    x = X[0]
    Y = np.zeros((N, d))
    for i in range(nH):
        sl = slice(i * dH, (i + 1) * dH)
        fused = WDQ @ WUQ[:, sl] @ WUK[:, sl].T                              # [d, dck]
        for m in range(N):
            s = np.array([x[m] @ fused @ orc.rope_matrix(m, dck, base) @ orc.rope_matrix(n, dck, base).T
                          @ WDKV.T @ x[n] for n in range(m + 1)]) / math.sqrt(dH)
            p = np.exp(s - s.max())
            p /= p.sum()
            for n in range(m + 1):
                Y[m] += p[n] * (x[n] @ WDKV @ WUV[:, sl] @ WO[sl, :])
    close(got, Y)


# ---- truncated higher-order SVD ------------------------------------------------------------------

def test_sign_convention():
    U = np.array([[0.1, -0.2], [-0.9, 0.2], [0.3, 0.1]])
    F = cv.fix_signs(U)
    close(F[:, 0], -U[:, 0])
    close(F[:, 1], -U[:, 1])                    # tie between rows 0 and 1: the first decides
    assert F[1, 0] > 0 and F[0, 1] > 0


def test_unfoldings_index_the_right_modes():
    T = np.arange(24, dtype=float).reshape(2, 3, 4)
    assert cv.unfold(T, 0).shape == (2, 12) and cv.unfold(T, 1).shape == (3, 8) and cv.unfold(T, 2).shape == (4, 6)
    for k in range(3):
        M = cv.unfold(T, k)
        for j in range(T.shape[k]):
            assert sorted(M[j]) == sorted(np.take(T, j, axis=k).ravel())


def test_full_ranks_are_exact_and_the_core_is_all_orthogonal():
    rng = RNG(44)
    T = rng.standard_normal((3, 5, 4))
    C, U1, U2, U3, sv = cv.hosvd(T, (3, 5, 4))
    close(orc.tucker_tensor(C, U1, U2, U3), T, 1e-12)
    for k, U in enumerate((U1, U2, U3)):
        close(U.T @ U, np.eye(U.shape[1]), 1e-12)
        G = cv.unfold(C, k) @ cv.unfold(C, k).T                     # slices of the core are orthogonal,
        close(G, np.diag(sv[k] ** 2), 1e-10)                         # their norms the singular values, ordered
        assert np.all(np.diff(sv[k]) <= 0)


def test_a_planted_tucker_tensor_is_recovered_at_its_own_ranks():
    rng = RNG(45)
    nH, d, r = 4, 12, (2, 5, 3)
    P1, P2, P3 = orthonormal(rng, nH, r[0]), orthonormal(rng, d, r[1]), orthonormal(rng, d, r[2])
    core = rng.standard_normal(r)
    T = orc.tucker_tensor(core, P1, P2, P3)
    C, U1, U2, U3, _ = cv.hosvd(T, r)
    close(orc.tucker_tensor(C, U1, U2, U3), T, 1e-12)
    for U, P in ((U1, P1), (U2, P2), (U3, P3)):
        close(U @ U.T, P @ P.T, 1e-12)                                # same subspace


def test_one_head_reduces_to_a_planted_matrix_svd():
    # nH = 1: the tensor is one matrix P diag(s) Q^T; its higher-order SVD at rank (1, r, r) is the
    # truncated SVD (factors = leading columns of P and Q up to sign, core = diag(s))
    rng = RNG(46)
    d, r = 9, 4
    P, Q = orthonormal(rng, d, d), orthonormal(rng, d, d)
    s = np.array([9.0, 7.5, 5.0, 3.0, 2.0, 1.0, 0.5, 0.2, 0.1])
    T = (P * s) @ Q.T
    C, U1, U2, U3, sv = cv.hosvd(T[None], (1, r, r))
    close(np.abs(U1), [[1.0]])
    close(sv[1], s, 1e-12)
    close(sv[2], s, 1e-12)
    close(U2, cv.fix_signs(P[:, :r]), 1e-10)
    close(U3, cv.fix_signs(Q[:, :r]), 1e-10)
    close(np.abs(C[0]), np.diag(s[:r]), 1e-10)
    # Eckart-Young: the error of the truncation is the tail of the spectrum
    err = np.linalg.norm(orc.tucker_tensor(C, U1, U2, U3)[0] - T)
    close(err, math.sqrt(np.sum(s[r:] ** 2)), 1e-10)


def test_rank_one_closed_form():
    a, b, c = np.array([3.0, -4.0]), np.array([1.0, 2.0, -2.0]), np.array([0.0, -5.0, 12.0, 0.0])
    T = np.einsum("i,j,k->ijk", a, b, c)
    C, U1, U2, U3, _ = cv.hosvd(T, (1, 1, 1))
    close(U1[:, 0], [-0.6, 0.8])                                   # largest entry positive
    close(U2[:, 0], [1 / 3, 2 / 3, -2 / 3])                        # tie of magnitude: the first decides
    close(U3[:, 0], [0.0, -5 / 13, 12 / 13, 0.0])
    close(C, [[[-5.0 * 3.0 * 13.0]]])


def test_truncation_error_lies_between_the_bounds_of_the_decomposition():
    rng = RNG(47)
    WQ, WK, WV, WO = mha_weights(rng, 10, 3, 4)
    W, _ = cv.attention_tensors(WQ, WK, WV, WO, 3)
    ranks = (2, 6, 5)
    C, U1, U2, U3, sv = cv.hosvd(W, ranks)
    err2 = np.sum((orc.tucker_tensor(C, U1, U2, U3) - W) ** 2)
    tails = [np.sum(sv[k][ranks[k]:] ** 2) for k in range(3)]
    assert max(tails) * (1 - 1e-12) <= err2 <= sum(tails) * (1 + 1e-12)


def test_attention_tensors_follow_the_stacking_of_the_paper():
    rng = RNG(48)
    d, nH, dH = 6, 2, 3
    WQ, WK, WV, WO = mha_weights(rng, d, nH, dH)
    W, Wt = cv.attention_tensors(WQ, WK, WV, WO, nH)
    X = rng.standard_normal((4, d))
    # layer through the dense bilinear forms equals brute-force MHA: fixes the orientation of both tensors
    close(ca.bilinear_attention_reference(X, W, Wt, dH, causal=True), ca.mha_reference(X, WQ, WK, WV, WO, nH, True))


@pytest.mark.parametrize("shared", [False, True])
def test_conversion_at_full_ranks_reproduces_multi_head_attention(shared):
    rng = RNG(49)
    d, nH, dH, N = 8, 2, 4, 6
    WQ, WK, WV, WO = mha_weights(rng, d, nH, dH)
    X = rng.standard_normal((1, N, d))
    w = cv.mha_to_tucker_hosvd(WQ, WK, WV, WO, nH, (nH, d, d), (nH, d, d), shared_kv=shared)
    assert ("Ut3" in w) == (not shared)
    full = dict(w, Ut3=w["U3"]) if shared else w
    close(orc.per_head_forward(X, full, dH, True)[0], ca.mha_reference(X[0], WQ, WK, WV, WO, nH, True), 1e-9)


def test_shared_latent_is_exact_when_values_live_in_the_key_space():
    # WV_i = P R_i with P the span of all key matrices: the value mode of W~ lies inside the span of U3
    rng = RNG(50)
    d, nH, dH, r3 = 10, 2, 3, 5
    P = orthonormal(rng, d, r3)
    WK = P @ rng.standard_normal((r3, nH * dH))
    WV = P @ rng.standard_normal((r3, nH * dH))
    WQ, WO = rng.standard_normal((d, nH * dH)), rng.standard_normal((nH * dH, d))
    w = cv.mha_to_tucker_hosvd(WQ, WK, WV, WO, nH, (nH, nH * dH, r3), (nH, nH * dH, r3), shared_kv=True)
    W, Wt = cv.attention_tensors(WQ, WK, WV, WO, nH)
    close(w["U3"] @ w["U3"].T, P @ P.T, 1e-10)
    close(orc.tucker_tensor(w["C"], w["U1"], w["U2"], w["U3"]), W, 1e-10)
    close(orc.tucker_tensor(w["Ct"], w["Ut1"], w["Ut2"], w["U3"]), Wt, 1e-10)
    with pytest.raises(ValueError):
        cv.mha_to_tucker_hosvd(WQ, WK, WV, WO, nH, (1, 2, 3), (1, 2, 4), shared_kv=True)
