"""Pins for the gradient oracle: it is checked against derivatives of the forward oracle (which is
pinned on its own against the paper's definitions and special cases) taken by brute force, and
against closed forms.  All CPU, fp64, tiny."""
import math

import numpy as np
import pytest

from oracle import tucker_backward as bwd
from oracle import tucker_oracle as orc

RNG = np.random.default_rng

KEYS = ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")


def rand_weights(rng, d, nH, r, rt=None):
    r1, r2, r3 = r
    t1, t2, t3 = rt or r
    g = lambda *s: rng.standard_normal(s)
    return dict(C=g(r1, r2, r3) / math.sqrt(r2), U1=g(nH, r1), U2=g(d, r2) / math.sqrt(d), U3=g(d, r3) / math.sqrt(d),
                Ct=g(t1, t2, t3) / math.sqrt(t3), Ut1=g(nH, t1), Ut2=g(d, t2), Ut3=g(d, t3) / math.sqrt(d))


def loss(X, w, dY, shared, **kw):
    if shared:
        w = dict(w, Ut3=w["U3"])
    return float(np.sum(dY * orc.per_head_forward(X, w, **kw)))


def finite_difference(X, w, dY, name, shared, eps=1e-6, **kw):
    """Central differences of the forward oracle, one element at a time."""
    target = X if name == "X" else w[name]
    g = np.zeros_like(target)
    it = np.nditer(target, flags=["multi_index"])
    for _ in it:
        idx = it.multi_index
        old = target[idx]
        target[idx] = old + eps
        up = loss(X, w, dY, shared, **kw)
        target[idx] = old - eps
        dn = loss(X, w, dY, shared, **kw)
        target[idx] = old
        g[idx] = (up - dn) / (2 * eps)
    return g


@pytest.mark.parametrize("causal,rope,shared", [(True, 50.0, False), (False, None, False), (True, None, True),
                                                (False, 50.0, True)])
def test_every_gradient_equals_finite_differences_of_the_forward_oracle(causal, rope, shared):
    rng = RNG(21)
    d, nH, N, B = 6, 3, 5, 2
    w = rand_weights(rng, d, nH, (2, 3, 4), (2, 5, 4))
    X = rng.standard_normal((B, N, d))
    dY = rng.standard_normal((B, N, d))
    kw = dict(d_head=3, causal=causal, rope_base=rope, pos0=2)
    g = bwd.backward(X, dY, w, shared_kv=shared, **kw)
    names = ["X"] + [k for k in KEYS if not (shared and k == "Ut3")]
    assert set(g) == {"d" + n for n in names}
    for n in names:
        fd = finite_difference(X, w, dY, n, shared, **kw)
        ref = max(1e-3, float(np.max(np.abs(fd))))
        assert np.max(np.abs(g["d" + n] - fd)) <= 2e-7 * ref, n


@pytest.mark.parametrize("shared", [False, True])
def test_directional_derivatives_at_a_larger_size(shared):
    # <grad, v> against a central difference of the loss along v, for random v in every argument
    rng = RNG(22)
    d, nH, N, B = 24, 5, 33, 2
    w = rand_weights(rng, d, nH, (3, 8, 6), (2, 10, 6))
    X = rng.standard_normal((B, N, d))
    dY = rng.standard_normal((B, N, d))
    kw = dict(d_head=8, causal=True, rope_base=1e4, pos0=0)
    g = bwd.backward(X, dY, w, shared_kv=shared, **kw)
    names = ["X"] + [k for k in KEYS if not (shared and k == "Ut3")]
    for n in names:
        for trial in range(2):
            v = rng.standard_normal(g["d" + n].shape)
            eps = 1e-5

            def at(t):
                X2 = X + t * v if n == "X" else X
                w2 = dict(w)
                if n != "X":
                    w2[n] = w[n] + t * v
                return loss(X2, w2, dY, shared, **kw)

            fd = (at(eps) - at(-eps)) / (2 * eps)
            an = float(np.sum(g["d" + n] * v))
            assert abs(an - fd) <= 1e-6 * max(1.0, abs(fd)), (n, trial, an, fd)


def test_gradients_are_linear_in_the_upstream_gradient():
    rng = RNG(23)
    d, nH, N = 8, 2, 6
    w = rand_weights(rng, d, nH, (2, 4, 4))
    X = rng.standard_normal((1, N, d))
    a, b = rng.standard_normal((1, N, d)), rng.standard_normal((1, N, d))
    kw = dict(d_head=4, causal=True, rope_base=100.0)
    ga, gb = bwd.backward(X, a, w, **kw), bwd.backward(X, b, w, **kw)
    gs = bwd.backward(X, 2.0 * a - 3.0 * b, w, **kw)
    for k in gs:
        np.testing.assert_allclose(gs[k], 2.0 * ga[k] - 3.0 * gb[k], rtol=0, atol=1e-11 * max(1.0, np.abs(gs[k]).max()))
    zero = bwd.backward(X, np.zeros_like(a), w, **kw)
    assert all(np.all(v == 0.0) for v in zero.values())


def test_shared_latent_gradient_is_the_tied_weight_sum():
    # tying U~3 to U3 adds the two untied gradients (chain rule for a repeated argument)
    rng = RNG(24)
    d, nH, N = 10, 3, 9
    w = rand_weights(rng, d, nH, (2, 4, 6), (3, 5, 6))
    w["Ut3"] = w["U3"].copy()
    X = rng.standard_normal((2, N, d))
    dY = rng.standard_normal((2, N, d))
    kw = dict(d_head=5, causal=True, rope_base=1e3, pos0=1)
    untied = bwd.backward(X, dY, w, shared_kv=False, **kw)
    tied = bwd.backward(X, dY, w, shared_kv=True, **kw)
    np.testing.assert_allclose(tied["dU3"], untied["dU3"] + untied["dUt3"], rtol=0, atol=1e-12)
    for k in tied:
        if k != "dU3":
            np.testing.assert_allclose(tied[k], untied[k], rtol=0, atol=1e-12)


def test_one_token_sequences_reduce_to_the_linear_value_path():
    # With N = 1 the softmax of the single score is 1 whatever the query and key are, so
    # Y = x U~3 (sum_i G~_i^T) U~2^T: no gradient reaches C, U1, U2, U3, and the others are the
    # gradients of that product of matrices.
    rng = RNG(25)
    d, nH, B = 7, 4, 3
    w = rand_weights(rng, d, nH, (2, 3, 4), (3, 5, 2))
    X = rng.standard_normal((B, 1, d))
    dY = rng.standard_normal((B, 1, d))
    g = bwd.backward(X, dY, w, d_head=4, causal=True, rope_base=10.0, pos0=5)
    for k in ("dC", "dU1", "dU2", "dU3"):
        assert np.max(np.abs(g[k])) <= 1e-13, k
    x, dy = X[:, 0, :], dY[:, 0, :]
    Gs = np.einsum("ia,abc->bc", w["Ut1"], w["Ct"])               # sum over heads of G~_i, [rt2, rt3]
    M = w["Ut3"] @ Gs.T @ w["Ut2"].T                               # Y = x M
    np.testing.assert_allclose(g["dX"][:, 0, :], dy @ M.T, atol=1e-12)
    np.testing.assert_allclose(g["dUt3"], x.T @ (dy @ w["Ut2"] @ Gs), atol=1e-12)
    np.testing.assert_allclose(g["dUt2"], dy.T @ (x @ w["Ut3"] @ Gs.T), atol=1e-12)
    dGs = (dy @ w["Ut2"]).T @ (x @ w["Ut3"])                      # gradient of every G~_i
    np.testing.assert_allclose(g["dCt"], np.einsum("ia,bc->abc", w["Ut1"], dGs), atol=1e-12)
    np.testing.assert_allclose(g["dUt1"], np.tile(np.einsum("bc,abc->a", dGs, w["Ct"]), (nH, 1)), atol=1e-12)


def test_causal_gradient_of_x_respects_the_mask():
    # an upstream gradient on token m alone cannot reach tokens after m
    rng = RNG(26)
    d, nH, N, m = 8, 2, 7, 3
    w = rand_weights(rng, d, nH, (2, 4, 4))
    X = rng.standard_normal((1, N, d))
    dY = np.zeros((1, N, d))
    dY[0, m] = rng.standard_normal(d)
    g = bwd.backward(X, dY, w, d_head=4, causal=True, rope_base=100.0)
    assert np.all(g["dX"][0, m + 1:] == 0.0)
    assert np.any(g["dX"][0, :m + 1] != 0.0)


def test_mixed_core_gradients_and_the_cancellation_factor():
    # identity head factors: the head-mixed core IS the core, so dG must equal dC (itself pinned by finite
    # differences above), and likewise after the softmax
    rng = RNG(27)
    d, nH, N = 6, 3, 5
    w = rand_weights(rng, d, nH, (nH, 3, 4), (nH, 5, 4))
    w["U1"], w["Ut1"] = np.eye(nH), np.eye(nH)
    X, dY = rng.standard_normal((2, N, d)), rng.standard_normal((2, N, d))
    g = bwd.backward(X, dY, w, d_head=3, causal=True, rope_base=50.0, return_mixed=True)
    assert np.allclose(g["dG"], g["dC"], rtol=0, atol=1e-12) and np.allclose(g["dGt"], g["dCt"], rtol=0, atol=1e-12)
    fd = finite_difference(X, w, dY, "C", False, d_head=3, causal=True, rope_base=50.0)
    assert np.max(np.abs(g["dG"] - fd)) <= 2e-7 * max(1e-3, float(np.max(np.abs(fd))))
    # general head factors: the returned dC / dU1 are the contractions of dG the docstring states
    w = rand_weights(rng, d, nH, (2, 3, 4), (2, 5, 4))
    g = bwd.backward(X, dY, w, d_head=3, causal=False, return_mixed=True)
    assert np.allclose(g["dU1"], np.einsum("ibc,abc->ia", g["dG"], w["C"]), rtol=0, atol=1e-12)
    assert np.allclose(g["dCt"], np.einsum("ia,ibc->abc", w["Ut1"], g["dGt"]), rtol=0, atol=1e-12)
    assert set(bwd.backward(X, dY, w, d_head=3, causal=False)) == set(g) - {"dG", "dGt"}
    # cancellation factor by hand: terms (+3, -2) -> |3| + |-2| over |3 - 2|; same-sign terms give 1
    assert bwd.head_factor_cancellation(np.array([[[3.0, 2.0]]]), np.array([[[1.0, -1.0]]])) == 5.0
    assert bwd.head_factor_cancellation(np.array([[[3.0, 2.0]]]), np.array([[[1.0, 1.0]]])) == 1.0
    two = bwd.head_factor_cancellation(np.array([[[1.0, 1.0]], [[2.0, 0.0]]]), np.array([[[1.0, -1.0]]]))
    assert abs(two - math.sqrt(2.0 ** 2 + 2.0 ** 2) / 2.0) < 1e-15           # entries (0, 2): sums of |terms| (2, 2)
