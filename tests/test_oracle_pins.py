"""Pins for the CPU oracle: it is checked against what the paper and the mathematics fix,
never against itself or the HIP path.  All CPU, all fp64, all tiny."""
import math
import os

import numpy as np
import pytest

from oracle import classic_attention as ca
from oracle import sizes
from oracle import tucker_oracle as orc

RNG = np.random.default_rng


def rand_weights(rng, d, nH, r, rt=None, scale=1.0):
    r1, r2, r3 = r
    t1, t2, t3 = rt or r
    g = lambda *s: rng.standard_normal(s) * scale
    return dict(C=g(r1, r2, r3), U1=g(nH, r1), U2=g(d, r2) / math.sqrt(d), U3=g(d, r3) / math.sqrt(d),
                Ct=g(t1, t2, t3), Ut1=g(nH, t1), Ut2=g(d, t2), Ut3=g(d, t3) / math.sqrt(d))


def close(a, b, tol=1e-11):
    scale = max(1.0, float(np.max(np.abs(b))))
    assert np.max(np.abs(np.asarray(a) - np.asarray(b))) <= tol * scale


# --- brute force: the two oracle forms agree, and the dense form equals element-wise loops --------

@pytest.mark.parametrize("causal", [False, True])
@pytest.mark.parametrize("rope", [None, 100.0])
def test_per_head_equals_dense_definition(causal, rope):
    rng = RNG(11)
    d, nH, N = 12, 3, 7
    w = rand_weights(rng, d, nH, (2, 5, 4), (3, 6, 4))          # r2 != r3, tilde ranks differ
    X = rng.standard_normal((2, N, d))
    y1 = orc.dense_definition_forward(X, w, d_head=4, causal=causal, rope_base=rope, pos0=3)
    y2 = orc.per_head_forward(X, w, d_head=4, causal=causal, rope_base=rope, pos0=3)
    close(y2, y1)


@pytest.mark.parametrize("causal", [False, True])
def test_dense_definition_equals_elementwise_loops(causal):
    rng = RNG(12)
    d, nH, N = 6, 2, 5
    w = rand_weights(rng, d, nH, (2, 3, 4), (2, 4, 3))
    X = rng.standard_normal((1, N, d))
    W = np.zeros((nH, d, d))
    Wt = np.zeros((nH, d, d))
    for i in range(nH):                                              # Tucker representation, index by index
        for j in range(d):
            for k in range(d):
                W[i, j, k] = sum(w["C"][a, b, c] * w["U1"][i, a] * w["U2"][j, b] * w["U3"][k, c]
                                 for a in range(2) for b in range(3) for c in range(4))
                Wt[i, j, k] = sum(w["Ct"][a, b, c] * w["Ut1"][i, a] * w["Ut2"][j, b] * w["Ut3"][k, c]
                                  for a in range(2) for b in range(4) for c in range(3))
    close(orc.tucker_tensor(w["C"], w["U1"], w["U2"], w["U3"]), W)
    ref = ca.bilinear_attention_reference(X[0], W, Wt, d_head=3, causal=causal)
    close(orc.dense_definition_forward(X, w, 3, causal)[0], ref)
    close(orc.per_head_forward(X, w, 3, causal)[0], ref)


# --- special cases the paper proves ---------------------------------------------------------------

def selector_core(nH, dH, n_kv_groups=None):
    """C[i, n, m] = 1 iff n = (i,l) and m = (g(i), l): the core of the lemma on D_i = A_i B_i^T."""
    nG = n_kv_groups or nH
    per = nH // nG
    C = np.zeros((nH, nH * dH, nG * dH))
    for i in range(nH):
        for l in range(dH):
            C[i, i * dH + l, (i // per) * dH + l] = 1.0
    return C


@pytest.mark.parametrize("causal", [False, True])
def test_mha_is_a_special_case(causal):
    rng = RNG(21)
    d, nH, dH, N = 8, 2, 4, 6
    WQ, WK, WV = (rng.standard_normal((d, d)) for _ in range(3))
    WO = rng.standard_normal((d, d))
    X = rng.standard_normal((1, N, d))
    w = dict(C=selector_core(nH, dH), U1=np.eye(nH), U2=WQ, U3=WK,
             Ct=selector_core(nH, dH), Ut1=np.eye(nH), Ut2=WO.T, Ut3=WV)
    ref = ca.mha_reference(X[0], WQ, WK, WV, WO, nH, causal)
    close(orc.per_head_forward(X, w, dH, causal)[0], ref)
    close(orc.dense_definition_forward(X, w, dH, causal)[0], ref)


@pytest.mark.parametrize("nG", [1, 2])
def test_gqa_and_mqa_are_special_cases(nG):
    rng = RNG(22)
    d, nH, dH, N = 8, 4, 2, 5
    WQ = rng.standard_normal((d, nH * dH))
    WKg, WVg = rng.standard_normal((d, nG * dH)), rng.standard_normal((d, nG * dH))
    WO = rng.standard_normal((nH * dH, d))
    X = rng.standard_normal((1, N, d))
    core = selector_core(nH, dH, nG)                                  # ranks (nH, d, nG*dH)
    w = dict(C=core, U1=np.eye(nH), U2=WQ, U3=WKg, Ct=core, Ut1=np.eye(nH), Ut2=WO.T, Ut3=WVg)
    ref = ca.gqa_reference(X[0], WQ, WKg, WVg, WO, nH, nG, causal=True)
    close(orc.per_head_forward(X, w, dH, True)[0], ref)


@pytest.mark.parametrize("shared_kv", [True, False])
def test_mla_is_a_special_case(shared_kv):
    rng = RNG(23)
    d, nH, dH, N, dcq, dck = 8, 2, 4, 6, 5, 3
    WDQ, WUQ = rng.standard_normal((d, dcq)), rng.standard_normal((dcq, nH * dH))
    WDKV, WUK = rng.standard_normal((d, dck)), rng.standard_normal((dck, nH * dH))
    WDV = WDKV if shared_kv else rng.standard_normal((d, dck))
    WUV = rng.standard_normal((dck, nH * dH))
    WO = rng.standard_normal((nH * dH, d))
    X = rng.standard_normal((1, N, d))
    hs = lambda i: slice(i * dH, (i + 1) * dH)
    C = np.stack([WUQ[:, hs(i)] @ WUK[:, hs(i)].T for i in range(nH)])           # [nH, dcq, dck]
    Ct = np.stack([(WUV[:, hs(i)] @ WO[hs(i), :]).T for i in range(nH)])          # [nH, d(out), dck]
    w = dict(C=C, U1=np.eye(nH), U2=WDQ, U3=WDKV, Ct=Ct, Ut1=np.eye(nH), Ut2=np.eye(d), Ut3=WDV)
    ref = ca.mla_reference(X[0], WDQ, WUQ, WDKV, WUK, WDV, WUV, WO, nH, causal=True)
    close(orc.per_head_forward(X, w, dH, True)[0], ref)


def test_full_ranks_reproduce_arbitrary_bilinear_forms():
    rng = RNG(24)
    d, nH, N = 5, 2, 4
    W, Wt = rng.standard_normal((nH, d, d)), rng.standard_normal((nH, d, d))
    X = rng.standard_normal((1, N, d))
    I = np.eye
    w = dict(C=W, U1=I(nH), U2=I(d), U3=I(d), Ct=Wt, Ut1=I(nH), Ut2=I(d), Ut3=I(d))
    ref = ca.bilinear_attention_reference(X[0], W, Wt, d_head=2, causal=False)
    close(orc.per_head_forward(X, w, 2, False)[0], ref)


# --- RoPE ------------------------------------------------------------------------------------------

def test_rope_worked_values_and_group_property():
    # r = 2: theta_0 = 1, so position p rotates (1,0) to (cos p, sin p) and (0,1) to (-sin p, cos p)
    R = orc.rope_matrix(1, 2, 10000.0)
    close(np.array([1.0, 0.0]) @ R, [math.cos(1), math.sin(1)])
    close(np.array([0.0, 1.0]) @ R, [-math.sin(1), math.cos(1)])
    # r = 4, base 100: second pair turns at theta_1 = 100**(-2/4) = 0.1
    close(orc.rope_frequencies(4, 100.0), [1.0, 0.1])
    x = np.array([[0.0, 0.0, 2.0, 0.0]])
    close(orc.rope_rotate(x, np.array([5]), 100.0), [[0, 0, 2 * math.cos(0.5), 2 * math.sin(0.5)]])
    # relative-position property R(m) R(n)^T = R(m - n), orthogonality, pairwise == dense
    for m, n in [(7, 3), (2, 9), (0, 4)]:
        close(orc.rope_matrix(m, 8, 50.0) @ orc.rope_matrix(n, 8, 50.0).T, orc.rope_matrix(m - n, 8, 50.0))
    rng = RNG(31)
    v = rng.standard_normal((3, 8))
    pos = np.array([0, 6, 11])
    dense = np.stack([v[t] @ orc.rope_matrix(int(pos[t]), 8, 50.0) for t in range(3)])
    close(orc.rope_rotate(v, pos, 50.0), dense)
    close(orc.rope_rotate(v, np.zeros(3), 50.0), v)


@pytest.mark.parametrize("causal", [False, True])
def test_rope_relative_position_invariance(causal):
    rng = RNG(32)
    d, nH, N = 10, 3, 9
    w = rand_weights(rng, d, nH, (2, 4, 6))
    X = rng.standard_normal((1, N, d))
    y0 = orc.per_head_forward(X, w, 4, causal, rope_base=30.0, pos0=0)
    y1 = orc.per_head_forward(X, w, 4, causal, rope_base=30.0, pos0=1234)
    close(y1, y0, 1e-9)
    # and RoPE does change the result (it is not a no-op)
    y_plain = orc.per_head_forward(X, w, 4, causal, rope_base=None)
    assert np.max(np.abs(y_plain - y0)) > 1e-3


def test_rope_rotating_key_only_by_relative_matrix():
    # q R(m) . (k R(n)) == q . (k R(n) R(m)^T): the two printed forms of latent RoPE agree
    rng = RNG(33)
    q, k = rng.standard_normal(6), rng.standard_normal(6)
    Rm, Rn = orc.rope_matrix(5, 6, 20.0), orc.rope_matrix(2, 6, 20.0)
    close((q @ Rm) @ (k @ Rn), q @ (k @ Rn @ Rm.T))


# --- causal mask -----------------------------------------------------------------------------------

def test_causal_rows_ignore_the_future_and_row0_closed_form():
    rng = RNG(41)
    d, nH, N = 8, 2, 10
    w = rand_weights(rng, d, nH, (2, 3, 4))
    X = rng.standard_normal((1, N, d))
    y = orc.per_head_forward(X, w, 4, True, rope_base=10.0)
    X2 = X.copy()
    X2[0, 6:] += rng.standard_normal((N - 6, d))
    y2 = orc.per_head_forward(X2, w, 4, True, rope_base=10.0)
    close(y2[0, :6], y[0, :6])
    assert np.max(np.abs(y2[0, 6:] - y[0, 6:])) > 1e-3
    close(orc.per_head_forward(X[:, :4], w, 4, True, rope_base=10.0)[0], y[0, :4])
    # row 0 sees only itself: Y[0] = sum_i (X_0 Ut3) G~_i^T Ut2^T
    Gt = np.einsum("ia,abc->ibc", w["Ut1"], w["Ct"])
    v0 = X[0, 0] @ w["Ut3"]
    row0 = sum(v0 @ Gt[i].T @ w["Ut2"].T for i in range(nH))
    close(y[0, 0], row0)
    # non-causal rows DO depend on later tokens
    yn, yn2 = (orc.per_head_forward(Z, w, 4, False) for Z in (X, X2))
    assert np.max(np.abs(yn2[0, :6] - yn[0, :6])) > 1e-3


def test_zero_core_gives_uniform_attention():
    rng = RNG(42)
    d, nH, N = 6, 3, 7
    w = rand_weights(rng, d, nH, (2, 3, 4))
    w["C"] = np.zeros_like(w["C"])
    X = rng.standard_normal((1, N, d))
    V = X[0] @ w["Ut3"]
    M = sum(np.einsum("a,abc->bc", w["Ut1"][i], w["Ct"]).T for i in range(nH)) @ w["Ut2"].T   # [rt3, d]
    yc = orc.per_head_forward(X, w, 2, True, rope_base=10.0)[0]
    yn = orc.per_head_forward(X, w, 2, False)[0]
    for j in range(N):
        close(yc[j], V[: j + 1].mean(axis=0) @ M)
        close(yn[j], V.mean(axis=0) @ M)


def test_identical_tokens_make_softmax_irrelevant():
    rng = RNG(43)
    d, nH, N = 6, 2, 5
    w = rand_weights(rng, d, nH, (2, 3, 4), scale=3.0)
    X = np.repeat(rng.standard_normal((1, 1, d)), N, axis=1)
    M = sum(np.einsum("a,abc->bc", w["Ut1"][i], w["Ct"]).T for i in range(nH)) @ w["Ut2"].T
    expect = (X[0, 0] @ w["Ut3"]) @ M
    for causal, rope in [(True, 10.0), (False, None), (False, 10.0)]:
        y = orc.per_head_forward(X, w, 2, causal, rope_base=rope)[0]
        for j in range(N):
            close(y[j], expect, 1e-10)


# --- invariances of the Tucker form ----------------------------------------------------------------

def test_gauge_invariance():
    rng = RNG(51)
    d, nH, N = 8, 3, 6
    w = rand_weights(rng, d, nH, (2, 4, 4))
    X = rng.standard_normal((1, N, d))
    A2, A3, A1 = rng.standard_normal((4, 4)), rng.standard_normal((4, 4)), rng.standard_normal((2, 2))
    inv = np.linalg.inv
    y_rope = orc.per_head_forward(X, w, 4, True, rope_base=10.0)
    y = orc.per_head_forward(X, w, 4, True)
    w2 = dict(w, U2=w["U2"] @ A2, C=np.einsum("abc,db->adc", w["C"], inv(A2)))          # mode 2, RoPE on
    close(orc.per_head_forward(X, w2, 4, True, rope_base=10.0), y_rope, 1e-9)
    w3 = dict(w, U3=w["U3"] @ A3, C=np.einsum("abc,dc->abd", w["C"], inv(A3)))          # mode 3, RoPE off
    close(orc.per_head_forward(X, w3, 4, True), y, 1e-9)
    w1 = dict(w, U1=w["U1"] @ A1, C=np.einsum("abc,da->dbc", w["C"], inv(A1)))          # head mode
    close(orc.per_head_forward(X, w1, 4, True, rope_base=10.0), y_rope, 1e-9)
    wt = dict(w, Ut2=w["Ut2"] @ A2, Ct=np.einsum("abc,db->adc", w["Ct"], inv(A2)),
              Ut3=w["Ut3"] @ A3)
    wt["Ct"] = np.einsum("abc,dc->abd", wt["Ct"], inv(A3))
    close(orc.per_head_forward(X, wt, 4, True, rope_base=10.0), y_rope, 1e-9)


def test_token_permutation_equivariance_without_mask_and_rope():
    rng = RNG(52)
    d, nH, N = 8, 2, 7
    w = rand_weights(rng, d, nH, (2, 3, 4))
    X = rng.standard_normal((1, N, d))
    perm = rng.permutation(N)
    y = orc.per_head_forward(X, w, 4, False)
    close(orc.per_head_forward(X[:, perm], w, 4, False)[0], y[0, perm])


def test_sampled_rows_equal_rows_of_the_full_result():
    rng = RNG(53)
    d, nH, N = 8, 2, 9
    w = rand_weights(rng, d, nH, (2, 3, 4))
    X = rng.standard_normal((3, N, d))
    y = orc.per_head_forward(X, w, 4, True, rope_base=10.0, pos0=2)
    ys = orc.per_head_forward(X, w, 4, True, rope_base=10.0, pos0=2, rows=[0, 4, 8], batches=[2, 0])
    close(ys[0], y[2][[0, 4, 8]])
    close(ys[1], y[0][[0, 4, 8]])


# --- KV cache / decode -----------------------------------------------------------------------------

@pytest.mark.parametrize("rope", [None, 25.0])
def test_decode_equals_last_row_of_causal_prefill(rope):
    rng = RNG(61)
    d, nH, N, Lmax = 8, 3, 6, 9
    w = rand_weights(rng, d, nH, (2, 3, 4))
    X = rng.standard_normal((2, N, d))
    full = orc.per_head_forward(X, w, 4, True, rope_base=rope)
    K, V = orc.latent_kv(X, w, rope)
    Kc, Vc = np.zeros((2, Lmax, 4)), np.zeros((2, Lmax, 4))
    lens = np.array([N, N - 2])
    for b in range(2):
        Kc[b, : lens[b] - 1], Vc[b, : lens[b] - 1] = K[b, : lens[b] - 1], V[b, : lens[b] - 1]
    xs = np.stack([X[b, lens[b] - 1] for b in range(2)])
    y, Kn, Vn = orc.decode_step(xs, Kc, Vc, lens, w, 4, rope_base=rope)
    for b in range(2):
        close(y[b], full[b, lens[b] - 1], 1e-10)
        close(Kn[b, : lens[b]], K[b, : lens[b]])
        close(Vn[b, : lens[b]], V[b, : lens[b]])


@pytest.mark.parametrize("rope", [None, 25.0])
def test_shared_kv_decode_equals_last_row_of_prefill_with_one_basis(rope):
    # Sharing U3 between the two Tucker factorizations (value basis := key basis) is the shared
    # key-value down-projection; the one-cache decode must reproduce the last row of the ordinary
    # prefill evaluated with Ut3 = U3, and its cache must be the UNROTATED latent X U3.
    rng = RNG(62)
    d, nH, N, Lmax = 8, 3, 7, 9
    w = rand_weights(rng, d, nH, (2, 3, 4))
    w["Ut3"] = w["U3"].copy()
    X = rng.standard_normal((2, N, d))
    full = orc.per_head_forward(X, w, 4, True, rope_base=rope)
    Lat = X @ w["U3"]
    Lc = np.zeros((2, Lmax, 4))
    lens = np.array([N, N - 3])
    for b in range(2):
        Lc[b, : lens[b] - 1] = Lat[b, : lens[b] - 1]
    xs = np.stack([X[b, lens[b] - 1] for b in range(2)])
    w_no_value_basis = {k: v for k, v in w.items()}
    w_no_value_basis["Ut3"] = np.full_like(w["U3"], np.nan)          # must not be read
    y, Ln = orc.decode_step_shared_kv(xs, Lc, lens, w_no_value_basis, 4, rope_base=rope)
    for b in range(2):
        close(y[b], full[b, lens[b] - 1], 1e-10)
        close(Ln[b, : lens[b]], Lat[b, : lens[b]])
    # and it agrees with the two-cache decode fed the rotated and the plain copy of the same latent
    K, V = orc.latent_kv(X, w, rope)
    Kc, Vc = np.zeros((2, Lmax, 4)), np.zeros((2, Lmax, 4))
    for b in range(2):
        Kc[b, : lens[b] - 1], Vc[b, : lens[b] - 1] = K[b, : lens[b] - 1], V[b, : lens[b] - 1]
    y2, _, _ = orc.decode_step(xs, Kc, Vc, lens, w, 4, rope_base=rope)
    close(y, y2, 1e-10)


# --- robustness of the softmax ---------------------------------------------------------------------

def test_sharp_and_shifted_scores_stay_finite_and_exact():
    rng = RNG(71)
    d, nH, N = 6, 2, 8
    w = rand_weights(rng, d, nH, (2, 3, 4))
    w["C"] = w["C"] * 1e5                                             # huge scores: one-hot softmax
    X = rng.standard_normal((1, N, d))
    y = orc.per_head_forward(X, w, 1, True)
    assert np.all(np.isfinite(y))
    # one-hot limit: every head picks its arg-max visible key
    WQ, WK, WV, WO = orc.per_head_weights(w)
    expect = np.zeros_like(y[0])
    for i in range(nH):
        S = (X[0] @ WQ[i]) @ (X[0] @ WK).T
        for j in range(N):
            l = int(np.argmax(S[j, : j + 1]))
            expect[j] += (X[0, l] @ WV) @ WO[i]
    close(y[0], expect, 1e-6)


# --- closed-form sizes against the numbers the paper prints ------------------------------------------

def test_memory_closed_forms_match_printed_tables():
    path = os.path.join(os.path.dirname(__file__), "golden", "paper_memory_tables.txt")
    d, nH, dH, bytes_el = 768, 12, 64, 2
    n_rows = 0
    for line in open(path):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        table, method, a, b, c, N, layers, p_print, c_print = line.split()
        a, b, c, N, layers = int(a), int(b), int(c), int(N), int(layers)
        if method == "mha":
            p, kv = sizes.mha_params(d), sizes.mha_cache(N, d)
        elif method in ("gqa", "gqa_params"):
            p, kv = sizes.gqa_params(d, dH, a), sizes.gqa_cache(N, dH, a)
        elif method == "tucker":
            p, kv = sizes.tucker_params(d, nH, a, b, c), sizes.tucker_cache(N, c)
        elif method == "tucker_shared":
            p, kv = sizes.tucker_params(d, nH, a, b, c, True), sizes.tucker_cache(N, c, True)
        elif method == "mla_shared":
            p, kv = sizes.mla_params_train(d, a, True), sizes.mla_cache(N, a, True)
        elif method == "mla":
            p, kv = sizes.mla_params_train(d, a, False), sizes.mla_cache(N, a, False)
        else:
            raise AssertionError(method)
        cache_unit = 1e6 if table == "gpt2" else 2.0 ** 20
        if p_print != "-":
            assert abs(p * layers * bytes_el / 1e6 - float(p_print)) <= (0.05 if method == "mla_shared" else 0.03), line
        if c_print != "-":
            assert abs(kv * layers * bytes_el / cache_unit - float(c_print)) <= 0.03, line
        n_rows += 1
    assert n_rows == 26
    # the caption of the GPT-2 loss figure prints parameter counts in millions: MHA 28.31, GQA-2 16.51,
    # MLA (shared latent, dc = 128) 13.00
    assert abs(sizes.mha_params(d) * 12 / 1e6 - 28.31) < 0.01
    assert abs(sizes.gqa_params(d, dH, 2) * 12 / 1e6 - 16.51) < 0.01
    assert abs(sizes.mla_params_train(d, 128, True) * 12 / 1e6 - 13.00) < 0.03
    # separated minus shared latent = one d x dc down-projection; the cache doubles
    assert sizes.mla_params_train(d, 64, False) - sizes.mla_params_train(d, 64, True) == d * 64
    assert sizes.mla_cache(100, 64, False) == 2 * sizes.mla_cache(100, 64, True) == 2 * 100 * 64
    # table formula with r2 = r3 = r, and the LLaMA-1B rows (printed in millions of elements, 16 layers)
    assert sizes.tucker_params(d, nH, 8, 128, 128) == 2 * (nH * 8 + 2 * 128 * d + 8 * 128 * 128)
    assert abs(sizes.tucker_params(2048, 32, 32, 128, 128) * 16 / 1e6 - 33.5) < 0.1
    assert abs(sizes.tucker_params(2048, 32, 32, 64, 64) * 16 / 1e6 - 12.6) < 0.05
    assert abs(sizes.tucker_cache(4096, 128) * 16 / 1e6 - 16.7) < 0.1


# --- the error measure every GPU parity assertion goes through ---------------------------------------

def test_relative_l2_hand_values():
    # ||a - b|| / ||b|| with b the reference: a = (3, 4), b = (0, 4) -> ||(3, 0)|| / 4
    assert orc.relative_l2(np.array([3.0, 4.0]), np.array([0.0, 4.0])) == 0.75
    # not symmetric: the second argument is the denominator
    assert abs(orc.relative_l2(np.array([0.0, 4.0]), np.array([3.0, 4.0])) - 3.0 / 5.0) < 1e-15
    b = np.arange(1.0, 25.0).reshape(2, 3, 4)
    assert orc.relative_l2(b, b) == 0.0
    assert abs(orc.relative_l2(1.01 * b, b) - 0.01) < 1e-14                  # uniform 1 % error, any shape
    assert abs(orc.relative_l2(7.0 * 1.01 * b, 7.0 * b) - 0.01) < 1e-14      # scale invariance
    # one wrong element among many: sqrt of the sum of squares, not a mean and not a maximum
    a = np.ones(100)
    a[0] = 2.0
    assert abs(orc.relative_l2(a, np.ones(100)) - 0.1) < 1e-15
    # fp32 and bf16-rounded inputs are compared in double precision
    x = np.array([1.0, 1.0 + 2.0 ** -20], dtype=np.float32)
    assert abs(orc.relative_l2(x, np.array([1.0, 1.0])) - 2.0 ** -20 / np.sqrt(2.0)) < 1e-12


def test_per_row_relative_l2_hand_values():
    ref = np.array([[3.0, 4.0], [0.0, 2.0], [1.0, 0.0]])
    got = np.array([[3.0, 4.5], [0.0, 2.0], [0.0, 0.0]])
    rows = orc.relative_l2_rows(got, ref)
    assert rows.shape == (3,)
    assert np.allclose(rows, [0.1, 0.0, 1.0], atol=1e-15)
    # rows are the vectors along the last axis, whatever the leading shape
    assert orc.relative_l2_rows(got.reshape(3, 1, 2), ref.reshape(3, 1, 2)).shape == (3, 1)
    # a reference row of zeros is measured on the scale of the root-mean-square reference row
    z = orc.relative_l2_rows(np.array([[0.0, 0.0], [0.0, 1.0]]), np.array([[0.0, 0.0], [0.0, 0.0]]), floor=2.0)
    assert np.allclose(z, [0.0, 0.5])
