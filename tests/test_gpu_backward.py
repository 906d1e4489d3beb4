"""GPU parity of the backward pass: the HIP library's gradients, through the C ABI, against the
fp64 chain-rule oracle on the same seeded inputs.  The measure is the relative L2 error of each
returned array; the bars are those of the forward pass (1e-5 for fp32 storage, 2e-2 for bf16).

One documented exception, bf16 storage only: the head-factor gradients dU1 [nH, r1] and dU~1 are a handful
of numbers, each a sum of signed terms sum_bc dG_i[b,c] C[a][b,c].  The bf16 storage roundings of the
pipeline perturb the terms by about a unit roundoff (2^-9) each, so the result is off by that times the
cancellation factor kappa = |sum of absolute terms| / |sum| (computed by the oracle in fp64).  Their bar is
max(2e-2, 2^-10 kappa); tests/test_bf16_tolerance_model.py shows on the CPU that a plain fp64 chain rule with
nothing but those roundings exceeds 2e-2 in such cases.  With kappa below 20 it is the common bar."""
import numpy as np
import pytest
import torch

from oracle import tucker_backward as bwd
from oracle import tucker_oracle as orc
from paper_2603_30033_amd import workloads as wl
from paper_2603_30033_amd.device import Layer, to_device, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def upstream(w, seed):
    rng = np.random.default_rng(seed)
    return wl.round_to_storage(rng.standard_normal((w.B, w.N, w.d_model)).astype(np.float32), w.dtype)


def run_backward(w, inp, dY):
    with Layer(w, inp, max_positions=w.pos0 + w.N + 8) as layer:
        dX, grads = layer.backward(to_device(inp["X"], w.dtype), to_device(dY, w.dtype), pos0=w.pos0)
        torch.cuda.synchronize()
        out = {k: to_host(v) for k, v in grads.items()}
        out["dX"] = to_host(dX)
        return out


def oracle_backward(w, inp, dY):
    """The oracle's gradients, plus under "_bars" the bars of the head-factor gradients."""
    wts = wl.weights_of(inp)
    ref = bwd.backward(inp["X"], dY, wts, w.d_head, w.causal, w.rope_base, pos0=w.pos0, shared_kv=w.shared_kv,
                       return_mixed=True)
    dG, dGt = ref.pop("dG"), ref.pop("dGt")
    bars = {}
    if w.dtype == "bf16":
        for key, mixed, core in (("dU1", dG, "C"), ("dUt1", dGt, "Ct")):
            if np.linalg.norm(ref[key]) > 0:
                bars[key] = max(TOL["bf16"], 2.0 ** -10 * bwd.head_factor_cancellation(mixed, wts[core]))
    ref["_bars"] = bars
    return ref


def check_all(got, ref, dtype, what):
    ref = dict(ref)
    bars = ref.pop("_bars", {})
    assert set(got) == set(ref), (sorted(got), sorted(ref))
    errs = {}
    for k in sorted(ref):
        assert got[k].shape == ref[k].shape, (k, got[k].shape, ref[k].shape)
        assert np.all(np.isfinite(got[k])), f"{what}: {k} not finite"
        if np.linalg.norm(ref[k]) <= 1e-12 * np.sqrt(ref[k].size):
            # a gradient that is exactly zero (one-token sequences: the softmax of a single score is
            # constant): the relative measure has no scale, so compare with the scale of the input gradient
            errs[k] = float(np.linalg.norm(got[k]) / np.linalg.norm(ref["dX"]))
        else:
            errs[k] = orc.relative_l2(got[k], ref[k])
    bad = {k: f"{v:.2e} > {bars.get(k, TOL[dtype]):.1e}" for k, v in errs.items() if v > bars.get(k, TOL[dtype])}
    assert not bad, f"{what}: relative L2 above its bar: {bad} (all: { {k: f'{v:.1e}' for k, v in errs.items()} })"
    return errs


def test_backward_tiny_f32():
    w = wl.WORKLOADS["tiny_f32"]
    inp = wl.make_inputs(w)
    dY = upstream(w, 100)
    check_all(run_backward(w, inp, dY), oracle_backward(w, inp, dY), w.dtype, w.name)


def run_case(w, seed=100):
    inp = wl.make_inputs(w)
    dY = upstream(w, seed)
    return check_all(run_backward(w, inp, dY), oracle_backward(w, inp, dY), w.dtype, repr(w))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("causal,rope", [(True, 1e4), (False, None), (True, None), (False, 1e4)])
def test_backward_mode_switches_ragged_length(dtype, causal, rope):
    # two sequences, a length that is no multiple of any tile, unequal ranks, a start position
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=2, N=203, d_model=128, n_heads=5, d_head=32, r1=3, r2=48, r3=40,
                  rt1=2, rt2=72, rt3=56, dtype=dtype, causal=causal, rope_base=rope, pos0=7, seed=31)
    run_case(w)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("r3", [16, 64, 128])
def test_backward_every_latent_width_and_the_shared_latent(dtype, r3):
    base = wl.scaled(wl.WORKLOADS["tiny_f32"], B=1, N=150, d_model=96, n_heads=6, d_head=16, r1=2, r2=32, r3=r3,
                     rt1=3, rt2=32, rt3=r3, dtype=dtype, seed=32)
    run_case(base)
    run_case(wl.scaled(base, shared_kv=True, seed=33))


@pytest.mark.parametrize("n", [1, 31, 32, 33, 64, 65, 129])
def test_backward_short_sequences(n):
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=3, N=n, seed=34)
    run_case(w)


def test_backward_gpt2_shape_scaled():
    run_case(wl.scaled(wl.WORKLOADS["gpt2_small"], B=2, N=333))


def test_backward_vit_shape_scaled():
    run_case(wl.scaled(wl.WORKLOADS["vit_b"], B=3))


def test_backward_llama_shape_scaled():
    run_case(wl.scaled(wl.WORKLOADS["llama7b_n4096"], B=1, N=448))
    run_case(wl.scaled(wl.WORKLOADS["llama7b_n4096_shared_kv"], B=1, N=320))


def test_backward_paper_rank_shapes_scaled():
    run_case(wl.scaled(wl.WORKLOADS["gpt2_r8_128_64"], B=2, N=300))
    run_case(wl.scaled(wl.WORKLOADS["llama1b_r32_128_128"], B=1, N=320))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_from_saved_forward_state(dtype):
    # a training step: forward with save_for_backward, then backward without re-running the forward;
    # both results against their oracles, and the gradients equal to the self-contained call's bit for bit
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=2, N=203, d_model=128, n_heads=5, d_head=32, r1=3, r2=48, r3=40,
                  rt1=2, rt2=72, rt3=56, dtype=dtype, pos0=3, seed=41)
    inp = wl.make_inputs(w)
    dY = upstream(w, 101)
    with Layer(w, inp, max_positions=w.pos0 + w.N, save_for_backward=True) as layer:
        X, dYd = to_device(inp["X"], w.dtype), to_device(dY, w.dtype)
        Y = layer.forward(X, pos0=w.pos0)
        dX, grads = layer.backward(X, dYd, pos0=w.pos0, forward_state=True)
        torch.cuda.synchronize()
        got = {k: to_host(v) for k, v in grads.items()}
        got["dX"] = to_host(dX)
        y = to_host(Y)
        dX2, grads2 = layer.backward(X, dYd, pos0=w.pos0, forward_state=False)
        torch.cuda.synchronize()
        assert torch.equal(dX, dX2)
        for k in ("dU2", "dUt2", "dC", "dCt"):
            assert torch.equal(grads[k], grads2[k]), k
    ref_y = orc.per_head_forward(inp["X"], wl.weights_of(inp), w.d_head, w.causal, w.rope_base, pos0=w.pos0)
    assert orc.relative_l2(y, ref_y) <= TOL[dtype]
    check_all(got, oracle_backward(w, inp, dY), dtype, "saved forward state")


def test_backward_argument_errors():
    from paper_2603_30033_amd import binding as ta
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], N=40)
    inp = wl.make_inputs(w)
    with Layer(w, inp) as layer:
        X = to_device(inp["X"], w.dtype)
        dX = torch.empty_like(X)
        grads = {"d" + k: torch.empty(v.shape, dtype=torch.float32, device="cuda") for k, v in layer.weights.items()}
        ws = layer.workspace(ta.tucker_attn_backward_workspace_bytes(layer.ctx, w.B, w.N))
        ok = ta.tucker_attn_backward(layer.ctx, layer.weights, X, X, dX, grads, 0, ws, check=False)
        assert ok == 0
        # saved state asked of a context that does not save it
        assert ta.tucker_attn_backward(layer.ctx, layer.weights, X, X, dX, grads, 0, ws, check=False,
                                       forward_state=True) == -1
        # a missing gradient buffer, a workspace that is too small
        g2 = dict(grads); g2.pop("dU3")
        assert ta.tucker_attn_backward(layer.ctx, layer.weights, X, X, dX, g2, 0, ws, check=False) == -1
        assert ta.tucker_attn_backward(layer.ctx, layer.weights, X, X, dX, grads, 0, ws[:1024], check=False) == -3
        torch.cuda.synchronize()


def test_backward_gpt2_full_size():
    # the GPT-2-small-shaped workload as the benchmark launches it (B=8, N=1024), every gradient
    run_case(wl.WORKLOADS["gpt2_small"])


def test_backward_llama_full_size():
    # the LLaMA-7B-shaped workload at the size and launch configuration bench.py times (B=2, N=4096):
    # every gradient against the oracle (about a minute of fp64 work on the host)
    run_case(wl.WORKLOADS["llama7b_n4096"])


def test_backward_vit_shape_many_sequences():
    # enough sequences that the key/value gradient kernel gives several heads to one workgroup
    run_case(wl.scaled(wl.WORKLOADS["vit_b"], B=64))


@pytest.mark.parametrize("seed", range(16))
def test_backward_random_small_configurations(seed):
    rng = np.random.default_rng(5000 + seed)
    dtype = ["f32", "bf16"][seed % 2]
    shared = bool(rng.integers(0, 2))
    r3 = int(rng.choice([8, 16, 24, 40, 48, 64, 72, 96, 128]))
    rt3 = r3 if shared else int(rng.choice([8, 16, 32, 56, 64, 104, 128]))
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=int(rng.integers(1, 5)), N=int(rng.integers(1, 300)),
                  d_model=int(rng.choice([64, 96, 200])), n_heads=int(rng.integers(1, 11)),
                  d_head=int(rng.choice([16, 32, 64])), r1=int(rng.integers(1, 5)), r2=int(rng.choice([8, 32, 48, 80])),
                  r3=r3, rt1=int(rng.integers(1, 5)), rt2=int(rng.choice([8, 32, 64, 100])), rt3=rt3, dtype=dtype,
                  causal=bool(rng.integers(0, 2)), rope_base=[None, 1e4, 5e5][int(rng.integers(0, 3))],
                  seed=6000 + seed, shared_kv=shared, pos0=int(rng.integers(0, 50)))
    run_case(w, seed=7000 + seed)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_head_rank_one(dtype):
    # r1 = 1: every head uses the same core slice, scaled by U1[i, 0].  dU1[i] = <dG_i, C[0]> is then a
    # temperature-like gradient in which the row sums of dS cancel (cancellation factor about 70 here).
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=2, N=140, d_model=96, n_heads=6, d_head=16, r1=1, r2=80, r3=48,
                  rt1=1, rt2=8, rt3=128, dtype=dtype, rope_base=None, seed=6011)
    run_case(w, seed=7011)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_one_head_two_post_softmax_head_ranks(dtype):
    # one head, r~1 = 2, value rank 8: the two numbers of dU~1 cancel by a factor of about 75
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=2, N=242, d_model=96, n_heads=1, d_head=64, r1=4, r2=8, r3=128,
                  dtype=dtype, causal=False, rope_base=None, seed=6083, recipe="fan_in", rt1=2, rt2=64, rt3=8, pos0=3)
    run_case(w, seed=7083)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_backward_at_maximum_ranks(dtype):
    # r1 = 64, r2 = 512, r3 = 128 before and after the softmax, 64 heads
    w = wl.scaled(wl.WORKLOADS["tiny_f32"], B=1, N=70, n_heads=64, d_model=256, d_head=64, r1=64, r2=512, r3=128,
                  rt1=64, rt2=512, rt3=128, dtype=dtype, seed=41, recipe="fan_in")
    run_case(w)
