"""tucker_attn_decode_static, the decode entry point that allocates nothing (its workspace is a
static device array inside the library), against tucker_attn_decode on a caller-owned workspace:
same kernels, so results must be bit-identical, and both must meet the oracle's bar.  Two calls in a
row share the one static array, the second with a smaller input."""
import numpy as np
import pytest
import torch

from oracle import tucker_oracle as orc
from paper_2603_30033_amd import binding as ta
from paper_2603_30033_amd import workloads as wl
from paper_2603_30033_amd.device import Layer, to_device, to_host

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def _decode_both(layer, w, inp):
    """One decode step through both entry points on separate copies of the caches."""
    x = to_device(inp["X"][:, 0], w.dtype)
    lens = [int(v) for v in inp["kv_len"]]
    out = []
    for static in (False, True):
        Kc, Vc = to_device(inp["Kcache"], w.dtype), to_device(inp["Vcache"], w.dtype)
        y = torch.full_like(x, float("nan"))
        if static:
            ta.tucker_attn_decode_static(layer.ctx, layer.weights, x, y, Kc, Vc, lens)
        else:
            ws = layer.workspace(ta.tucker_attn_decode_workspace_bytes(layer.ctx, w.B))
            ta.tucker_attn_decode(layer.ctx, layer.weights, x, y, Kc, Vc, lens, ws)
        torch.cuda.synchronize()
        out.append((to_host(y), to_host(Kc), to_host(Vc)))
    return out


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_static_scratch_decode_equals_workspace_decode_twice_in_a_row(dtype):
    big = wl.scaled(wl.WORKLOADS["decode_32k"], d_model=512, n_heads=12, d_head=64, r1=4, r2=96, r3=64,
                    B=5, kv_len=1500, dtype=dtype, seed=31)
    small = wl.scaled(big, d_model=512, B=2, kv_len=130, seed=32)
    for w in (big, small):                                  # the second call is the smaller one
        inp = wl.make_inputs(w)
        inp["kv_len"] = np.array([w.kv_len, 1, w.kv_len // 2 + 1, 77, 64][: w.B], dtype=np.int32)
        with Layer(w, inp, max_positions=w.kv_len + 1) as layer:
            (y0, K0, V0), (y1, K1, V1) = _decode_both(layer, w, inp)
        assert np.all(np.isfinite(y1))
        assert np.array_equal(y0, y1) and np.array_equal(K0, K1) and np.array_equal(V0, V1)
        y_ref, _, _ = orc.decode_step(inp["X"][:, 0], inp["Kcache"], inp["Vcache"], inp["kv_len"], wl.weights_of(inp),
                                      w.d_head, w.rope_base)
        err = orc.relative_l2(y1, y_ref)
        assert err <= TOL[dtype], f"{w.B} sequences: relative L2 {err:.3e}"


def test_static_scratch_decode_refuses_what_does_not_fit_and_bad_arguments():
    # operand-layout copies of the weights alone exceed the 32 MiB array: refused, nothing enqueued
    w = wl.scaled(wl.WORKLOADS["decode_32k"], d_model=8192, n_heads=64, d_head=128, r1=2, r2=512, r3=128,
                  B=1, kv_len=8, dtype="bf16", seed=33, recipe="fan_in")
    ctx = ta.tucker_attn_create(d_model=w.d_model, n_heads=w.n_heads, d_head=w.d_head, r1=w.r1, r2=w.r2, r3=w.r3,
                                rope_base=None, dtype="bf16", max_positions=16)
    try:
        assert ta.tucker_attn_decode_workspace_bytes(ctx, 1) > 32 << 20
        t = torch.zeros(8192 * 512, dtype=torch.bfloat16, device="cuda")
        weights = {k: t for k in ("C", "U1", "U2", "U3", "Ct", "Ut1", "Ut2", "Ut3")}
        x = torch.zeros((1, 8192), dtype=torch.bfloat16, device="cuda")
        Kc = torch.zeros((1, 8, 128), dtype=torch.bfloat16, device="cuda")
        assert ta.tucker_attn_decode_static(ctx, weights, x, torch.empty_like(x), Kc, Kc.clone(), [8], check=False) == -3
    finally:
        ta.tucker_attn_destroy(ctx)
    small = wl.scaled(wl.WORKLOADS["decode_32k"], d_model=128, n_heads=4, d_head=32, r1=2, r2=32, r3=32, B=2, kv_len=20,
                      seed=34, recipe="fan_in")
    inp = wl.make_inputs(small)
    with Layer(small, inp, max_positions=32) as layer:
        x = to_device(inp["X"][:, 0], small.dtype)
        Kc, Vc = to_device(inp["Kcache"], small.dtype), to_device(inp["Vcache"], small.dtype)
        y = torch.empty_like(x)
        assert ta.tucker_attn_decode_static(layer.ctx, layer.weights, x, y, Kc, Vc, [20, 21], check=False) == -1
        assert ta.tucker_attn_decode_static(layer.ctx, layer.weights, x, y, Kc, Vc, [20, 0], check=False) == -1
        assert ta.tucker_attn_decode_static(layer.ctx, layer.weights, x, y, Kc, Vc, [20, 20], check=True) == 0
        torch.cuda.synchronize()
