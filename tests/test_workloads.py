"""The seeded generators: shapes, recipes, determinism and the bf16 storage rounding."""
import numpy as np
import torch

from paper_2603_30033_amd import workloads as wl


def small(name, **kw):
    return wl.scaled(wl.WORKLOADS[name], **kw)


def test_shapes_determinism_and_recipes():
    w = small("gpt2_small", B=2, N=16)
    a, b = wl.make_inputs(w), wl.make_inputs(w)
    for k in a:
        assert np.array_equal(a[k], b[k]), k
    assert a["X"].shape == (2, 16, 768) and a["C"].shape == (4, 64, 64)
    assert a["U1"].shape == (12, 4) and a["Ut2"].shape == (768, 64)
    # LayerNorm-scaled tokens (before bf16 rounding: zero mean, unit variance per token)
    assert np.max(np.abs(a["X"].mean(-1))) < 2e-3 and np.max(np.abs(a["X"].std(-1) - 1)) < 5e-3
    # orthonormal columns survive bf16 rounding to ~2^-9
    for k in ("U1", "U2", "U3", "Ut2", "Ut3"):
        g = a[k].astype(np.float64).T @ a[k].astype(np.float64)
        assert np.max(np.abs(g - np.eye(g.shape[0]))) < 2e-2, k
    assert abs(a["C"].std() - 1 / 8.0) < 0.01

    t = wl.make_inputs(wl.WORKLOADS["tiny_f32"])
    assert t["X"].shape == (1, 128, 256) and t["X"].dtype == np.float32
    assert abs(t["U2"].std() * 16 - 1) < 0.05 and abs(t["C"].std() * np.sqrt(32) - 1) < 0.05


def test_decode_workload_has_caches():
    w = small("decode_32k", B=2, kv_len=64, d_model=256, n_heads=4, r1=2, r2=32, r3=32)
    a = wl.make_inputs(w)
    assert a["X"].shape == (2, 1, 256)
    assert a["Kcache"].shape == (2, 64, 32) and a["Vcache"].shape == (2, 64, 32)
    assert np.all(a["Kcache"][:, 63] == 0) and list(a["kv_len"]) == [64, 64]
    assert abs(a["Kcache"][:, :63].std() - 1) < 0.05


def test_bf16_rounding_is_round_to_nearest_even():
    rng = np.random.default_rng(5)
    x = np.concatenate([rng.standard_normal(4096).astype(np.float32) * 37.0,
                        np.array([1.0, 1.00390625, 1.01171875, -1.00390625, 0.0, 3.3895314e38], np.float32)])
    ours = wl.round_to_storage(x, "bf16")
    theirs = torch.from_numpy(x).to(torch.bfloat16).to(torch.float32).numpy()
    assert np.array_equal(ours, theirs)
    assert np.array_equal(wl.bf16_bits(x), torch.from_numpy(x).to(torch.bfloat16).view(torch.int16).numpy().view(np.uint16))
    # ties go to even: 1 + 2^-8 -> 1.0, 1 + 3*2^-8 -> 1 + 2^-6
    assert ours[4097] == 1.0 and ours[4098] == 1.015625


def test_classic_weights_are_deterministic_rounded_and_have_a_decaying_spectrum():
    a = wl.make_classic_weights(96, 6, 16, 5, "bf16")
    b = wl.make_classic_weights(96, 6, 16, 5, "bf16")
    assert all(np.array_equal(a[k], b[k]) for k in a)
    assert a["WQ"].shape == (96, 96) and a["WK"].shape == (96, 96) and a["WO"].shape == (96, 96)
    g = wl.make_classic_weights(96, 6, 16, 5, "bf16", kv_width=32)
    assert g["WK"].shape == (96, 32) and g["WV"].shape == (96, 32) and g["WQ"].shape == (96, 96)
    for k in a:                                                   # values the storage type holds exactly
        assert np.array_equal(wl.round_to_storage(a[k], "bf16"), a[k]), k
    f = wl.make_classic_weights(96, 6, 16, 5, "f32")
    assert abs(np.mean(np.sum(f["WQ"].astype(np.float64) ** 2, axis=0)) - 1.0) < 0.2   # unit expected column norm
    s = np.linalg.svd(f["WQ"].astype(np.float64), compute_uv=False)
    assert s[0] / s[47] > 4.0 and np.all(np.diff(s) <= 0)         # power-law weighting, not a flat Gaussian spectrum
