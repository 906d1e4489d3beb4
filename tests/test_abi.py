"""The C-ABI library loads and exports every symbol the header declares; host-side argument
checks that need no GPU."""
import ctypes as C
import os
import re

import pytest

from paper_2603_30033_amd import binding as ta

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def header_functions(header="tucker_attn.h", prefix="tucker_attn_"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(" + prefix + r"[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = ta.load_library()
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["tucker_attn.h", "tucker_convert.h"]
    names = header_functions()
    assert sorted(ta.EXPORTED) == names
    convert = header_functions("tucker_convert.h", "tucker_convert_")
    assert sorted(ta.EXPORTED_CONVERT) == convert
    for n in names + convert:
        assert getattr(lib, n) is not None


def test_conversion_entry_points_reject_bad_arguments_on_the_host():
    lib = ta.load_library()
    out = ta.tucker_convert_weights_out(*([256] * 8))
    o = C.byref(out)
    assert lib.tucker_convert_from_gqa(0, 64, 4, 16, 3, 256, 256, 256, 256, o, None) == -1        # 3 does not divide 4
    assert lib.tucker_convert_from_gqa(2, 64, 4, 16, 2, 256, 256, 256, 256, o, None) == -1        # unknown storage type
    assert lib.tucker_convert_from_gqa(0, 64, 4, 16, 2, None, 256, 256, 256, o, None) == -1
    assert lib.tucker_convert_from_mla(0, 64, 4, 16, 0, 8, 256, 256, 256, 256, None, 256, 256, o, None) == -1
    no_ut3 = ta.tucker_convert_weights_out(*([256] * 7 + [None]))
    assert lib.tucker_convert_from_mla(0, 64, 4, 16, 8, 8, 256, 256, 256, 256, 256, 256, 256, C.byref(no_ut3), None) == -1
    assert ta.tucker_convert_hosvd_workspace_bytes(0, 4, 16) == 0
    assert ta.tucker_convert_hosvd_workspace_bytes(16384, 4, 16) == 0
    nbytes = ta.tucker_convert_hosvd_workspace_bytes(64, 4, 16)
    assert nbytes > 0 and nbytes % 256 == 0
    hosvd = lambda *a: lib.tucker_convert_from_mha_hosvd(*a)
    W = [256] * 4
    assert hosvd(0, 64, 4, 16, *W, 5, 8, 8, 4, 8, 8, 0, o, None, None, 256, 1 << 40, None) == -1         # r1 > nH
    assert hosvd(0, 64, 4, 16, *W, 4, 65, 8, 4, 8, 8, 0, o, None, None, 256, 1 << 40, None) == -1        # r2 > d
    assert hosvd(0, 64, 4, 16, *W, 4, 8, 8, 4, 8, 4, 1, o, None, None, 256, 1 << 40, None) == -1         # shared needs rt3 == r3
    assert hosvd(0, 64, 4, 16, *W, 4, 8, 8, 4, 8, 8, 0, o, None, None, 256, 16, None) == -3              # workspace too small
    assert hosvd(0, 64, 4, 16, *W, 4, 8, 8, 4, 8, 8, 0, o, None, None, 257, 1 << 40, None) == -1         # misaligned workspace
    assert hosvd(0, 16384, 4, 16, *W, 4, 8, 8, 4, 8, 8, 0, o, None, None, 256, 1 << 40, None) == -2


def test_status_strings():
    assert ta.tucker_attn_status_string(0) == "ok"
    for s in (-1, -2, -3, -4):
        assert ta.tucker_attn_status_string(s) not in ("ok", "unknown status")
    assert ta.tucker_attn_status_string(-99) == "unknown status"


def _cfg(**kw):
    base = dict(d_model=256, n_heads=4, d_head=64, r1=2, r2=32, r3=32, causal=True, rope_base=None,
                dtype="f32", max_positions=128)
    base.update(kw)
    return base


def test_create_rejects_bad_configs_without_touching_the_gpu():
    lib = ta.load_library()
    assert lib.tucker_attn_create(None, None) == -1
    for bad, status in [(dict(d_model=0), -1), (dict(r3=0), -1), (dict(r3=160), -2), (dict(r2=1024), -2),
                        (dict(d_model=100), -2), (dict(n_heads=0), -1)]:
        with pytest.raises(ta.TuckerAttnError) as e:
            ta.tucker_attn_create(**_cfg(**bad))
        assert f"status {status} " in str(e.value)
    cfg = ta.tucker_attn_config(256, 4, 64, 2, 32, 31, 2, 32, 32, 1, 1, 1e4, 0, 128)   # odd r3 with RoPE
    ctx = C.c_void_p()
    assert lib.tucker_attn_create(C.byref(cfg), C.byref(ctx)) == -2


def test_workspace_sizes_and_host_side_argument_checks():
    ctx = ta.tucker_attn_create(**_cfg())          # no RoPE table -> no device allocation
    try:
        assert ta.tucker_attn_workspace_bytes(ctx, 0, 16) == 0
        assert ta.tucker_attn_workspace_bytes(ctx, 1, 0) == 0
        small, big = ta.tucker_attn_workspace_bytes(ctx, 1, 64), ta.tucker_attn_workspace_bytes(ctx, 2, 128)
        assert 0 < small < big and small % 256 == 0
        assert ta.tucker_attn_workspace_bytes(ctx, 1, 1) == small          # tokens are padded to 64
        assert ta.tucker_attn_decode_workspace_bytes(ctx, 0) == 0
        assert 0 < ta.tucker_attn_decode_workspace_bytes(ctx, 4) <= ta.tucker_attn_decode_workspace_bytes(ctx, 32)
        # batches above 32 sequences run in passes of 32 that share the workspace
        assert ta.tucker_attn_decode_workspace_bytes(ctx, 1000) == ta.tucker_attn_decode_workspace_bytes(ctx, 32)
        lib = ta.load_library()
        w = ta.tucker_attn_weights(*([1] * 8))
        # null X / Y / workspace, bad sizes: rejected on the host before any launch
        assert lib.tucker_attn_forward(ctx, C.byref(w), None, None, 1, 16, 0, None, None, 0, None, 0, None) == -1
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 0, 16, 0, None, None, 0, 256, 1 << 30, None) == -1
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 1, 16, -1, None, None, 0, 256, 1 << 30, None) == -1
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 1, 16, 0, 256, None, 64, 256, 1 << 30, None) == -1
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 1, 16, 0, None, None, 0, 256, 16, None) == -3
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 1, 16, 0, None, None, 0, 257, 1 << 30, None) == -1
        lens = (C.c_int32 * 2)(5, 0)
        assert lib.tucker_attn_decode(ctx, C.byref(w), 256, 256, 256, 256, 8, lens, 2, 256, 1 << 30, None) == -1
        lens = (C.c_int32 * 2)(5, 9)
        assert lib.tucker_attn_decode(ctx, C.byref(w), 256, 256, 256, 256, 8, lens, 2, 256, 1 << 30, None) == -1
        lens = (C.c_int32 * 2)(5, 8)
        assert lib.tucker_attn_decode(ctx, C.byref(w), 256, 256, 256, 256, 8, lens, 2, 256, 16, None) == -3
        # more padded tokens than the launch grids can index: refused before anything is enqueued
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 1, 65535 * 32 + 1, 0, None, None, 0, 256, 1 << 60, None) == -2
        assert lib.tucker_attn_forward(ctx, C.byref(w), 256, 256, 70000, 16, 0, None, None, 0, 256, 1 << 60, None) == -2
        # the attended part of one sequence's cache must stay below 2 GiB (r3 = 32 fp32 channels = 128 bytes per row)
        lens = (C.c_int32 * 1)(1 << 24)
        assert lib.tucker_attn_decode(ctx, C.byref(w), 256, 256, 256, 256, 1 << 24, lens, 1, 256, 1 << 30, None) == -2
        lens = (C.c_int32 * 1)((1 << 24) - 1)
        assert lib.tucker_attn_decode(ctx, C.byref(w), 256, 256, 256, 256, 1 << 24, lens, 1, 256, 16, None) == -3
    finally:
        ta.tucker_attn_destroy(ctx)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "one-GPU" in r.stderr and r.stdout.strip() == ""


def test_shared_kv_config_is_validated_on_the_host():
    with pytest.raises(ta.TuckerAttnError) as e:                  # value rank must equal the key rank
        ta.tucker_attn_create(**_cfg(rt3=16, shared_kv=True))
    assert "status -1 " in str(e.value)
    ctx = ta.tucker_attn_create(**_cfg(shared_kv=True))
    ta.tucker_attn_destroy(ctx)


def test_memory_footprint_helpers_match_the_closed_forms_and_the_printed_gpt2_figures():
    from oracle import sizes
    d, nH, layers, N = 768, 12, 12, 1024
    # GPT-2 table of the paper: attention parameters and KV cache in MB (bf16, 12 layers, N = 1024)
    for ranks, p_mb, kv_mb in (((8, 128, 128), 15.74, 6.28), ((8, 128, 64), 10.24, 3.14), ((8, 64, 64), 6.31, 3.14)):
        r1, r2, r3 = ranks
        n = ta.tucker_attn_parameter_count(d_model=d, n_heads=nH, r1=r1, r2=r2, r3=r3)
        assert n == sizes.tucker_params(d, nH, r1, r2, r3)
        assert abs(n * 2 * layers / 1e6 - p_mb) < 0.02           # printed to two decimals, 10.24 for 10.228
        ctx = ta.tucker_attn_create(**_cfg(d_model=d, n_heads=nH, r1=r1, r2=r2, r3=r3, dtype="bf16", max_positions=N))
        try:
            b = ta.tucker_attn_cache_bytes(ctx, 1, N)
            assert b == sizes.tucker_cache(N, r3) * 2
            assert abs(b * layers / 1e6 - kv_mb) < 0.02            # the table prints 6.28 for 6.2915
            assert ta.tucker_attn_cache_bytes(ctx, 0, N) == 0 and ta.tucker_attn_cache_bytes(ctx, 1, 0) == 0
        finally:
            ta.tucker_attn_destroy(ctx)
    # shared key-value latent: one d x r3 factor and one cache fewer; separate post-softmax ranks
    assert ta.tucker_attn_parameter_count(d_model=d, n_heads=nH, r1=8, r2=128, r3=128, shared_kv=True) == \
        sizes.tucker_params(d, nH, 8, 128, 128, True)
    assert ta.tucker_attn_parameter_count(d_model=64, n_heads=4, r1=2, r2=8, r3=16, rt1=3, rt2=24, rt3=32) == \
        (4 * 2 + 64 * (8 + 16) + 2 * 8 * 16) + (4 * 3 + 64 * (24 + 32) + 3 * 24 * 32)
    ctx = ta.tucker_attn_create(**_cfg(r3=32, shared_kv=True, dtype="f32"))
    try:
        assert ta.tucker_attn_cache_bytes(ctx, 3, 100) == 3 * 100 * 32 * 4
    finally:
        ta.tucker_attn_destroy(ctx)
    assert ta.load_library().tucker_attn_parameter_count(None) == 0
