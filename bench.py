#!/usr/bin/env python3
"""Benchmark of the Tucker-attention forward hot path on one MI355X.

One "step" = one call of the whole path (weight prep, factor projection, latent RoPE, fused
attention, head merge, output projection) on one batch of synthetic input that is already
resident in HBM.  Default workload: the LLaMA-7B-shaped causal layer at N=4096 (bf16).
Prints ONE JSON line on stdout; progress and the per-kernel table go to stderr.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# MI355X published dense peaks.  The bf16 figure is the rounded 2.5 PFLOP/s; at 256 compute units x 4096
# FLOP/clock x 2.4 GHz it is 2516.6, so fractions quoted here are 0.7 % (relative) above that basis.
PEAK_BF16_TFLOPS = 2500.0
PEAK_FP32_MFMA_TFLOPS = 157.3
PEAK_HBM_GBS = 8000.0

TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic.json")


def library_build_id():
    """Hash of the kernel sources the loaded library was built from (the library is built in-tree from
    exactly these files), so that figures measured with one build are not reported for another."""
    import hashlib
    csrc = os.path.join(ROOT, "paper_2603_30033_amd", "csrc")
    h = hashlib.sha1()
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            h.update(open(os.path.join(csrc, name), "rb").read())
    return h.hexdigest()[:16]


def measured_traffic(workload, kernel):
    """HBM bytes per launch of `kernel` (read + written) from the hardware-counter runs recorded in
    profiles/hbm_traffic.json (written by `bench.py --pmc-summary`), or None if there is no record for this
    workload and kernel made with the library build that is loaded now."""
    try:
        rec = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        return None
    e = rec.get(f"{workload}:{kernel}")
    if not e or e.get("build_id") != library_build_id():
        return None
    return e.get("bytes")


def pmc_summary(args):
    """Turn two rocprofv3 --pmc runs (FETCH_SIZE, WRITE_SIZE; KiB per dispatch) of `bench.py --workload W
    --copy-calibration-mib M` into HBM bytes per launch of the kernels named by --pmc-kernels, scaled by what
    the same counters read for the plain copy of known size, and record them in profiles/hbm_traffic.json."""
    import csv
    import glob

    def per_kernel(root, counter):
        """mean and largest reading per kernel name, and the number of dispatches"""
        tot, cnt, top = {}, {}, {}
        for f in glob.glob(os.path.join(root, "**", "*counter_collection.csv"), recursive=True):
            for row in csv.DictReader(open(f)):
                if row.get("Counter_Name") != counter:
                    continue
                k, v = row["Kernel_Name"], float(row["Counter_Value"])
                tot[k] = tot.get(k, 0.0) + v
                cnt[k] = cnt.get(k, 0) + 1
                top[k] = max(top.get(k, 0.0), v)
        return {k: tot[k] / cnt[k] for k in tot}, cnt, top

    fetch, nf, fetch_top = per_kernel(args.pmc_summary[0], "FETCH_SIZE")
    write, nw, write_top = per_kernel(args.pmc_summary[1], "WRITE_SIZE")
    copy_bytes = args.copy_calibration_mib << 20
    # the calibration copy is the largest dispatch of the runtime's buffer-copy kernel (smaller ones move inputs)
    ck = [k for k in fetch_top if "copybuffer" in k.lower()]
    assert ck and copy_bytes > 0, "the counter runs must include the calibration copy (--copy-calibration-mib)"
    ck = max(ck, key=lambda k: fetch_top[k])
    f_scale, w_scale = copy_bytes / (fetch_top[ck] * 1024.0), copy_bytes / (write_top[ck] * 1024.0)
    try:
        rec = json.load(open(TRAFFIC_JSON))
    except (OSError, ValueError):
        rec = {}
    for spec in args.pmc_kernels:
        label, pattern = spec.split("=", 1)
        pats = pattern.split("+")
        fk = [k for k in fetch if any(p in k for p in pats)]
        assert fk, f"no kernel matches {pattern}"
        rd = sum(fetch[k] for k in fk) * 1024.0 * f_scale
        wr = sum(write.get(k, 0.0) for k in fk) * 1024.0 * w_scale
        rec[f"{args.workload}:{label}"] = {
            "bytes": int(rd + wr), "read_bytes": int(rd), "written_bytes": int(wr), "dispatches": int(nf[fk[0]]),
            "fetch_scale": round(f_scale, 4), "write_scale": round(w_scale, 4), "build_id": library_build_id(),
            "kernels": sorted(fk)}
        log(f"{args.workload}:{label}: read {rd / 2**20:.1f} MiB, written {wr / 2**20:.1f} MiB per launch "
            f"(scales {f_scale:.4f}, {w_scale:.4f})")
    json.dump(rec, open(TRAFFIC_JSON, "w"), indent=1, sort_keys=True)


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def flops(w, N=None, B=None):
    """Algorithmic FLOPs of one forward (multiply-add = 2), per step of the path.
    The per-head query and the head merge are counted in their cheaper form factored through
    the head rank r1; causal attention counts only visible pairs."""
    B = w.B if B is None else B
    N = w.N if N is None else N
    rt1, rt2, rt3 = w.ranks_post()
    d, nH = w.d_model, w.n_heads
    if w.mode == "decode":
        T = B
        pairs = w.kv_len
    else:
        T = B * N
        pairs = N * (N + 1) // 2 if w.causal else N * N
    proj = 2 * T * d * (w.r2 + w.r3 + (0 if w.shared_kv else rt3))      # a shared latent is projected once
    qhat = min(2 * T * nH * w.r2 * w.r3, 2 * T * w.r1 * w.r2 * w.r3 + 2 * T * nH * w.r1 * w.r3)
    attn = B * nH * pairs * (2 * w.r3 + 2 * rt3)
    merge = min(2 * T * nH * rt2 * rt3, 2 * T * rt1 * rt2 * rt3 + 2 * T * nH * rt1 * rt3)
    out = 2 * T * rt2 * d
    return dict(proj=proj, qhat=qhat, attn=attn, merge=merge, out=out,
                total=proj + qhat + attn + merge + out)


def backward_flops(w):
    """Algorithmic FLOPs of one backward: every product of the forward has two gradient products of the
    same size, and the attention has five products per visible (query, key) pair (scores and dP are
    recomputed once, then dQ, dK, dV) against the forward's two.  Re-running the forward, which this
    library's backward does inside the call, is not counted."""
    f = flops(w)
    rt3 = w.ranks_post()[2]
    pairs = w.N * (w.N + 1) // 2 if w.causal else w.N * w.N
    attn = w.B * w.n_heads * pairs * (6 * w.r3 + 4 * rt3)
    dense = 2 * (f["proj"] + f["qhat"] + f["merge"] + f["out"])
    return dict(attn=attn, dense=dense, total=attn + dense)


def mandatory_bytes(w):
    es = 2 if w.dtype == "bf16" else 4
    rt1, rt2, rt3 = w.ranks_post()
    wts = (w.r1 * w.r2 * w.r3 + rt1 * rt2 * rt3 + w.n_heads * (w.r1 + rt1)
           + w.d_model * (w.r2 + w.r3 + rt2 + rt3)) * es
    if w.mode == "decode":
        return w.B * w.kv_len * (w.r3 + (0 if w.shared_kv else rt3)) * es + wts + 2 * w.B * w.d_model * es
    return 2 * w.B * w.N * w.d_model * es + wts


def cpu_baseline(w, backward=False):
    """The oracle as it stands, timed on the host cores on a bounded sample of the workload."""
    import numpy as np
    from threadpoolctl import threadpool_info

    from oracle import tucker_oracle as orc
    from paper_2603_30033_amd import workloads as wl
    if w.mode == "decode":
        ws = wl.scaled(w, B=2)
        inp = wl.make_inputs(ws)
        t0 = time.perf_counter()
        if ws.shared_kv:
            orc.decode_step_shared_kv(inp["X"][:, 0], inp["Lcache"], inp["kv_len"], wl.weights_of(inp),
                                      ws.d_head, ws.rope_base)
        else:
            orc.decode_step(inp["X"][:, 0], inp["Kcache"], inp["Vcache"], inp["kv_len"], wl.weights_of(inp),
                            ws.d_head, ws.rope_base)
        dt = time.perf_counter() - t0
        f = flops(ws)["total"]
        sample = f"decode step of {ws.B} of the {w.B} sequences at kv_len={w.kv_len} (cache given, as for the GPU)"
    elif backward:
        from oracle import tucker_backward as orb
        n = min(w.N, 2048)
        b = 1 if w.N >= 1024 else min(w.B, 8)
        ws = wl.scaled(w, B=b, N=n)
        inp = wl.make_inputs(ws)
        dY = np.random.default_rng(1).standard_normal(inp["X"].shape).astype(np.float32)
        t0 = time.perf_counter()
        orb.backward(inp["X"], dY, wl.weights_of(inp), ws.d_head, ws.causal, ws.rope_base, shared_kv=ws.shared_kv)
        dt = time.perf_counter() - t0
        f = backward_flops(ws)["total"]
        sample = f"full oracle backward of {b} sequence(s) of {n} tokens of the same layer shape"
    else:
        n = min(w.N, 4096)
        b = min(w.B, 2) if w.N >= 1024 else min(w.B, 16)        # about 10 s of host time at the LLaMA-7B shape
        ws = wl.scaled(w, B=b, N=n)
        inp = wl.make_inputs(ws)
        t0 = time.perf_counter()
        orc.per_head_forward(inp["X"], wl.weights_of(inp), ws.d_head, ws.causal, ws.rope_base)
        dt = time.perf_counter() - t0
        f = flops(ws)["total"]
        sample = f"full oracle forward of {b} sequence(s) of {n} tokens of the same layer shape"
    threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    # cores = threads of the BLAS pool the oracle's matrix products ran on; host_cpus = what the box reports
    return {"value": f / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "cores_kind": "BLAS threads",
            "host_cpus": os.cpu_count(), "kind": "oracle", "sample": sample, "seconds": round(dt, 3)}


def bench_convert_hosvd(w, args):
    """Time the MHA -> Tucker conversion at the layer shape and ranks of workload `w`."""
    import numpy as np
    import torch

    from paper_2603_30033_amd import device as dev
    from paper_2603_30033_amd import workloads as wl

    d, nH, dH = w.d_model, w.n_heads, w.d_head
    ranks, ranks_t = (w.r1, w.r2, w.r3), w.ranks_post()
    log(f"generating MHA weights d={d} nH={nH} dH={dH} ...")
    host = wl.make_classic_weights(d, nH, dH, w.seed + 7, w.dtype)
    D = {k: dev.to_device(v, w.dtype) for k, v in host.items()}
    K, W = args.steps, args.warmup
    infos = []

    def step():
        dev.from_mha_hosvd(D["WQ"], D["WK"], D["WV"], D["WO"], nH, ranks, ranks_t, w.shared_kv)
        infos.append(dev.from_mha_hosvd.last_info)

    for _ in range(W):
        step()
    torch.cuda.synchronize()
    infos.clear()
    t0 = time.perf_counter()
    for _ in range(K):
        step()
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / K
    launches = sum(i["jacobi_launches"] for i in infos) / K
    jac_ms = sum(i["jacobi_ms"] for i in infos) / K
    jac_bytes = sum(i["jacobi_bytes"] for i in infos) / K
    ach = jac_bytes / (jac_ms * 1e-3) / 1e9 if jac_ms > 0 else 0.0
    log(f"{w.name}: {dt:.3f} s per conversion; Jacobi iterations {jac_ms:.1f} ms in {launches:.0f} launches, "
        f"sweeps {infos[-1]['sweeps']}, {ach:.0f} GB/s")
    out = {
        "metric": "hosvd_conversion_seconds", "value": dt, "unit": "s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": dt * 1e3, "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": w.name, "d_model": d, "n_heads": nH, "d_head": dH, "ranks": list(ranks),
                   "ranks_post": list(ranks_t), "shared_kv": w.shared_kv, "storage": w.dtype},
        "pass": "convert_hosvd", "sweeps": infos[-1]["sweeps"],
        "roofline": {"kernel": "jacobi_block_kernel", "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS,
                     "unit": "GB/s", "frac": ach / PEAK_HBM_GBS,
                     "traffic": measured_traffic(w.name, "jacobi_block_kernel"),
                     "algorithmic_bytes": jac_bytes / max(launches, 1), "avg_us": jac_ms * 1e3 / max(launches, 1),
                     "launches": launches},
    }
    if not args.no_cpu_baseline:
        # the oracle builds the dense nH x d x d tensors: bounded to a layer of at most 768 channels
        from threadpoolctl import threadpool_info

        from oracle import conversions as cv
        ds = min(d, 768)
        hs = max(1, min(nH, ds // dH))
        sample = wl.make_classic_weights(ds, hs, dH, w.seed + 7, w.dtype)
        rs = (min(ranks[0], hs), min(ranks[1], ds), min(ranks[2], ds))
        rts = (min(ranks_t[0], hs), min(ranks_t[1], ds), min(ranks_t[2], ds))
        log("timing the CPU oracle on a bounded sample ...")
        t0 = time.perf_counter()
        cv.mha_to_tucker_hosvd(sample["WQ"], sample["WK"], sample["WV"], sample["WO"], hs, rs, rts, shared_kv=w.shared_kv)
        cpu = time.perf_counter() - t0
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        out["cpu_baseline"] = {"value": cpu, "unit": "s", "cores": int(threads), "cores_kind": "BLAS threads",
                               "host_cpus": os.cpu_count(), "kind": "oracle",
                               "sample": f"oracle conversion of a layer with d={ds}, {hs} heads of width {dH} "
                                         f"(dense tensors, LAPACK SVD of the three unfoldings)"}
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="llama7b_n4096")
    ap.add_argument("--batch", type=int, default=0, help="override the workload's number of sequences")
    ap.add_argument("--seq-len", type=int, default=0,
                    help="override the workload's tokens per sequence (prefill) or cache length (decode)")
    ap.add_argument("--pass", dest="which",
                    choices=["forward", "backward", "backward_self_contained", "convert_hosvd"],
                    default="forward",
                    help="convert_hosvd: one step = one conversion of synthetic MHA weights of the workload's layer "
                         "shape into Tucker weights of the workload's ranks (tucker_convert_from_mha_hosvd); "
                         "backward: one step = one tucker_attn_backward call on the state a forward call left in "
                         "the shared workspace (the forward is run once, untimed); backward_self_contained: the "
                         "backward call re-runs the forward inside (prefill workloads only)")
    ap.add_argument("--frozen-weights", action="store_true",
                    help="prepare the operand-layout copies of the weights once, outside the timed region "
                         "(tucker_attn_prepare_weights); the default keeps that step inside every call")
    ap.add_argument("--hip-graph", action="store_true",
                    help="capture the launches of one step into a HIP graph once and time replays of it (the library "
                         "only enqueues kernels on the caller's stream, so a step can be captured as it is)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--mfma-ceiling", action="store_true",
                    help="only measure what the matrix pipe of this board sustains on a bf16 MFMA loop with random "
                         "operands (registers only, and fed from LDS like the attention kernel) and print it as JSON")
    ap.add_argument("--pmc-summary", nargs=2, metavar=("FETCH_DIR", "WRITE_DIR"),
                    help="no GPU work: read the counter CSVs of two rocprofv3 --pmc runs of this script (FETCH_SIZE, "
                         "WRITE_SIZE) and record HBM bytes per launch in profiles/hbm_traffic.json")
    ap.add_argument("--pmc-kernels", nargs="*", default=[],
                    help="with --pmc-summary: label=substring[+substring] of the kernel names to record")
    ap.add_argument("--copy-calibration-mib", type=int, default=0,
                    help="also launch a plain device-to-device copy of this many MiB (three times), so that a "
                         "hardware-counter run holds a kernel of known HBM traffic to scale its readings by")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py measures the one-GPU hot path only; run it with --gpus 1 "
            "(batch, head and sequence sharding are described in the repository's design notes)")
        sys.exit(2)

    if args.pmc_summary:
        pmc_summary(args)
        return

    import numpy as np
    import torch

    from paper_2603_30033_amd import binding as ta
    from paper_2603_30033_amd import workloads as wl
    from paper_2603_30033_amd.device import Layer, to_device

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.mfma_ceiling:
        regs = ta.tucker_attn_measure_mfma_ceiling(False)
        lds = ta.tucker_attn_measure_mfma_ceiling(True)
        print(json.dumps({"metric": "mfma_ceiling_bf16", "unit": "TFLOP/s", "operands_in_registers": regs,
                          "one_operand_from_lds": lds, "published_peak": PEAK_BF16_TFLOPS,
                          "frac_registers": regs / PEAK_BF16_TFLOPS, "frac_lds": lds / PEAK_BF16_TFLOPS,
                          "what": "bf16 32x32x16 MFMA loop, pseudo-random operands, 8 waves per compute unit, best of 5"}),
              flush=True)
        return
    w = wl.WORKLOADS[args.workload]
    if args.batch > 0:
        w = wl.scaled(w, B=args.batch, name=f"{w.name}_B{args.batch}")
    if args.seq_len > 0:
        w = wl.scaled(w, name=f"{w.name}_L{args.seq_len}",
                      **({"kv_len": args.seq_len} if w.mode == "decode" else {"N": args.seq_len}))
    if args.which == "convert_hosvd":
        print(json.dumps(bench_convert_hosvd(w, args)), flush=True)
        return
    log(f"generating {w.name} ...")
    inp = wl.make_inputs(w)
    K, W = args.steps, args.warmup
    fl = flops(w)
    backward = args.which != "forward"
    saved = args.which == "backward"
    if backward and w.mode == "decode":
        log("a decode step has no backward pass")
        sys.exit(2)
    if backward:
        fb = backward_flops(w)

    if args.copy_calibration_mib > 0:
        src = torch.randint(0, 255, (args.copy_calibration_mib << 20,), dtype=torch.uint8, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    with Layer(w, inp, save_for_backward=backward and saved) as layer:
        if args.frozen_weights:
            layer.freeze_weights()
        if w.mode == "decode":
            x = to_device(inp["X"][:, 0], w.dtype)
            y = torch.empty_like(x)
            # three cache copies in rotation so that a step streams its cache from HBM, not from
            # the last-level cache that the previous step filled
            if w.shared_kv:
                caches = [(to_device(inp["Lcache"], w.dtype), None) for _ in range(3)]
            else:
                caches = [(to_device(inp["Kcache"], w.dtype), to_device(inp["Vcache"], w.dtype)) for _ in range(3)]
            lens = [int(v) for v in inp["kv_len"]]
            ws = layer.workspace(ta.tucker_attn_decode_workspace_bytes(layer.ctx, w.B))
            step_i = [0]

            def step():
                kc, vc = caches[step_i[0] % 3]
                step_i[0] += 1
                ta.tucker_attn_decode(layer.ctx, layer.weights, x, y, kc, vc, lens, ws)
            units = w.B
        else:
            X = to_device(inp["X"], w.dtype)
            Y = torch.empty_like(X)
            ws = layer.workspace(ta.tucker_attn_workspace_bytes(layer.ctx, w.B, w.N))
            if backward:
                dY = to_device(wl.round_to_storage(
                    np.random.default_rng(w.seed + 1000).standard_normal(inp["X"].shape).astype(np.float32), w.dtype),
                    w.dtype)
                grads = {"d" + k: torch.empty(v.shape, dtype=torch.float32, device="cuda")
                         for k, v in layer.weights.items()}
                ws = layer.workspace(ta.tucker_attn_backward_workspace_bytes(layer.ctx, w.B, w.N))
                dX = torch.empty_like(X)
                if saved:
                    ta.tucker_attn_forward(layer.ctx, layer.weights, X, Y, w.pos0, None, None, ws)

                def step():
                    ta.tucker_attn_backward(layer.ctx, layer.weights, X, dY, dX, grads, w.pos0, ws,
                                            forward_state=saved)
            else:
                def step():
                    ta.tucker_attn_forward(layer.ctx, layer.weights, X, Y, w.pos0, None, None, ws)
            units = w.B * w.N

        timed_step = step
        if args.hip_graph:
            # one captured step per cache buffer, replayed in rotation (a decode step keeps streaming its cache
            # from HBM; a prefill workload has one buffer set, i.e. one graph)
            n_graphs = 3 if w.mode == "decode" else 1
            for _ in range(n_graphs):
                step()                                          # first calls outside the capture
            torch.cuda.synchronize()
            graphs = []
            side = torch.cuda.Stream()
            side.wait_stream(torch.cuda.current_stream())
            with torch.cuda.stream(side):
                for _ in range(n_graphs):
                    gr = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(gr, stream=side):
                        step()
                    graphs.append(gr)
            torch.cuda.current_stream().wait_stream(side)
            replay_i = [0]

            def timed_step():
                graphs[replay_i[0] % n_graphs].replay()
                replay_i[0] += 1

        def event_times(n):
            """n steps, each between its own pair of HIP events on the stream the library launches on."""
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(n)]
            for a, b in ev:
                a.record()
                timed_step()
                b.record()
            torch.cuda.synchronize()
            return [a.elapsed_time(b) for a, b in ev]

        # Clock warm-up (untimed, before --warmup): the first launches after idle run at a lower shader clock, and
        # under back-to-back launches the clock then settles at what the power limit allows.  Blocks of 10
        # back-to-back steps (timed as the K steps below are: wall clock, device synchronised on both sides) are
        # run until the last three blocks agree within 1 %, at least 5 and at most 60 blocks.
        clock_steps, blocks = 0, []
        for _ in range(60):
            torch.cuda.synchronize()
            tb = time.perf_counter()
            for _ in range(10):
                timed_step()
            torch.cuda.synchronize()
            blocks.append(time.perf_counter() - tb)
            clock_steps += 10
            last = blocks[-3:]
            if len(blocks) >= 5 and max(last) - min(last) <= 0.01 * min(last):
                break
        for _ in range(W):
            timed_step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            timed_step()
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        ms = dt / K * 1e3
        # the same K steps once more, each timed by its own event pair: median and minimum
        per_step = event_times(K)
        median_ms, min_ms = float(np.median(per_step)), float(np.min(per_step))

        # per-kernel durations: K more steps with HIP events around every launch.  Reading a step's events
        # means waiting for it, and a step that starts on an idle device runs at another clock than one in a
        # back-to-back stream (the attention launch was seen 10 % slower that way), so every profiled step is
        # preceded by three ordinary ones queued with it.
        acc = {}
        order = []
        for _ in range(K):
            for _ in range(3):
                step()
            ta.tucker_attn_profile_enable(layer.ctx, True)
            step()
            for name, t in ta.tucker_attn_profile_read(layer.ctx):
                if name not in acc:
                    acc[name] = 0.0
                    order.append(name)
                acc[name] += t
            ta.tucker_attn_profile_enable(layer.ctx, False)
        kern_ms = {n: acc[n] / K for n in order}
        # entries "<name>_kernel": a kernel alone, from events attached to its dispatch (not a step of its own)
        alone_ms = {n: kern_ms.pop(n) for n in list(kern_ms) if n.endswith("_kernel")}
        order = [n for n in order if n in kern_ms]

        # the same K steps once more with the weights prepared beforehand (what a serving loop with fixed weights
        # runs: step a0 hoisted out of the call); reported beside `value`, never as `value`
        prepared_ms = None
        if not args.frozen_weights and not backward and not args.hip_graph:
            layer.freeze_weights()
            for _ in range(max(W, 20)):
                step()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(K):
                step()
            torch.cuda.synchronize()
            prepared_ms = (time.perf_counter() - t0) / K * 1e3

    total_flops = fb["total"] if backward else fl["total"]
    tflops = total_flops / (ms * 1e-3) / 1e12
    log(f"{w.name}: {ms:.4f} ms/step (events: median {median_ms:.4f}, min {min_ms:.4f}; {clock_steps} clock warm-up "
        f"steps), {tflops:.1f} TFLOP/s algorithmic, {units / (ms * 1e-3):.3e} tokens/s")
    if prepared_ms is not None:
        log(f"  with prepared weights (step a0 hoisted out of the call): {prepared_ms:.4f} ms/step")
    for n in order:
        log(f"  {n:20s} {kern_ms[n] * 1e3:9.1f} us" +
            (f"   (the kernel alone: {alone_ms[n + '_kernel'] * 1e3:.1f} us)" if n + "_kernel" in alone_ms else ""))
    log(f"  sum of kernels       {sum(kern_ms.values()) * 1e3:9.1f} us")

    if backward:
        # the two attention-gradient kernels together, against the five products per visible pair
        dom = "attention_bwd_dq+attention_bwd_dkv"
        t_ms = kern_ms["attention_bwd_dq"] + kern_ms["attention_bwd_dkv"]
        peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
        alg = fb["attn"] + 2 * fl["qhat"]
        ach = alg / (t_ms * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": measured_traffic(w.name, dom), "algorithmic_flops": alg,
                "avg_us": t_ms * 1e3}
    elif w.mode == "decode":
        dom = "decode_attention"
        es = 2 if w.dtype == "bf16" else 4
        rt3 = w.ranks_post()[2]
        alg_bytes = w.B * w.kv_len * (w.r3 + (0 if w.shared_kv else rt3)) * es
        t_ms = alone_ms.get(dom + "_kernel", kern_ms[dom])
        ach = alg_bytes / (t_ms * 1e-3) / 1e9
        roof = {"kernel": dom, "bound": "hbm", "achieved": ach, "peak": PEAK_HBM_GBS, "unit": "GB/s",
                "frac": ach / PEAK_HBM_GBS, "traffic": measured_traffic(w.name, dom),
                "algorithmic_bytes": alg_bytes, "avg_us": t_ms * 1e3, "between_events_us": kern_ms[dom] * 1e3}
    else:
        dom = "attention"
        peak = PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS
        t_ms = alone_ms.get(dom + "_kernel", kern_ms[dom])
        ach = (fl["attn"] + fl["qhat"]) / (t_ms * 1e-3) / 1e12
        roof = {"kernel": dom, "bound": "mfma", "achieved": ach, "peak": peak, "unit": "TFLOP/s",
                "frac": ach / peak, "traffic": measured_traffic(w.name, dom),
                "algorithmic_flops": fl["attn"] + fl["qhat"], "avg_us": t_ms * 1e3,
                "between_events_us": kern_ms[dom] * 1e3}

    out = {
        "metric": ("tucker_attn_bwd_tflops" if backward else
                   "tucker_attn_fwd_tflops" if w.mode != "decode" else "tucker_attn_decode_tflops"),
        "value": tflops, "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W, "ms_per_step": ms,
        "median_ms": median_ms, "min_ms": min_ms, "clock_warmup_steps": clock_steps,
        "ms_per_step_prepared_weights": prepared_ms,
        "timing": "value and ms_per_step: wall clock around the K steps, device synchronised on both sides; "
                  "median_ms and min_ms: one HIP event pair per step on the launch stream, K further steps; "
                  "clock_warmup_steps untimed steps ran first, until the step time settled",
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": w.name, "B": w.B, "N": w.N if w.mode != "decode" else w.kv_len,
                   "d_model": w.d_model, "n_heads": w.n_heads, "d_head": w.d_head,
                   "ranks": [w.r1, w.r2, w.r3], "causal": w.causal, "rope_base": w.rope_base, "mode": w.mode,
                   "shared_kv": w.shared_kv},
        "tokens_per_s": units / (ms * 1e-3),
        "pass": args.which, "frozen_weights": bool(args.frozen_weights), "hip_graph": bool(args.hip_graph),
        "pct_mfma_peak": 100.0 * tflops / (PEAK_BF16_TFLOPS if w.dtype == "bf16" else PEAK_FP32_MFMA_TFLOPS),
        "hbm_gbs_mandatory": mandatory_bytes(w) / (ms * 1e-3) / 1e9,
        "algorithmic_gflop": total_flops / 1e9,
        "kernel_us": {n: kern_ms[n] * 1e3 for n in order},
        "peak_basis": "published dense peaks: bf16 MFMA 2500 TFLOP/s (2516.6 at 2.4 GHz), HBM 8000 GB/s",
        "library_build_id": library_build_id(),
        "roofline": roof,
    }
    if not args.no_cpu_baseline:
        log("timing the CPU oracle on a bounded sample ...")
        out["cpu_baseline"] = cpu_baseline(w, backward)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
