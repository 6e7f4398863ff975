#!/usr/bin/env python3
"""Bench: Flash-Attention forward on one MI355X, headline workload.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--config 4] [--no-cpu-baseline]
    python bench.py --config N                          # baseline workloads 1..5 (4 = headline)
    python bench.py --config 4 --inputs zeros           # same launch on all-zero tensors (power-limit evidence)
    python bench.py --paper-seq 16384 [--dtype f16]     # the paper's own sweep shape (Section 6.2)
    python bench.py --probe-mfma                        # matrix-pipe ceiling: MFMA-only loop of the debug build
    python bench.py --probe-dq-atomics                  # cost of a single-pass backward's atomic dQ reduction alone
    python bench.py --timeline --config 3               # per-workgroup phase timing of one forward launch (debug build)
    python bench.py --config 3 --compare-lib old.so     # A/B against another build of the library, same process

A "step" is one attn_fwd call (the whole hot path) over one batch of seeded
synthetic Q/K/V that is already resident in HBM.  Prints ONE JSON line.

--paper-seq S times the shape of the paper's forward-attention figures instead
(BATCH=4, NUM_HEADS=32, HEAD_DIM=128, non-causal, S queries and keys, fp16 by
default): N(0,1) values drawn on the device with torch's seeded generator (the
host generator would need minutes for 3 x 268M elements at S = 16384).
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA peak
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.json")  # measured with rocprofv3 --pmc, see profiles/


def measured_traffic(workload):
    """HBM bytes per launch from the committed rocprofv3 counter summary (None if not measured)."""
    try:
        with open(TRAFFIC_FILE) as f:
            t = json.load(f).get(workload)
        return None if t is None else float(t["hbm_bytes_per_launch"])
    except (OSError, ValueError, KeyError):
        return None


def cpu_baseline(cfg, q, k, v, scale, target_seconds=15.0):
    """Time the fp64 oracle (as it stands) on a bounded sample of rows of the same workload."""
    from oracle import attn_oracle
    from paper_2512_18134_amd import synth

    total_rows = cfg["B"] * cfg["H"] * cfg["S_q"]
    rng = np.random.default_rng(1234)
    cores = attn_oracle.max_threads()

    def run(n):
        rows = np.sort(rng.choice(total_rows, size=min(n, total_rows), replace=False)).astype(np.int64)
        t0 = time.perf_counter()
        attn_oracle.attn_ref(q, k, v, cfg["causal"], scale, rows=rows, dtype=cfg.get("dtype", "bf16"))
        dt = time.perf_counter() - t0
        i = rows % cfg["S_q"]
        pairs = np.minimum(i + 1, cfg["S_kv"]).sum() if cfg["causal"] else len(rows) * cfg["S_kv"]
        return dt, 4.0 * cfg["D"] * float(pairs), len(rows)

    dt, fl, n = run(16 * cores)                      # calibration
    n2 = int(max(16 * cores, min(total_rows, n * target_seconds / max(dt, 1e-6))))
    dt, fl, n = run(n2)
    return {"value": fl / dt / 1e12, "unit": "TFLOP/s", "cores": cores, "kind": "oracle",
            "sample": "%d of %d rows (uniform random, seed 1234), %.1f s wall, fp64 two-pass oracle, OpenMP" % (n, total_rows, dt)}


def cpu_baseline_bwd(cfg, q, k, v, d_o, scale, target_seconds=15.0):
    """Time the fp64 backward oracle on whole heads of the same workload (bounded)."""
    from oracle import attn_oracle
    BH = cfg["B"] * cfg["H"]
    per_head = 2.5 * 4.0 * cfg["D"] * (cfg["S_q"] * (cfg["S_q"] + 1) // 2 if cfg["causal"] and cfg["S_q"] == cfg["S_kv"]
                                       else cfg["S_q"] * cfg["S_kv"])
    t0 = time.perf_counter()
    dt_name = cfg.get("dtype", "bf16")
    attn_oracle.attn_bwd_ref(q, k, v, d_o, cfg["causal"], scale, heads=np.array([0], dtype=np.int64), dtype=dt_name)
    dt1 = time.perf_counter() - t0
    n = int(max(1, min(BH - 1, target_seconds / max(dt1, 1e-6))))
    t0 = time.perf_counter()
    attn_oracle.attn_bwd_ref(q, k, v, d_o, cfg["causal"], scale, heads=np.arange(1, 1 + n, dtype=np.int64) % BH,
                             dtype=dt_name)
    dt = time.perf_counter() - t0
    return {"value": n * per_head / dt / 1e12, "unit": "TFLOP/s", "cores": attn_oracle.max_threads(), "kind": "oracle",
            "sample": "%d of %d heads in full, %.1f s wall, fp64 backward oracle, OpenMP" % (n, BH, dt)}


def bench_bwd(args, cfg, qd, kd, vd, scale, stream, fwd_flops, host_qkv):
    """One step = one attn_bwd call (Delta kernel, key-owner sweep, query-owner sweep).  Algorithmic work:
    the five products of the backward pass = 2.5x the forward FLOP (the library computes seven)."""
    import torch
    from paper_2512_18134_amd import binding

    gen = torch.Generator(device=qd.device)
    gen.manual_seed(cfg["seed"] + 1000)
    d_o = torch.randn(qd.shape, generator=gen, device=qd.device, dtype=torch.float32).to(qd.dtype)
    f16 = cfg["dtype"] == "f16"
    fwd, bwd = (binding.attn_fwd_f16, binding.attn_bwd_f16) if f16 else (binding.attn_fwd, binding.attn_bwd)
    o, lse = fwd(qd, kd, vd, causal=cfg["causal"], scale=scale, stream=stream)
    dq, dk, dv = torch.empty_like(qd), torch.empty_like(kd), torch.empty_like(vd)
    ws = torch.empty((2,) + tuple(qd.shape[:3]), dtype=torch.float32, device=qd.device)
    step = lambda: bwd(qd, kd, vd, o, d_o, lse, dq, dk, dv, ws, causal=cfg["causal"], scale=scale, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record(stream)
        step()
        e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    flops = 2.5 * fwd_flops
    ms_per_step = wall * 1e3 / args.steps
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (float(np.mean(kern_ms)) * 1e-3) / 1e12
    out = {
        "metric": "attention bwd TFLOP/s at 1 GPU (%s, D=%d, S=%d, %s)" % (cfg["dtype"], cfg["D"], cfg["S_q"], "causal" if cfg["causal"] else "non-causal"),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"] + "_bwd", "B": cfg["B"], "H": cfg["H"], "S_q": cfg["S_q"], "S_kv": cfg["S_kv"],
                   "D": cfg["D"], "causal": cfg["causal"], "flop_per_step": flops,
                   "kernel_ms_avg": float(np.mean(kern_ms)), "kernel_ms_min": float(np.min(kern_ms))},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(cfg["name"] + "_bwd")},
    }
    if not args.no_cpu_baseline:
        to_bits = lambda t: t.cpu().view(torch.int16).numpy().view(np.uint16)
        q, k, v = host_qkv if host_qkv[0] is not None else (to_bits(qd), to_bits(kd), to_bits(vd))
        out["cpu_baseline"] = cpu_baseline_bwd(cfg, q, k, v, to_bits(d_o), scale)
    print(json.dumps(out), flush=True)


def probe_mfma(args, dev):
    """Matrix-pipe ceiling: the MFMA-only loop of the debug build (attn_probe_mfma: no LDS, no VALU work, no
    memory traffic), 256 CUs x 4 workgroups, one or two waves per SIMD, on random N(0,1), constant and zero bf16
    operands.  Prints one JSON line; run it under rocprofv3 --pmc GRBM_GUI_ACTIVE for the clock."""
    import ctypes
    import torch
    path = os.path.join(ROOT, "paper_2512_18134_amd", "libmi355attn_debug.so")
    lib = ctypes.CDLL(path)
    lib.attn_probe_mfma.restype = ctypes.c_int
    lib.attn_probe_mfma.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    stream = torch.cuda.current_stream(dev)
    gen = torch.Generator(device=dev)
    gen.manual_seed(11)
    n_wg, iters = 1024, 4096
    res = {}
    for waves in (4, 8):
        out = torch.empty((n_wg * waves * 64,), dtype=torch.float32, device=dev)
        for kind in ("random", "constant", "zero"):
            ops = {"random": torch.randn((8 * 64 * 8,), generator=gen, device=dev, dtype=torch.float32),
                   "constant": torch.full((8 * 64 * 8,), 1.0, device=dev),
                   "zero": torch.zeros((8 * 64 * 8,), device=dev)}[kind].to(torch.bfloat16)
            call = lambda: lib.attn_probe_mfma(ops.data_ptr(), out.data_ptr(), n_wg, waves, iters, stream.cuda_stream)
            for _ in range(3):
                assert call() == 0
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for e0, e1 in evs:
                e0.record(stream)
                call()
                e1.record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
            flop = float(n_wg) * waves * iters * 8 * 32768
            res["%d_waves_per_simd_%s" % (waves // 4, kind)] = {"ms": ms, "tflops": flop / ms / 1e9,
                                                               "frac_of_peak": flop / ms / 1e9 / PEAK_BF16_TFLOPS}
    # what the rate on random operands depends on: the operand pattern of consecutive MFMAs, the tile shape of
    # the instruction, the element type (one wave per SIMD; attn_probe_mfma_pattern of the debug build)
    lib.attn_probe_mfma_pattern.restype = ctypes.c_int
    lib.attn_probe_mfma_pattern.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p]
    out = torch.empty((n_wg * 4 * 64,), dtype=torch.float32, device=dev)
    rnd = torch.randn((8 * 64 * 8,), generator=gen, device=dev, dtype=torch.float32)
    patterns = {}
    for pattern, name in enumerate(("both_operands_change", "a_shared_by_pairs", "a_fixed_b_changes", "both_fixed",
                                    "16x16x32_both_change", "f16_both_change")):
        ops = rnd.to(torch.float16 if pattern == 5 else torch.bfloat16)
        call = lambda: lib.attn_probe_mfma_pattern(ops.data_ptr(), out.data_ptr(), n_wg, pattern, iters, stream.cuda_stream)
        for _ in range(3):
            assert call() == 0
        torch.cuda.synchronize()
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
        for e0, e1 in evs:
            e0.record(stream)
            call()
            e1.record(stream)
        torch.cuda.synchronize()
        ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
        flop = float(n_wg) * 4 * iters * 8 * 32768
        patterns[name] = {"ms": ms, "tflops": flop / ms / 1e9, "frac_of_peak": flop / ms / 1e9 / PEAK_BF16_TFLOPS}
    print(json.dumps({"probe": "v_mfma_f32_32x32x16_bf16 issue ceiling (registers only)", "n_wg": n_wg,
                      "iters": iters, "results": res, "random_operand_patterns": patterns}), flush=True)


def probe_dq_atomics(args, dev):
    """What the fp32 atomic reduction of dQ in a single-pass backward (the paper's Section 6.3 form) costs alone:
    attn_probe_dq_atomics of the debug build on the paper's shape (B4 H32 D128), every (128-key tile, 64-query
    tile) pair adding a 64 x 128 fp32 block.  Prints one JSON line."""
    import ctypes
    import torch
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2512_18134_amd", "libmi355attn_debug.so"))
    lib.attn_probe_dq_atomics.restype = ctypes.c_int
    lib.attn_probe_dq_atomics.argtypes = [ctypes.c_void_p] + [ctypes.c_int] * 4 + [ctypes.c_void_p]
    stream = torch.cuda.current_stream(dev)
    res = {}
    for S in (2048, 4096, 8192):
        for causal in (0, 1):
            dq = torch.zeros((128, S, 128), dtype=torch.float32, device=dev)
            call = lambda: lib.attn_probe_dq_atomics(dq.data_ptr(), 128, S, S, causal, stream.cuda_stream)
            assert call() == 0
            torch.cuda.synchronize()
            rows = torch.arange(S, device=dev)
            want = (rows // 64 // 2 + 1 if causal else torch.full((S,), S // 128, device=dev)).to(torch.float32)
            assert torch.equal(dq, want[None, :, None].expand_as(dq)), "atomic sums are wrong"
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(5)]
            for e0, e1 in evs:
                e0.record(stream)
                call()
                e1.record(stream)
            torch.cuda.synchronize()
            ms = float(np.median([e0.elapsed_time(e1) for e0, e1 in evs]))
            nbytes = float(want.sum().item()) * 128 * 128 * 4
            res["S%d_%s" % (S, "causal" if causal else "full")] = {"ms": ms, "atomic_GB": nbytes / 1e9,
                                                                   "TB_per_s": nbytes / ms / 1e9}
    print(json.dumps({"probe": "fp32 atomic dQ reduction of a single-pass backward, B4 H32 D128", "results": res}), flush=True)


def timeline(args, dev):
    """Where the time of one forward launch goes: attn_fwd_trace of the debug build records, per workgroup,
    a constant-rate clock (10 ns) when a tile is taken up, when its first loads are issued, after K(0) and Q
    have landed, before and after the main loop, after O is staged, and when O is stored, plus the CU it ran on
    (behind a finished tile the persistent kernels issue the next tile's loads before they write the finished
    one out, so the two tiles' records overlap there).  Prints one JSON line: the launch's span,
    the mean and maximum of every phase, and per CU the start of its first workgroup (dispatch ramp), the gaps
    between its workgroups and the end of its last one (tail)."""
    import ctypes
    import torch
    from paper_2512_18134_amd import synth
    lib = ctypes.CDLL(os.path.join(ROOT, "paper_2512_18134_amd", "libmi355attn_debug.so"))
    lib.attn_fwd_trace.restype = ctypes.c_int
    lib.attn_fwd_trace.argtypes = ([ctypes.c_void_p] * 5 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p,
                                                                                ctypes.c_void_p, ctypes.c_longlong])
    if args.paper_seq:
        # the paper's Section 6.2 shape (bf16 here: the trace entry point takes bf16)
        S = args.paper_seq
        cfg = {"name": "paper_B4_H32_S%d_D128_%s_bf16" % (S, "causal" if args.causal else "full"), "B": 4, "H": 32,
               "S_q": S, "S_kv": S, "D": 128, "causal": bool(args.causal)}
        scale = synth.default_scale(128)
        gen = torch.Generator(device=dev)
        gen.manual_seed(5)
        qd, kd, vd = [torch.randn((4, 32, S, 128), generator=gen, device=dev, dtype=torch.float32).to(torch.bfloat16)
                      for _ in range(3)]
    else:
        cfg, q, k, v, scale = synth.make_config(args.config)
        to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(torch.bfloat16)
        qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    B, H, S_q, S_kv, D = cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"]
    o = torch.empty_like(qd)
    lse = torch.empty((B, H, S_q), dtype=torch.float32, device=dev)
    n_rec = B * H * ((S_q + 127) // 128)                    # at least one record per workgroup of any tiling
    trace = torch.zeros((n_rec, 8), dtype=torch.int64, device=dev)
    stream = torch.cuda.current_stream(dev)
    call = lambda: lib.attn_fwd_trace(qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o.data_ptr(), lse.data_ptr(), B, H,
                                      S_q, S_kv, D, int(cfg["causal"]), scale, stream.cuda_stream, trace.data_ptr(),
                                      trace.numel())
    for _ in range(max(args.warmup, 3)):
        assert call() == 0
    torch.cuda.synchronize()
    trace.zero_()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    assert call() == 0
    e1.record(stream)
    torch.cuda.synchronize()
    t = trace.cpu().numpy()
    t = t[t[:, 0] != 0]
    us = (t[:, :6] - t[:, 0].min()) / 100.0                 # microseconds since the first workgroup started
    hw, xcc = t[:, 7] & 0xFFFFFFFF, (t[:, 7] >> 32) & 0xF
    issued = (t[:, 6] - t[:, 0].min()) / 100.0
    cu_key = (xcc << 16) | (((hw >> 13) & 7) << 8) | (((hw >> 12) & 1) << 4) | ((hw >> 8) & 0xF)
    phases = {"take_up_to_loads_issued": issued - us[:, 0], "loads_issued_to_k0_q_landed": us[:, 1] - issued,
              "s0_and_setup": us[:, 2] - us[:, 1], "loop": us[:, 3] - us[:, 2],
              "loop_end_to_o_staged": us[:, 4] - us[:, 3], "store_o": us[:, 5] - us[:, 4]}
    # a CU's first tile starts cold; later tiles of a persistent workgroup are taken up behind the previous loop
    is_first = np.zeros(len(t), dtype=bool)
    for key in np.unique(cu_key):
        idx = np.nonzero(cu_key == key)[0]
        is_first[idx[np.argmin(us[idx, 0])]] = True
    first, last, gaps, per_cu = [], [], [], []
    for key in np.unique(cu_key):
        w = us[cu_key == key]
        w = w[np.argsort(w[:, 0])]
        first.append(w[0, 0])
        last.append(w[:, 5].max())
        per_cu.append(len(w))
        # workgroups of one CU that do not overlap: idle time between the end of one and the start of the next
        ends = np.maximum.accumulate(w[:, 5])
        gaps += [max(0.0, float(w[i + 1, 0] - ends[i])) for i in range(len(w) - 1)]
    span = float(us[:, 5].max())
    xcd_of = {int(key): int(key) >> 16 for key in np.unique(cu_key)}
    keys = [int(key) for key in np.unique(cu_key)]
    end_by_xcd = {}
    for key, e in zip(keys, last):
        end_by_xcd.setdefault(xcd_of[key], []).append(e)
    out = {"timeline": cfg["name"], "workgroups": int(len(t)), "cus_used": int(len(first)),
           "event_ms": e0.elapsed_time(e1), "span_us": span,
           "phase_us_mean_max": {k: [float(x.mean()), float(x.max())] for k, x in phases.items()},
           "phase_us_mean_first_tile_of_cu": {k: float(x[is_first].mean()) for k, x in phases.items()},
           "phase_us_mean_later_tiles": {k: (float(x[~is_first].mean()) if (~is_first).any() else None) for k, x in phases.items()},
           "workgroups_per_cu_min_mean_max": [int(min(per_cu)), float(np.mean(per_cu)), int(max(per_cu))],
           "first_start_per_cu_us_mean_max": [float(np.mean(first)), float(np.max(first))],
           "gap_between_workgroups_us_mean_max": [float(np.mean(gaps)) if gaps else 0.0, float(np.max(gaps)) if gaps else 0.0],
           "idle_before_span_end_per_cu_us_mean_max": [float(np.mean(span - np.array(last))), float(np.max(span - np.array(last)))],
           "last_end_per_xcd_us_mean_min_max": {str(x): [float(np.mean(v)), float(np.min(v)), float(np.max(v))]
                                                for x, v in sorted(end_by_xcd.items())},
           "loop_share_of_cu_time": float(phases["loop"].sum() / (len(first) * span))}
    print(json.dumps(out), flush=True)


def compare_lib(args, cfg, entry, qd, kd, vd, o, lse, scale, stream):
    """The same forward call through another build of the library (say the one of an earlier commit), in this
    process on this machine: three rounds, each timing `steps` calls of this build, then of the other (HIP events
    per call); medians over all rounds, and whether the two builds agree bit for bit."""
    import ctypes
    import torch
    def raw_call(path, o_, lse_):
        # both builds through the bare C entry point, so that the host side of a call costs the same
        lib = ctypes.CDLL(os.path.abspath(path))
        fn = lib.attn_fwd_f16 if cfg["dtype"] == "f16" else lib.attn_fwd
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.c_void_p] * 5 + [ctypes.c_int] * 6 + [ctypes.c_float, ctypes.c_void_p]
        args_ = (qd.data_ptr(), kd.data_ptr(), vd.data_ptr(), o_.data_ptr(), lse_.data_ptr(), cfg["B"], cfg["H"],
                 cfg["S_q"], cfg["S_kv"], cfg["D"], int(cfg["causal"]), scale, stream.cuda_stream)

        def call():
            rc = fn(*args_)
            assert rc == 0, rc
        return call
    o2, lse2 = torch.empty_like(o), torch.empty_like(lse)
    call_this = raw_call(os.path.join(ROOT, "paper_2512_18134_amd", "libmi355attn.so"), o, lse)
    call_other = raw_call(args.compare_lib, o2, lse2)
    times = {"this": [], "other": []}
    for _ in range(3):
        for name, call in (("this", call_this), ("other", call_other)):
            for _ in range(3):
                call()
            torch.cuda.synchronize()
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
            for e0, e1 in evs:
                e0.record(stream)
                call()
                e1.record(stream)
            torch.cuda.synchronize()
            times[name] += [e0.elapsed_time(e1) for e0, e1 in evs]
    this_ms, other_ms = float(np.median(times["this"])), float(np.median(times["other"]))
    return {"lib": args.compare_lib, "this_kernel_ms_median": this_ms, "other_kernel_ms_median": other_ms,
            "other_over_this": other_ms / this_ms,
            "same_bits": bool(torch.equal(o.view(torch.int16), o2.view(torch.int16)) and torch.equal(lse, lse2))}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=4, choices=[1, 2, 3, 4, 5],
                    help="baseline workload 1..5 (4 = headline D=128 S=16384 non-causal)")
    ap.add_argument("--inputs", choices=["synth", "zeros"], default="synth",
                    help="zeros: time the same launch on all-zero q, k, v (the matrix pipe then toggles no operand "
                         "bits: what the schedule sustains when the chip is not power limited)")
    ap.add_argument("--probe-mfma", action="store_true",
                    help="time the MFMA-only loop of the debug build on random, constant and zero operands")
    ap.add_argument("--probe-dq-atomics", action="store_true",
                    help="time the fp32 atomic dQ reduction a single-pass backward would issue (debug build)")
    ap.add_argument("--timeline", action="store_true",
                    help="per-workgroup phase timing of one forward launch of --config (debug build)")
    ap.add_argument("--paper-seq", type=int, default=0,
                    help="time the paper's Section 6.2 shape (B=4, H=32, D=128, non-causal) at this sequence length")
    ap.add_argument("--causal", action="store_true", help="with --paper-seq: the causal variant of that shape")
    ap.add_argument("--dtype", choices=["bf16", "f16"], default=None,
                    help="element type (default: bf16 for --config, f16 for --paper-seq)")
    ap.add_argument("--bwd", action="store_true",
                    help="time the backward pass (attn_bwd / attn_bwd_f16: Delta kernel + two sweeps) instead")
    ap.add_argument("--splitkv", type=int, default=0,
                    help="time attn_fwd_splitkv with this many key ranges on the long-context shape "
                         "(B=1, H=8, S_q=256, S_kv=131072, D=128, non-causal; --long-skv changes S_kv)")
    ap.add_argument("--long-skv", type=int, default=131072)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--compare-lib", default="",
                    help="also time the forward call through this other build of libmi355attn.so, interleaved "
                         "with this build's, in the same process")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run a plain 256 MiB device copy instead (to scale rocprofv3's FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (a single attention kernel; nothing is sharded); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2512_18134_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    if args.calibrate_copy:
        n = 256 << 20
        src = torch.randint(0, 255, (n,), dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(args.steps):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "launches": args.steps}))
        return
    dev = torch.device("cuda:0")
    if args.probe_mfma:
        return probe_mfma(args, dev)
    if args.probe_dq_atomics:
        return probe_dq_atomics(args, dev)
    if args.timeline:
        return timeline(args, dev)
    if args.splitkv:
        cfg = dict(name="long_B1_H8_Sq256_Skv%d_D128_full_split%d" % (args.long_skv, args.splitkv), B=1, H=8, S_q=256,
                   S_kv=args.long_skv, D=128, causal=False, seed=300, sharp=False, dtype="bf16")
        tdt = torch.bfloat16
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg["seed"])
        draw = lambda S: torch.randn((1, cfg["H"], S, cfg["D"]), generator=gen, device=dev, dtype=torch.float32).to(tdt)
        qd, kd, vd = draw(cfg["S_q"]), draw(cfg["S_kv"]), draw(cfg["S_kv"])
        scale = synth.default_scale(cfg["D"])
        q = k = v = None
    elif args.paper_seq:
        cfg = synth.paper_workload(args.paper_seq, causal=args.causal)
        cfg["dtype"] = args.dtype or "f16"
        cfg["name"] = cfg["name"].replace("_f16", "_" + cfg["dtype"])
        tdt = torch.float16 if cfg["dtype"] == "f16" else torch.bfloat16
        gen = torch.Generator(device=dev)
        gen.manual_seed(cfg["seed"])
        draw = lambda S: torch.cat([torch.randn((1, cfg["H"], S, cfg["D"]), generator=gen, device=dev,
                                                dtype=torch.float32).to(tdt) for _ in range(cfg["B"])])
        qd, kd, vd = draw(cfg["S_q"]), draw(cfg["S_kv"]), draw(cfg["S_kv"])
        scale = synth.default_scale(cfg["D"])
        q = k = v = None
    else:
        cfg, q, k, v, scale = synth.make_config(args.config)
        cfg = dict(cfg, dtype=args.dtype or "bf16")
        tdt = torch.float16 if cfg["dtype"] == "f16" else torch.bfloat16
        if cfg["dtype"] == "f16":
            q, k, v = synth.make_qkv(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["seed"], cfg["sharp"],
                                     dtype="f16")
            cfg["name"] += "_f16"
        to_dev = lambda bits: torch.from_numpy(bits.view(np.int16)).to(dev).view(tdt)
        qd, kd, vd = to_dev(q), to_dev(k), to_dev(v)
    if args.inputs == "zeros":
        qd, kd, vd = torch.zeros_like(qd), torch.zeros_like(kd), torch.zeros_like(vd)
        cfg = dict(cfg, name=cfg["name"] + "_zero_inputs")
        q = k = v = None
    entry = binding.attn_fwd_f16 if cfg["dtype"] == "f16" else binding.attn_fwd
    o = torch.empty_like(qd)
    lse = torch.empty(qd.shape[:3], dtype=torch.float32, device=dev)
    flops = synth.attention_flops(cfg["B"], cfg["H"], cfg["S_q"], cfg["S_kv"], cfg["D"], cfg["causal"])

    stream = torch.cuda.current_stream(dev)
    if args.bwd:
        return bench_bwd(args, cfg, qd, kd, vd, scale, stream, flops, (q, k, v))
    if args.splitkv:
        ws = torch.empty((binding.attn_fwd_splitkv_workspace_bytes(cfg["B"], cfg["H"], cfg["S_q"], cfg["D"], args.splitkv),),
                         dtype=torch.uint8, device=dev)
        entry = lambda q_, k_, v_, o_, lse_, causal, scale, stream: binding.attn_fwd_splitkv(
            q_, k_, v_, args.splitkv, o_, lse_, ws, causal=causal, scale=scale, stream=stream)
    step = lambda: entry(qd, kd, vd, o, lse, causal=cfg["causal"], scale=scale, stream=stream)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # HIP events on the launch stream around every launch (kernel duration), wall clock around all K steps
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for e0, e1 in evs:
        e0.record(stream)
        step()
        e1.record(stream)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    kern_ms = [e0.elapsed_time(e1) for e0, e1 in evs]
    per_launch_ms = float(np.mean(kern_ms))
    if np.median(kern_ms) < 0.25:
        # A launch this short ends before the host has issued the next one: an event pair around ONE launch then
        # times the host's call path, not the kernel.  Time K launches between one pair of events instead (the
        # host runs ahead of the GPU after the first few), five times over.
        kern_ms = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(args.steps):
                step()
            e1.record(stream)
            torch.cuda.synchronize()
            kern_ms.append(e0.elapsed_time(e1) / args.steps)
    avg_kern_ms = float(np.mean(kern_ms))
    ms_per_step = wall * 1e3 / args.steps
    value = flops / (ms_per_step * 1e-3) / 1e12
    achieved = flops / (avg_kern_ms * 1e-3) / 1e12

    out = {
        "metric": "attention fwd TFLOP/s at 1 GPU (%s, D=%d, S=%d, %s)" % (cfg["dtype"], cfg["D"], cfg["S_q"], "causal" if cfg["causal"] else "non-causal"),
        "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg["dtype"], "data": "synthetic",
        "config": {"workload": cfg["name"], "B": cfg["B"], "H": cfg["H"], "S_q": cfg["S_q"], "S_kv": cfg["S_kv"],
                   "D": cfg["D"], "causal": cfg["causal"], "flop_per_step": flops,
                   "pct_of_bf16_mfma_peak": 100.0 * value / PEAK_BF16_TFLOPS,
                   "kernel_ms_avg": avg_kern_ms, "kernel_ms_min": float(np.min(kern_ms)), "kernel_ms_median": float(np.median(kern_ms)),
                   "kernel_ms_events_around_each_launch": per_launch_ms},
        "roofline": {"bound": "mfma", "achieved": achieved, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": achieved / PEAK_BF16_TFLOPS, "traffic": measured_traffic(cfg["name"])},
    }
    if args.compare_lib and not args.splitkv:
        out["compare"] = compare_lib(args, cfg, entry, qd, kd, vd, o, lse, scale, stream)
    if not args.no_cpu_baseline:
        if q is None:  # device-generated inputs: the oracle reads the same bits back
            q, k, v = (t.cpu().view(torch.int16).numpy().view(np.uint16) for t in (qd, kd, vd))
        out["cpu_baseline"] = cpu_baseline(cfg, q, k, v, scale)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
