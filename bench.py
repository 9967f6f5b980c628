#!/usr/bin/env python3
"""Benchmark of the OVGGT streaming hot path on one MI355X.

A step is one frame through the whole path for every layer of the workload:
ovggt_global_attn (append + attention) -> ovggt_score_select -> ovggt_cache_compact,
called through the C ABI with all inputs already resident in HBM.  The default
workload is the VGGT-sized single global layer (1374 tokens/frame, 16x64 heads,
budget 16384, bf16).  Prints ONE JSON line with the throughput in frames/s, the
roofline of the dominant kernel (attention, MFMA-bound) measured with HIP
events inside the timed region, and the CPU oracle timed on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

from paper_2603_05959_amd import synth  # noqa: E402

MFMA_BF16_PEAK_TFLOPS = 2500.0       # MI355X dense bf16
HBM_PEAK_GBS = 8000.0


def gen_frames(cfg, frames, layers, pool):
    """Host generation of the (layer, frame) inputs of a few frames, threaded
    (numpy releases the GIL in the heavy parts)."""
    jobs = [(l, t) for t in frames for l in range(layers)]
    return dict(zip(jobs, pool.map(lambda lt: synth.frame_inputs(cfg, lt[0], lt[1]), jobs)))


def profiled_figure(what, kernel, workload, layers):
    """A per-launch figure of `kernel` from the committed rocprofv3 summary of this workload, or
    None: "traffic_bytes_per_launch" (FETCH_SIZE + WRITE_SIZE, calibrated there against a plain
    copy) or "trace_avg_kernel_us" (steady-state duration in the kernel trace)."""
    path = os.path.join(ROOT, "profiles", "bench_%s_kernels_and_traffic.md" % workload)
    tag = "%s %s %s layers=%d:" % (what, kernel, workload, layers)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith(tag):
                    return float(line[len(tag):].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(cfg, warm_frames, timed_frames, smooth=None, hybrid_beta=None, threads=None):
    """The oracle as it stands: attention-free warm-up to reach the steady-state
    cache, then whole steps (fp64 attention + score + select + compact) timed.
    threads: cap on the BLAS thread pool (None: whatever the box gives)."""
    from oracle import ovggt_oracle as oc            # cpu_baseline leg only
    limit = None
    try:
        import threadpoolctl
        if threads:
            limit = threadpoolctl.threadpool_limits(limits=int(threads))
        cores = max((p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()), default=1)
    except Exception:
        cores = os.cpu_count() or 1
    orc = oc.OracleCache(cfg.M, cfg.H, cfg.d, cfg.B, smooth=smooth, hybrid_beta=hybrid_beta)
    for t in range(warm_frames):
        f = synth.frame_inputs(cfg, 0, t, want=("k", "v", "r", "a"))
        orc.append(f["k"], f["v"])
        orc.update(f["r"], f["a"])
    fs = [synth.frame_inputs(cfg, 0, warm_frames + i) for i in range(timed_frames)]
    t0 = time.perf_counter()
    for f in fs:
        orc.step(f["q"], f["k"], f["v"], f["r"], f["a"])
    dt = time.perf_counter() - t0
    if limit is not None:
        limit.restore_original_limits()
    return {"value": timed_frames / dt, "unit": "frames/s", "cores": int(cores), "kind": "oracle",
            "sample": f"{timed_frames} steady-state frames (t={warm_frames}..{warm_frames + timed_frames - 1}, "
                      f"{orc.n + cfg.M} resident keys) of the same workload, layer 0, after an attention-free "
                      f"{warm_frames}-frame warm-up; numpy/OpenBLAS fp64",
            "seconds": dt}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=170)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--config", type=int, default=1, help="workload preset (1 = the headline layer)")
    ap.add_argument("--layers", type=int, default=None, help="override the preset's layer count")
    ap.add_argument("--budget", type=int, default=None)
    ap.add_argument("--hybrid-beta", type=float, default=None,
                    help="rank by hybrid scoring (Eq. 7) with this beta instead of the stored Eq. 5 scores")
    ap.add_argument("--smooth-alpha", type=float, default=None,
                    help="activation smoothing (Eq. 6) with this alpha and a 3x3 Gaussian (sigma 1) over the patch map")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-frames", type=int, default=12)
    ap.add_argument("--cpu-threads", type=int, default=None, help="cap the oracle's BLAS threads (default: all the box gives)")
    ap.add_argument("--detail-steps", type=int, default=40, help="extra untimed steps with per-kernel events")
    ap.add_argument("--flatness", action="store_true",
                    help="also bracket every 8th timed step with events and report the slope of step latency over the stream")
    ap.add_argument("--rising-scores", action="store_true",
                    help="worst case for compaction: residual norms grow with t, so every new token survives and "
                         "M cached entries move per frame (all frames of the run are generated: keep the run short)")
    ap.add_argument("--standalone-compact", action="store_true",
                    help="apply every frame's compaction with the stand-alone kernel (ovggt_cache_flush after each step) "
                         "instead of letting the next frame's append carry it")
    ap.add_argument("--mfma-loop", action="store_true",
                    help="also measure what a loop of nothing but the attention kernel's MFMA sustains on this box "
                         "(random and constant operands): the reachable denominator beside the published peak")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run a plain 256 MiB device copy (reference dispatch for rocprofv3 FETCH_SIZE/WRITE_SIZE)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one GPU only (no collectives, no sharding); run with --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2603_05959_amd import binding as B
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    B.lib()                                              # fail loudly if the HIP library is missing

    over = {}
    if args.layers:
        over["L"] = args.layers
    if args.budget:
        over["B"] = args.budget
    cfg = synth.preset(args.config, **over)
    W, K = args.warmup, args.steps
    T = W + K
    L = cfg.L
    dev = torch.device("cuda:0")

    # ---- inputs: generated on the host, staged to HBM before anything is timed
    distinct = min(T, max(64, 2 * (cfg.B // cfg.M) + 8)) if L > 1 else T
    if args.rising_scores:
        distinct = T + args.detail_steps                 # a reused frame would rank below the cache and break the pattern
    t_gen = time.perf_counter()
    staged = []
    with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 8)) as pool:
        for t0_ in range(0, distinct, 8):
            batch = range(t0_, min(distinct, t0_ + 8))
            host = gen_frames(cfg, batch, L, pool)
            if args.rising_scores:
                for (l, t), f in host.items():
                    f["r"] = synth.rising_resid(cfg, l, t)
            for t in batch:
                fs = [host[(l, t)] for l in range(L)]
                pack = lambda key: B.to_device(np.stack([f[key] for f in fs]), cfg.dtype, dev)
                staged.append((pack("q"), pack("k"), pack("v"), pack("r"),
                               torch.from_numpy(np.stack([f["a"] for f in fs])).to(dev)))
            del host
    torch.cuda.synchronize()
    gen_s = time.perf_counter() - t_gen

    if args.calibrate_copy:                              # known traffic: reads 256 MiB, writes 256 MiB
        src = torch.ones(64 * 1024 * 1024, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    smooth = None
    if args.smooth_alpha:
        ph, pw = synth.patch_grid(cfg)
        smooth = (args.smooth_alpha, ph, pw, cfg.M - ph * pw, synth.gaussian_kernel3(1.0))
    cache = B.Cache(L, cfg.H, cfg.d, cfg.M, cfg.C, cfg.B, cfg.dtype, smooth=smooth, hybrid_beta=args.hybrid_beta)
    out = cache.new_output()                             # fp32 outputs (fp32 accumulators stored unrounded)
    layer = B.OVGGT_ALL_LAYERS if L > 1 else 0

    def step(t):
        q, k, v, r, a = staged[t % distinct]
        # frames reused past `distinct` keep their anchor bits only in frame 0's first use
        cache.step(q, k, v, r, a if t < distinct else None, out, layer)
        if args.standalone_compact:
            cache.flush(layer)

    for t in range(W):
        step(t)
    torch.cuda.synchronize()
    B.ovggt_profile_enable(cache.h, 1, 4)                # attention kernel of every 4th step
    flat_ev = []
    t0 = time.perf_counter()
    for t in range(W, T):
        if args.flatness and (t - W) % 8 == 0:
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            step(t)
            e1.record()
            flat_ev.append((t, e0, e1))
        else:
            step(t)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    prof = B.ovggt_profile_read(cache.h, cache.stream)
    # what an event bracket reports beyond the bracketed kernel's own execution (empty launch)
    bracket_overhead_ms = B.ovggt_profile_overhead(cache.h, 64, cache.stream)
    status = [cache.status(l) for l in range(L)]
    assert not any(status), f"device status {status}"
    n_res = cache.size(0)
    assert n_res == min(T * cfg.M, cfg.B)

    # ---- per-kernel detail on further (untimed) steady-state steps
    B.ovggt_profile_enable(cache.h, 2, 1)
    ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.detail_steps)]
    for i in range(args.detail_steps):
        ev[i][0].record()
        step(T + i)
        ev[i][1].record()
    torch.cuda.synchronize()
    detail = B.ovggt_profile_read(cache.h, cache.stream)
    B.ovggt_profile_enable(cache.h, 0, 1)
    lat = sorted(a.elapsed_time(b) for a, b in ev) if ev else [0.0]

    # ---- roofline of the dominant kernel (attention): algorithmic FLOP = 4*M*N*H*d per layer
    n_keys = min(cfg.B, T * cfg.M) + cfg.M if T * cfg.M > cfg.B else T * cfg.M
    attn_ms, attn_cnt = prof["attn"]
    flop = 4.0 * cfg.M * n_keys * cfg.H * cfg.d * L
    bracket_ms = attn_ms / max(attn_cnt, 1)
    attn_avg_ms = max(bracket_ms - bracket_overhead_ms, 1e-6)
    achieved = flop / (attn_avg_ms * 1e-3) / 1e12 if attn_cnt else 0.0
    # from the committed rocprofv3 summary of this workload (stored-score ranking, no smoothing): HBM
    # bytes per launch, and the kernel's steady-state duration in the trace (the profiled run is a
    # few per cent slower than a plain one)
    wl = cfg.name.split("-")[0]
    traffic = profiled_figure("traffic_bytes_per_launch", "attn_bf16_kernel", wl, L)
    traffic = None if traffic is None else int(traffic)
    trace_us = profiled_figure("trace_avg_kernel_us", "attn_bf16_kernel", wl, L)
    roofline = {"bound": "mfma", "kernel": "attn_bf16_kernel", "achieved": achieved, "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / MFMA_BF16_PEAK_TFLOPS,
                "traffic": traffic, "avg_kernel_ms": attn_avg_ms,
                "profiled_kernel_ms": None if trace_us is None else trace_us * 1e-3, "event_bracket_ms": bracket_ms,
                "event_bracket_of_empty_launch_ms": bracket_overhead_ms, "launches_timed": int(attn_cnt),
                "flop_per_launch": flop, "keys_per_launch": int(n_keys)}

    kernels = {}
    for name, (ms, cnt) in detail.items():
        if cnt:
            kernels[name] = {"avg_us": 1e3 * ms / cnt, "launches": int(cnt)}
    esz = 2 if cfg.dtype == "bf16" else 4
    hbm = {}
    if "score_select" in kernels:
        byts = L * (cfg.M * cfg.C * esz + 4 * cfg.M + 9 * n_keys)
        hbm["score_select"] = {"algorithmic_bytes": byts, "GB/s": byts / (kernels["score_select"]["avg_us"] * 1e-6) / 1e9}
    move_bytes = 0
    if args.rising_scores:
        moves = len(cache.last_moves(0)[0])
        assert moves == cfg.M, f"rising scores: {moves} of {cfg.M} entries moved in the last frame"
        move_bytes = L * moves * (2 * cfg.H * cfg.d * esz + 9) * 2           # K, V, id, score, flag: read and written
        if "compact" in kernels:
            hbm["compact"] = {"algorithmic_bytes": move_bytes, "GB/s": move_bytes / (kernels["compact"]["avg_us"] * 1e-6) / 1e9,
                              "entries_moved_per_layer": moves}
    if "append" in kernels:
        byts = L * 4 * cfg.M * cfg.H * cfg.d * esz
        if move_bytes and not args.standalone_compact:                       # the append carries the moves as well
            byts += move_bytes
        hbm["append"] = {"algorithmic_bytes": byts, "GB/s": byts / (kernels["append"]["avg_us"] * 1e-6) / 1e9}
    for v in hbm.values():
        v["frac_of_8TBs"] = v["GB/s"] / HBM_PEAK_GBS

    res = {
        "metric": "streamed frames/sec at fixed cache budget",
        "value": K / elapsed,
        "unit": "frames/s",
        "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": 1e3 * elapsed / K,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: {L} layer(s) x (M={cfg.M} tokens/frame, {cfg.H}x{cfg.d} heads, "
                               f"C={cfg.C}, budget B={cfg.B}), {T}-frame stream, {cfg.dtype}",
                   "tokens_per_frame": cfg.M, "budget": cfg.B, "layers": L, "frames": T,
                   "resident_keys_steady": int(n_keys), "out_dtype": "f32",
                   "ranking": ("hybrid Eq. 7, beta=%g" % args.hybrid_beta) if args.hybrid_beta is not None
                              else "stored Eq. 5 scores",
                   "smoothing": ("Eq. 6, alpha=%g, 3x3 Gaussian sigma 1" % args.smooth_alpha) if smooth else "off",
                   "scores": "rising with t (worst case for compaction)" if args.rising_scores else "workload's own",
                   "compaction": "stand-alone kernel after every frame" if args.standalone_compact
                                 else "carried by the next frame's append"},
        "roofline": roofline,
        "kernels_us": kernels,
        "hbm_kernels": hbm,
        "step_latency_ms": {"p50": lat[len(lat) // 2], "p99": lat[min(len(lat) - 1, int(0.99 * len(lat)))],
                            "note": "per-step events on untimed steady-state steps with per-kernel events enabled"},
        "cache_bytes": {"kv": cache.bytes[0], "meta": cache.bytes[1], "workspace": cache.bytes[2]},
        "input_staging_s": gen_s,
    }
    if flat_ev:
        # steady state only: the resident key count is constant once the cache is full
        full_from = cfg.B // cfg.M + 1
        pts = [(t, a.elapsed_time(b)) for t, a, b in flat_ev if t >= full_from]
        if len(pts) >= 8:
            tt = np.array([p[0] for p in pts], dtype=np.float64)
            ms = np.array([p[1] for p in pts], dtype=np.float64)
            slope, icpt = np.polyfit(tt, ms, 1)
            q = len(pts) // 4
            res["flatness"] = {"samples": len(pts), "first_frame": int(tt[0]), "last_frame": int(tt[-1]),
                               "mean_ms": float(ms.mean()), "mean_ms_first_quarter": float(ms[:q].mean()),
                               "mean_ms_last_quarter": float(ms[-q:].mean()),
                               "slope_us_per_1000_frames": float(slope * 1e6),
                               "note": "event-bracketed whole steps, every 8th timed step, frames with a full cache"}
    if args.mfma_loop:
        rnd = B.ovggt_profile_mfma_loop(cache.h, True, 20000, cache.stream)
        cst = B.ovggt_profile_mfma_loop(cache.h, False, 20000, cache.stream)
        res["mfma_loop"] = {"random_operands_TFLOPs": rnd, "constant_operands_TFLOPs": cst, "unit": "TFLOP/s",
                            "instruction": "v_mfma_f32_32x32x16_f16", "waves_per_simd": 2,
                            "attention_frac_of_random_operand_rate": res["roofline"]["achieved"] / rnd}
    cache.close()
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(cfg, warm_frames=max(cfg.B // cfg.M + 2, 2), timed_frames=args.cpu_frames,
                                           smooth=smooth, hybrid_beta=args.hybrid_beta, threads=args.cpu_threads)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
