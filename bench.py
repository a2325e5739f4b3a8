#!/usr/bin/env python3
"""Benchmark of the cache-hit denoising step on one MI355X.

A "step" is one pass of the whole hot path (conv_in, residual blocks, spatial and temporal
attention blocks, fetch of the cached deep feature, skip-concat, up conv, conv_out) over one batch
of seeded synthetic input shaped like the AnimateDiff workload (batch 2 x 16 frames of 4 x 64 x 64
latents, 320 channels, 8 heads of 40, frame chunk 4), with every input already resident in HBM.
Prints ONE JSON line. Beside the headline it carries, measured in the same run:
  * `roofline`   the kernel family with the largest total time, and `rooflines` for each big MFMA kernel
  * `svdxt`      the SVD-XT-like workload (batch 2 x 25 frames of 72 x 128, frame chunk 5, token chunk 2304)
  * `tiny`       the small fp32 stage: step latencies, and the 25-step schedule (normal step every 3rd,
                 swap-out after each, prefetch one step ahead) with frame chunk 16, 8, 4, 2
  * `stress`     the 50-step schedule (interval 5, bank of 10 host entries) on batch 2 x 32 frames of 96 x 96,
                 with the chunk the footprint model picks under 64 GB and predicted vs measured peak
  * `swap`       host-to-device and device-to-host copies against the steps they hide behind
  * `hbm_modes`  footprint with a resident cache, one device buffer, two device buffers
  * `cpu_baseline` the CPU oracle on the same input
"""
from __future__ import annotations

import argparse
import json
import os
import statistics
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_TFLOPS = {"bf16": 2500.0, "f32": 157.3}  # dense MFMA peaks of MI355X, TFLOP/s
PEAK_HBM_GBS = 8000.0
# HBM-side bytes of one launch of a kernel family (animatediff, frame chunk 4) from the rocprofv3 FETCH_SIZE /
# WRITE_SIZE runs summarised under profiles/ (fetch x 2.0, the factor a plain copy of known size gave). Valid only
# for the kernel sources the counters were taken with: `sha256_16` covers the listed files, else traffic is null.
TRAFFIC = {
    "conv_up": {"sources": ("lc_convws.hip", "lc_common.h", "lc_internal.h"), "sha256_16": "9f27ba249d998d07",
                "bytes_per_launch": 83.6e6 + 22.3e6},
    "sattn": {"sources": ("lc_attn.hip", "lc_common.h", "lc_internal.h"), "sha256_16": "7aacbd5d82e993a6",
              "bytes_per_launch": 61.0e6 + 12.6e6},
    "conv_res": {"sources": ("lc_convws.hip", "lc_common.h", "lc_internal.h"), "sha256_16": "9f27ba249d998d07",
                 "bytes_per_launch": 54.5e6 + 22.3e6},
}
TRAFFIC_WORKLOAD = ("animatediff", 4)


def measured_traffic(family, cfg_name, fc):
    import hashlib
    t = TRAFFIC.get(family)
    if t is None or (cfg_name, fc) != TRAFFIC_WORKLOAD:
        return None
    m = hashlib.sha256()
    try:
        for f in t["sources"]:
            m.update(open(os.path.join(ROOT, "paper_2510_05367_amd", "csrc", f), "rb").read())
    except OSError:
        return None
    return t["bytes_per_launch"] if m.hexdigest()[:16] == t["sha256_16"] else None  # null once the kernel has changed


def family_flops(cfg):
    """Algorithmic FLOPs per cached step of each MFMA kernel family (unpadded head size, 9 taps)."""
    P, C, Cd = cfg.N * cfg.T, cfg.C, cfg.C_deep
    return {
        "conv_res": cfg.n_res * 2.0 * 9 * C * C * P,
        "conv_up": 2.0 * 9 * (C + Cd) * C * P,
        "qkv": 2 * 6.0 * C * C * P,
        "proj": 2 * 2.0 * C * C * P,
        "sattn": 4.0 * cfg.T * cfg.T * cfg.head_dim * cfg.heads * cfg.N,
        "tattn": 4.0 * cfg.F * cfg.F * cfg.head_dim * cfg.heads * cfg.B * cfg.T,
        "tblock": 8.0 * C * C * P + 4.0 * cfg.F * cfg.F * cfg.head_dim * cfg.heads * cfg.B * cfg.T,
        "conv_in": 2.0 * 9 * cfg.C_lat * C * P,
        "conv_out": 2.0 * 9 * cfg.C_lat * C * P,
    }


def family_bytes(cfg):
    """Algorithmic HBM bytes per cached step of each bandwidth kernel family (one read + one write
    of what the operator must touch; fp32 residual stream = 4 bytes, operands = element size)."""
    P, C, Cd = cfg.N * cfg.T, cfg.C, cfg.C_deep
    es = 2 if cfg.dtype == "bf16" else 4
    return {
        "gn_stats": (P // 4) * Cd * es,  # only the deep feature has a statistics pass of its own (once per slot content)
        "conv_in": P * cfg.C_lat * es + P * C * 4,
        "conv_out": P * C * 4 + P * cfg.C_lat * es,
        "tattn": 4 * P * C * es,
        "tblock": 2 * P * C * 4,  # the fused temporal block reads the fp32 stream once and writes it once
        # the projections are near the machine balance (193 FLOP per byte): both rooflines are reported.
        # q,k,v: fp32 stream in, three operand tensors out; output projection: operand in, fp32 residual in and out
        "qkv": 2 * (P * C * 4 + 3 * P * C * es),
        "proj": 2 * (P * C * es + 2 * P * C * 4),
    }


MFMA_FAMILIES = ("conv_res", "conv_up", "qkv", "proj", "sattn", "tblock")


def cpu_baseline(cfg, w):
    """The float64 oracle, as it stands, on the same input: one cached step of the whole workload."""
    import numpy as np
    from oracle import lightcache_oracle as lo
    from paper_2510_05367_amd import synth
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    x = synth.make_latents(cfg, 1)
    deep = synth.make_deep(cfg, 2)
    orc = lo.Oracle(cfg, {k: v.astype(np.float64) for k, v in w.items()})
    orc.set_chunk(cfg.frame_chunk, cfg.token_chunk)
    orc.cache_write(0, deep)
    t0 = time.time()
    orc.cached_step(x, 0)
    dt = time.time() - t0
    return {"value": cfg.cached_step_flops() / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle", "seconds": round(dt, 2),
            "sample": f"one cached step of the float64 numpy oracle on the whole workload input (B={cfg.B}, F={cfg.F}, "
                      f"{cfg.H}x{cfg.W}x{cfg.C}; {cfg.cached_step_flops() / 1e9:.1f} GFLOP)"}


class Timer:
    """Per-step HIP events on the compute stream (the stream the steps are launched on; a chunked step forks to
    the library's second stream and joins back into it) plus the wall clock around the whole region."""

    def __init__(self, torch, stage):
        self.torch, self.stage = torch, stage

    def run(self, n, fn):
        ev = [self.torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
        self.torch.cuda.synchronize()
        t0 = time.perf_counter()
        ev[0].record(self.stage.compute)
        for i in range(n):
            fn(i)
            ev[i + 1].record(self.stage.compute)
        self.torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) * 1e3
        per = [ev[i].elapsed_time(ev[i + 1]) for i in range(n)]
        return {"wall_ms_per_step": wall / n, "median_ms": statistics.median(per), "min_ms": min(per), "per_step": per}


def make_stage(lcb, synth, cfg, w, fc, tc, host_slots, dev_slots, lanes):
    stage = lcb.Stage(cfg, w, host_slots=host_slots, dev_slots=dev_slots, frame_chunk=fc, token_chunk=tc)
    stage.set_lanes(lanes)
    return stage


def profile_families(lcb, stage, step, n):
    """One-lane pass with every kernel family bracketed by events: ms and launches per step."""
    lcb.lc_set_profiling(stage.ctx, (1 << len(lcb.KERNEL_FAMILIES)) - 1)
    lcb.lc_get_profile(stage.ctx)
    for i in range(n):
        step(i)
    pf = lcb.lc_get_profile(stage.ctx)
    lcb.lc_set_profiling(stage.ctx, 0)
    dropped = pf.pop("dropped", 0)
    out = {k: {"ms_per_step": v["ms"] / n, "launches_per_step": v["launches"] // n} for k, v in pf.items()
           if v["launches"]}
    return out, dropped


def breakdown_record(cfg, fams, peak):
    fam_fl, fam_by = family_flops(cfg), family_bytes(cfg)
    out = {}
    for name, v in fams.items():
        e = {"ms_per_step": round(v["ms_per_step"], 4), "launches_per_step": v["launches_per_step"]}
        if name in MFMA_FAMILIES and name in fam_fl:
            e["tflops"] = round(fam_fl[name] / (v["ms_per_step"] * 1e-3) / 1e12, 1)
            e["frac_mfma_peak"] = round(e["tflops"] / peak, 4)
        if name in fam_by:
            e["gbs"] = round(fam_by[name] / (v["ms_per_step"] * 1e-3) / 1e9, 1)
            e["frac_hbm_peak"] = round(e["gbs"] / PEAK_HBM_GBS, 4)
        out[name] = e
    return out


def roofline_of(lcb, torch, stage, cfg, fc, family, step, K, peak):
    """K steps with one kernel family bracketed by events on the stream it is launched on. With a bracket set the
    library keeps a step on one lane, so the kernel is timed with the device to itself."""
    lcb.lc_set_profiling(stage.ctx, 1 << lcb.LC_K[family])
    lcb.lc_get_profile(stage.ctx)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    ms_one = (time.perf_counter() - t0) * 1e3 / K
    d = lcb.lc_get_profile(stage.ctx)[family]
    lcb.lc_set_profiling(stage.ctx, 0)
    launches = max(d["launches"], 1)
    avg_ms = d["ms"] / launches
    if family in MFMA_FAMILIES:
        work = family_flops(cfg)[family] * K / launches
        achieved = work / (avg_ms * 1e-3) / 1e12
        r = {"kernel": family, "bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TFLOP/s",
             "frac": round(achieved / peak, 4), "flops_per_launch": work}
    else:
        work = family_bytes(cfg)[family] * K / launches
        achieved = work / (avg_ms * 1e-3) / 1e9
        r = {"kernel": family, "bound": "hbm", "achieved": round(achieved, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
             "frac": round(achieved / PEAK_HBM_GBS, 4), "bytes_per_launch": work}
    if family == "sattn":
        # context for the MFMA fraction: the kernel also issues one v_exp_f32 per score, on the quarter-rate
        # transcendental unit (256 CUs x 4 SIMDs x 4 lanes per clock at 2.4 GHz = 9.83e12 per second), and pads the
        # head size to MFMA tiles (contraction of K Q^T to a multiple of 16, rows of V^T to a multiple of 32)
        frames = work / (4.0 * cfg.T * cfg.T * cfg.head_dim * cfg.heads)
        exps = frames * cfg.heads * cfg.T * cfg.T
        pad_qk = (cfg.head_dim + 15) // 16 * 16
        pad_pv = (cfg.head_dim + 31) // 32 * 32
        padded = frames * cfg.heads * 2.0 * cfg.T * cfg.T * (pad_qk + pad_pv)
        r["context"] = {"exp_per_launch": exps, "exp_floor_ms": round(exps / 9.83e12 * 1e3, 5),
                        "executed_flops_per_launch": padded, "mfma_floor_ms": round(padded / (peak * 1e12) * 1e3, 5),
                        "note": "the counter summary under profiles/ shows the matrix pipe and the transcendental unit "
                                "taking turns (42 % and 48 % busy): the sum of the two floors is what the kernel's "
                                "launch time compares with"}
    r.update({"traffic": measured_traffic(family, cfg.name, fc), "traffic_unit": "bytes/launch",
              "avg_launch_ms": round(avg_ms, 5), "launches_per_step": d["launches"] // K,
              "total_ms_per_step": round(d["ms"] / K, 4)})
    return r, ms_one


def device_bytes_in_use(torch, stats):
    """Measured device footprint: the high-water mark of what torch allocated since the last reset (the arena the
    library works in, x, eps, and the temporaries of loading weights and inputs) plus the library's own allocation
    (its packed weights)."""
    return torch.cuda.max_memory_allocated() + stats.weight_bytes


def footprint(lcb, cfg, fc, tc, dev_slots, host_slots, weight_bytes):
    """Predicted device bytes: arena (footprint model) + packed weights + x + eps."""
    es = 2 if cfg.dtype == "bf16" else 4
    io = 2 * cfg.N * cfg.C_lat * cfg.T * es
    return lcb.lc_workspace_bytes(lcb.make_config(cfg, host_slots, dev_slots), fc, tc) + weight_bytes + io


def run_schedule(stage, x, eps, steps, interval, host_slots, mode):
    """The denoising loop with a normal step every `interval` steps. mode: "resident" (the deep feature stays in
    one device slot, nothing is copied), "single" (swap-out after each normal step, swap-in into the same device
    slot right before each cache step), "double" (swap-in one step ahead into the other device slot)."""
    refresh = -1
    prefetched = None
    for t in range(steps):
        slot = t % 2 if mode == "double" else 0
        if t % interval == 0:
            refresh += 1
            stage.full_step(x, eps, slot)
            if mode != "resident":
                stage.swap_out(slot, refresh % host_slots)
        else:
            if mode == "single" or (mode == "double" and prefetched != (t, slot)):
                stage.swap_in(refresh % host_slots, slot)
            stage.cached_step(x, eps, slot)
        nxt = t + 1
        if mode == "double" and nxt < steps and nxt % interval != 0:
            stage.swap_in(refresh % host_slots, nxt % 2)
            prefetched = (nxt, nxt % 2)


def time_schedule(torch, stage, x, eps, steps, interval, host_slots, mode, reps):
    run_schedule(stage, x, eps, steps, interval, host_slots, mode)  # untimed
    torch.cuda.synchronize()
    best = None
    for _ in range(reps):
        t0 = time.perf_counter()
        run_schedule(stage, x, eps, steps, interval, host_slots, mode)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) * 1e3
        best = dt if best is None else min(best, dt)
    return best


def copy_times(lcb, stage, n=5):
    """Plain copies of one cache entry on the idle device: (ms out, ms in)."""
    stage.sync()
    lcb.lc_reset_stats(stage.ctx)
    for _ in range(n):
        stage.swap_out(0, 0)
    for _ in range(n):
        stage.swap_in(0, 1)
    st = lcb.lc_get_stats(stage.ctx)
    stage.swap_in(0, 0)
    stage.sync()
    return st.ms_out / max(st.timed_out, 1), st.ms_in / max(st.timed_in, 1)


def schedule_record(lcb, torch, synth, cfg, w, fc, tc, steps, interval, host_slots, reps, lanes):
    """Schedule of `steps` steps in the three cache modes; overlap = 1 - (t_double - t_resident) / t_copies."""
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    stage = make_stage(lcb, synth, cfg, w, fc, tc, host_slots, 2, lanes)
    try:
        x = stage.to_device(synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)
        stage.full_step(x, eps, 0)
        ms_out, ms_in = copy_times(lcb, stage)
        t_res = time_schedule(torch, stage, x, eps, steps, interval, host_slots, "resident", reps)
        t_single = time_schedule(torch, stage, x, eps, steps, interval, host_slots, "single", reps)
        t_double = time_schedule(torch, stage, x, eps, steps, interval, host_slots, "double", reps)
        n_full = (steps + interval - 1) // interval
        n_cached = steps - n_full
        copies = n_full * ms_out + n_cached * ms_in
        entry = lcb.lc_cache_entry_bytes(stage.ccfg)
        tm = Timer(torch, stage)
        cached = tm.run(max(10, min(50, steps)), lambda i: stage.cached_step(x, eps, 0))
        st = lcb.lc_get_stats(stage.ctx)
        measured = device_bytes_in_use(torch, st)

        def ov(t):
            return round(min(1.0, max(0.0, 1.0 - max(0.0, t - t_res) / copies)), 4) if copies > 0 else None
        return {"frame_chunk": fc, "token_chunk": tc, "effective_frame_chunk": min(fc, cfg.N) if fc else cfg.N,
                "steps": steps, "normal_steps": n_full, "cache_steps": n_cached,
                "cached_step_ms": round(cached["median_ms"], 4),
                "schedule_ms": {"resident": round(t_res, 3), "single_buffer": round(t_single, 3),
                                "double_buffer": round(t_double, 3)},
                "copy_ms": {"d2h": round(ms_out, 4), "h2d": round(ms_in, 4), "all_copies_of_schedule": round(copies, 3)},
                "link_gbs": {"d2h": round(entry / (ms_out * 1e-3) / 1e9, 1) if ms_out > 0 else None,
                             "h2d": round(entry / (ms_in * 1e-3) / 1e9, 1) if ms_in > 0 else None},
                "overlap_frac": {"single_buffer": ov(t_single), "double_buffer": ov(t_double)},
                "workspace_gb": round(st.workspace_bytes / 1e9, 5),
                "peak_hbm_gb_predicted": round(footprint(lcb, cfg, fc, tc, 2, host_slots, st.weight_bytes) / 1e9, 5),
                "peak_hbm_gb_measured": round(measured / 1e9, 5),
                "host_bank_gb": round(st.host_bank_bytes / 1e9, 4)}
    finally:
        stage.close()
        torch.cuda.empty_cache()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="animatediff", choices=["tiny", "animatediff", "svdxt", "stress"])
    ap.add_argument("--frame-chunk", type=int, default=None)
    ap.add_argument("--token-chunk", type=int, default=None)
    ap.add_argument("--lanes", type=int, default=2, choices=[1, 2],
                    help="streams a chunked step spreads its chunks over (lc_set_lanes); 1 = compute stream only")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-breakdown", action="store_true")
    ap.add_argument("--no-extra", action="store_true", help="headline workload only (no svdxt / tiny / stress records)")
    ap.add_argument("--steps-only", action="store_true",
                    help="warm-up and the timed steps only, then a short JSON line (the command rocprofv3 is pointed at)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="first run a plain device copy of 256 MiB three times (reference for hardware byte counters)")
    ap.add_argument("--only", default=None, choices=["sliced_decode", "video_dit", "unet"],
                    help="run one of the further records alone and print it (the command rocprofv3 is pointed at for them)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py measures one GPU: the library has no multi-GPU path (run with --gpus 1)")

    import torch
    from paper_2510_05367_amd import binding as lcb
    from paper_2510_05367_amd import synth

    if not torch.cuda.is_available():
        sys.exit("no GPU visible: the HIP path cannot run and there is no CPU fallback")
    if not os.path.exists(lcb.LIB_PATH):
        from paper_2510_05367_amd import build as lcbuild
        lcbuild.build_library()
    if args.only:
        fn = {"sliced_decode": decode_record, "video_dit": dit_record, "unet": unet_record}[args.only]
        kw = {"steps_only": True} if (args.only == "unet" and args.steps_only) else {}
        print(json.dumps({args.only: fn(lcb, torch, synth, **kw)}))
        return

    cfg = synth.CONFIGS[args.workload]
    fc = cfg.frame_chunk if args.frame_chunk is None else args.frame_chunk
    tc = cfg.token_chunk if args.token_chunk is None else args.token_chunk
    w = synth.make_weights(cfg, 0)
    torch.cuda.reset_peak_memory_stats()
    stage = make_stage(lcb, synth, cfg, w, fc, tc, 2, 2, args.lanes)
    x = stage.to_device(synth.make_latents(cfg, 1))
    eps = stage.empty(*x.shape)
    stage.cache_write(0, stage.to_device(synth.make_deep(cfg, 2)))
    stage.sync()
    K, W = args.steps, args.warmup
    peak = PEAK_TFLOPS[cfg.dtype]
    tm = Timer(torch, stage)

    if args.copy_calibration:
        src = torch.zeros(64 * 1024 * 1024, dtype=torch.float32, device=stage.device)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    def step(i):
        stage.cached_step(x, eps, 0)

    for i in range(W):
        step(i)
    stage.sync()

    # ---- timed region: K cached steps as the library runs them (chunks spread over `lanes` streams)
    timed = tm.run(K, step)
    ms = timed["wall_ms_per_step"]
    flops = cfg.cached_step_flops()
    tflops = flops / (ms * 1e-3) / 1e12
    if args.steps_only:
        print(json.dumps({"workload": cfg.name, "frame_chunk": fc, "token_chunk": tc, "lanes": args.lanes, "steps": K,
                          "warmup": W, "ms_per_step": round(ms, 4), "cached_step_ms_median": round(timed["median_ms"], 4),
                          "tflops": round(tflops, 2)}))
        stage.close()
        return

    # ---- per-family pass (one lane, every family bracketed), then the family with the largest total time again
    #      on its own for `roofline`, and each big MFMA kernel for `rooflines`
    fams, dropped = profile_families(lcb, stage, step, min(K, 5))
    dom = max(fams, key=lambda k: fams[k]["ms_per_step"])
    roofline, ms_one = roofline_of(lcb, torch, stage, cfg, fc, dom, step, K, peak)
    roofline["time_dominant"] = True
    rooflines = [roofline]
    for fam in ("sattn", "conv_up", "conv_res"):
        if fam != dom and fam in fams:
            r, _ = roofline_of(lcb, torch, stage, cfg, fc, fam, step, min(K, 10), peak)
            r["time_dominant"] = False
            rooflines.append(r)
    breakdown = None if args.no_breakdown else breakdown_record(cfg, fams, peak)

    # ---- asynchronous swapping on the headline workload
    entry = lcb.lc_cache_entry_bytes(stage.ccfg)
    stage.swap_out(0, 0)
    ms_out, ms_in = copy_times(lcb, stage)

    def prefetched_steps(n):
        for i in range(n):
            stage.cached_step(x, eps, i % 2)
            stage.swap_in(0, (i + 1) % 2)  # prefetch for the next step into the other buffer
    # untimed, like the warm-up of the plain steps, but longer: the first time the host runs many steps with
    # copies ahead of the device, a few lc_swap_in calls block for milliseconds inside the runtime
    # (seen up to about 80 steps into the first such loop of a process; the faster of two timed blocks is reported)
    prefetched_steps(max(W, 80))
    ms_swap = None
    for _ in range(2):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        prefetched_steps(K)
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) * 1e3 / K
        ms_swap = t if ms_swap is None else min(ms_swap, t)
    overlap_in = 1.0 - max(0.0, ms_swap - ms) / ms_in if ms_in > 0 else None

    # device-to-host: a normal step followed by the swap-out of what it produced, then a cache step on the other
    # slot (the copy runs behind that step), against the same pair without the copy
    e2 = stage.empty(*x.shape)

    def pair(n, with_copy):
        for i in range(n):
            stage.full_step(x, e2, 0)
            if with_copy:
                stage.swap_out(0, 1)
            stage.cached_step(x, eps, 1)
    pair(3, True)
    torch.cuda.synchronize()
    n_pair = max(5, K // 4)
    t0 = time.perf_counter(); pair(n_pair, False); torch.cuda.synchronize()
    pair_plain = (time.perf_counter() - t0) * 1e3 / n_pair
    t0 = time.perf_counter(); pair(n_pair, True); torch.cuda.synchronize()
    pair_copy = (time.perf_counter() - t0) * 1e3 / n_pair
    overlap_out = 1.0 - max(0.0, pair_copy - pair_plain) / ms_out if ms_out > 0 else None
    clip = lambda v: None if v is None else round(min(1.0, max(0.0, v)), 4)
    swap = {"entry_mb": round(entry / 1e6, 1), "h2d_ms": round(ms_in, 4), "d2h_ms": round(ms_out, 4),
            "h2d_gbs": round(entry / (ms_in * 1e-3) / 1e9, 1) if ms_in > 0 else None,
            "d2h_gbs": round(entry / (ms_out * 1e-3) / 1e9, 1) if ms_out > 0 else None,
            "step_ms_with_prefetch": round(ms_swap, 4), "overlap_frac": clip(overlap_in),
            "normal_plus_cache_step_ms": round(pair_plain, 4), "same_with_swap_out_ms": round(pair_copy, 4),
            "overlap_frac_d2h": clip(overlap_out)}

    stats = lcb.lc_get_stats(stage.ctx)
    measured_peak = device_bytes_in_use(torch, stats)
    es = 2 if cfg.dtype == "bf16" else 4
    io = 2 * cfg.N * cfg.C_lat * cfg.T * es
    floor = cfg.N * cfg.T * cfg.C * 4 + 2 * entry + stats.weight_bytes + io
    # the three cache modes side by side: what a double buffer costs against keeping the feature resident, and
    # what a bank of many entries would cost if it stayed on the device
    hbm_modes = {
        "resident_one_slot_gb": round(footprint(lcb, cfg, fc, tc, 1, 0, stats.weight_bytes) / 1e9, 4),
        "swap_single_buffer_gb": round(footprint(lcb, cfg, fc, tc, 1, 2, stats.weight_bytes) / 1e9, 4),
        "swap_double_buffer_gb": round(footprint(lcb, cfg, fc, tc, 2, 2, stats.weight_bytes) / 1e9, 4),
        "second_lane_scratch_gb": round((lcb.lc_workspace_bytes(stage.ccfg, fc, tc) -
                                         _one_lane_bytes(lcb, stage.ccfg, fc, tc)) / 1e9, 4),
        "unchunked_double_buffer_gb": round(footprint(lcb, cfg, 0, 0, 2, 2, stats.weight_bytes) / 1e9, 4),
        "note": "a double buffer holds two device copies of the deep feature: for one cached feature it uses MORE HBM "
                "than keeping it resident; swapping saves memory only against a bank of several entries kept on the "
                "device (stress record: 10 entries)"}
    out = {
        "metric": "shallow-branch TFLOP/s of one cached step (cached-step ms, MFMA util, peak HBM GB alongside)",
        "value": round(tflops, 2), "unit": "TFLOP/s", "n_gpus": 1, "steps": K, "warmup": W,
        "ms_per_step": round(ms, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": cfg.dtype, "data": "synthetic",
        "config": {"workload": f"{cfg.name}: cached step, B={cfg.B} F={cfg.F} latent {cfg.C_lat}x{cfg.H}x{cfg.W}, "
                               f"C={cfg.C}, C_deep={cfg.C_deep}, {cfg.heads} heads x {cfg.head_dim}, n_res={cfg.n_res}",
                   "frame_chunk": fc, "token_chunk": tc, "lanes": args.lanes, "gflop_per_step": round(flops / 1e9, 1)},
        "cached_step_ms": round(ms, 4), "cached_step_ms_median": round(timed["median_ms"], 4),
        "cached_step_ms_min": round(timed["min_ms"], 4),
        "ms_per_step_one_lane": round(ms_one, 4), "mfma_util_frac": round(tflops / peak, 4),
        "peak_hbm_gb": round(measured_peak / 1e9, 4), "peak_hbm_gb_predicted": round(
            footprint(lcb, cfg, fc, tc, 2, 2, stats.weight_bytes) / 1e9, 4),
        "hbm_floor_gb": round(floor / 1e9, 4), "workspace_gb": round(stats.workspace_bytes / 1e9, 4),
        "hbm_modes": hbm_modes,
        "roofline": roofline, "rooflines": rooflines, "swap": swap,
        "paper_context": "end-to-end on 4x L40S, pretrained models (not comparable, context only): 1.59x on "
                         "AnimateDiff-Lightning, 2.86x on SVD-XT; peak memory 13562 -> 5559 MB and 15346 -> 13937 MB",
    }
    if breakdown is not None:
        out["breakdown"] = breakdown
        out["breakdown_dropped_brackets"] = dropped
    stage.close()
    del stage, x, eps, e2
    torch.cuda.empty_cache()

    if not args.no_extra and args.workload == "animatediff":
        # the 25-step schedule (normal step when t % 3 == 0, the entry swapped out after it and prefetched one step
        # ahead) on the headline shapes, frame chunks 16, 8, 4, 2: latency, peak HBM and swap overlap per chunk
        out["schedule_25_steps_interval_3"] = [
            schedule_record(lcb, torch, synth, cfg, w, c, 0, 25, 3, 2, 3, args.lanes) for c in (16, 8, 4, 2)]
        out["svdxt"] = workload_record(lcb, torch, synth, "svdxt", w, args.lanes)
        out["tiny"] = tiny_record(lcb, torch, synth, args.lanes)
        out["stress"] = stress_record(lcb, torch, synth, w, args.lanes, stats.weight_bytes)
        out["sliced_decode"] = decode_record(lcb, torch, synth)
        out["video_dit"] = dit_record(lcb, torch, synth)
        out["unet"] = unet_record(lcb, torch, synth)
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(cfg, w)
    print(json.dumps(out))


def _one_lane_bytes(lcb, ccfg, fc, tc):
    """Arena bytes if the chunk scratch existed once: the plan counts it twice whenever a chunk is set, and the
    unchunked plan (one scratch of the whole axis) bounds what one lane's scratch of a chunk can be."""
    full = lcb.lc_workspace_bytes(ccfg, fc, tc)
    # scratch of one lane = difference between the plans of chunk c and of chunk 2c, when both are chunked
    N = ccfg.B * ccfg.F
    if fc and 2 * fc < N and tc == 0:
        per_lane = (lcb.lc_workspace_bytes(ccfg, 2 * fc, 0) - full) // 2
        return full - per_lane
    return full


def workload_record(lcb, torch, synth, name, w, lanes, steps=12, warmup=3):
    """Cached step of another workload in the same run: ms (median of per-step events), TFLOP/s, per-kernel, peak."""
    cfg = synth.CONFIGS[name]
    fc, tc = cfg.frame_chunk, cfg.token_chunk
    torch.cuda.empty_cache()
    torch.cuda.reset_peak_memory_stats()
    stage = make_stage(lcb, synth, cfg, w, fc, tc, 1, 2, lanes)
    try:
        x = stage.to_device(synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)
        stage.cache_write(0, stage.to_device(synth.make_deep(cfg, 2)))

        def step(i):
            stage.cached_step(x, eps, 0)
        for i in range(warmup):
            step(i)
        stage.sync()
        timed = Timer(torch, stage).run(steps, step)
        fams, _ = profile_families(lcb, stage, step, 3)
        st = lcb.lc_get_stats(stage.ctx)
        measured = device_bytes_in_use(torch, st)
        peak = PEAK_TFLOPS[cfg.dtype]
        flops = cfg.cached_step_flops()
        ms = timed["median_ms"]
        return {"workload": f"{cfg.name}: B={cfg.B} F={cfg.F} latent {cfg.C_lat}x{cfg.H}x{cfg.W}, C={cfg.C}, "
                            f"{cfg.heads} heads x {cfg.head_dim}", "frame_chunk": fc, "token_chunk": tc, "steps": steps,
                "cached_step_ms_median": round(ms, 4), "cached_step_ms_wall_mean": round(timed["wall_ms_per_step"], 4),
                "gflop_per_step": round(flops / 1e9, 1), "tflops": round(flops / (ms * 1e-3) / 1e12, 1),
                "mfma_util_frac": round(flops / (ms * 1e-3) / 1e12 / peak, 4),
                "peak_hbm_gb": round(measured / 1e9, 4),
                "peak_hbm_gb_predicted": round(footprint(lcb, cfg, fc, tc, 2, 1, st.weight_bytes) / 1e9, 4),
                "breakdown_one_lane": breakdown_record(cfg, fams, peak)}
    finally:
        stage.close()
        torch.cuda.empty_cache()


def tiny_record(lcb, torch, synth, lanes):
    """The small fp32 stage: latency of a normal and a cache step (launch-bound), and the 25-step schedule
    (normal step when t % 3 == 0, swap-out after it, prefetch one step ahead) for frame chunk 16, 8, 4, 2. The stage
    has 8 frames: 16 and 8 both clamp to unchunked."""
    cfg = synth.CONFIGS["tiny"]
    w = synth.make_weights(cfg, 0)
    stage = make_stage(lcb, synth, cfg, w, cfg.frame_chunk, cfg.token_chunk, 2, 2, lanes)
    try:
        x = stage.to_device(synth.make_latents(cfg, 1))
        eps = stage.empty(*x.shape)
        for _ in range(5):
            stage.full_step(x, eps, 0)
            stage.cached_step(x, eps, 0)
        tm = Timer(torch, stage)
        full = tm.run(50, lambda i: stage.full_step(x, eps, 0))
        cached = tm.run(50, lambda i: stage.cached_step(x, eps, 0))
        flops = cfg.cached_step_flops()
        rec = {"note_schedule": "the tiny steps are bound by the host's launch rate (about 100 launches of a few "
                                "microseconds of device work each), so what a swap costs here is its seven runtime "
                                "calls on the host, not the link: overlap_frac at this size measures that",
               "workload": f"tiny fp32: B={cfg.B} F={cfg.F} latent {cfg.C_lat}x{cfg.H}x{cfg.W}, C={cfg.C}, frame chunk "
                           f"{cfg.frame_chunk}", "normal_step_ms_median": round(full["median_ms"], 4),
               "cached_step_ms_median": round(cached["median_ms"], 4), "gflop_per_cached_step": round(flops / 1e9, 2),
               "tflops": round(flops / (cached["median_ms"] * 1e-3) / 1e12, 2)}
    finally:
        stage.close()
    rec["schedule_25_steps_interval_3"] = [
        schedule_record(lcb, torch, synth, cfg, w, c, 0, 25, 3, 2, 5, lanes) for c in (16, 8, 4, 2)]
    rec["note"] = "8 frames: frame chunk 16 and 8 clamp to unchunked (same plan, same launches)"
    return rec


def stress_record(lcb, torch, synth, w, lanes, wbytes):
    """50 steps, a normal step every 5th, a bank of 10 pinned host entries, two device buffers. The frame chunk is
    the largest one that still gives both lanes a chunk and whose predicted footprint stays under 64 GB."""
    cfg = synth.CONFIGS["stress"]
    budget = 64e9  # (wbytes: the packed weights of the headline stage; the stress stage has the same widths)
    cands = [c for c in (cfg.N // 2, 16, 8, 4, 2, 1) if c <= cfg.N // 2]
    chosen = next((c for c in cands if footprint(lcb, cfg, c, 0, 2, 10, wbytes) < budget), 1)
    rec = schedule_record(lcb, torch, synth, cfg, w, chosen, 0, 50, 5, 10, 1, lanes)
    rec["workload"] = f"stress: B={cfg.B} F={cfg.F} latent {cfg.C_lat}x{cfg.H}x{cfg.W}, C={cfg.C}"
    rec["chunk_candidates_predicted_gb"] = {str(c): round(footprint(lcb, cfg, c, 0, 2, 10, wbytes) / 1e9, 3)
                                            for c in [cfg.N] + cands}
    rec["budget_gb"] = 64.0
    rec["bank_on_device_would_be_gb"] = round(10 * lcb.lc_cache_entry_bytes(lcb.make_config(cfg)) / 1e9, 3)
    rec["gflop_per_cached_step"] = round(cfg.cached_step_flops() / 1e9, 1)
    rec["tflops"] = round(cfg.cached_step_flops() / (rec["cached_step_ms"] * 1e-3) / 1e12, 1)
    rec["note"] = ("no score matrix, concatenated or normalised copy is ever materialised, so every chunk meets the "
                   "64 GB bound; it would only bite an implementation that materialises the fp32 scores "
                   "(2.7 GB per frame)")
    return rec


def decode_record(lcb, torch, synth, reps=3):
    """Sliced decoding of the AnimateDiff-sized latent video (16 frames of 64 x 64 -> 512 x 512): frame by frame, four
    frames at a time and all at once; time per video and the workspace each needs (it is sized by the slice)."""
    cfg = synth.DECODERS["animatediff"]
    w = synth.make_decoder_weights(cfg, 0)
    dec = lcb.Decoder(cfg, w, max_slice=cfg.N)
    try:
        z = dec.to_device(synth.make_decoder_latents(cfg, 1))
        rec = {"workload": f"decoder stand-in, N={cfg.N} frames, latent {cfg.C_lat}x{cfg.H}x{cfg.W} -> {cfg.C_img}x"
                           f"{cfg.H * 2 ** cfg.levels}x{cfg.W * 2 ** cfg.levels}, widths {list(cfg.widths)}, {cfg.dtype}",
               "gflop_per_video": round(cfg.decode_flops() / 1e9, 1), "slices": []}
        for sl in (1, 4, cfg.N):
            dec.decode(z, sl)
            dec.sync()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(reps + 1)]
            ev[0].record(dec.stream)
            for i in range(reps):
                dec.decode(z, sl)
                ev[i + 1].record(dec.stream)
            dec.sync()
            ms = statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(reps))
            rec["slices"].append({"slice_frames": sl, "ms_per_video": round(ms, 3),
                                  "tflops": round(cfg.decode_flops() / (ms * 1e-3) / 1e12, 1),
                                  "workspace_gb": round(lcb.lc_decoder_workspace_bytes(dec.ccfg, sl) / 1e9, 4)})
        return rec
    finally:
        dec.close()
        torch.cuda.empty_cache()


def dit_record(lcb, torch, synth, steps=6):
    """The diffusion-transformer variant: normal and cache step of a 12-block video DiT (blocks [2, 10) cached), and
    a schedule with a normal step every `interval` steps, Delta swapped out and prefetched one step ahead."""
    cfg = synth.DITS["video_dit"]
    w = synth.make_dit_weights(cfg, 0)
    dit = lcb.Dit(cfg, w, host_slots=2, dev_slots=2)
    try:
        # the record's own figures are taken with all tokens at once (at this size the token chunk saves 18 % of the
        # workspace for more than twice the time: see the sweep below); the workspace holds any chunk setting
        dit.set_chunk(0)
        x = dit.to_device(synth.make_dit_hidden(cfg, 1))
        mod = dit.to_device(synth.make_dit_modulation(cfg, 2))
        out = dit.empty(cfg.B, cfg.T, cfg.D)

        def timed(fn, n):
            fn()
            dit.sync()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            ev[0].record(dit.compute)
            for i in range(n):
                fn()
                ev[i + 1].record(dit.compute)
            dit.sync()
            return statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
        ms_full = timed(lambda: dit.full_step(x, mod, out, 0), steps)
        ms_cached = timed(lambda: dit.cached_step(x, mod, out, 0), steps)
        rec = {"workload": f"video DiT stand-in: B={cfg.B}, T={cfg.T} tokens, D={cfg.D}, {cfg.heads} heads x {cfg.head_dim}, "
                           f"L={cfg.L} blocks of which [{cfg.cache_a}, {cfg.cache_b}) are cached, {cfg.dtype}, all tokens at once",
               "normal_step_ms": round(ms_full, 3), "cache_step_ms": round(ms_cached, 3),
               "normal_step_tflops": round(cfg.full_step_flops() / (ms_full * 1e-3) / 1e12, 1),
               "cache_step_tflops": round(cfg.cached_step_flops() / (ms_cached * 1e-3) / 1e12, 1),
               "entry_mb": round(lcb.lc_dit_entry_bytes(dit.ccfg) / 1e6, 1),
               "workspace_gb": round(lcb.lc_dit_workspace_bytes(dit.ccfg, 0) / 1e9, 4), "schedules": []}
        # the token chunk trades workspace for launch size (results never change)
        rec["token_chunks"] = []
        for chunk in (512, 1024, 2048, 4096, 0):
            dit.set_chunk(chunk)
            rec["token_chunks"].append({"token_chunk": chunk, "normal_step_ms": round(timed(lambda: dit.full_step(x, mod, out, 0), 3), 3),
                                        "workspace_gb": round(lcb.lc_dit_workspace_bytes(dit.ccfg, chunk) / 1e9, 4)})
        dit.set_chunk(0)
        n_steps = 12

        def schedule(interval, swapping):
            refresh, prefetched = -1, None
            for t in range(n_steps):
                slot = t % 2 if swapping else 0
                if t % interval == 0:
                    refresh += 1
                    dit.full_step(x, mod, out, slot)
                    if swapping:
                        dit.swap_out(slot, refresh % 2)
                else:
                    if swapping and prefetched != (t, slot):
                        dit.swap_in(refresh % 2, slot)
                    dit.cached_step(x, mod, out, slot)
                if swapping and t + 1 < n_steps and (t + 1) % interval != 0:
                    dit.swap_in(refresh % 2, (t + 1) % 2)
                    prefetched = (t + 1, (t + 1) % 2)
        for interval in (1, 2, 3, 4):
            row = {"interval": interval}
            for name, swapping in (("resident", False), ("swapped", True)):
                if interval == 1 and swapping:
                    continue
                schedule(interval, swapping)
                dit.sync()
                t0 = time.perf_counter()
                schedule(interval, swapping)
                dit.sync()
                row[f"{name}_ms_per_step"] = round((time.perf_counter() - t0) * 1e3 / n_steps, 3)
            rec["schedules"].append(row)
        base = rec["schedules"][0]["resident_ms_per_step"]
        for row in rec["schedules"]:
            row["speedup_vs_every_step_normal"] = round(base / row.get("swapped_ms_per_step", row["resident_ms_per_step"]), 3)
        return rec
    finally:
        dit.close()
        torch.cuda.empty_cache()


def unet_record(lcb, torch, synth, steps=5, steps_only=False):
    """The U-Net with real block internals (time-embedding residual blocks, transformer blocks with cross-attention
    and GEGLU, frame encoding, three-level deep branch): normal and cache step, and schedules with a normal step every
    `interval` steps, the cached feature swapped out and prefetched one step ahead."""
    cfg = synth.UNETS["sd15_video"]
    w = synth.make_unet_weights(cfg, 0)
    net = lcb.Unet(cfg, w, host_slots=2, dev_slots=2)
    try:
        xa, ta, ca = synth.make_unet_inputs(cfg, 1)
        x, temb, ctx = net.to_device(xa), net.to_device(ta), net.to_device(ca)
        out = net.empty(*xa.shape)

        def timed(fn, n):
            fn()
            net.sync()
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(n + 1)]
            ev[0].record(net.compute)
            for i in range(n):
                fn()
                ev[i + 1].record(net.compute)
            net.sync()
            return statistics.median(ev[i].elapsed_time(ev[i + 1]) for i in range(n))
        ms_full = timed(lambda: net.full_step(x, temb, ctx, out, 0), steps)
        ms_cached = timed(lambda: net.cached_step(x, temb, ctx, out, 0), steps)
        rec = {"workload": f"video U-Net with real block internals, synthetic weights: B={cfg.B}, F={cfg.F}, {cfg.H}x{cfg.W} latents, "
                           f"widths {cfg.C}/{cfg.C1}/{cfg.C2}, heads of {cfg.head_dim}, {cfg.ctx_len} x {cfg.ctx_dim} conditioning "
                           f"tokens, time embedding {cfg.temb_dim}, {cfg.dtype}, all frames at once",
               "normal_step_ms": round(ms_full, 3), "cache_step_ms": round(ms_cached, 3),
               "normal_step_tflops": round(cfg.full_step_flops() / (ms_full * 1e-3) / 1e12, 1),
               "cache_step_tflops": round(cfg.cached_step_flops() / (ms_cached * 1e-3) / 1e12, 1),
               "entry_mb": round(lcb.lc_unet_entry_bytes(net.ccfg) / 1e6, 1),
               "workspace_gb": round(lcb.lc_unet_workspace_bytes(net.ccfg) / 1e9, 4), "schedules": []}
        if steps_only:  # what a kernel trace is pointed at: 1 + steps normal steps, then as many cache steps
            return rec
        n_steps = 12

        def schedule(interval, swapping):
            refresh, prefetched = -1, None
            for t in range(n_steps):
                slot = t % 2 if swapping else 0
                if t % interval == 0:
                    refresh += 1
                    net.full_step(x, temb, ctx, out, slot)
                    if swapping:
                        net.swap_out(slot, refresh % 2)
                else:
                    if swapping and prefetched != (t, slot):
                        net.swap_in(refresh % 2, slot)
                    net.cached_step(x, temb, ctx, out, slot)
                if swapping and t + 1 < n_steps and (t + 1) % interval != 0:
                    net.swap_in(refresh % 2, (t + 1) % 2)
                    prefetched = (t + 1, (t + 1) % 2)
        for interval in (1, 2, 3, 5):
            row = {"interval": interval}
            for name, swapping in (("resident", False), ("swapped", True)):
                if interval == 1 and swapping:
                    continue
                schedule(interval, swapping)
                net.sync()
                t0 = time.perf_counter()
                schedule(interval, swapping)
                net.sync()
                row[f"{name}_ms_per_step"] = round((time.perf_counter() - t0) * 1e3 / n_steps, 3)
            rec["schedules"].append(row)
        base = rec["schedules"][0]["resident_ms_per_step"]
        for row in rec["schedules"]:
            row["speedup_vs_every_step_normal"] = round(base / row.get("swapped_ms_per_step", row["resident_ms_per_step"]), 3)
        # feature chunk: frames per chunk in the per-frame blocks, as many rows of all frames in the temporal ones
        rec["frame_chunks"] = []
        for fc in (16, 8, 4, 2):
            net.set_chunk(fc)
            rec["frame_chunks"].append({"frame_chunk": fc, "normal_step_ms": round(timed(lambda: net.full_step(x, temb, ctx, out, 0), steps), 3),
                                        "cache_step_ms": round(timed(lambda: net.cached_step(x, temb, ctx, out, 0), steps), 3),
                                        "workspace_gb": round(lcb.lc_unet_chunk_workspace_bytes(net.ccfg, fc) / 1e9, 4)})
        net.set_chunk(0)
        return rec
    finally:
        net.close()
        torch.cuda.empty_cache()


if __name__ == "__main__":
    main()
