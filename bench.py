#!/usr/bin/env python3
"""Benchmark of the ModeT hot path on one MI355X.

A step is one modet_fwd (phi + log-normaliser) followed by one modet_bwd (dQ, dK) on the
brain-MRI full-resolution level (1 x 160 x 192 x 224, C=8, 1 head, k=3, fp32, synthetic
seeded inputs already resident in HBM).  Prints ONE JSON line:

  value      voxel-neighbourhoods/s = B*D*H*W*heads / (time of fwd + bwd)
  roofline   the dominant kernel (the backward) against the 8 TB/s HBM peak, from its
             algorithmic bytes and its live HIP-event duration inside the timed region
  cpu_baseline   the CPU oracle (fp64 loops, OpenMP over slabs) on the same inputs
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
PREWARM_MS = 60.0

PROFILE_FILE = os.path.join(ROOT, "profiles", "config3_fwd_bwd_warp_kernels.txt")


def traffic_from_profile(kernel):
    """HBM bytes per launch of `kernel` as the committed rocprofv3 --pmc summary records them (FETCH_SIZE +
    WRITE_SIZE, scaled by what the same counters read for a plain copy): its line `hbm_bytes_per_launch <kernel>
    <bytes>`.  None if the summary has no such line (the kernel that ran is not the one that was profiled)."""
    try:
        with open(PROFILE_FILE) as f:
            for line in f:
                w = line.split()
                if len(w) == 3 and w[0] == "hbm_bytes_per_launch" and w[1] == kernel:
                    return int(w[2])
    except OSError:
        pass
    return None


def sclk_under(step, torch, seconds=1.2):
    """Shader clock in MHz as `rocm-smi --showclocks` reports it while `step` loops (median of the samples), or
    None if the tool is missing or prints something else.  Context for the roofline figures: the published peaks
    assume 2.4 GHz, the box lowers the clock under sustained vector load."""
    import re
    import subprocess
    import threading
    samples, stop = [], threading.Event()

    def watch():
        while not stop.is_set():
            try:
                out = subprocess.run(["rocm-smi", "--showclocks"], capture_output=True, text=True, timeout=5).stdout
            except Exception:
                return
            m = re.search(r"sclk clock level: \d+: \((\d+)Mhz\)", out)
            if m:
                samples.append(int(m.group(1)))
            stop.wait(0.2)

    th = threading.Thread(target=watch, daemon=True)
    th.start()
    t0 = time.perf_counter()
    while time.perf_counter() - t0 < seconds:
        for _ in range(20):
            step()
        torch.cuda.synchronize()
    stop.set()
    th.join(timeout=10)
    samples = sorted(samples[1:] or samples)          # (the first sample may predate the load)
    return samples[len(samples) // 2] if samples else None


def bench_pyramid(args, np, torch, modet, synth):
    """Config 4: the five-level coarse-to-fine loop for a 160x192x224 pair (Section 3.1); a step is one
    iteration over all levels (warp, forward, composition, backward, update), `--steps` of them are timed (50
    by default: the number of fine-tuning iterations per pair of Section 4.4)."""
    from paper_2403_16526_amd.pyramid import PyramidLoop
    t0 = time.time()
    pyr = synth.make_pyramid()
    t_gen = time.time() - t0
    levels = [dict(Q=torch.from_numpy(l["Q"]).cuda(), K=torch.from_numpy(l["K"]).cuda(), heads=l["heads"]) for l in pyr]
    loop = PyramidLoop(levels, eta=1.0)
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < PREWARM_MS:
        loop.iteration()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        loop.iteration()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        loop.iteration()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    ms_per_iter = wall * 1e3 / args.steps

    # the split: the same loop with HIP events around every library call (a run of its own: the events perturb it)
    spans = {}

    def timer(l, name, fn):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        out = fn()
        e1.record()
        spans.setdefault((l, name), []).append((e0, e1))
        return out

    loop.timer = timer
    nsplit = 10
    e_a, e_b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e_a.record()
    for _ in range(nsplit):
        loop.iteration()
    e_b.record()
    torch.cuda.synchronize()
    loop.timer = None
    split_iter_ms = e_a.elapsed_time(e_b) / nsplit
    us = {k: 1e3 * sum(a.elapsed_time(b) for a, b in v) / nsplit for k, v in spans.items()}
    per_level, lib_us = [], 0.0
    nvn_total, alg_bytes, alg_bytes_survey = 0, 0, 0
    for l, lv in enumerate(pyr):
        n, C, heads = lv["D"] * lv["H"] * lv["W"], lv["C"], lv["heads"]
        nvn_total += n * heads
        fwd_b, bwd_b = n * (8 * C + 12 * heads), n * (8 * C + 12 * heads + 8 * C)
        # warp: source and result once, the coarse field once (1/8 of 12 bytes per fine voxel); composition: the
        # residual field, the coarse field, the result
        warp_b = n * (8 * C) + n * 12 // 8 if l else 0
        comp_b = n * 24 + n * 12 // 8 if l else 0
        alg_bytes += fwd_b + bwd_b + warp_b + comp_b
        alg_bytes_survey += fwd_b + bwd_b + (n * (8 * C + 12) if l else 0)
        row = {"level": l + 1, "grid": f"{lv['D']}x{lv['H']}x{lv['W']}", "C": C, "heads": heads}
        for name in ("warp", "fwd", "compose", "bwd"):
            if (l, name) in us:
                row[name + "_us"] = round(us[(l, name)], 1)
                lib_us += us[(l, name)]
        per_level.append(row)
    top = pyr[-1]
    ntop = top["D"] * top["H"] * top["W"]
    dom_bytes = ntop * (8 * top["C"] + 12 * top["heads"] + 8 * top["C"])
    dom_ms = us[(len(pyr) - 1, "bwd")] * 1e-3
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": "modet_bwd of level 5 (bwd_sym_kernel)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": None,
                "algorithmic_bytes": dom_bytes, "avg_launch_ms": round(dom_ms, 4)}
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from oracle.pyramid_loop import OraclePyramidLoop
        ol = OraclePyramidLoop([dict(Q=l["Q"].copy(), K=l["K"], heads=l["heads"]) for l in pyr], eta=1.0)
        t0 = time.perf_counter()
        nit = 2
        for _ in range(nit):
            ol.iteration()
        dt = (time.perf_counter() - t0) / nit
        cpu = {"value": round(nvn_total / dt, 1), "unit": "voxel-neighbourhoods/s", "cores": oracle.threads(),
               "kind": "oracle",
               "sample": f"{nit} of the {synth.PYRAMID_ITERS} iterations of the oracle-side loop over all five levels, "
                         f"{dt:.2f} s per iteration ({dt * synth.PYRAMID_ITERS:.0f} s extrapolated to the whole loop)"}
    line = {
        "metric": "ModeT fwd+bwd voxel-neighbourhoods/sec and achieved HBM GB/s (% of peak), 1 GPU",
        "value": round(nvn_total / (ms_per_iter * 1e-3), 1), "unit": "voxel-neighbourhoods/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_iter, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": "config 4: five-level pairwise-optimisation loop for a 160x192x224 pair, C=64,32,32,16,8 "
                               "heads=8,4,4,2,1 k=3 f32; one step = one iteration over all levels (warp by the "
                               "upsampled field, fwd, composition, bwd, update)",
                   "untimed_prewarm_ms": PREWARM_MS, "logits": "fp64"},
        "roofline": roofline,
        "cpu_baseline": cpu,
        "loop_ms_total": round(ms_per_iter * args.steps, 3),
        "per_level": per_level,
        "libmodet_us_per_iteration": round(lib_us, 1),
        "glue_share": round(1.0 - lib_us * 1e-3 / split_iter_ms, 4),
        "iteration_ms_with_events": round(split_iter_ms, 4),
        "bytes_per_iteration": alg_bytes,
        "bytes_per_iteration_full_res_field": alg_bytes_survey,
        "hbm_gbs": round(alg_bytes / (ms_per_iter * 1e-3) / 1e9, 1),
        "hbm_frac": round(alg_bytes / (ms_per_iter * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "input_gen_s": round(t_gen, 1),
    }
    print(json.dumps(line))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    # the timed region is long enough to average over the box's jitter
    ap.add_argument("--steps", type=int, default=None, help="default: 300 (config 4: its 50 iterations)")
    ap.add_argument("--warmup", type=int, default=None, help="default: 100 (config 4: 5)")
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-clock-sample", action="store_true", help="do not sample the shader clock under load")
    ap.add_argument("--generic", action="store_true", help="force the generic kernels")
    ap.add_argument("--fast-logits", action="store_true",
                    help="fp32 instead of fp64 logits (does not meet the parity tolerance; for information)")
    ap.add_argument("--recompute-stats", action="store_true", help="do not hand phi/lse of the forward to the backward")
    # variants of the workload (not the headline configuration): the paper's own head sizes, the learned bias
    ap.add_argument("--head-dim", type=int, default=0, choices=[0, 6, 8, 12],
                    help="channels per head: the configuration's shape with C = heads * this (0: as configured)")
    ap.add_argument("--bias", action="store_true",
                    help="add a bias B (Eq. 3) to the logits; the backward then also returns its gradient")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (--gpus 1); a multi-GPU figure is not produced.",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2403_16526_amd import modet, synth

    assert torch.cuda.is_available(), "bench.py needs the GPU"
    torch.cuda.set_device(0)
    if args.config == 4:
        args.steps = synth.PYRAMID_ITERS if args.steps is None else args.steps
        args.warmup = 5 if args.warmup is None else args.warmup
        return bench_pyramid(args, np, torch, modet, synth)
    args.steps = 300 if args.steps is None else args.steps
    args.warmup = 100 if args.warmup is None else args.warmup
    cfg = synth.CONFIGS[args.config]
    t0 = time.time()
    over = {"C": cfg["heads"] * args.head_dim} if args.head_dim else {}
    c = synth.make_config(args.config, **over)
    t_gen = time.time() - t0
    B, D, H, W, C, heads, k, dtype = (c[n] for n in ("B", "D", "H", "W", "C", "heads", "k", "dtype"))
    nvox = B * D * H * W
    nvn = nvox * heads
    esz = 2 if dtype == "bf16" else 4

    def up(a):
        if a.dtype == np.uint16:
            return torch.from_numpy(a.view(np.int16)).cuda().view(torch.bfloat16)
        return torch.from_numpy(a).cuda()

    Q, K, g = up(c["Q"]), up(c["K"]), up(c["dphi"])
    f32 = dict(device="cuda", dtype=torch.float32)
    phi = torch.empty((B, D, H, W, heads, 3), **f32)
    lse = torch.empty((B, D, H, W, heads), **f32)
    dQ = torch.empty((B, D, H, W, C), **f32)
    dK = torch.empty((B, D, H, W, C), **f32)
    in_dt = modet.MODET_BF16 if dtype == "bf16" else modet.MODET_F32
    have_stats = not args.recompute_stats
    wsb = modet.modet_bwd_workspace_bytes(B, D, H, W, C, heads, k, in_dt, have_stats, want_dbias=args.bias)
    ws = torch.empty(max(wsb, 16), device="cuda", dtype=torch.uint8)
    bias = (torch.from_numpy((0.5 * synth.normal(synth.BASE_SEED + args.config, 9, (heads, k ** 3))).astype(np.float32))
            .cuda() if args.bias else None)
    if args.generic:
        modet.modet_set_kernel_path(1)
    if args.fast_logits:
        modet.modet_set_math_mode(1)

    def fwd():
        modet.modet_fwd(Q, K, heads, k, bias=bias, out=(phi, lse))

    def bwd():
        if have_stats:
            modet.modet_bwd(Q, K, g, heads, k, bias=bias, phi=phi, lse=lse, want_dbias=args.bias, out=(dQ, dK),
                            workspace=ws)
        else:
            modet.modet_bwd(Q, K, g, heads, k, bias=bias, want_dbias=args.bias, out=(dQ, dK), workspace=ws)

    # The first ~20 ms of GPU work after an idle period run ~15 % slower while the clocks ramp up.  Whatever
    # --warmup says, keep the GPU busy with the same step for PREWARM_MS before the warm-up steps (untimed, and
    # reported in the JSON line) so that short runs measure the same machine state as long ones.
    t0 = time.perf_counter()
    while (time.perf_counter() - t0) * 1e3 < PREWARM_MS:
        for _ in range(10):
            fwd()
            bwd()
        torch.cuda.synchronize()
    for _ in range(args.warmup):
        fwd()
        bwd()
    torch.cuda.synchronize()

    # timed region: exactly `steps` steps; HIP events on the launch stream bracket every call
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ev[i][0].record()
        fwd()
        ev[i][1].record()
        bwd()
        ev[i][2].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    t_fwd = sum(e[0].elapsed_time(e[1]) for e in ev) / args.steps          # ms
    t_bwd = sum(e[1].elapsed_time(e[2]) for e in ev) / args.steps
    ms_per_step = wall * 1e3 / args.steps
    sclk = None if args.no_clock_sample else sclk_under(lambda: (fwd(), bwd()), torch)

    # algorithmic bytes (each tensor moved once, no stored attention)
    fwd_bytes = nvox * (2 * C * esz + 12 * heads)
    bwd_bytes = nvox * (2 * C * esz + 12 * heads + 8 * C)
    hs = heads * (2 if C // heads == 12 else 1)       # fused columns per voxel (twelve channels: two half-heads)
    tiled = not args.generic and modet.modet_has_tiled_kernels(C, heads, k, in_dt) == 3
    bwd_kernel = ("generic kernels" if not tiled else "bwd_sym_kernel" if k == 3 and hs == 1 else
                  "bwd_fused_kernel" if k == 3 and hs == 2 else "bwd_shared_kernel" if k == 3 else "march_pair_kernel")
    dom_bytes, dom_ms, dom_name = ((bwd_bytes, t_bwd, f"modet_bwd ({bwd_kernel})") if t_bwd >= t_fwd
                                  else (fwd_bytes, t_fwd, "modet_fwd"))
    achieved = dom_bytes / (dom_ms * 1e-3) / 1e9
    roofline = {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": (traffic_from_profile(bwd_kernel)
                            if (args.config == 3 and t_bwd >= t_fwd and not args.generic and not args.bias
                                and not args.head_dim) else None),
                "algorithmic_bytes": dom_bytes, "avg_launch_ms": round(dom_ms, 4)}

    # the same step against the vector-ALU roofline.  Algorithmic flops per window: k^3 pairs, each a d-term dot
    # product in the forward, one in the backward, and d-term updates of dQ and dK (2 flops per FMA), plus ~16 for
    # the two softmax evaluations.  Peak: the published vector rate of the arithmetic type, fp64 78.6 TFLOP/s
    # (fp32 inputs: logits in fp64, and unpacked fp32 FMAs issue at that same rate) or fp32 157.3 TFLOP/s
    # (bf16 inputs: everything in fp32; reachable only with packed instructions, which this build does not use).
    d = C // heads
    flops = nvn * (k ** 3) * (8 * d + 16)
    alu_peak = 157.3 if dtype == "bf16" else 78.6
    alu_ach = flops / ((t_fwd + t_bwd) * 1e-3) / 1e12
    roofline_alu = {"bound": "alu", "kernel": "modet_fwd + modet_bwd", "achieved": round(alu_ach, 2), "peak": alu_peak,
                    "unit": "TFLOP/s", "frac": round(alu_ach / alu_peak, 4), "traffic": None,
                    "algorithmic_flops": flops, "avg_launch_ms": round(t_fwd + t_bwd, 4)}
    if args.config == 5:      # 125 pairs per window: arithmetic, not memory, bounds this workload
        roofline, roofline_other = roofline_alu, ("roofline_hbm", roofline)
    else:
        roofline_other = ("roofline_alu", roofline_alu)

    # a plain device copy of the same byte count: the attainable ceiling on this machine
    nb = (fwd_bytes + bwd_bytes) // 2
    a = torch.empty(nb // 4, **f32)
    b = torch.empty_like(a)
    for _ in range(3):
        b.copy_(a)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(10):
        b.copy_(a)
    e1.record()
    torch.cuda.synchronize()
    copy_gbs = 2 * nb * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9
    del a, b

    # warp at the same shape (reported beside the metric, not part of `value`)
    field = torch.from_numpy(synth.smooth_real_field(synth.BASE_SEED + args.config, B, D, H, W, 1.5)).cuda()
    Kw = torch.empty_like(K)
    for _ in range(3):
        modet.modet_warp(K, field, out=Kw)
    e0.record()
    for _ in range(10):
        modet.modet_warp(K, field, out=Kw)
    e1.record()
    torch.cuda.synchronize()
    t_warp = e0.elapsed_time(e1) / 10
    warp_bytes = nvox * (2 * C * esz + 12)

    # the warp's adjoint (scatter with atomics), source gradient alone and with the field gradient
    dsrc = torch.empty((B, D, H, W, C), **f32)
    dKw = torch.empty((B, D, H, W, C), **f32).normal_()
    t_wb = []
    for want in (False, True):
        for _ in range(2):
            modet.modet_warp_bwd(K, field, dKw, want_dfield=want, out=dsrc)
        e0.record()
        for _ in range(5):
            modet.modet_warp_bwd(K, field, dKw, want_dfield=want, out=dsrc)
        e1.record()
        torch.cuda.synchronize()
        t_wb.append(e0.elapsed_time(e1) / 5)
    del dsrc, dKw

    # field composition and scaling-and-squaring at the same shape (also beside the metric)
    comp, tmp = torch.empty_like(field), torch.empty_like(field)
    for _ in range(3):
        modet.modet_compose(field, field, out=comp)
    e0.record()
    for _ in range(10):
        modet.modet_compose(field, field, out=comp)
    e1.record()
    torch.cuda.synchronize()
    t_comp = e0.elapsed_time(e1) / 10
    modet.modet_integrate_velocity(field, 7, out=comp, tmp=tmp)
    e0.record()
    for _ in range(5):
        modet.modet_integrate_velocity(field, 7, out=comp, tmp=tmp)
    e1.record()
    torch.cuda.synchronize()
    t_int = e0.elapsed_time(e1) / 5

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        # bounded sample: a slab of D planes sized so the oracle runs for roughly 10-20 s
        Ds = D if nvn * (k ** 3) <= 6_881_280 * 27 else max(2 * k, int(D * 6_881_280 * 27 / (nvn * k ** 3)))
        sl = slice(0, Ds)
        Qs, Ks, gs = c["Q"][:, sl].copy(), c["K"][:, sl].copy(), c["dphi"][:, sl].copy()
        best = 1e30
        for _ in range(2):
            t0 = time.perf_counter()
            oracle.modet_fwd(Qs, Ks, heads, k, dtype=dtype)
            oracle.modet_bwd(Qs, Ks, gs, heads, k, dtype=dtype, form="gather")
            best = min(best, time.perf_counter() - t0)
        nthreads = oracle.threads()
        cpu = {"value": round(B * Ds * H * W * heads / best, 1), "unit": "voxel-neighbourhoods/s",
               "cores": nthreads, "kind": "oracle",
               "sample": f"fwd+bwd(gather form) of the fp64 oracle on planes 0..{Ds - 1} of {D} "
                         f"({B}x{Ds}x{H}x{W}), best of 2, {best:.2f} s"}
        # the same oracle on one thread, on a slab 1/threads as deep (about the same wall time)
        D1 = min(Ds, max(2 * k, Ds // max(1, nthreads)))
        Q1, K1, g1 = c["Q"][:, :D1].copy(), c["K"][:, :D1].copy(), c["dphi"][:, :D1].copy()
        oracle.set_threads(1)
        try:
            t0 = time.perf_counter()
            oracle.modet_fwd(Q1, K1, heads, k, dtype=dtype)
            oracle.modet_bwd(Q1, K1, g1, heads, k, dtype=dtype, form="gather")
            one = time.perf_counter() - t0
        finally:
            oracle.set_threads(nthreads)
        cpu["one_thread"] = {"value": round(B * D1 * H * W * heads / one, 1), "cores": 1,
                             "sample": f"planes 0..{D1 - 1}, one run, {one:.2f} s"}

    value = nvn / (wall / args.steps)
    line = {
        "metric": "ModeT fwd+bwd voxel-neighbourhoods/sec and achieved HBM GB/s (% of peak), 1 GPU",
        "value": round(value, 1), "unit": "voxel-neighbourhoods/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "f32" if dtype == "f32" else "bf16-in/f32-acc", "data": "synthetic",
        "config": {"workload": f"config {args.config}{' (variant)' if (args.bias or args.head_dim) else ''}: "
                               f"{cfg['name']} B={B} {D}x{H}x{W} C={C} heads={heads} k={k} {dtype}, "
                               + ("fwd(phi,lse)+bwd(dQ,dK,dbias) with bias" if args.bias else "fwd(phi,lse)+bwd(dQ,dK)"),
                   "kernel_path": "generic" if args.generic else "auto",
                   "stats_from_forward": have_stats, "untimed_prewarm_ms": PREWARM_MS,
                   "logits": ("fp32" if dtype == "bf16" else
                              "fp32 (outside the parity tolerance)" if args.fast_logits else "fp64")},
        "roofline": roofline,
        roofline_other[0]: roofline_other[1],
        "cpu_baseline": cpu,
        "fwd_ms": round(t_fwd, 4), "bwd_ms": round(t_bwd, 4), "sclk_mhz_under_load": sclk,
        "hbm_gbs_fwd_bwd": round((fwd_bytes + bwd_bytes) / ((t_fwd + t_bwd) * 1e-3) / 1e9, 1),
        "hbm_frac_fwd_bwd": round((fwd_bytes + bwd_bytes) / ((t_fwd + t_bwd) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "hbm_gbs_fwd": round(fwd_bytes / (t_fwd * 1e-3) / 1e9, 1),
        "hbm_gbs_bwd": round(bwd_bytes / (t_bwd * 1e-3) / 1e9, 1),
        "pairs_per_s": round(value * k ** 3, 1),
        "device_copy_gbs": round(copy_gbs, 1),
        "warp": {"ms": round(t_warp, 4), "gbs": round(warp_bytes / (t_warp * 1e-3) / 1e9, 1)},
        "warp_bwd": {"ms": round(t_wb[0], 4), "gbs": round(warp_bytes / (t_wb[0] * 1e-3) / 1e9, 1),
                     "ms_with_field_gradient": round(t_wb[1], 4)},
        "compose": {"ms": round(t_comp, 4), "gbs": round(nvox * 24 / (t_comp * 1e-3) / 1e9, 1),
                    "integrate_T7_ms": round(t_int, 4)},
        "input_gen_s": round(t_gen, 1),
    }
    print(json.dumps(line))


if __name__ == "__main__":
    main()
