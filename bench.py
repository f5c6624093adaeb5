#!/usr/bin/env python3
"""Benchmark of the Flash Window Attention forward on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

A step is one pass of the whole forward hot path (load Q/K/V, scores, softmax,
PV, store O -- one kernel launch through the C ABI) over one Swin-T stage-1
batch: 128 images of 56x56 tokens, 7x7 windows -> N = 8192 windows, L = 49,
C = 96 = 3 heads x 32, bf16 data, fp32 accumulation, synthetic N(0,1) inputs
already resident in HBM.  The step cycles through several distinct Q/K/V/O
buffer sets whose total size exceeds twice the 256 MB last-level cache, so every
step streams from HBM.

Prints ONE JSON line: whole-job window-heads/s, plus the roofline object of the
forward kernel (HIP-event time per launch against the 8 TB/s HBM peak) and the
fp64 CPU oracle timed on this machine's host cores as a baseline.
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

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E bandwidth
LLC_BYTES = 256 * 2 ** 20       # Infinity Cache
# HBM bytes per launch of the forward kernel on this workload, from two rocprofv3 --pmc runs
# (FETCH_SIZE, then WRITE_SIZE, each scaled by what the same counter reads for a plain elementwise
# kernel of known size; figures and commands in profiles/fwd_bf16_staged_kernel_swin_t_stage1.md):
# 232.7 MB read + 77.1 MB written.
MEASURED_TRAFFIC_BYTES = 309.8e6
# Matrix-core busy fraction of the same kernel on the same workload, from the SQ counters in the same
# file (SQ_VALU_MFMA_BUSY_CYCLES over SIMDs x active cycles).  tests/test_bench_constants.py holds both
# constants to the figures in that file.
MEASURED_MFMA_BUSY_FRAC = 0.084
PROFILE_FILE = "profiles/fwd_bf16_staged_kernel_swin_t_stage1.md"
EVENT_GROUP = 100               # launches between two HIP events, at most
PREWARM_SECONDS = 0.3           # un-timed launches in front of the warm-up: the clocks ramp up over the first ones


def ensure_built():
    from paper_2501_06480_amd import binding
    if not os.path.exists(binding.library_path()):
        from paper_2501_06480_amd import build
        build.build(verbose=False)


def cpu_baseline(workload):
    """The fp64 oracle, as it stands, on the host cores, over the same batch shape."""
    import numpy as np
    import torch
    import oracle
    g = torch.Generator().manual_seed(workload.seed)
    q, k, v = (torch.randn((workload.N, workload.L, workload.C), generator=g).bfloat16().double().numpy()
               for _ in range(3))
    oracle.load()
    oracle.forward(q[:64], k[:64], v[:64], workload.heads, workload.scale)   # spin the thread pool up
    reps, t0 = 0, time.perf_counter()
    while True:
        o = oracle.forward(q, k, v, workload.heads, workload.scale)
        reps += 1
        dt = time.perf_counter() - t0
        if dt >= 1.5 or reps >= 50:
            break
    assert np.isfinite(o).all()
    cores = oracle.threads_used()
    return {"value": reps * workload.N * workload.heads / dt, "unit": "window-heads/s",
            "cores": cores, "kind": "oracle",
            "sample": f"whole batch ({workload.N} windows x {workload.heads} heads, fp64) x {reps} passes, "
                      f"{dt:.2f} s wall = {dt * cores:.0f} core-seconds"}


def device_info(torch, dev):
    """What the runtime reports for the device, next to the published peaks the fractions are taken against."""
    p = torch.cuda.get_device_properties(dev)
    khz = getattr(p, "clock_rate", None)
    mem_khz = bus_bits = None
    try:  # the HIP runtime torch has already loaded; attribute numbers of hipDeviceAttribute_t (hip_runtime_api.h)
        import ctypes
        hip = ctypes.CDLL("libamdhip64.so")
        def attr(which):
            v = ctypes.c_int(0)
            return v.value if hip.hipDeviceGetAttribute(ctypes.byref(v), which, dev.index or 0) == 0 else None
        khz = khz or attr(5)                   # hipDeviceAttributeClockRate, kHz
        mem_khz, bus_bits = attr(60), attr(59)  # hipDeviceAttributeMemoryClockRate (kHz), ...MemoryBusWidth (bits)
    except OSError:
        pass
    return {"name": p.name, "arch": getattr(p, "gcnArchName", None), "compute_units": p.multi_processor_count,
            "max_clock_mhz": None if not khz else khz / 1e3,
            "memory_clock_mhz": None if not mem_khz else mem_khz / 1e3, "memory_bus_bits": bus_bits,
            "hbm_bytes": p.total_memory,
            "published_peaks": {"hbm_GBps": HBM_PEAK_GBPS, "bf16_mfma_dense_TFLOPs": 2500.0,
                                "compute_units": 256, "clock_mhz": 2400}}


def copy_ceiling(torch, sets, iters=60):
    """A plain elementwise kernel that reads three tensors and writes one, each the size of Q, over the
    same rotating buffer sets: the HBM rate a 3-in / 1-out streaming kernel reaches on this machine."""
    n = len(sets)
    for i in range(5):
        q, k, v, o = sets[i % n]
        torch.addcmul(q, k, v, out=o)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for i in range(iters):
        q, k, v, o = sets[i % n]
        torch.addcmul(q, k, v, out=o)
    e1.record()
    torch.cuda.synchronize()
    us = e0.elapsed_time(e1) / iters * 1e3
    gbps = 4 * sets[0][0].numel() * 2 / us / 1e3
    return {"kernel": "torch.addcmul(q, k, v, out=o), bf16, same bytes as one step", "us_per_call": round(us, 2),
            "GBps": gbps, "frac_of_hbm_peak": gbps / HBM_PEAK_GBPS}


def time_other_workloads(torch, fwa, synth, dev):
    """Short HIP-event timings of the other configurations (context next to the headline line):
    Swin-T stage 1 with bias + shift mask, the large windows, and the backward.  Same buffer
    rotation rule as the headline (cycle larger than twice the last-level cache)."""
    out = []

    def run(name, w, backward, iters, want_dbias=True, as_labels=False, bias_bf16=False):
        shape = (w.N, w.L, w.C)
        tdt, esz = {"f32": (torch.float32, 4), "bf16": (torch.bfloat16, 2), "f16": (torch.float16, 2)}[w.dtype]
        per_set = (7 if backward else 4) * w.N * w.L * w.C * esz
        nsets = max(2, -(-2 * LLC_BYTES // per_set) + 1)
        g = torch.Generator(device=dev).manual_seed(w.seed)
        sets = [[torch.randn(shape, device=dev, generator=g).to(tdt) for _ in range(4 if backward else 3)]
                for _ in range(nsets)]
        outs = [torch.empty(shape, device=dev, dtype=tdt) for _ in range(nsets)]
        bias = mask = labels = ws = None
        if w.use_bias:
            bias = fwa.fwa_bias_gather(torch.from_numpy(synth.bias_table(w.heads, w.k, w.seed)).to(dev), w.k)
            if bias_bf16:
                bias = bias.to(torch.bfloat16)
        if w.shift and as_labels:  # the mask as region labels, formed inside the kernels
            labels = torch.from_numpy(synth.shift_labels(w.map_hw, w.map_hw, w.k, w.shift)).to(dev)
        elif w.shift:
            mask = torch.from_numpy(synth.shift_mask(w.map_hw, w.map_hw, w.k, w.shift)).to(dev)
        if backward:
            need = fwa.fwa_backward_workspace_bytes(w.N, w.L, w.C, w.heads, {"f32": 0, "bf16": 1, "f16": 2}[w.dtype], want_dbias)
            ws = torch.empty(max(need, 16), dtype=torch.uint8, device=dev)

        def step(i):
            t = sets[i % nsets]
            if backward:
                fwa.fwa_backward(t[0], t[1], t[2], t[3], w.heads, w.scale, bias, mask, want_dbias=want_dbias, workspace=ws,
                                 labels=labels)
            else:
                fwa.fwa_forward(t[0], t[1], t[2], w.heads, w.scale, bias, mask, out=outs[i % nsets], labels=labels)

        t_warm = time.perf_counter()  # at least 0.3 s of warm-up: the clocks ramp up over the first launches
        while True:
            for i in range(40):
                step(i)
            torch.cuda.synchronize()
            if time.perf_counter() - t_warm > 0.3:
                break
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for i in range(iters):
            step(i)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) / iters * 1e3
        wh = w.N * w.heads
        algo = (7 if backward else 4) * w.L * (w.C // w.heads) * esz * wh
        out.append({"workload": name, "us_per_call": round(us, 2), "window_heads_per_s": wh / us * 1e6,
                    "algorithmic_GBps": algo / us / 1e3, "frac_of_hbm_peak": algo / us / 1e3 / HBM_PEAK_GBPS})

    def run_small(name, w, launches=16, replays=60):
        """A launch-bound shape, eager and as one HIP graph of `launches` forward calls (distinct buffers)."""
        shape = (w.N, w.L, w.C)
        g = torch.Generator(device=dev).manual_seed(w.seed)
        sets = [[torch.randn(shape, device=dev, generator=g).to(torch.bfloat16) for _ in range(3)] for _ in range(launches)]
        outs = [torch.empty(shape, device=dev, dtype=torch.bfloat16) for _ in range(launches)]
        bias = fwa.fwa_bias_gather(torch.from_numpy(synth.bias_table(w.heads, w.k, w.seed)).to(dev), w.k)

        def chain(stream=None):
            for t, o in zip(sets, outs):
                fwa.fwa_forward(t[0], t[1], t[2], w.heads, w.scale, bias, None, out=o, stream=stream)

        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)

        def timed(fn):
            for _ in range(5):
                fn()
            torch.cuda.synchronize()
            e0.record()
            for _ in range(replays):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / (replays * launches) * 1e3

        us_eager = timed(chain)
        side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            chain(torch.cuda.current_stream())
        us_graph = timed(graph.replay)
        wh = w.N * w.heads
        algo = 4 * w.L * 32 * 2 * wh
        for label, us in (("eager", us_eager), (f"HIP graph of {launches} launches", us_graph)):
            out.append({"workload": f"{name}, {label}", "us_per_call": round(us, 2), "window_heads_per_s": wh / us * 1e6,
                        "algorithmic_GBps": algo / us / 1e3, "frac_of_hbm_peak": algo / us / 1e3 / HBM_PEAK_GBPS})

    run("swin_t_stage1_fwd_bias_shiftmask (N=8192, L=49, 3 heads)", synth.swin_t_stage(1, shifted=True), False, 400)
    run("swin_t_stage1_fwd_bias_shiftlabels (N=8192, L=49, 3 heads; mask from region labels)",
        synth.swin_t_stage(1, shifted=True), False, 400, as_labels=True)
    run_small("swin_t_stage3_fwd_bias (N=512, L=49, 12 heads)", synth.swin_t_stage(3))
    run_small("swin_t_stage4_fwd_bias (N=128, L=49, 24 heads)", synth.swin_t_stage(4))
    l144, l256 = synth.config4()
    run("window12_fwd_bias (N=1024, L=144, 4 heads)", l144, False, 100)
    run("window16_fwd_bias (N=1024, L=256, 4 heads)", l256, False, 50)
    s1, s3 = synth.config5()
    run("swin_t_stage1_bwd_bias_shiftmask_dbias (N=8192, L=49, 3 heads)", s1, True, 200)
    run("swin_t_stage3_bwd_bias_shiftmask_dbias (N=512, L=49, 12 heads)", s3, True, 200)
    run("window12_bwd_bias (N=1024, L=144, 4 heads; dQ, dK, dV)", l144, True, 30, want_dbias=False)
    run("window16_bwd_bias (N=1024, L=256, 4 heads; dQ, dK, dV)", l256, True, 20, want_dbias=False)
    # shifted 16 x 16 windows of a 32 x 32 map: the dense mask against region labels
    w16s = synth.Workload("window16_shift", 1024, 256, 128, 4, "bf16", 1300, 16, 32, True, 8, True)
    for form, lab, b16 in (("bias_shiftmask", False, False), ("bias_shiftlabels", True, False),
                           ("bf16bias_shiftlabels", True, True)):
        run(f"window16_fwd_{form} (N=1024, L=256, 4 heads)", w16s, False, 50, as_labels=lab, bias_bf16=b16)
        run(f"window16_bwd_{form}_dbias (N=1024, L=256, 4 heads)", w16s, True, 20, as_labels=lab, bias_bf16=b16)
    # the shapes of the paper's own kernel benchmark (section 3.1): L = 64, 4 heads, width per head 64 and 256
    paper_shapes(run)
    # stage 1 on the token map of an 896 x 896 input (224 x 224 tokens: 1024 windows per image, batch 8): a mask
    # period that no workgroup stride over the windows is a multiple of; the mask as region labels
    hr = synth.Workload("stage1_map224", 8192, 49, 96, 3, "bf16", 1400, 7, 224, True, 3, True)
    run("swin_t_stage1_fwd_bias_shiftlabels, 1024 windows per image (N=8192, L=49, 3 heads)", hr, False, 200, as_labels=True)
    run("swin_t_stage1_bwd_bias_shiftlabels_dbias, 1024 windows per image (N=8192, L=49, 3 heads)", hr, True, 100,
        as_labels=True)
    return out


def paper_shapes(run):
    from paper_2501_06480_amd import synth
    for d in (64, 256):
        pw = synth.Workload(f"paper_L64_d{d}", 4096, 64, 4 * d, 4, "bf16", 1100 + d, 8)
        run(f"paper_benchmark_shape_fwd (N=4096, L=64, 4 heads x {d})", pw, False, 50)
        run(f"paper_benchmark_shape_bwd (N=4096, L=64, 4 heads x {d}; dQ, dK, dV)", pw, True, 30, want_dbias=False)
        # IEEE half data, the precision of the paper's comparison with flash-attention (section 3.3)
        ph = synth.Workload(f"paper_L64_d{d}_f16", 4096, 64, 4 * d, 4, "f16", 1150 + d, 8)
        run(f"paper_benchmark_shape_fwd_fp16 (N=4096, L=64, 4 heads x {d})", ph, False, 50)
        run(f"paper_benchmark_shape_bwd_fp16 (N=4096, L=64, 4 heads x {d}; dQ, dK, dV)", ph, True, 30, want_dbias=False)
        # the same in the paper's own precision (fp32 data and arithmetic), half the windows
        pf = synth.Workload(f"paper_L64_d{d}_f32", 2048, 64, 4 * d, 4, "f32", 1200 + d, 8)
        run(f"paper_benchmark_shape_fwd_fp32 (N=2048, L=64, 4 heads x {d})", pf, False, 20)
        run(f"paper_benchmark_shape_bwd_fp32 (N=2048, L=64, 4 heads x {d}; dQ, dK, dV)", pf, True, 10, want_dbias=False)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--no-other-workloads", action="store_true", help="skip the short timings of the other configs")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch 5 plain elementwise kernels that read and write one tensor of known size, "
                         "so that a counter run can scale FETCH_SIZE / WRITE_SIZE against known traffic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py measures one GPU: this build has no multi-GPU path (the workload is data-parallel "
              "over windows: each GPU would take a contiguous range of them, with one all-reduce of dBias). "
              "Run with --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import torch
    ensure_built()
    import paper_2501_06480_amd as fwa
    from paper_2501_06480_amd import synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU: there is no CPU path.", file=sys.stderr)
        sys.exit(3)
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    w = synth.config2()
    shape = (w.N, w.L, w.C)
    set_bytes = 4 * w.N * w.L * w.C * 2
    nsets = max(2, -(-2 * LLC_BYTES // set_bytes) + 1)
    g = torch.Generator(device=dev).manual_seed(w.seed)
    sets = []
    for _ in range(nsets):
        q, k, v = (torch.randn(shape, device=dev, dtype=torch.float32, generator=g).to(torch.bfloat16)
                   for _ in range(3))
        sets.append((q, k, v, torch.empty(shape, device=dev, dtype=torch.bfloat16)))

    def step(i):
        q, k, v, o = sets[i % nsets]
        fwa.fwa_forward(q, k, v, w.heads, w.scale, out=o)

    # Whatever --warmup says, the device first gets PREWARM_SECONDS of the same launches: a fresh
    # process starts at idle clocks, and a short timed region (the default K, W of a driver run are
    # a millisecond of work) would otherwise measure the ramp.
    t_warm, i = time.perf_counter(), 0
    while True:
        for _ in range(50):
            step(i)
            i += 1
        torch.cuda.synchronize()
        if time.perf_counter() - t_warm >= PREWARM_SECONDS:
            break
    prewarm_steps = i
    for i in range(args.warmup):
        step(i)
    # HIP events on the launch stream bracket groups of launches (an event between every two kernels
    # would itself put a bubble between them): at most EVENT_GROUP per group, at least 4 groups when
    # the run is long enough for groups of 5.  The kernel's average duration is the summed event time
    # over the whole timed region divided by the number of launches; median and minimum are over the
    # groups' per-launch times.
    group = max(1, min(EVENT_GROUP, max(5, args.steps // 20)))
    bounds = list(range(0, args.steps, group)) + [args.steps]
    marks = [torch.cuda.Event(enable_timing=True) for _ in bounds]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for gi in range(len(bounds) - 1):
        marks[gi].record()
        for i in range(bounds[gi], bounds[gi + 1]):
            step(i)
    marks[-1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    group_ms = [marks[gi].elapsed_time(marks[gi + 1]) / (bounds[gi + 1] - bounds[gi]) for gi in range(len(bounds) - 1)]
    kernel_ms = sum(marks[gi].elapsed_time(marks[gi + 1]) for gi in range(len(bounds) - 1)) / args.steps
    kernel_ms_median, kernel_ms_min = sorted(group_ms)[len(group_ms) // 2], min(group_ms)
    assert all(torch.isfinite(s[3].float()).all().item() for s in sets)

    if args.calibrate_copy:
        for i in range(5):
            q, _, _, o = sets[i % nsets]
            torch.neg(q, out=o)                  # reads w.N*w.L*w.C*2 bytes, writes as many
        torch.cuda.synchronize()

    wh = w.N * w.heads
    algo_bytes = 4 * w.L * 32 * 2 * wh           # Q, K, V in and O out, once each, bf16
    achieved = algo_bytes / (kernel_ms * 1e-3) / 1e9
    line = {
        "metric": "fwd window-heads/sec, Swin-T stage-1 shapes bf16",
        "value": wh * args.steps / wall,
        "unit": "window-heads/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "swin_t_stage1_fwd: N=8192 windows, L=49, C=96, heads=3, head_dim=32, "
                               "no bias/mask, batch 128 of 56x56", "buffer_sets": nsets,
                   "window_heads_per_step": wh},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": MEASURED_TRAFFIC_BYTES,
                     "kernel": "fwd_bf16_staged_kernel<4,false,1>", "kernel_ms": kernel_ms,
                     "kernel_ms_median": kernel_ms_median, "kernel_ms_min": kernel_ms_min,
                     "event_groups": len(group_ms), "launches_per_group": group,
                     "frac_at_median": algo_bytes / (kernel_ms_median * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "frac_at_min": algo_bytes / (kernel_ms_min * 1e-3) / 1e9 / HBM_PEAK_GBPS,
                     "algorithmic_bytes_per_launch": algo_bytes,
                     "mfma_busy_frac": MEASURED_MFMA_BUSY_FRAC, "counters_from": PROFILE_FILE},
        "prewarm": {"seconds": PREWARM_SECONDS, "steps": prewarm_steps},
        "device": device_info(torch, dev),
    }
    line["copy_ceiling"] = copy_ceiling(torch, sets)
    line["paper_context"] = ("paper (one RTX 4090, Triton, fp32): forward up to 300 % faster than Swin's window "
                             "attention at L=64, 4 heads; end-to-end Swin 10-30 %; no absolute throughput published")
    if not args.no_other_workloads:
        del sets
        torch.cuda.empty_cache()
        line["other_workloads"] = time_other_workloads(torch, fwa, synth, dev)
    if not args.no_cpu_baseline:
        line["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(line))


if __name__ == "__main__":
    main()
