#!/usr/bin/env python3
"""Benchmark of the per-block distillation step and of the all-block schedule on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch resident in HBM: frozen teacher block forward +
student forward, local loss, backward and SGD-momentum update (pbkd_distill_step); for the all-block schedule one step
is one batch through the teacher chain and all five student steps (pbkd_distill_step_all).

The default run prints ONE JSON line that carries the whole metric ("images/s per block + all-block step time"):
  * value / ms_per_step: the largest block configuration, the ImageNet-shaped VGG16 block 1 at batch 32 (cfg4);
  * config.blocks: the CIFAR-shaped VGG16 block 2 (cfg2) and the ResNet-18 downsampling block (cfg3), each with the
    student step alone beside the whole step;
  * config.all_block_step: the five CIFAR-shaped VGG16 blocks (cfg5) on three student streams packed by
    worst-fit-decreasing, teacher chain on its own stream;
  every figure is the MEDIAN over `--repeats` timed regions of exactly `--steps` steps each (a device synchronisation on
  both sides of every region), after a warm-up that runs until the clocks have ramped (at least `--warmup` steps and at
  least half a second), so the figure does not depend on --warmup being large;
  * roofline: the dominant kernel (3x3 implicit-GEMM convolution on the fp32 matrix cores) of the cfg4 step, timed with
    HIP events carried by each of its launches on ONE stream; roofline.hbm: the bandwidth-bound kernels of the same
    step (first-layer convolution, depthwise forward/backward, pointwise, BatchNorm backward, block head, update) as
    algorithmic bytes per launch / event time / 8 TB/s; roofline.blocks: the same convolution figure for cfg2 and cfg3;
  * cpu_baseline: the CPU oracle as it stands on the host cores, per reported workload (cfg5 = all five blocks), with
    OpenMP over all cores and single-threaded (the latter on a smaller batch, stated), core counts beside it.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--repeats R] [--workload all|cfg1|cfg2|cfg3|cfg4|cfg5|vgg13|vgg16_imagenet]
                    [--overlap 0|1] [--streams S] [--policy 0|1|2] [--measured-weights] [--breakdown] [--no-cpu-baseline]
                    [--min-warmup-seconds T] [--graph 0|1]
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

MFMA_F32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
MFMA_BF16_PEAK_TFLOPS = 2500.0    # MI355X dense bf16 matrix peak
# The teacher's 3x3 convolution forms every fp32 product from six bf16 MFMA products of operands split three ways (fp32
# accumulation): its ceiling in fp32-equivalent flops is a sixth of the bf16 peak.
SPLIT_PRODUCTS = 6
MFMA_SPLIT_PEAK_TFLOPS = round(MFMA_BF16_PEAK_TFLOPS / SPLIT_PRODUCTS, 1)


def conv_split_in_use():
    """The library's rule for the frozen teacher's 3x3 convolutions: the bf16-split kernel unless PBKD_CONV_SPLIT=0."""
    return os.environ.get("PBKD_CONV_SPLIT", "") != "0"
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of a kernel (reads + writes) from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs of this benchmark,
# scaled by what the same counters read for a device copy of known size: written by
# `python -m paper_2012_03096_amd.profile_summary traffic ...` (the commands are in the file), read here.
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "hbm_traffic.json")

SINGLE = {"cfg1": "cfg1_tiny", "cfg2": "cfg2_vgg_block2", "cfg3": "cfg3_resnet_down", "cfg4": "cfg4_imagenet_vgg_block1"}


def measured_traffic(workload_name, kernel):
    """Counter-measured HBM bytes per launch of `kernel` in `workload_name`, or None if no profile has been summarised."""
    if kernel in ("conv1x1_mfma", "pw_dgrad_mfma"):     # one kernel serves both: the counters cannot tell them apart
        kernel = "pw_mfma (forward and data gradient)"
    try:
        with open(TRAFFIC_JSON) as f:
            rec = json.load(f)["workloads"][workload_name]["kernels"][kernel]
        return int(rec["fetch_bytes_per_launch"] + rec["write_bytes_per_launch"])
    except (OSError, KeyError, ValueError):
        return None


# ---------------------------------------------------------------------------------------------- algorithmic work
def wgrad_takes_bn_backward(arch, shapes, l):
    """The library's rule (layer 0 a trainable full 3x3 convolution with at most three input channels, stride 1, width a
    multiple of 4, tensors of at most 2 GiB, a depthwise-separable layer behind it): its weight-gradient kernel then
    folds the BatchNorm backward in and the elementwise kernel is not launched."""
    from paper_2012_03096_amd import workloads as wl
    if l != 0 or len(arch.layers) < 2:
        return False
    L = arch.layers[0]
    ci, hi, wi, co, ho, wo = shapes[0]
    return (L.kind == wl.CONV3X3 and L.trainable and L.stride == 1 and 9 * ci <= 32 and wo % 4 == 0
            and arch.layers[1].kind == wl.DWSEP3X3 and 4 * arch.n * co * ho * wo <= 2 ** 31)


def kernel_work(w):
    """Per kernel kind of the library (pbkd_kernel_kind_name): algorithmic bytes (every input tensor read once, every
    output written once, fp32), convolution FLOPs and launches of ONE step = teacher forward + student step."""
    from paper_2012_03096_amd import workloads as wl
    work = {}

    def add(kind, nbytes, flops=0):
        rec = work.setdefault(kind, {"bytes": 0, "flops": 0, "launches": 0})
        rec["bytes"] += 4 * nbytes
        rec["flops"] += flops
        rec["launches"] += 1

    def forward(arch, training):
        n = arch.n
        shapes = wl.layer_shapes(arch)
        for l, ((ci, hi, wi, co, ho, wo), L) in enumerate(zip(shapes, arch.layers)):
            a, u, z = n * ci * hi * wi, n * ci * ho * wo, n * co * ho * wo
            if L.kind == wl.CONV3X3:
                first = l == 0 and L.stride == 1 and 9 * ci <= 32
                add("conv3x3_first" if first else "conv3x3_mfma", a + z, 2 * 9 * ci * co * n * ho * wo)
            else:
                add("dw3x3_fwd", a + u, 2 * 9 * ci * n * ho * wo)
                add("conv1x1_mfma", u + z, 2 * ci * co * n * ho * wo)
        ci, hi, wi, co, ho, wo = shapes[-1]
        z = n * co * ho * wo
        t = z // 4 if arch.pool == 2 else z
        zs = 0
        if arch.shortcut == 1:
            add("conv1x1_mfma", n * arch.c * ho * wo + z, 2 * arch.c * co * n * ho * wo)
            zs = z
        elif arch.shortcut == 2:
            zs = z
        if training:
            add("head_loss", z + zs + t)
            add("head_bwd", z + zs + t + z)
        else:
            add("head_out", z + zs + t)

    forward(w.teacher, False)
    forward(w.student, True)
    arch = w.student
    n = arch.n
    shapes = wl.layer_shapes(arch)
    params = 0
    for l in range(len(arch.layers) - 1, -1, -1):
        (ci, hi, wi, co, ho, wo), L = shapes[l], arch.layers[l]
        if not L.trainable:
            break
        a, u, z = n * ci * hi * wi, n * ci * ho * wo, n * co * ho * wo
        if L.kind == wl.DWSEP3X3:
            add("pw_wgrad_mfma", z + u, 2 * ci * co * n * ho * wo)
            add("pw_dgrad_mfma", z + u, 2 * ci * co * n * ho * wo)
            add("dw3x3_bwd", u + a if l == 0 else u + 2 * a, 2 * 9 * ci * n * ho * wo * (1 if l == 0 else 2))
            if l > 0 and arch.layers[l - 1].trainable and not wgrad_takes_bn_backward(arch, shapes, l - 1):
                add("bn_bwd_apply", 3 * a)
            params += 9 * ci + ci * co + 2 * co
        else:
            # behind a depthwise-separable layer the first layer's weight gradient reads g and z (BatchNorm backward
            # folded in) instead of a dz written by a kernel of its own
            fused = wgrad_takes_bn_backward(arch, shapes, l)
            add("conv3x3_wgrad", (2 * z if fused else z) + a, 2 * 9 * ci * co * n * ho * wo * (2 if fused else 1))
            params += 9 * ci * co + 2 * co
    add("sgd_momentum", 5 * params)      # theta and momentum read and written, the gradient written
    return work


HBM_KINDS = ["conv3x3_first", "dw3x3_fwd", "conv1x1_mfma", "head_out", "head_loss", "head_bwd", "pw_wgrad_mfma", "pw_dgrad_mfma",
             "dw3x3_bwd", "bn_bwd_apply", "conv3x3_wgrad", "sgd_momentum"]


# ---------------------------------------------------------------------------------------------- timing helpers
def touch_first(torch, stream):
    """Makes `stream` submit a first (tiny) piece of work and waits for it."""
    with torch.cuda.stream(stream):
        torch.zeros(256, device="cuda").add_(1.0)
    torch.cuda.synchronize()


MIN_WARMUP_SECONDS = 0.5


def warm_up(torch, step, min_steps, min_seconds=None):
    """Untimed steps until the shader and memory clocks have ramped: at least min_steps and at least min_seconds."""
    if min_seconds is None:
        min_seconds = MIN_WARMUP_SECONDS
    min_seconds = min(min_seconds, MIN_WARMUP_SECONDS)
    t0 = time.perf_counter()
    n = 0
    while n < min_steps or time.perf_counter() - t0 < min_seconds:
        step()
        n += 1
        if n % 16 == 0:
            torch.cuda.synchronize()
    torch.cuda.synchronize()
    return n


def timed_regions(torch, step, steps, repeats):
    """`repeats` regions of exactly `steps` steps, a device synchronisation on both sides of each.
    Returns (seconds per region, host seconds spent enqueueing per region)."""
    el, host = [], []
    for _ in range(repeats):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            step()
        t1 = time.perf_counter()
        torch.cuda.synchronize()
        el.append(time.perf_counter() - t0)
        host.append(t1 - t0)
    return el, host


def summary(el, steps, batch):
    med = statistics.median(el)
    return {"images_per_s": round(batch * steps / med, 1), "ms_per_step": round(med / steps * 1e3, 4),
            "ms_per_step_repeats": [round(e / steps * 1e3, 4) for e in el]}


# ---------------------------------------------------------------------------------------------- one block
def run_block(args, w, kernel_roofline=True):
    """One block: whole steps (teacher on a second stream beside the student unless --overlap 0), the student step
    alone, and -- on ONE stream, where every kernel has the GPU to itself -- HIP-event times of every kernel kind."""
    import torch
    from paper_2012_03096_amd import binding as pb, workloads as wl
    x, tp, sp = w.tensors()
    # the teacher's stream submits work before the student's ever does: streams get their hardware queues in the
    # order of their first submission, and the overlap is better when the teacher's queue is the earlier one
    tstream = torch.cuda.Stream() if args.overlap else None
    if tstream is not None:
        touch_first(torch, tstream)
    stream = torch.cuda.Stream()
    if tstream is None:
        tstream = stream
    blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum, stream=stream)
    blk.set_graph_mode(bool(args.graph))
    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    n = w.teacher.n

    def step():
        blk.distill_step(xd, td, w.lr, want_loss=False, student_stream=stream, teacher_stream=tstream)

    def step_one_stream():
        blk.distill_step(xd, td, w.lr, want_loss=False, student_stream=stream, teacher_stream=stream)

    def student_only():
        blk.student_step(xd, td, w.lr, want_loss=False, stream=stream)

    warm_up(torch, step, args.warmup)
    el, host = timed_regions(torch, step, args.steps, args.repeats)
    res = summary(el, args.steps, n)
    res.update({"workload": w.name, "batch": n, "input": [n, w.teacher.c, w.teacher.h, w.teacher.w],
                "streams": 2 if args.overlap else 1, "hip_graph": bool(args.graph), "block_flops_per_step": blk.flops(3),
                "host_enqueue_ms_per_step": round(statistics.median(host) / args.steps * 1e3, 4),
                "loss_after": blk.last_loss()})
    if args.plain:                       # for profiler runs: nothing but the warm-up and the timed whole steps
        blk.close()
        return res, None
    if args.overlap:
        warm_up(torch, step_one_stream, 4, 0.05)
        el1, _ = timed_regions(torch, step_one_stream, args.steps, args.repeats)
        res["one_stream"] = summary(el1, args.steps, n)
    warm_up(torch, student_only, 4, 0.05)
    el_s, _ = timed_regions(torch, student_only, args.steps, args.repeats)
    res["student_step_alone"] = summary(el_s, args.steps, n)

    roof = None
    if kernel_roofline:
        # every launch of every kernel kind between a pair of HIP events on the stream it runs on (the 3x3
        # convolutions carry their events themselves), all on ONE stream
        work = kernel_work(w)
        n_launch = sum(r["launches"] for r in work.values()) + 16
        k_prof = max(4, min(args.steps, 40))
        warm_up(torch, step_one_stream, 4, 0.05)
        blk.profile_enable(None, capacity=n_launch * k_prof + 64)
        for _ in range(k_prof):
            step_one_stream()
        torch.cuda.synchronize()
        prof = blk.profile_read()
        blk.profile_enable(None, 0)
        roof = {"per_kind": {}, "steps": k_prof}
        for kind, (ms, launches) in prof.items():
            rec = {"launches_per_step": round(launches / k_prof, 2), "avg_launch_us": round(ms / max(launches, 1) * 1e3, 2),
                   "us_per_step": round(ms / k_prof * 1e3, 2)}
            wk = work.get(kind)
            if wk:
                sec = ms * 1e-3 / k_prof
                rec["algorithmic_bytes_per_step"] = wk["bytes"]
                rec["GBps"] = round(wk["bytes"] / sec / 1e9, 1)
                rec["frac_of_hbm_peak"] = round(wk["bytes"] / sec / 1e9 / HBM_PEAK_GBS, 4)
                if wk["flops"]:
                    rec["flops_per_step"] = wk["flops"]
                    rec["TFLOPps"] = round(wk["flops"] / sec / 1e12, 2)
                    rec["frac_of_mfma_peak"] = round(wk["flops"] / sec / 1e12 / MFMA_F32_PEAK_TFLOPS, 4)
            roof["per_kind"][kind] = rec
    blk.close()
    del blk, xd, td
    torch.cuda.empty_cache()
    return res, roof


def mfma_roofline(w, roof, region_note):
    """The `roofline` object for the dominant kernel: the 3x3 implicit-GEMM convolution on the matrix cores."""
    rec = roof["per_kind"].get("conv3x3_mfma")
    if not rec:
        return {"bound": "mfma", "achieved": None, "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": None, "traffic": None}
    lps = max(int(round(rec["launches_per_step"])), 1)
    out = {"bound": "mfma", "kernel": "pbkd::conv_mfma_kernel (3x3 implicit GEMM, v_mfma_f32_32x32x2_f32)",
           "workload": w.name, "achieved": rec["TFLOPps"], "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
           "frac": rec["frac_of_mfma_peak"], "traffic": measured_traffic(w.name, "conv_mfma_kernel"),
           "launches_per_step": lps, "avg_launch_ms": round(rec["avg_launch_us"] * 1e-3, 5),
           "flops_per_launch": rec["flops_per_step"] // lps, "flops_per_step": rec["flops_per_step"],
           "algorithmic_bytes_per_launch": rec["algorithmic_bytes_per_step"] // lps, "region": region_note}
    if conv_split_in_use():
        # `achieved` stays the convolution's own (fp32) flops over its time; the peak is the bf16 one over the six bf16
        # products each of them costs.  The same rate against the fp32 matrix peak is given beside it.
        out.update({"kernel": "pbkd::conv_split_kernel (3x3 implicit GEMM, fp32 operands split into three bf16 terms, "
                              "six v_mfma_f32_32x32x16_bf16 products per fp32 product, fp32 accumulation)",
                    "peak": MFMA_SPLIT_PEAK_TFLOPS, "frac": round(rec["TFLOPps"] / MFMA_SPLIT_PEAK_TFLOPS, 4),
                    "peak_is": "dense bf16 MFMA peak %.0f TFLOP/s / %d bf16 products per fp32 product" % (MFMA_BF16_PEAK_TFLOPS, SPLIT_PRODUCTS),
                    "frac_of_fp32_mfma_peak": rec["frac_of_mfma_peak"],
                    "bf16_TFLOPps_issued": round(rec["TFLOPps"] * SPLIT_PRODUCTS, 1),
                    "traffic": measured_traffic(w.name, "conv_split_kernel")})
    return out


def hbm_list(w, roof):
    out = []
    for kind in HBM_KINDS:
        rec = roof["per_kind"].get(kind)
        if not rec or "GBps" not in rec:
            continue
        lps = max(rec["launches_per_step"], 1e-9)
        item = {"kernel": kind, "bound": "hbm", "launches_per_step": rec["launches_per_step"],
                "algorithmic_bytes_per_launch": int(rec["algorithmic_bytes_per_step"] / lps),
                "avg_launch_us": rec["avg_launch_us"], "achieved": rec["GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": rec["frac_of_hbm_peak"], "traffic": measured_traffic(w.name, kind)}
        if "TFLOPps" in rec:
            item["TFLOPps"] = rec["TFLOPps"]
            item["frac_of_mfma_peak"] = rec["frac_of_mfma_peak"]
        out.append(item)
    return out


# ---------------------------------------------------------------------------------------------- all blocks
def run_all_blocks(args, workload):
    """cfg5: all five VGG16 blocks, one concurrent distillation step per 'step' (teacher chain once, students on
    streams).  vgg13: the paper's own granularity (section 3.3, 4.4): one task per 3x3 convolution, 13 tasks, the
    student two depthwise-separable layers; every task has its own synthetic input (no chain)."""
    import torch
    from paper_2012_03096_amd import binding as pb, workloads as wl
    chain = workload in ("cfg5", "vgg16_imagenet")
    if workload == "vgg16_imagenet":       # the five VGG16 stages at ImageNet size: 224x224 images, batch 32
        ws = wl.cfg5_vgg16_blocks(n=32, hw=224)
    else:
        ws = wl.cfg5_vgg16_blocks() if chain else wl.paper_granularity_vgg16_tasks()
    blocks, xs, ts = [], [], []
    for i, w in enumerate(ws):
        x, tp, sp = w.tensors()
        blocks.append(pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum))
        blocks[-1].set_graph_mode(bool(args.graph) and args.policy != 2 and not args.measured_weights)
        if i == 0 or not chain:
            xs.append(torch.from_numpy(x).cuda())
        ts.append(torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda"))
    if chain:
        xs = [xs[0]] + ts[:-1]
    n_streams = args.streams
    # the teacher's stream submits work before any student stream does: streams get their hardware queues in the
    # order of their first submission, and the overlap is better when the teacher's queue is the earlier one (measured)
    tstream = torch.cuda.Stream()
    if chain:                       # (without a chain there is no teacher stream to favour: it stays unused)
        touch_first(torch, tstream)
    streams = [torch.cuda.Stream() for _ in range(n_streams)]
    for st_ in streams:
        touch_first(torch, st_)
    weights = None
    if args.measured_weights:
        # the paper's own bin-packing weight: each task's measured run time (microseconds for 5 steps, alone)
        one = streams[0]          # no extra stream: the process has few hardware queues, more streams would share them
        weights = []
        if chain:
            pb.distill_step_all(blocks, xs, ts, 0.01, [one], [0] * len(blocks), list(range(len(blocks))), True, one)
        for b, x, t in zip(blocks, xs, ts):
            for rep in range(2):
                torch.cuda.synchronize()
                t0 = time.perf_counter()
                for _ in range(5):
                    b.distill_step(x, t, 0.01, want_loss=False, student_stream=one, teacher_stream=one)
                torch.cuda.synchronize()
                dt = time.perf_counter() - t0
            weights.append(max(int(dt * 1e6), 1))
    sob, order, load = pb.schedule_blocks(weights, n_streams, min(args.policy, 1), blocks=blocks)
    # bins are interchangeable: the fullest one goes to the stream that submitted first (the earliest hardware queue
    # of the student streams, which the command processor serves best), the next to the second, ...
    rank = {b_: r_ for r_, b_ in enumerate(sorted(range(n_streams), key=lambda k: (-load[k], k)))}
    sob = [rank[b_] for b_ in sob]
    load = [l_ for _, l_ in sorted((rank[k], load[k]) for k in range(n_streams))]
    torch.cuda.synchronize()

    # With a chain the targets are double buffered (--target-sets 2): consecutive steps write their teacher activations
    # into alternate sets, so the next step's teacher chain does not wait for this step's students to let go of them.
    sets = [(xs, ts)]
    if chain and args.target_sets == 2:
        ts2 = [torch.empty_like(t) for t in ts]
        sets.append(([xs[0]] + ts2[:-1], ts2))
    parity = [0]

    def step():
        xs_, ts_ = sets[parity[0] % len(sets)]
        parity[0] += 1
        pb.distill_step_all(blocks, xs_, ts_, 0.01, streams, sob, order, chain, tstream)

    steals = None
    n = ws[0].teacher.n
    if args.policy == 2:
        # work stealing: every task = one whole run of K steps of its block on its own copy of the input (with the
        # chained workload the inputs are the teacher prefix's activations, computed once here); all tasks start in
        # the queue the round-robin deal gives them
        step()
        torch.cuda.synchronize()
        xs = [x.clone() for x in xs]
        q0 = [i % n_streams for i in range(len(blocks))]
        pb.run_tasks_work_stealing(blocks, xs, ts, 0.01, [max(args.warmup, 10)] * len(blocks), streams, q0)
        el = []
        for _ in range(args.repeats):
            t0 = time.perf_counter()
            sob, steals = pb.run_tasks_work_stealing(blocks, xs, ts, 0.01, [args.steps] * len(blocks), streams, q0)
            el.append(time.perf_counter() - t0)
        host = el
    else:
        warm_up(torch, step, args.warmup)
        el, host = timed_regions(torch, step, args.steps, args.repeats)
    flops = sum(b.flops(3) for b in blocks)
    res = summary(el, args.steps, n)
    med = statistics.median(el)
    name = ("vgg16_imagenet_all_blocks" if workload == "vgg16_imagenet" else "cfg5_vgg16_all_blocks") if chain else "vgg16_13_conv_tasks"
    res.update({"workload": name, "batch": n, "tasks": len(blocks), "streams": n_streams, "target_sets": len(sets),
                "hip_graph": bool(args.graph) and args.policy != 2 and not args.measured_weights,
                "policy": ["wfd", "round_robin", "work_stealing"][args.policy], "steals": steals,
                "weights": "measured_us_per_5_steps" if weights else "flops", "stream_load": load, "stream_of_block": sob,
                "flops_per_step": flops, "host_enqueue_ms_per_step": round(statistics.median(host) / args.steps * 1e3, 4),
                "whole_schedule_TFLOPps": round(flops * args.steps / med / 1e12, 2),
                "whole_schedule_frac_of_mfma_peak": round(flops * args.steps / med / 1e12 / MFMA_F32_PEAK_TFLOPS, 4),
                "losses": [round(b.last_loss(), 6) for b in blocks]})
    for b in blocks:
        b.close()
    del blocks, xs, ts
    torch.cuda.empty_cache()
    return res


# ---------------------------------------------------------------------------------------------- CPU oracle
def physical_cores():
    try:
        pairs = set()
        phys = core = None
        with open("/proc/cpuinfo") as f:
            for line in f:
                if line.startswith("physical id"):
                    phys = line.split(":")[1].strip()
                elif line.startswith("core id"):
                    core = line.split(":")[1].strip()
                elif not line.strip():
                    if phys is not None and core is not None:
                        pairs.add((phys, core))
                    phys = core = None
        return len(pairs) or None
    except OSError:
        return None


def _set_omp_threads(n):
    """Thread count of the oracle's OpenMP loops (the oracle itself is left as it stands)."""
    import ctypes
    ctypes.CDLL("libgomp.so.1").omp_set_num_threads(int(n))


def oracle_steps(ws, steps, chain):
    """`steps` full steps (teacher forward + student step) of every workload in ws on the CPU oracle; seconds taken."""
    import numpy as np
    from oracle import block as ob
    refs, xs = [], []
    for w in ws:
        x, tp, sp = w.tensors()
        refs.append(ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum))
        xs.append(x)
    t0 = time.perf_counter()
    for _ in range(steps):
        x = xs[0]
        for i, (w, ref) in enumerate(zip(ws, refs)):
            xin = x if (chain or i == 0) else xs[i]
            t = ref.teacher_forward(xin)
            ref.student_step(xin, t.astype(np.float32), w.lr)
            x = t.astype(np.float32)
    return time.perf_counter() - t0


def cpu_baseline_for(make, chain, all_threads, label):
    """OpenMP over all cores on the full-size workload (as many steps as fit a few seconds) and single-threaded on
    a smaller batch of the same shapes (stated)."""
    from oracle import block as ob
    ws = make(None)
    n = ws[0].teacher.n
    _set_omp_threads(all_threads)
    el = oracle_steps(ws, 1, chain)
    steps = 1
    if el < 1.5:
        steps = max(1, min(16, int(3.0 / el)))
        el = oracle_steps(ws, steps, chain)
    used = ob.num_threads()
    small = max(1, n // 16)
    ws1 = make(small)
    _set_omp_threads(1)
    el1 = oracle_steps(ws1, 1, chain)
    _set_omp_threads(all_threads)
    return {"value": round(n * steps / el, 2), "unit": "images/s", "cores": used, "kind": "oracle",
            "sample": f"{steps} full step(s) of {label} at batch {n}, fp64, OpenMP, {el:.1f} s",
            "single_thread": {"value": round(small / el1, 3), "unit": "images/s", "cores": 1,
                              "sample": f"1 full step of {label} at batch {small} (same shapes), fp64, {el1:.1f} s"}}


def cpu_baselines(names):
    from oracle import block as ob
    from paper_2012_03096_amd import workloads as wl
    all_threads = ob.num_threads()
    makers = {
        "cfg1": (lambda n: [wl.cfg1_tiny()], False, "cfg1_tiny_block"),
        "cfg2": (lambda n: [wl.cfg2_vgg_block2(**({"n": n} if n else {}))], False, "cfg2_cifar_vgg16_block2"),
        "cfg3": (lambda n: [wl.cfg3_resnet_down(**({"n": n} if n else {}))], False, "cfg3_cifar_resnet18_down"),
        "cfg4": (lambda n: [wl.cfg4_imagenet_vgg_block1(**({"n": n} if n else {}))], False, "cfg4_imagenet_vgg16_block1"),
        "cfg5": (lambda n: wl.cfg5_vgg16_blocks(**({"n": n} if n else {})), True, "cfg5_vgg16_all_blocks (five blocks, teacher chain)"),
        "vgg13": (lambda n: wl.paper_granularity_vgg16_tasks(**({"n": n} if n else {})), False, "vgg16_13_conv_tasks"),
    }
    out = {}
    for name in names:
        make, chain, label = makers[name]
        out[label.split(" ")[0]] = cpu_baseline_for(make, chain, all_threads, label)
    return out, {"logical_cpus": os.cpu_count(), "physical_cores": physical_cores(), "omp_threads": all_threads}


# ---------------------------------------------------------------------------------------------- main
def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="steps per timed region")
    ap.add_argument("--warmup", type=int, default=10, help="least number of untimed steps before the timed regions")
    ap.add_argument("--repeats", type=int, default=5, help="timed regions per figure; the median is reported")
    ap.add_argument("--min-warmup-seconds", type=float, default=0.5,
                    help="the warm-up also lasts at least this long (clock ramp); 0 under a profiler keeps traces short")
    ap.add_argument("--workload", default="all", choices=["all", "cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "vgg13", "vgg16_imagenet"])
    ap.add_argument("--streams", type=int, default=3, help="cfg5 / vgg13: number of student streams")
    ap.add_argument("--overlap", type=int, default=1,
                    help="single block: 1 (default) = teacher on a second stream beside the student; 0 = everything on one stream")
    ap.add_argument("--target-sets", type=int, default=2, choices=[1, 2],
                    help="cfg5: sets of target buffers the all-block step alternates between (2 = double buffered)")
    ap.add_argument("--policy", type=int, default=0, help="cfg5 / vgg13: 0 worst-fit-decreasing, 1 round robin, 2 work stealing (whole K-step runs as tasks)")
    ap.add_argument("--measured-weights", action="store_true",
                    help="cfg5 / vgg13: pack by each task's measured run time (the paper's weight) instead of its FLOP count")
    ap.add_argument("--graph", type=int, default=0,
                    help="1: steps are captured into HIP graphs and replayed (pbkd_block_set_graph_mode); 0 (default): every launch "
                         "issued by the host (measured on this ROCm: a graph launch costs the host as much as the launches it replaces)")
    ap.add_argument("--plain", action="store_true",
                    help="single block: only the warm-up and the timed whole steps (no student-alone, one-stream or kernel-timing "
                         "regions, no roofline): what a profiler run should trace")
    ap.add_argument("--breakdown", action="store_true", help="add the per-kernel-kind event times of every reported block")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="run 20 plain device-to-device copies of MIB mebibytes and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (blocks are spread over HIP streams of one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.steps < 1 or args.repeats < 1 or args.warmup < 0:
        print("bench.py: --steps and --repeats must be at least 1", file=sys.stderr)
        sys.exit(2)
    global MIN_WARMUP_SECONDS
    MIN_WARMUP_SECONDS = max(args.min_warmup_seconds, 0.0)
    if args.workload != "all" or args.calibrate_copy:
        import torch
        if not torch.cuda.is_available():
            print("bench.py: no GPU visible", file=sys.stderr)
            sys.exit(1)
    if args.calibrate_copy:
        n = args.calibrate_copy << 20
        src = torch.arange(n // 4, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        for _ in range(20):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": n, "calibrate_copy_bytes_written": n, "copies": 20}))
        return
    from paper_2012_03096_amd import workloads as wl

    common = {"n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "higher_is_better": True, "scaling": "weak",
              "vs_baseline": None, "dtype": "f32", "data": "synthetic"}
    region = "%d steps on ONE stream, every launch between HIP events (the 3x3 convolutions carry theirs)"
    if args.workload == "all":
        # every workload in a process of its own, one after the other (this process never touches the GPU): a process
        # has four hardware queues and a stream keeps the queue it first submitted to, so in a shared process the
        # later workloads' streams would inherit whichever queues the earlier ones left them
        import subprocess
        parts = {}
        for key in ("cfg4", "cfg2", "cfg3", "cfg5"):
            cmd = [sys.executable, os.path.abspath(__file__), "--workload", key, "--steps", str(args.steps), "--warmup", str(args.warmup),
                   "--repeats", str(args.repeats), "--overlap", str(args.overlap), "--streams", str(args.streams),
                   "--policy", str(args.policy), "--graph", str(args.graph), "--min-warmup-seconds", str(args.min_warmup_seconds),
                   "--target-sets", str(args.target_sets),
                   "--no-cpu-baseline", "--breakdown"]
            out = subprocess.run(cmd, stdout=subprocess.PIPE, text=True)
            if out.returncode != 0:
                print("bench.py: the %s run failed with status %d" % (key, out.returncode), file=sys.stderr)
                sys.exit(out.returncode or 1)
            parts[key] = json.loads(out.stdout.strip().splitlines()[-1])
        p4 = parts["cfg4"]
        roofline = dict(p4["roofline"])
        roofline["blocks"] = {parts[k]["config"]["workload"]: {"mfma": {kk: vv for kk, vv in parts[k]["roofline"].items() if kk != "hbm"},
                                                              "hbm": parts[k]["roofline"].get("hbm", [])} for k in ("cfg2", "cfg3")}
        res = {"metric": "distill images/sec per block (teacher forward + student step) + all-block step time",
               "value": p4["value"], "unit": "images/s", "ms_per_step": p4["ms_per_step"], **common, "repeats": args.repeats,
               "config": {**p4["config"], "all_block_step": parts["cfg5"]["config"],
                          "blocks": {parts[k]["config"]["workload"]: parts[k]["config"] for k in ("cfg2", "cfg3")}},
               "roofline": roofline}
        if args.breakdown:
            res["breakdown"] = {parts[k]["config"]["workload"]: parts[k].get("breakdown") for k in ("cfg4", "cfg2", "cfg3")}
        base_names = ["cfg4", "cfg5", "cfg2", "cfg3"]
        primary = p4["config"]["workload"]
    elif args.workload in SINGLE:
        w = getattr(wl, SINGLE[args.workload])()
        r, roof = run_block(args, w)
        if roof is None:
            roof = {"per_kind": {}, "steps": 0}
        roofline = mfma_roofline(w, roof, region % roof["steps"])
        roofline["hbm"] = hbm_list(w, roof)
        res = {"metric": "distill images/sec per block (teacher forward + student step)", "value": r["images_per_s"],
               "unit": "images/s", "ms_per_step": r["ms_per_step"], **common, "repeats": args.repeats, "config": r,
               "roofline": roofline}
        if args.breakdown:
            res["breakdown"] = roof["per_kind"]
        base_names = [args.workload]
        primary = w.name
    else:
        r = run_all_blocks(args, args.workload)
        res = {"metric": ("distill images/sec, all 5 VGG16 blocks concurrently (teacher chain + 5 student steps)"
                          if args.workload != "vgg13" else
                          "distill images/sec, 13 per-convolution VGG16 tasks concurrently (teacher conv + two-DS-layer student step each)"),
               "value": r["images_per_s"], "unit": "images/s", "ms_per_step": r["ms_per_step"], **common,
               "repeats": args.repeats, "config": r,
               "roofline": {"bound": "mfma", "achieved": r["whole_schedule_TFLOPps"], "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": r["whole_schedule_frac_of_mfma_peak"], "traffic": None,
                            "note": "whole schedule: all convolution FLOPs / wall time (not a single kernel)"}}
        base_names = ["cfg5" if args.workload != "vgg13" else "vgg13"] if args.workload != "vgg16_imagenet" else []
        primary = r["workload"]
    if not args.no_cpu_baseline and base_names:
        per, cores = cpu_baselines(base_names)
        first = per[primary] if primary in per else next(iter(per.values()))
        res["cpu_baseline"] = {**first, **cores, "per_workload": per}
    print(json.dumps(res))


if __name__ == "__main__":
    main()
