#!/usr/bin/env python3
"""Benchmark of the per-block distillation step on one MI355X.

One "step" = one pass of the whole hot path over one synthetic batch: frozen teacher block forward + student
forward, local loss, backward and SGD-momentum update (pbkd_distill_step), inputs resident in HBM.  Default
workload: the CIFAR-shaped VGG16 block 2 at batch 128 (fp32).  Prints ONE JSON line with
  * value: whole-job throughput in images/s over K timed steps, the teacher on a second stream (--overlap 1);
  * roofline: the dominant kernel (the 3x3 implicit-GEMM convolution on the fp32 matrix cores) timed with HIP
    events around every one of its launches over K timed steps on ONE stream, where it has the GPU to itself
    (with --overlap 1 that is a second timed region; the first region's event figures are reported beside it);
  * cpu_baseline: the CPU oracle timed on the host cores on a bounded sample.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--overlap 0|1] [--workload cfg2|cfg3|cfg4|cfg5|vgg13] [--breakdown]
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

MFMA_F32_PEAK_TFLOPS = 157.3      # MI355X dense fp32 matrix peak
HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the 3x3 convolution kernel (reads + writes), from rocprofv3 --pmc FETCH_SIZE and
# WRITE_SIZE of this benchmark, scaled by what the same counters read for a device copy of known size
# (bench.py --calibrate-copy); the runs and the scale factors are in profiles/.  None: not measured.
CONV_TRAFFIC_BYTES = {"cfg2_cifar_vgg16_block2": 37445632}


def conv3x3_flops(arch):
    """2*MACs of the 3x3 full convolutions of a teacher block, and their number."""
    from paper_2012_03096_amd import workloads as wl
    total, count = 0, 0
    for (ci, hi, wi, co, ho, wo), L in zip(wl.layer_shapes(arch), arch.layers):
        if L.kind == wl.CONV3X3:
            total += 2 * 9 * ci * co * arch.n * ho * wo
            count += 1
    return total, count


def cpu_baseline(w, budget_s=12.0):
    """The CPU oracle as it stands, on the host cores: teacher forward + student steps of the same workload."""
    from oracle import block as ob
    x, tp, sp = w.tensors()
    ref = ob.RefBlock(w.teacher, tp, w.student, sp, momentum=w.momentum)
    t0 = time.perf_counter()
    steps = 0
    while True:
        t = ref.teacher_forward(x)
        ref.student_step(x, t, w.lr)
        steps += 1
        el = time.perf_counter() - t0
        if el > budget_s or steps >= 64:
            break
    return {"value": w.teacher.n * steps / el, "unit": "images/s", "cores": ob.num_threads(), "kind": "oracle",
            "sample": f"{steps} full step(s) (teacher forward + student step) of {w.name} at batch {w.teacher.n}, fp64, {el:.1f} s"}


def touch_first(torch, stream):
    """Makes `stream` submit a first (tiny) piece of work and waits for it."""
    with torch.cuda.stream(stream):
        torch.zeros(256, device="cuda").add_(1.0)
    torch.cuda.synchronize()


def run_single(args, w):
    import torch
    from paper_2012_03096_amd import binding as pb, workloads as wl
    x, tp, sp = w.tensors()
    # the teacher's stream submits work before the student's ever does: streams get their hardware queues in the
    # order of their first submission, and the overlap is better when the teacher's queue is the earlier one
    # (measured: 7 % on the ResNet block, nothing on the VGG block)
    tstream_own = torch.cuda.Stream() if args.overlap else None
    if tstream_own is not None:
        touch_first(torch, tstream_own)
    stream = torch.cuda.Stream()
    tstream = tstream_own if args.overlap else stream
    blk = pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum, stream=stream)
    xd = torch.from_numpy(x).cuda()
    td = torch.empty(wl.output_shape(w.teacher), dtype=torch.float32, device="cuda")
    torch.cuda.synchronize()
    conv_flops, n_conv = conv3x3_flops(w.teacher)
    # a student layer 0 may be a full conv too (ImageNet-shaped block): same kernel, its flops count as well
    s_flops, s_n = conv3x3_flops(w.student)
    per_step_flops = conv_flops + s_flops

    def timed_region(teacher_stream):
        """K steps of pbkd_distill_step (teacher forward + student step) between two device synchronisations, with
        HIP events around every launch of the 3x3 convolution kernel on the stream it runs on."""
        def step():
            blk.distill_step(xd, td, w.lr, want_loss=False, student_stream=stream, teacher_stream=teacher_stream)
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        blk.profile_enable(["conv3x3_mfma"], capacity=(n_conv + s_n + 1) * args.steps + 8)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        host_el = time.perf_counter() - t0
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
        ms_conv, launches = blk.profile_read().get("conv3x3_mfma", (0.0, 0))
        achieved = per_step_flops * args.steps / (ms_conv * 1e-3) / 1e12 if ms_conv > 0 else 0.0
        return {"el": el, "host_el": host_el, "achieved": achieved, "launches": launches,
                "avg_ms": ms_conv / max(launches, 1), "step": step}

    # region 1 gives `value`: with --overlap 1 the teacher runs on a second stream (the student's forward does not
    # need the label, and the next step's teacher convolutions run beside this step's backward pass)
    r1 = timed_region(tstream)
    el, host_el, step = r1["el"], r1["host_el"], r1["step"]
    loss = blk.last_loss()
    # the roofline is that of the kernel ALONE: when two streams share the GPU the event pair around a launch also
    # measures the time the kernel waits for, or shares, compute units with the other stream's kernels.  So with
    # --overlap 1 a second timed region runs the same K steps on one stream and the roofline is taken there.
    rr = timed_region(stream) if args.overlap else r1
    launches = rr["launches"]
    roof = {"bound": "mfma", "kernel": "pbkd::conv_mfma_kernel (3x3 implicit GEMM, v_mfma_f32_32x32x2_f32)",
            "achieved": round(rr["achieved"], 3), "peak": MFMA_F32_PEAK_TFLOPS, "unit": "TFLOP/s",
            "frac": round(rr["achieved"] / MFMA_F32_PEAK_TFLOPS, 4), "traffic": CONV_TRAFFIC_BYTES.get(w.name),
            "launches_per_step": launches // max(args.steps, 1), "avg_launch_ms": round(rr["avg_ms"], 5),
            "flops_per_launch": per_step_flops // max(launches // max(args.steps, 1), 1),
            "flops_per_step": per_step_flops,
            "region": ("second timed region: the same %d steps on ONE stream (kernel alone), %.4f ms/step"
                       % (args.steps, rr["el"] / args.steps * 1e3)) if args.overlap else "the timed region (one stream)"}
    if args.overlap:
        roof["in_value_region"] = {"achieved": round(r1["achieved"], 3), "frac": round(r1["achieved"] / MFMA_F32_PEAK_TFLOPS, 4),
                                   "avg_launch_ms": round(r1["avg_ms"], 5),
                                   "note": "two streams share the GPU: event time includes waiting for and sharing compute units"}
    # the student step alone (the teacher's target already in HBM), on one stream with timing off: the second
    # figure the per-block metric is quoted with
    blk.profile_enable(None, 0)
    k_student = max(args.steps // 2, 1)
    for _ in range(min(args.warmup, 10)):
        blk.student_step(xd, td, w.lr, want_loss=False, stream=stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(k_student):
        blk.student_step(xd, td, w.lr, want_loss=False, stream=stream)
    torch.cuda.synchronize()
    el_student = time.perf_counter() - t0
    breakdown = None
    if args.breakdown:
        blk.profile_enable(None, capacity=64 * 8)
        for _ in range(8):
            step()
        torch.cuda.synchronize()
        pr = blk.profile_read()
        breakdown = {k: {"ms_per_step": round(v[0] / 8, 5), "launches_per_step": v[1] / 8} for k, v in pr.items()}
    blk.profile_enable(None, 0)
    ms_per_step = el / args.steps * 1e3
    res = {"metric": "distill images/sec per block (teacher forward + student step)",
           "value": round(w.teacher.n * args.steps / el, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
           "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak",
           "vs_baseline": None, "dtype": "f32", "data": "synthetic",
           "config": {"workload": w.name, "batch": w.teacher.n, "input": [w.teacher.n, w.teacher.c, w.teacher.h, w.teacher.w],
                      "streams": 2 if args.overlap else 1,
                      "block_flops_per_step": blk.flops(3), "loss_after": loss,
                      "host_enqueue_ms_per_step": round(host_el / args.steps * 1e3, 4),
                      "student_step_alone": {"images_per_s": round(w.teacher.n * k_student / el_student, 1),
                                             "ms_per_step": round(el_student / k_student * 1e3, 4), "steps": k_student}},
           "roofline": roof}
    if breakdown:
        res["breakdown"] = breakdown
    blk.close()
    return res


def run_all_blocks(args):
    """cfg5: all five VGG16 blocks, one concurrent distillation step per 'step' (teacher chain once, students on
    streams).  vgg13: the paper's own granularity (section 3.3, 4.4): one task per 3x3 convolution, 13 tasks, the
    student two depthwise-separable layers; every task has its own synthetic input (no chain)."""
    import torch
    from paper_2012_03096_amd import binding as pb, workloads as wl
    chain = args.workload in ("cfg5", "vgg16_imagenet")
    if args.workload == "vgg16_imagenet":       # the five VGG16 stages at ImageNet size: 224x224 images, batch 32
        ws = wl.cfg5_vgg16_blocks(n=32, hw=224)
    else:
        ws = wl.cfg5_vgg16_blocks() if chain else wl.paper_granularity_vgg16_tasks()
    blocks, xs, ts = [], [], []
    for i, w in enumerate(ws):
        x, tp, sp = w.tensors()
        blocks.append(pb.Block(w.teacher, tp, w.student, sp, momentum=w.momentum))
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

    def step():
        pb.distill_step_all(blocks, xs, ts, 0.01, streams, sob, order, chain, tstream)

    steals = None
    if args.policy == 2:
        # work stealing: every task = one whole run of K steps of its block on its own copy of the input (with the
        # chained workload the inputs are the teacher prefix's activations, computed once here); all tasks start in
        # the queue the round-robin deal gives them
        step()
        torch.cuda.synchronize()
        xs = [x.clone() for x in xs]
        q0 = [i % n_streams for i in range(len(blocks))]
        pb.run_tasks_work_stealing(blocks, xs, ts, 0.01, [args.warmup] * len(blocks), streams, q0)
        t0 = time.perf_counter()
        sob, steals = pb.run_tasks_work_stealing(blocks, xs, ts, 0.01, [args.steps] * len(blocks), streams, q0)
        el = time.perf_counter() - t0
    else:
        for _ in range(args.warmup):
            step()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        el = time.perf_counter() - t0
    flops = sum(b.flops(3) for b in blocks)
    n = ws[0].teacher.n
    res = {"metric": ("distill images/sec, all 5 VGG16 blocks concurrently (teacher chain + 5 student steps)" if chain else
                      "distill images/sec, 13 per-convolution VGG16 tasks concurrently (teacher conv + two-DS-layer student step each)"),
           "value": round(n * args.steps / el, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
           "ms_per_step": round(el / args.steps * 1e3, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
           "dtype": "f32", "data": "synthetic",
           "config": {"workload": ("vgg16_imagenet_all_blocks" if args.workload == "vgg16_imagenet" else "cfg5_vgg16_all_blocks") if chain else "vgg16_13_conv_tasks", "batch": n, "streams": n_streams, "policy": ["wfd", "round_robin", "work_stealing"][args.policy], "steals": steals, "weights": "measured_us_per_5_steps" if weights else "flops", "stream_load": load,
                      "stream_of_block": sob, "flops_per_step": flops, "losses": [round(b.last_loss(), 6) for b in blocks]},
           "roofline": {"bound": "mfma", "achieved": round(flops * args.steps / el / 1e12, 3), "peak": MFMA_F32_PEAK_TFLOPS,
                        "unit": "TFLOP/s", "frac": round(flops * args.steps / el / 1e12 / MFMA_F32_PEAK_TFLOPS, 4), "traffic": None,
                        "note": "whole schedule: all convolution FLOPs / wall time (not a single kernel)"}}
    for b in blocks:
        b.close()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=30)
    ap.add_argument("--workload", default="cfg2", choices=["cfg1", "cfg2", "cfg3", "cfg4", "cfg5", "vgg13", "vgg16_imagenet"])
    ap.add_argument("--streams", type=int, default=3, help="cfg5 / vgg13: number of student streams")
    ap.add_argument("--overlap", type=int, default=1,
                    help="single block: 1 (default) = teacher on a second stream beside the student; 0 = everything on one stream")
    ap.add_argument("--policy", type=int, default=0, help="cfg5 / vgg13: 0 worst-fit-decreasing, 1 round robin, 2 work stealing (whole K-step runs as tasks)")
    ap.add_argument("--measured-weights", action="store_true",
                    help="cfg5 / vgg13: pack by each task's measured run time (the paper's weight) instead of its FLOP count")
    ap.add_argument("--breakdown", action="store_true", help="add a per-kernel time breakdown (extra untimed steps)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", type=int, default=0, metavar="MIB",
                    help="run 20 plain device-to-device copies of MIB mebibytes and exit (reference for HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (blocks are spread over HIP streams of one device); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
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
    if args.workload in ("cfg5", "vgg13", "vgg16_imagenet"):
        res = run_all_blocks(args)
        base_w = wl.cfg5_vgg16_blocks()[1]
    else:
        w = {"cfg1": wl.cfg1_tiny, "cfg2": wl.cfg2_vgg_block2, "cfg3": wl.cfg3_resnet_down, "cfg4": wl.cfg4_imagenet_vgg_block1}[args.workload]()
        res = run_single(args, w)
        base_w = w
    if not args.no_cpu_baseline:
        res["cpu_baseline"] = cpu_baseline(base_w)
    print(json.dumps(res))


if __name__ == "__main__":
    main()
