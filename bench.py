#!/usr/bin/env python3
"""Benchmark of the integer complex-Winograd F(4x4,3x3) convolution on one MI355X.

One "step" is one pass of the whole hot path (input transform, Winograd-domain
contraction on the int8 matrix cores, output transform) over one batch of the
ResNet-style 56x56x64 layer (N=8, C=K=64, lossless mode, channels-last), with
activations and the packed Winograd-domain filters already resident in HBM.
The filter transform is done once before timing, as the paper prescribes
(Section 4.3: off the inference path); its time is reported separately.

Prints ONE JSON line.  `value` is direct-equivalent int8 TOPS,
2*9*N*K*C*H*W / time.  `roofline` describes the kernel that takes the most
time; `cpu_baseline` is the CPU oracle timed on this machine's host cores.
"""
import argparse
import json
import os
import re
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

# Kernel arguments in device memory rather than in host memory: the waves' first scalar loads then
# stay on the GPU.  Launches replayed from a HIP graph (the timed path) are unaffected; launches
# made one by one (--eager) take 8.7 instead of 9.8 us per step on the default workload.  Has to be
# in the environment before the HIP runtime starts.
os.environ.setdefault("HIP_FORCE_DEV_KERNARG", "1")

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E
INT8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8

STAGES = ("input_transform", "contraction", "output_transform", "fused_conv")


def algorithmic_bytes(case, mode):
    """Algorithmic HBM bytes per launch of each kernel (the unavoidable traffic):
    input transform: 16 B read + 72 B written per (tile, channel) (36 planes of 12 bits as two int8 limbs);
    contraction: 72 B read per (tile, channel), the packed filters once, 144 B written per (tile, filter);
    output transform: 144 B read + 64 B written per (tile, filter);
    fused kernel: 16 B read per (tile, channel), the packed filters once, 64 B written per (tile, filter)."""
    T, C, K = case.tiles, case.C, case.K
    filt = (72 if mode == "lossless" else 36) * K * C
    return {
        "input_transform": (16 + 72) * T * C,
        "contraction": 72 * T * C + filt + 144 * T * K,
        "output_transform": (144 + 64) * T * K,
        "fused_conv": 16 * T * C + filt + 64 * T * K,
    }


def layout_bytes(case, mode):
    """Bytes per launch that the kernels' own data layout moves when nothing is cached (same padding-free
    counting): the staged pipeline stores 138 (lossless) or 72 (scaled) int8 operand planes per (tile, channel)
    and 46 or 36 int32 accumulator planes per (tile, filter); the fused kernel has no intermediate arrays."""
    T, C, K = case.tiles, case.C, case.K
    vp, mp, fp = (138, 46, 138) if mode == "lossless" else (72, 36, 46)
    return {
        "input_transform": (16 + vp) * T * C,
        "contraction": vp * T * C + fp * K * C + 4 * mp * T * K,
        "output_transform": (4 * mp + 64) * T * K,
        "fused_conv": 16 * T * C + fp * K * C + 64 * T * K,
    }


def contraction_int8_ops(case, mode):
    """int8 multiply-adds x2 the method needs on the matrix cores: 46 real products per tile and channel
    pair (Section 3.4), each three int8 limb products in lossless mode (138), 112 in scaled mode."""
    per_pair = 138 if mode == "lossless" else 112
    return 2 * per_pair * case.tiles * case.C * case.K


def capture_steps(torch, step, count):
    """`count` calls of step() recorded into one HIP graph on a side stream; None if capture is not possible."""
    try:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for _ in range(count):
                step()
        return graph
    except Exception as exc:   # fall back to eager launches, and say so
        print("bench.py: HIP graph capture failed (%s); timing eager launches" % exc, file=sys.stderr)
        torch.cuda.synchronize()
        return None


def kernel_sources_sha16():
    """Fingerprint of the HIP sources the library is built from (names and contents of csrc/*, in order)."""
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_1901_01965_amd", "csrc")
    for name in sorted(os.listdir(csrc)):
        if name.endswith((".hip", ".h")):
            h.update(name.encode())
            with open(os.path.join(csrc, name), "rb") as f:
                h.update(f.read())
    return h.hexdigest()[:16]


TRAFFIC_PROFILE = os.path.join("profiles", "hbm_traffic_cfg2.txt")


def read_profiled_traffic(kernel):
    """(bytes per launch or None, note): HBM traffic of `kernel` from the committed rocprofv3 counter summary.
    The summary is stamped with the fingerprint of the kernel sources it was measured on; if the sources have
    changed since, the figure is stale and None is reported instead."""
    path = os.path.join(ROOT, TRAFFIC_PROFILE)
    found, stamp = None, None
    try:
        with open(path) as f:
            for line in f:
                m = re.match(r"^traffic_bytes_per_launch\s+%s\s+(\d+)" % kernel, line)
                if m:
                    found = int(m.group(1))
                m = re.match(r"^kernel_sources_sha16\s+([0-9a-f]{16})", line)
                if m:
                    stamp = m.group(1)
    except OSError:
        return None, "no counter summary at %s" % TRAFFIC_PROFILE
    if found is None:
        return None, "%s has no line for %s" % (TRAFFIC_PROFILE, kernel)
    now = kernel_sources_sha16()
    if stamp != now:
        return None, "%s was measured on kernel sources %s, the library is built from %s: figure withheld" % (
            TRAFFIC_PROFILE, stamp, now)
    return found, "rocprofv3 FETCH_SIZE + WRITE_SIZE, calibrated, from %s (kernel sources %s)" % (TRAFFIC_PROFILE, stamp)


SETTLE_MS = 30.0   # untimed replays before the timed one: the device's clocks take some 10 ms of load to settle


def time_replay(torch, step, count, eager=False, settle_ms=SETTLE_MS):
    """Milliseconds per call of step(): `count` calls recorded into one HIP graph, replayed untimed until the device has
    been busy for `settle_ms` (measured: a 20-step replay of the 7.5 us layer right after start-up runs 6 % slower than
    the same replay 10 ms later), then once between two synchronisations: the timed region is exactly `count` calls
    (launched one by one when `eager` or when capture is not possible)."""
    graph = None if eager else capture_steps(torch, step, count)
    busy0 = time.perf_counter()
    while True:
        if graph is not None:
            graph.replay()
        else:
            for _ in range(count):
                step()
        torch.cuda.synchronize()
        if graph is None or (time.perf_counter() - busy0) * 1e3 >= settle_ms:   # eager (profiling) runs: one untimed pass
            break
    t0 = time.perf_counter()
    if graph is not None:
        graph.replay()
    else:
        for _ in range(count):
            step()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / count * 1e3, graph is not None


def time_stage(torch, wg, stage, iters, xd, packed, layout, y, ws):
    """Mean milliseconds per launch of one kernel of the path: `iters` untimed launches (settled clocks), then
    `iters` launches between two events recorded on the stream the launches go to (torch's current stream, the
    one the binding hands to the library)."""
    wg.enqueue_stage(xd, packed, stage, iters, layout, out=y, workspace=ws)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    wg.enqueue_stage(xd, packed, stage, iters, layout, out=y, workspace=ws)
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / iters


def run_stack(args):
    """--stack: the VGG-16-shaped stack (13 layers, batch 16, requantisation + ReLU after every layer, 2x2 max-pool
    after layers 2, 4, 7, 10, 13).  A step is one pass of the batch through all 13 layers, each layer one launch of
    the convolution with the int8 epilogue; filters are transformed once beforehand."""
    import numpy as np
    import torch
    import paper_1901_01965_amd as wg
    from paper_1901_01965_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    wg.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    mode = wg.LOSSLESS if args.mode == "lossless" else wg.SCALED
    batch = args.batch or wl.VGG16_BATCH
    x_np, gs = wl.make_vgg16(batch=batch)
    x0 = torch.from_numpy(wl.to_nhwc(x_np)).to(dev)
    gd = [torch.from_numpy(wl.to_krsc(g)).to(dev) for g in gs]
    packed = [wg.winograd_filter_transform(g, wg.NHWC, mode) for g in gd]
    acts, y32 = [x0], []
    for cin, cout, hw, pool in wl.VGG16_LAYERS:
        ho = hw // 2 if pool else hw
        acts.append(torch.empty((batch, ho, ho, cout), dtype=torch.int8, device=dev))
        y32.append(None)
    ops = sum(2 * 9 * batch * cout * cin * hw * hw for cin, cout, hw, _ in wl.VGG16_LAYERS)

    def layer(i):
        wg.winograd_conv2d_int8_requant(acts[i], packed[i], wl.VGG16_SHIFTS[i], True, wl.VGG16_LAYERS[i][3], wg.NHWC,
                                        out=acts[i + 1])

    def step():
        for i in range(13):
            layer(i)

    def timed(fn, count):
        for _ in range(max(1, args.warmup // 4)):
            fn()
        torch.cuda.synchronize()
        return time_replay(torch, fn, count, args.eager)

    steps = min(args.steps, 50)
    ms, graphed = timed(step, steps)
    layers = []
    for i, (cin, cout, hw, pool) in enumerate(wl.VGG16_LAYERS):
        lms, _ = timed(lambda i=i: layer(i), 20)
        lops = 2 * 9 * batch * cout * cin * hw * hw
        layers.append({"layer": "%d->%d @%d%s" % (cin, cout, hw, " +pool" if pool else ""), "ms": round(lms, 4),
                       "TOPS": round(lops / (lms * 1e-3) / 1e12, 1)})

    # the same stack as 13 int32 convolutions + 13 requantisation launches, and with the direct convolution
    outs32 = [torch.empty((batch, hw, hw, cout), dtype=torch.int32, device=dev) for _, cout, hw, _ in wl.VGG16_LAYERS]
    wss = [wg.make_workspace(batch, cin, hw, hw, cout, mode, dev) for cin, cout, hw, _ in wl.VGG16_LAYERS]

    def two_kernel_step():
        for i in range(13):
            wg.winograd_conv2d_int8(acts[i], packed[i], wg.NHWC, out=outs32[i], workspace=wss[i])
            wg.requant_relu_pool_int8(outs32[i], wl.VGG16_SHIFTS[i], True, wl.VGG16_LAYERS[i][3], wg.NHWC, out=acts[i + 1])

    def direct_step():
        for i in range(13):
            wg.direct_conv2d_int8(acts[i], gd[i], wg.NHWC, out=outs32[i])
            wg.requant_relu_pool_int8(outs32[i], wl.VGG16_SHIFTS[i], True, wl.VGG16_LAYERS[i][3], wg.NHWC, out=acts[i + 1])

    final = acts[13].clone()
    two_ms, _ = timed(two_kernel_step, 10)
    same = bool(torch.equal(final, acts[13]))
    direct_ms, _ = timed(direct_step, 10)
    same_direct = bool(torch.equal(final, acts[13])) if mode == wg.LOSSLESS else None
    print(json.dumps({
        "metric": "direct-equivalent int8 conv TOPS, VGG-16-shaped stack, 1 GPU", "value": round(ops / (ms * 1e-3) / 1e12, 2),
        "unit": "TOPS", "n_gpus": 1, "steps": steps, "warmup": args.warmup, "ms_per_step": round(ms, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": "cfg5: VGG-16-shaped stack of 13 3x3 convolutions, N=%d, NHWC, %s mode, int8 between layers "
                               "(power-of-two requantisation, ReLU, 2x2 max-pool after layers 2,4,7,10,13)" % (batch, args.mode)},
        "launch": ("hip graph of %d steps: untimed replays for %d ms, then one timed replay" % (steps, SETTLE_MS)
                   if graphed else "eager"),
        "layers": layers,
        "int32_conv_plus_requant_kernel_ms": round(two_ms, 4), "final_activations_equal": same,
        "direct_conv_plus_requant_kernel_ms": round(direct_ms, 4), "final_activations_equal_direct": same_direct,
        "nonzero_fraction_of_final_activations": round(float((final != 0).float().mean().item()), 3),
    }))


def run_f2x2(args):
    """--algorithm f2x2: the same layer through the rational F(2x2,3x3) integer path (one kernel per step)."""
    import torch
    import paper_1901_01965_amd as wg
    from paper_1901_01965_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    wg.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    case = wl.CASES[args.case]
    if args.batch is not None:
        import dataclasses
        case = dataclasses.replace(case, name="%s@N=%d" % (case.name, args.batch), N=args.batch)
    layout = wg.NHWC if args.layout == "nhwc" else wg.NCHW
    mode = wg.LOSSLESS if args.mode == "lossless" else wg.SCALED
    both = args.mode == "both-scaled"
    x_np, g_np = wl.make_case(case)
    xd = torch.from_numpy(wl.to_nhwc(x_np) if layout == wg.NHWC else x_np).to(dev)
    gd = torch.from_numpy(wl.to_krsc(g_np) if layout == wg.NHWC else g_np).to(dev)
    out_shape = (case.N, case.H, case.W, case.K) if layout == wg.NHWC else (case.N, case.K, case.H, case.W)
    y = torch.empty(out_shape, dtype=torch.int32, device=dev)
    packed = wg.f2x2_filter_transform(gd, layout, mode)

    def step():
        if both:
            wg.f2x2_conv2d_int8_act_scaled(xd, packed, layout, out=y)
        else:
            wg.f2x2_conv2d_int8(xd, packed, layout, out=y)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ms, graphed = time_replay(torch, step, args.steps, args.eager)
    yd = wg.direct_conv2d_int8(xd, gd, layout)
    tiles2 = case.N * ((case.H + 1) // 2) * ((case.W + 1) // 2)
    alg = 4 * tiles2 * case.C + (32 if mode == wg.LOSSLESS else 16) * case.K * case.C + 16 * tiles2 * case.K
    # int8 products per tile and channel pair: two limbs on both sides, on the activations only, on neither
    mfma_ops = 2 * (64 if mode == wg.LOSSLESS else 16 if both else 32) * tiles2 * case.C * case.K
    print(json.dumps({
        "metric": "direct-equivalent int8 conv TOPS, %s, 1 GPU, F(2x2,3x3)" % args.case,
        "value": round(case.direct_ops / (ms * 1e-3) / 1e12, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: 3x3 s1 p1 conv N=%d C=%d K=%d H=W=%d, %s, %s mode, rational F(2x2,3x3)" % (
            case.name, case.N, case.C, case.K, case.H, args.layout.upper(), args.mode)},
        "launch": ("hip graph of %d steps: untimed replays for %d ms, then one timed replay" % (args.steps, SETTLE_MS)
                   if graphed else "eager"),
        "roofline": {"kernel": "f2_conv", "bound": "hbm", "achieved": round(alg / (ms * 1e-3) / 1e9, 1), "peak": HBM_PEAK_GBS,
                     "unit": "GB/s", "frac": round(alg / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4), "traffic": None,
                     "algorithmic_bytes": alg, "kernel_ms": round(ms, 5)},
        "int8_mfma_TOPS": round(mfma_ops / (ms * 1e-3) / 1e12, 1),
        "mfma_frac": round(mfma_ops / (ms * 1e-3) / 1e12 / INT8_MFMA_PEAK_TOPS, 4),
        "gpu_lossless_equals_gpu_direct": bool(torch.equal(y, yd)) if mode == wg.LOSSLESS else None,
    }))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--case", default="cfg2", help="workload (default: the 56x56x64 layer the metric is quoted on)")
    ap.add_argument("--mode", default="lossless", choices=("lossless", "scaled", "both-scaled"),
                    help="both-scaled: filters and activations scaled (Section 4.1's closing remark), int32 output")
    ap.add_argument("--layout", default="nhwc", choices=("nhwc", "nchw"))
    ap.add_argument("--batch", type=int, default=None,
                    help="override the workload's batch size N (batch sweeps; the default is the quoted configuration)")
    ap.add_argument("--rotate", type=int, default=1,
                    help="cycle the timed steps over this many separate input/output buffer sets (a working set above "
                         "256 MB defeats the Infinity Cache; the default, 1, is the resident case)")
    ap.add_argument("--eager", action="store_true", help="launch the timed steps one by one instead of as one HIP graph")
    ap.add_argument("--no-rotated-figure", action="store_true",
                    help="skip the second timed run over a working set above 512 MB")
    ap.add_argument("--no-large-batch-figure", action="store_true",
                    help="skip the extra measurement of the default layer at N = 256 (both modes)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one 256 MiB device-to-device tensor copy, the known-size kernel that "
                         "rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled by")
    ap.add_argument("--algorithm", default="f4x4", choices=("f4x4", "f2x2"),
                    help="f4x4: the complex F(4x4,3x3) path (the headline); f2x2: the rational F(2x2,3x3) path")
    ap.add_argument("--lossless-variant", type=int, default=0, choices=(0, 1, 2),
                    help="lossless single-kernel form: 0 the library's choice, 1 limb-pair form wherever possible, 2 never")
    ap.add_argument("--scaled-variant", type=int, default=0, choices=(0, 1, 2),
                    help="role-specialised kernel: 0 the library's choice, 1 the form with eight product "
                         "waves wherever possible, 2 never")
    ap.add_argument("--stack", action="store_true",
                    help="time the VGG-16-shaped stack (cfg5) instead of one layer; prints its own JSON line")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build measures one GPU only (the path has no cross-GPU step); use --gpus 1")
    if args.mode == "both-scaled" and args.stack:
        sys.exit("bench.py: --mode both-scaled times one layer, not the stack")
    if args.lossless_variant:
        import paper_1901_01965_amd as wg_
        wg_.lossless_variant(args.lossless_variant)
    if args.scaled_variant:
        import paper_1901_01965_amd as wg_
        wg_.scaled_variant(args.scaled_variant)
    if args.stack:
        return run_stack(args)
    if args.algorithm == "f2x2":
        return run_f2x2(args)

    import numpy as np
    import torch
    import paper_1901_01965_amd as wg
    from paper_1901_01965_amd import workloads as wl

    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")
    wg.load_library()
    dev = torch.device("cuda:0")
    torch.cuda.set_device(dev)
    case = wl.CASES[args.case]
    if args.batch is not None:
        import dataclasses
        case = dataclasses.replace(case, name="%s@N=%d" % (case.name, args.batch), N=args.batch)
    layout = wg.NHWC if args.layout == "nhwc" else wg.NCHW
    mode = wg.LOSSLESS if args.mode == "lossless" else wg.SCALED
    both = args.mode == "both-scaled"   # the blob is the scaled one; the timed call scales the activations as well

    x_np, g_np = wl.make_case(case)
    xd = torch.from_numpy(wl.to_nhwc(x_np) if layout == wg.NHWC else x_np).to(dev)
    gd = torch.from_numpy(wl.to_krsc(g_np) if layout == wg.NHWC else g_np).to(dev)
    ws = wg.make_workspace(case.N, case.C, case.H, case.W, case.K, mode, dev)
    out_shape = (case.N, case.H, case.W, case.K) if layout == wg.NHWC else (case.N, case.K, case.H, case.W)
    y = torch.empty(out_shape, dtype=torch.int32, device=dev)

    # offline filter transform (timed on its own)
    packed = wg.winograd_filter_transform(gd, layout, mode)
    packed.check()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(10):
        wg.winograd_filter_transform(gd, layout, mode, blob=packed.blob)
    torch.cuda.synchronize()
    filter_ms = (time.perf_counter() - t0) / 10 * 1e3

    # rotation over several buffer sets (same contents) takes the caches out of the picture
    def make_sets(count):
        return [(xd, y)] + [(xd.clone(), torch.empty_like(y)) for _ in range(max(1, count) - 1)]

    def stepper(sets):
        turn = [0]

        def step():
            xi, yi = sets[turn[0] % len(sets)]
            turn[0] += 1
            if both:
                wg.winograd_conv2d_int8_act_scaled(xi, packed, layout, out=yi)
            else:
                wg.winograd_conv2d_int8(xi, packed, layout, out=yi, workspace=ws)
        return step

    sets = make_sets(args.rotate)
    step = stepper(sets)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    # The K timed steps are recorded into one HIP graph (the steps are a few microseconds each, so
    # an interpreter loop would be launch-bound) and replayed once inside the timed region.
    ms_per_step, graphed = time_replay(torch, step, args.steps, args.eager)
    tops = case.direct_ops / (ms_per_step * 1e-3) / 1e12

    # The same steps over enough separate buffer sets that the working set (inputs + outputs) is above 512 MB,
    # twice the Infinity Cache: every step then reads its activations from HBM and its output lines are new.
    rotated = None
    if args.rotate == 1 and not args.no_rotated_figure:
        per_set = xd.numel() + 4 * y.numel()
        count = min(512, -(-(520 << 20) // per_set))
        if count * per_set < (64 << 30):
            rsets = make_sets(count)
            rstep = stepper(rsets)
            for _ in range(count):
                rstep()
            torch.cuda.synchronize()
            rms, _ = time_replay(torch, rstep, max(args.steps, count), args.eager)
            rotated = {"buffer_sets": count, "working_set_MB": round(count * per_set / 2**20, 1), "ms_per_step": round(rms, 5),
                       "TOPS": round(case.direct_ops / (rms * 1e-3) / 1e12, 2)}
            del rsets, rstep

    # per-kernel durations: events on the launch stream around back-to-back launches of one kernel; the three
    # staged kernels run once in order first, so that each finds its input in the workspace
    wg.force_path(wg.STAGED)
    try:
        wg.winograd_conv2d_int8(xd, packed, layout, out=y, workspace=ws)
    finally:
        wg.force_path(wg.AUTO)
    iters = max(20, args.steps // 2)
    stage = {name: time_stage(torch, wg, i, iters, xd, packed, layout, y, ws) for i, name in enumerate(STAGES)}
    alg = algorithmic_bytes(case, args.mode)
    path = wg.conv2d_path(case.N, case.C, case.H, case.W, case.K, mode)
    used = ("fused_conv",) if path == wg.FUSED else STAGES[:3]
    dominant = max(used, key=lambda s: stage[s])
    achieved = alg[dominant] / (stage[dominant] * 1e-3) / 1e9
    default_workload = (args.case == "cfg2" and args.batch is None and args.mode == "lossless"
                        and args.layout == "nhwc")
    roofline = {
        "kernel": dominant, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
        "frac": round(achieved / HBM_PEAK_GBS, 4),
        "traffic": None, "algorithmic_bytes": alg[dominant], "kernel_ms": round(stage[dominant], 5),
    }
    # the committed counter summary covers the default workload only, and only the sources it was measured on
    if both:
        # the stage measurement above timed the filter-scaled kernels; the kernel this mode runs is the timed step itself
        roofline.update({"kernel": "fused_conv_act_scaled", "kernel_ms": round(ms_per_step, 5),
                         "achieved": round(alg["fused_conv"] / (ms_per_step * 1e-3) / 1e9, 1),
                         "frac": round(alg["fused_conv"] / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                         "algorithmic_bytes": alg["fused_conv"],
                         "traffic_source": "no counter summary for this workload; kernel_ms is the step time"})
    elif default_workload:
        roofline["traffic"], roofline["traffic_source"] = read_profiled_traffic(dominant)
    else:
        roofline["traffic_source"] = "no counter summary for this workload"
    kernels = {
        s: {"ms": round(stage[s], 5), "algorithmic_GBps": round(alg[s] / (stage[s] * 1e-3) / 1e9, 1),
            "hbm_frac": round(alg[s] / (stage[s] * 1e-3) / 1e9 / HBM_PEAK_GBS, 4)}
        for s in STAGES if stage[s] > 0
    }
    lay = layout_bytes(case, args.mode)
    for s in kernels:
        kernels[s]["on_timed_path"] = s in used
        kernels[s]["layout_GBps"] = round(lay[s] / (stage[s] * 1e-3) / 1e9, 1)
    for s in ("contraction", "fused_conv"):
        if s in kernels:
            mfma_tops = contraction_int8_ops(case, args.mode) / (stage[s] * 1e-3) / 1e12
            kernels[s]["int8_mfma_TOPS"] = round(mfma_tops, 1)
            kernels[s]["mfma_frac"] = round(mfma_tops / INT8_MFMA_PEAK_TOPS, 4)

    if args.calibration_copy:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # direct convolution on the same inputs, for context
    yd = torch.empty_like(y)

    def direct_step():
        wg.direct_conv2d_int8(xd, gd, layout, out=yd)

    for _ in range(3):
        direct_step()
    torch.cuda.synchronize()
    direct_ms, _ = time_replay(torch, direct_step, max(20, args.steps), args.eager)
    same_as_direct = bool(torch.equal(y, yd)) if mode == wg.LOSSLESS else None

    # the same convolution with requantisation and ReLU applied before the store (int8 output), for context
    shift = max(0, int(y.abs().max().item()).bit_length() - 7)
    y8 = torch.empty(out_shape, dtype=torch.int8, device=dev)

    def int8_step():
        wg.winograd_conv2d_int8_requant(xd, packed, shift, True, False, layout, out=y8)

    for _ in range(3):
        int8_step()
    torch.cuda.synchronize()
    int8_ms, _ = time_replay(torch, int8_step, args.steps, args.eager)
    int8_matches = bool(torch.equal(y8, wg.requant_relu_pool_int8(y, shift, True, False, layout)))

    result = {
        "metric": "direct-equivalent int8 conv TOPS, 56x56x64 layer, 1 GPU" if args.case == "cfg2"
                  else "direct-equivalent int8 conv TOPS, %s, 1 GPU" % args.case,
        "value": round(tops, 2), "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 5), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8", "data": "synthetic",
        "config": {"workload": "%s: 3x3 s1 p1 conv N=%d C=%d K=%d H=W=%d, %s, %s mode" % (
            case.name, case.N, case.C, case.K, case.H, args.layout.upper(), args.mode)},
        "path": "fused" if path == wg.FUSED else "staged",
        "launch": ("hip graph of %d steps: untimed replays for %d ms, then one timed replay" % (args.steps, SETTLE_MS)
                   if graphed else "eager"),
        "buffer_sets": len(sets),
        "rotated": rotated,
        "roofline": roofline,
        "kernels": kernels,
        "filter_transform_ms": round(filter_ms, 4),
        "direct_conv_ms": round(direct_ms, 4),
        "int8_epilogue": {"ms_per_step": round(int8_ms, 5), "TOPS": round(case.direct_ops / (int8_ms * 1e-3) / 1e12, 2),
                          "shift": shift, "relu": True, "pool": False,
                          "equals_int32_path_then_requantisation": int8_matches},
        "gpu_lossless_equals_gpu_direct": same_as_direct,
    }

    # The same layer at N = 256, both modes, for context: where the headline batch (196 workgroups, one round) is bound by
    # launch and per-workgroup latency, this shows what the kernels sustain once every compute unit has a dozen tile blocks.
    if default_workload and not args.no_large_batch_figure:
        import dataclasses
        big = dataclasses.replace(case, N=256)
        xb_np, _ = wl.make_case(big)
        xb = torch.from_numpy(wl.to_nhwc(xb_np)).to(dev)
        yb = torch.empty((big.N, big.H, big.W, big.K), dtype=torch.int32, device=dev)
        figure = {"workload": "N=256 C=%d K=%d H=W=%d, NHWC" % (big.C, big.K, big.H)}
        for name, m in (("lossless", wg.LOSSLESS), ("scaled", wg.SCALED)):
            pk = packed if m == mode else wg.winograd_filter_transform(gd, layout, m)
            wsb = wg.make_workspace(big.N, big.C, big.H, big.W, big.K, m)

            def big_step():
                wg.winograd_conv2d_int8(xb, pk, layout, out=yb, workspace=wsb)

            for _ in range(10):
                big_step()
            torch.cuda.synchronize()
            bms, _ = time_replay(torch, big_step, 100, args.eager)   # as `--batch 256 --steps 100` measures it
            figure[name] = {"ms_per_step": round(bms, 5), "TOPS": round(big.direct_ops / (bms * 1e-3) / 1e12, 2)}
        result["large_batch"] = figure
        del xb, yb

    if not args.no_cpu_baseline:
        import oracle
        omode = oracle.BOTH_SCALED if both else oracle.LOSSLESS if mode == wg.LOSSLESS else oracle.SCALED
        oracle.winograd_conv2d(x_np[:1], g_np, omode)           # build + page in
        runs, t_cpu = 0, 0.0
        want = None
        while t_cpu < args.cpu_seconds or runs < 2:
            t0 = time.perf_counter()
            want, _ = oracle.winograd_conv2d(x_np, g_np, omode)
            t_cpu += time.perf_counter() - t0
            runs += 1
        cpu_tops = case.direct_ops * runs / t_cpu / 1e12
        got = y.cpu().numpy()
        got = wl.from_nhwc(got) if layout == wg.NHWC else got
        result["gpu_equals_oracle"] = bool(np.array_equal(got, want))
        result["cpu_baseline"] = {
            "value": round(cpu_tops, 5), "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": "the whole %s batch through the oracle's Gaussian-integer Winograd path, %d runs, %.1f s"
                      % (case.name, runs, t_cpu),
        }
        # the same oracle on one thread (OpenMP's own switch; the oracle is not touched), a few runs
        import ctypes
        try:
            gomp = ctypes.CDLL("libgomp.so.1")
            threads = oracle.num_threads()
            gomp.omp_set_num_threads(1)
            try:
                runs1, t1 = 0, 0.0
                while t1 < min(3.0, args.cpu_seconds) or runs1 < 1:
                    t0 = time.perf_counter()
                    oracle.winograd_conv2d(x_np, g_np, omode)
                    t1 += time.perf_counter() - t0
                    runs1 += 1
            finally:
                gomp.omp_set_num_threads(threads)
            result["cpu_baseline_1thread"] = {
                "value": round(case.direct_ops * runs1 / t1 / 1e12, 5), "unit": "TOPS", "cores": 1, "kind": "oracle",
                "sample": "the same, %d runs, %.1f s" % (runs1, t1)}
        except OSError:
            result["cpu_baseline_1thread"] = None
    print(json.dumps(result))


if __name__ == "__main__":
    main()
