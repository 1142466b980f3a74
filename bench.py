#!/usr/bin/env python3
"""Benchmark of the int8 quantised-convolution path on one MI355X.

A step = one pass of the online hot path over one resident batch: Q on the fp32 input
image, every fused int8 convolution of the network (bias, ReLU, residual sum, requantise
in the epilogue), D on the output that leaves the int8 domain.  The offline steps (BN
fold, max-abs calibration, weight/bias quantisation) are run once before the timed
region and timed separately (reported under "offline").  Default workload: the full
ResNet-50 conv stack at batch 64 (config 3), the configuration the headline metric names.

Prints ONE JSON line on stdout; per-layer detail goes to stderr (and --layers-out).
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_INT8_TOPS = 5000.0     # MI355X dense int8 MFMA, POP/s -> TOP/s
PEAK_HBM_GBS = 8000.0
RIDGE = PEAK_INT8_TOPS * 1e12 / (PEAK_HBM_GBS * 1e9)

# What arxiv 1805.08691 itself reports (Tables 1 and 2 and the evaluation text): whole-network
# CPU figures on other hardware, printed beside this machine's numbers as context.  They are
# not the target of this build and enter no ratio above.
PAPER_CONTEXT = {
    "source": "arxiv 1805.08691, Tables 1-2 (inference throughput and latency) and evaluation text",
    "hardware": "AWS c5.18xlarge, one socket: 18 cores of an Intel Xeon Platinum 8124M, "
                "IntelCaffe with MKL-DNN, fake random input data",
    "throughput_images_per_s": {        # batch 64 / 64 / 32
        "resnet50": {"bvlc_caffe_fp32": 6.1, "intelcaffe_fp32": 158, "all_optimizations_int8": 462},
        "inception_v3": {"bvlc_caffe_fp32": 5.0, "intelcaffe_fp32": 126, "all_optimizations_int8": 282},
        "ssd_vgg16": {"bvlc_caffe_fp32": None, "intelcaffe_fp32": 31, "all_optimizations_int8": 43}},
    "latency_ms_batch1": {
        "resnet50": {"bvlc_caffe_fp32": 131.8, "intelcaffe_fp32": 10.7, "all_optimizations_int8": 3.5},
        "inception_v3": {"bvlc_caffe_fp32": 158.96, "intelcaffe_fp32": 14.3, "all_optimizations_int8": 5.9},
        "ssd_vgg16": {"bvlc_caffe_fp32": None, "intelcaffe_fp32": 33.7, "all_optimizations_int8": 24.8}},
    "speedups_quoted": {"throughput_over_intelcaffe_fp32": "1.38X-2.9X",
                        "latency_over_intelcaffe_fp32": "1.35X-3X",
                        "throughput_over_bvlc_caffe": "56X-75X", "latency_over_bvlc_caffe": "26X-37X"},
    "note": "context only: another machine, whole networks including the non-convolution layers",
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def conv_work(net, op, N):
    """Algorithmic int8 ops and HBM bytes of one conv launch (true C and K, no padding)."""
    s, d = net.tensors[op.src], net.tensors[op.dst]
    npix = N * d.H * d.W
    ops = 2 * npix * op.K * op.C * op.R * op.S
    if op.R == 1 and op.S == 1 and op.stride > 1:
        in_bytes = npix * op.C                     # only the pixels a strided 1x1 touches
    else:
        in_bytes = N * s.H * s.W * op.C
    byts = in_bytes + npix * op.K + op.K * op.R * op.S * op.C + 4 * op.K
    if op.res:
        byts += npix * op.K
    return ops, byts


def measured_traffic(kernel, net_name, batch):
    """HBM bytes per launch of ``kernel`` from the committed counter summary (rocprofv3 --pmc
    FETCH_SIZE and WRITE_SIZE, scaled by a plain copy), or None when no summary covers it."""
    path = os.path.join(ROOT, "profiles", f"conv_i8_{net_name}_b{batch}_hbm_traffic.txt")
    try:
        for line in open(path):
            f = line.split("|")
            if len(f) >= 3 and f[0].strip() == "traffic_bytes_per_launch" and f[1].strip() == kernel:
                return int(f[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--config", type=int, default=3, help="workload: 1..5 (BASELINE configs)")
    ap.add_argument("--batch", type=int, default=0, help="override the config's batch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-cold", action="store_true",
                    help="skip the per-layer timing with caches flushed before every layer")
    ap.add_argument("--no-graph", action="store_true", help="launch eagerly instead of a HIP graph")
    ap.add_argument("--fuse-dequant", action="store_true",
                    help="Eq. D on the output inside the last layer's launches instead of a pass "
                         "of its own (same values; measured slower on ResNet-50: the layer then "
                         "takes the general epilogue and writes five times the bytes)")
    ap.add_argument("--no-fuse-head", action="store_true",
                    help="quantise the input, run the first layer and its max-pool as three "
                         "launches instead of one")
    ap.add_argument("--streams", type=int, default=2, choices=(1, 2, 3, 4),
                    help="number of concurrent part-batch pipelines the layers run as (2: two "
                         "half-batch pipelines, the default and the headline configuration)")
    ap.add_argument("--layers-out", default="", help="write the per-layer table (JSON) here")
    ap.add_argument("--sparsity-removal", action="store_true",
                    help="config 3 only: run the graph after the paper's sparsity-removal "
                         "transformation (reported as its own workload, not the headline)")
    ap.add_argument("--unsigned-activations", action="store_true",
                    help="unsigned p = 8 codes on the outputs of ReLU layers (the paper's "
                         "precision for non-negative tensors); reported as its own workload")
    ap.add_argument("--per-channel-weights", action="store_true",
                    help="one weight factor per output channel instead of one per tensor; "
                         "reported as its own workload")
    ap.add_argument("--fuse-pairs", action="store_true",
                    help="a convolution and the 1x1 layer that alone reads it run as one launch")
    ap.add_argument("--fuse-duals", action="store_true",
                    help="two independent convolutions on the same input run as one launch")
    ap.add_argument("--own-sum-factor", action="store_true",
                    help="a fused sum's output factor from its own max-abs instead of the "
                         "max(q1, q2) rule; reported as its own workload")
    ap.add_argument("--real-output", action="store_true",
                    help="the output convolution writes fp32 itself (no int8 code, no separate "
                         "dequantise pass); reported as its own workload")
    ap.add_argument("--pmc-probe", action="store_true",
                    help="one eager pass plus one plain 256 MiB device copy, then exit: the "
                         "program to run under rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE (the copy "
                         "gives the counters' scale)")
    ap.add_argument("--probe-layers", default="",
                    help="with --pmc-probe: comma-separated convolution names; each runs five "
                         "times alone on the first part-batch, after the pass and before the "
                         "copy (the dispatches a counter run picks up for one layer)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (batch data-parallel sharding is a "
              "design note, not code); run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_1805_08691_amd import binding as B, workloads as wl
    from paper_1805_08691_amd.engine import Engine

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(3)
    torch.cuda.set_device(0)
    cfg = wl.CONFIGS[args.config]
    net = cfg["make"]()
    if args.sparsity_removal:
        assert args.config == 3, "--sparsity-removal applies to config 3"
        net = wl.resnet50(sparsity_removal=True)       # same filters (seeded by config 3)
    N = args.batch or cfg["batch"]
    convs = net.convs()
    log(f"workload: {net.name} batch {N}: {len(convs)} convs, "
        f"{net.macs_per_image() / 1e9:.3f} GMAC/image")

    # ---------------- offline: parameters, fold, calibrate, quantise weights ---------------
    params = {op.name: wl.conv_params(args.config, i, op) for i, op in enumerate(convs)}
    eng = Engine(net, N, n_streams=args.streams, unsigned_activations=args.unsigned_activations,
                 per_channel_weights=args.per_channel_weights, real_outputs=args.real_output,
                 own_sum_factor=args.own_sum_factor, fuse_pairs=args.fuse_pairs,
                 fuse_duals=args.fuse_duals,
                 fuse_head=not (args.no_fuse_head or args.unsigned_activations
                                or args.per_channel_weights),
                 fuse_dequant=args.fuse_dequant)
    eng.load_params(params)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.fold()
    torch.cuda.synchronize()
    t_fold = time.perf_counter() - t0
    if args.config >= 3:
        calib = [torch.from_numpy(wl.input_batch(args.config, net, 8, 100 + i)).cuda()
                 for i in range(8)]                       # 8 seeded batches of 8 images
    else:
        calib = [torch.from_numpy(wl.input_batch(args.config, net, N, 0,
                                                 relu=cfg["relu_input"])).cuda()]
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    eng.calibrate(calib)
    torch.cuda.synchronize()
    t_cal = time.perf_counter() - t0
    t0 = time.perf_counter()
    eng.quantize_weights()
    torch.cuda.synchronize()
    t_qw = time.perf_counter() - t0
    del calib
    eng.allocate()

    x = torch.from_numpy(wl.input_batch(args.config, net, N, 0, relu=cfg["relu_input"])).cuda()
    out_name = net.outputs[0]
    out_f32 = torch.empty(eng.act[out_name].shape, dtype=torch.float32, device="cuda")

    if args.real_output:
        assert out_name in eng.real, "this network's output is not written whole by a convolution"

    # what leaves the int8 domain in a step (nothing when the last convolution writes fp32)
    dequant = {} if args.real_output else {out_name: out_f32}

    def step():
        eng.run_step(x, dequant)

    step()
    torch.cuda.synchronize()
    if args.pmc_probe:
        src = torch.ones(256 << 20, dtype=torch.int8, device="cuda")
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        step()
        # the calibration reduction over a 205 MB tensor (conv1's real-valued output at batch 64)
        big = torch.randn(64 * 112 * 112 * 64, dtype=torch.float32, device="cuda")
        slot = torch.zeros(1, dtype=torch.float32, device="cuda")
        torch.cuda.synchronize()
        B.calibrate_maxabs(big, slot)
        by_name = {o.name: o for o in convs}
        for name in filter(None, args.probe_layers.split(",")):
            lo, n = eng.parts[0]
            for _ in range(5):
                eng.run_conv(by_name[name], lo, n, fuse=False)
        torch.cuda.synchronize()
        dst.copy_(src)                      # 256 MiB read + 256 MiB written
        torch.cuda.synchronize()
        log("pmc probe pass done")
        return
    graph = None
    if not args.no_graph:
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            step()
    run = graph.replay if graph is not None else step

    # ---------------- timed region ---------------------------------------------------------
    for _ in range(args.warmup):
        run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        run()
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0
    ms_per_step = elapsed / args.steps * 1e3
    images_per_s = N * args.steps / elapsed

    # the same launches on ONE stream (the half-batch pipelines one after the other): the
    # total the per-launch intervals below must add up to
    serial_us = ms_per_step * 1e3
    if graph is not None and eng.n_streams > 1:
        g1 = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g1):
            eng.run_step(x, dequant, serial=True)
        for _ in range(3):
            g1.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            g1.replay()
        torch.cuda.synchronize()
        serial_us = (time.perf_counter() - t0) / 20 * 1e6

    # ---------------- per-launch durations with HIP events on the launch stream ------------
    # The host enqueues a whole chained pass behind a spin kernel so the GPU runs the
    # layers back to back; events between launches give each kernel's duration.
    ops_list = [o for o in net.ops]
    fused_deq = {k: v for k, v in dequant.items() if eng._dequant_writer(k)}
    reps = 7
    # an event record costs GPU time of its own: measure the interval between back-to-back
    # records on the busy stream and take it off every interval below
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(33)]
    torch.cuda._sleep(20_000_000)
    for e in evs:
        e.record()
    torch.cuda.synchronize()
    ev_cost = float(np.median([evs[i].elapsed_time(evs[i + 1]) * 1e3 for i in range(32)]))
    dur = np.zeros((reps, len(ops_list) + 2))
    for r in range(reps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(len(ops_list) + 3)]
        torch.cuda._sleep(20_000_000)
        ev[0].record()
        eng.set_input(x)                  # Eq. Q now, or inside the first layer's launches
        eng._deq = dict(fused_deq)        # Eq. D inside the last layer's launches, or below
        ev[1].record()
        for i, op in enumerate(ops_list):
            # the launches of one layer (one per half-batch when split) back to back on
            # this stream; the interval is divided by their number below
            for lo, n in (eng.parts if i >= eng.n_unsplit else [(0, N)]):
                eng.run_ops([op], lo, n)
            ev[i + 2].record()
        for name, buf in dequant.items():
            if name not in fused_deq:
                eng.dequantize(name, out=buf)
        ev[-1].record()
        eng._x, eng._deq = None, {}
        torch.cuda.synchronize()
        for i in range(len(ops_list) + 2):
            dur[r, i] = ev[i].elapsed_time(ev[i + 1]) * 1e3      # us
    raw = np.median(dur, axis=0)
    # between busy kernels a record costs less than between empty ones: take off the amount
    # that makes the intervals add up to the timed step (never more than the measured cost)
    ev_take = float(np.clip((raw.sum() - serial_us) / len(raw), 0.0, ev_cost))
    med = np.maximum(raw - ev_take, 0.0)
    log(f"event record cost {ev_cost:.2f} us between empty intervals; {ev_take:.2f} us taken off "
        f"each launch interval: sum {med.sum():.1f} us vs one-stream step {serial_us:.1f} us "
        f"(timed step, {eng.n_streams} stream(s): {ms_per_step * 1e3:.1f} us)")

    # ---------------- the same launches cold: caches flushed before every layer -------------
    # A 1 GiB device copy (four times the 256 MB last-level cache) runs before each layer's
    # launches, so activations, residual and filters come from HBM.
    cold = np.zeros(len(ops_list))
    if not args.no_cold:
        flush_src = torch.ones(512 << 20, dtype=torch.int8, device="cuda")
        flush_dst = torch.empty_like(flush_src)
        cold_reps = 5
        cdur = np.zeros((cold_reps, len(ops_list)))
        for r in range(cold_reps):
            eng._x = x if eng.head else None
            eng._deq = dict(fused_deq)
            e0 = [torch.cuda.Event(enable_timing=True) for _ in ops_list]
            e1 = [torch.cuda.Event(enable_timing=True) for _ in ops_list]
            for i, op in enumerate(ops_list):
                flush_dst.copy_(flush_src)
                e0[i].record()
                for lo, n in (eng.parts if i >= eng.n_unsplit else [(0, N)]):
                    eng.run_ops([op], lo, n)
                e1[i].record()
            eng._x, eng._deq = None, {}
            torch.cuda.synchronize()
            for i in range(len(ops_list)):
                cdur[r, i] = e0[i].elapsed_time(e1[i]) * 1e3
        cold = np.maximum(np.median(cdur, axis=0) - ev_take, 0.0)
        del flush_src, flush_dst

    # ---------------- measured ceilings: a plain device copy, a register-resident MFMA loop --
    def timed_us(fn, reps=20):
        fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / reps
    cp_src = torch.ones(1 << 30, dtype=torch.int8, device="cuda")
    cp_dst = torch.empty_like(cp_src)
    t_copy = timed_us(lambda: cp_dst.copy_(cp_src), reps=10)
    del cp_src, cp_dst
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    n_cu = torch.cuda.get_device_properties(0).multi_processor_count
    probe_ops = [0]
    def mfma_probe():
        probe_ops[0] = B.probe_mfma_i8(2 * n_cu, 20000, sink)
    t_mfma = timed_us(mfma_probe, reps=3)
    ceilings = {"device_copy_gbs": round(2 * (1 << 30) / t_copy / 1e3, 1),
                "mfma_int8_loop_tops": round(probe_ops[0] / t_mfma / 1e6, 1),
                "compute_units": n_cu}
    log(f"measured ceilings: 1 GiB device copy {ceilings['device_copy_gbs']:.0f} GB/s (read + write), "
        f"register-resident int8 MFMA loop {ceilings['mfma_int8_loop_tops']:.0f} TOP/s on {n_cu} CUs")

    # ---------------- HBM-bound passes: max-abs (calibration), quantise, dequantise ---------
    big = torch.randn(64 * 112 * 112 * 64, dtype=torch.float32, device="cuda")   # 205 MB
    slot = torch.zeros(1, dtype=torch.float32, device="cuda")
    t_maxabs = timed_us(lambda: B.calibrate_maxabs(big, slot))
    del big
    n_in = x.numel()
    n_out = out_f32.numel()
    # with the fused head Eq. Q on the input is not a launch of the step: timed on its own
    t_qin = timed_us(lambda: eng.quantize_input(x)) if eng.head else float(med[0])
    passes = {
        "maxabs": dict(bytes=4 * 64 * 112 * 112 * 64, us=round(t_maxabs, 2)),
        "quantize_input": dict(bytes=5 * n_in + n_in // 3, us=round(t_qin, 2),
                               in_step=not eng.head),
        "dequantize_output": dict(bytes=5 * n_out, in_step=not fused_deq,
                                  us=round(timed_us(lambda: eng.dequantize(out_name, out=out_f32))
                                           if fused_deq else float(med[-1]), 2)),
    }
    if args.real_output:
        del passes["dequantize_output"]
    for k, v in passes.items():
        v["gbs"] = round(v["bytes"] / v["us"] / 1e3, 1)
        v["frac_of_hbm_peak"] = round(v["gbs"] / PEAK_HBM_GBS, 3)
        log(f"pass {k}: {v['bytes'] / 1e6:.1f} MB in {v['us']:.2f} us = {v['gbs']:.0f} GB/s "
            f"({100 * v['frac_of_hbm_peak']:.0f}% of HBM peak)")

    layers = []
    by_variant = {}
    tot_ops = tot_us = tot_bytes = tot_cold = 0.0
    roof_us = 0.0
    helpers = []          # the pooling launches between convolutions (not the paper's method)
    for i, op in enumerate(ops_list):
        if eng.head and op is eng.head[1]:
            continue                      # ran inside the first layer's launch
        if op.kind != "conv":
            n_launch = len(eng.parts) if i >= eng.n_unsplit else 1
            s_t, d_t = net.tensors[op.src], net.tensors[op.dst]
            byts = N * (s_t.H * s_t.W * s_t.C + d_t.H * d_t.W * s_t.C) / n_launch
            us = float(med[i + 1]) / n_launch
            helpers.append(dict(name=op.name, mode=op.mode, H=s_t.H, C=s_t.C, R=op.R, stride=op.stride,
                                us=round(us, 2), gbs=round(byts / us / 1e3, 1), launches=n_launch))
            continue
        if op.name in eng.paired or op.name in eng.dualed:
            continue                      # counted with the layer in front of it
        n_launch = len(eng.parts) if i >= eng.n_unsplit else 1
        n_img = eng.parts[0][1] if i >= eng.n_unsplit else N
        ops, byts = conv_work(net, op, N)
        if op.name in eng.duals:          # one launch for two layers on the same input
            ops2, byts2 = conv_work(net, eng.duals[op.name], N)
            s_t = net.tensors[op.src]
            ops, byts = ops + ops2, byts + byts2
        if op.name in eng.pairs:          # one launch for two layers: the tensor between
            ops2, byts2 = conv_work(net, eng.pairs[op.name], N)     # them is not moved
            mid = net.tensors[op.dst]
            ops, byts = ops + ops2, byts + byts2 - 2 * N * mid.H * mid.W * mid.C
        fused_head = bool(eng.head and op is eng.head[0])
        if fused_head:                    # reads the fp32 image, writes the pooled tensor
            t_img = net.tensors[net.input]
            out_t = net.tensors[eng.head[1].dst] if eng.head[1] else net.tensors[op.dst]
            byts = (4 * N * t_img.H * t_img.W * t_img.C + N * out_t.H * out_t.W * op.K
                    + op.K * op.R * op.S * op.C + 4 * op.K)
        if op.dst in fused_deq:           # also writes the fp32 values of its codes
            byts += 4 * N * net.tensors[op.dst].H * net.tensors[op.dst].W * op.K
        ops, byts = ops / n_launch, byts / n_launch          # per launch
        us = float(med[i + 1]) / n_launch
        us_cold = float(cold[i]) / n_launch
        variant = B.conv_variant(eng.conv_desc(op, n_img)) + ("+pair" if op.name in eng.pairs else "")
        if fused_head:
            variant += "<Q" + (",pool>" if eng.head[1] else ">")
        if op.dst in fused_deq:
            variant += "+D"
        bound = "mfma" if ops / byts > RIDGE else "hbm"
        t_roof = max(ops / (PEAK_INT8_TOPS * 1e12), byts / (PEAK_HBM_GBS * 1e9)) * 1e6
        layers.append(dict(name=op.name, C=op.C, K=op.K, R=op.R, S=op.S, stride=op.stride,
                           H=net.tensors[op.src].H, variant=variant, us=round(us, 2),
                           cold_us=round(us_cold, 2),
                           tops=round(ops / us / 1e6, 1), gbs=round(byts / us / 1e3, 1),
                           bound=bound, roof_us=round(t_roof, 2), frac=round(t_roof / us, 3)))
        v = by_variant.setdefault(variant, dict(ops=0.0, us=0.0, bytes=0.0, launches=0))
        v["ops"] += ops * n_launch; v["us"] += us * n_launch; v["bytes"] += byts * n_launch
        v["launches"] += n_launch
        tot_ops += ops * n_launch; tot_us += us * n_launch; tot_bytes += byts * n_launch
        roof_us += t_roof * n_launch
        tot_cold += us_cold * n_launch
    for Hh in helpers:
        log("{name:22s} {mode}-pool {R}x{R}/{stride} H={H:<3d} C={C:<4d} {us:8.2f} us {gbs:7.1f} GB/s x{launches}"
            .format(**Hh))
    for L in layers:
        log("{name:22s} C={C:<4d} K={K:<4d} {R}x{S}/{stride} H={H:<3d} {variant:30s} {us:8.2f} us "
            "(cold {cold_us:7.2f}) {tops:7.1f} TOP/s {gbs:7.1f} GB/s  {bound:4s} roof {roof_us:6.2f} us frac {frac:.3f}"
            .format(**L))
    dom_name, dom = max(by_variant.items(), key=lambda kv: kv[1]["us"])
    for k, v in by_variant.items():
        log(f"variant {k}: {v['launches']} launches, avg {v['us'] / v['launches']:.2f} us, "
            f"{v['ops'] / v['us'] / 1e6:.1f} TOP/s")
    agg_tops = tot_ops / tot_us / 1e6
    log(f"conv kernels: sum {tot_us:.1f} us per pass, {agg_tops:.1f} TOP/s aggregate "
        f"({100 * agg_tops / PEAK_INT8_TOPS:.1f}% of int8 MFMA peak), "
        f"roofline sum {roof_us:.1f} us; quantize {med[0]:.1f} us; dequantize {med[-1]:.1f} us; "
        f"graph step {ms_per_step * 1e3:.1f} us")

    # the kernel with the largest share of the step; its launches together decide which
    # roofline bounds it (algorithmic ops / algorithmic bytes against the ridge)
    dom_tops = dom["ops"] / dom["us"] / 1e6
    dom_gbs = dom["bytes"] / dom["us"] / 1e3
    traffic = measured_traffic(dom_name, net.name, N)
    if dom["ops"] / dom["bytes"] > RIDGE:
        roofline = dict(bound="mfma", achieved=round(dom_tops, 2), peak=PEAK_INT8_TOPS,
                        unit="TOP/s", frac=round(dom_tops / PEAK_INT8_TOPS, 4))
    else:
        roofline = dict(bound="hbm", achieved=round(dom_gbs, 1), peak=PEAK_HBM_GBS, unit="GB/s",
                        frac=round(dom_gbs / PEAK_HBM_GBS, 4))
    roofline.update(traffic=traffic, kernel=dom_name, launches_per_step=dom["launches"],
                    avg_launch_us=round(dom["us"] / dom["launches"], 3),
                    algorithmic_bytes_per_launch=round(dom["bytes"] / dom["launches"]),
                    algorithmic_ops_per_launch=round(dom["ops"] / dom["launches"]),
                    tops=round(dom_tops, 2), pct_of_mfma_int8_peak=round(100 * dom_tops / PEAK_INT8_TOPS, 2),
                    hbm_gbs=round(dom_gbs, 1))

    # the same figures for every kernel variant of the step, largest share first
    def variant_roofline(name, v):
        tops, gbs = v["ops"] / v["us"] / 1e6, v["bytes"] / v["us"] / 1e3
        mfma = v["ops"] / v["bytes"] > RIDGE
        return dict(kernel=name, launches_per_step=v["launches"],
                    avg_launch_us=round(v["us"] / v["launches"], 3),
                    share_of_conv_time=round(v["us"] / tot_us, 3), bound="mfma" if mfma else "hbm",
                    achieved=round(tops, 2) if mfma else round(gbs, 1),
                    peak=PEAK_INT8_TOPS if mfma else PEAK_HBM_GBS, unit="TOP/s" if mfma else "GB/s",
                    frac=round(tops / PEAK_INT8_TOPS if mfma else gbs / PEAK_HBM_GBS, 4),
                    traffic=measured_traffic(name, net.name, N))
    kernels = [variant_roofline(k, v)
               for k, v in sorted(by_variant.items(), key=lambda kv: -kv[1]["us"])]

    # ---------------- the oracle on the host cores, bounded sample --------------------------
    cpu = None
    if not args.no_cpu_baseline:
        import oracle as orc
        from oracle import net as onet
        sample = {1: 1, 2: 32, 3: 64, 4: 32, 5: 4}[args.config]
        sample = min(sample, N)
        xs = x[:sample].cpu().numpy()
        folded = onet.fold_all(net, params)
        q = {k: np.float32(v) for k, v in eng.q.items()}
        qparams = onet.quantize_params(net, folded, q, per_channel=args.per_channel_weights)
        U = onet.unsigned_tensors(net) if args.unsigned_activations else set()
        t0 = time.perf_counter()
        z_in = orc.Q(xs, q[net.input], 7)
        acts = onet.forward_i8(net, qparams, q, z_in, unsigned=U)
        (orc.D_u8 if out_name in U else orc.D)(acts[out_name], q[out_name])
        t_cpu = time.perf_counter() - t0
        # the tensor compared: the output's codes, or (fp32 output) the codes its conv reads
        cmp_name = out_name
        if args.real_output:
            cmp_name = next(o.src for o in convs if o.dst == out_name)
        gpu_out = eng.act[cmp_name][:sample].cpu().numpy()
        if cmp_name in U:
            gpu_out = (gpu_out.astype(np.int16) + 128).astype(np.uint8)
        same = bool(np.array_equal(acts[cmp_name], gpu_out))
        log(f"oracle: {sample} image(s) in {t_cpu:.2f} s on {orc.num_threads()} threads; "
            f"output equals the GPU's: {same}")
        cpu = dict(value=round(sample / t_cpu, 3), unit="images/s", cores=orc.num_threads(),
                   kind="oracle", sample=f"{sample} image(s) of the same batch, whole conv stack",
                   matches_gpu=same)

    result = {
        "metric": "ResNet-50 int8 images/sec at batch 64"
                  if args.config == 3 and N == 64 and not (args.sparsity_removal or args.unsigned_activations
                                               or args.per_channel_weights or args.real_output
                                               or args.own_sum_factor)
                  else f"{net.name}{' (unsigned activations)' if args.unsigned_activations else ''}"
                       f"{' (per-channel weights)' if args.per_channel_weights else ''}"
                       f"{' (fp32 output from the last conv)' if args.real_output else ''}"
                       f"{' (sums at their own factor)' if args.own_sum_factor else ''} "
                       f"int8 images/sec at batch {N}",
        "value": round(images_per_s, 1), "unit": "images/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "int8", "data": "synthetic",
        "config": {"workload": f"{net.name} conv stack, batch {N}, NHWC int8, "
                               f"{len(convs)} fused convs"
                               + (", unsigned p=8 ReLU outputs" if args.unsigned_activations else "")
                               + (", per-channel weight factors" if args.per_channel_weights else "")
                               + (f", {len(eng.pairs)} fused layer pairs" if eng.pairs else "")
                               + (", fp32 output written by the last conv" if args.real_output else ""),
                   "batch": N,
                   "launch": "eager" if graph is None else "hip_graph",
                   "streams": eng.n_streams},
        # every convolution's algorithmic ops over the timed step (which also holds the
        # quantise, pooling and dequantise launches), and over the convolutions' own
        # back-to-back launch durations on one stream
        "int8_conv_tops": round(tot_ops / (ms_per_step * 1e-3) / 1e12, 1),
        "pct_of_mfma_int8_peak": round(100 * tot_ops / (ms_per_step * 1e-3) / 1e12 / PEAK_INT8_TOPS, 2),
        "int8_conv_tops_one_stream": round(agg_tops, 1),
        "hbm_passes": passes,
        "conv_kernel_us_per_step": round(tot_us, 1),
        "helper_kernel_us_per_step": round(sum(h["us"] * h["launches"] for h in helpers), 1),
        "conv_kernel_us_per_step_cold": round(tot_cold, 1) if not args.no_cold else None,
        "measured_ceilings": ceilings,
        "one_stream_step_us": round(serial_us, 1),
        "conv_roofline_us_per_step": round(roof_us, 1),
        "roofline": roofline,
        "kernels": kernels,
        "cpu_baseline": cpu,
        "paper_context": PAPER_CONTEXT,
        "offline": {"fold_bn_ms": round(t_fold * 1e3, 2), "calibrate_ms": round(t_cal * 1e3, 2),
                    "quantize_weights_ms": round(t_qw * 1e3, 2)},
    }
    if args.layers_out:
        with open(args.layers_out, "w") as f:
            json.dump(dict(result=result, layers=layers, helpers=helpers, variants=by_variant), f,
                      indent=1)
    print(json.dumps(result), flush=True)


if __name__ == "__main__":
    main()
