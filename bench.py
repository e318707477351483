#!/usr/bin/env python3
"""Benchmark of the sliding-window-sum hot path on one MI355X.

A "step" is one pass of the hot path over configuration 5 (the largest single-GPU
workload, 2 GiB of input, genuinely HBM-cold): sliding add and sliding max with
w in {16, 64, 255} over x[256,128,16384] plus the 31-tap depthwise convolution —
seven launches through the C ABI.  Inputs are resident in HBM before the clock starts.

    value    = algorithmic bytes of a step / wall time of a step            [GB/s]
    roofline = the dominant kernel's algorithmic bytes per launch / its mean launch
               duration (HIP events on the launch stream, inside the timed region),
               against the 8 TB/s HBM peak
    ops      = every operator of all five configurations timed on its own (pooling in
               GB/s, convolution in GFLOP/s, each with its fraction of roofline)
    cpu_baseline = the fp64 oracle on a bounded sample of the same workload

Prints ONE JSON line on stdout.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0
FP32_PEAK_GFLOPS = 157300.0
BF16_PEAK_GFLOPS = 2.5e6
ROWS5, LEN5, CH5, K5 = 256 * 128, 16384, 128, 31
WINDOWS5 = (16, 64, 255)


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-ops", action="store_true", help="skip the per-operator table of configs 1-4")
    ap.add_argument("--cold", action="store_true",
                    help="with --only cfg2_* / cfg3_* / cfg4_*: go round enough distinct buffer pairs that more than "
                         "512 MB is touched between reuses (the tensors of those configurations fit the last-level cache)")
    ap.add_argument("--only", default=None,
                    help="profiling aid: launch just this operator --steps times and print nothing but a "
                         "short note (names: the keys of 'kernels' and 'ops', or 'copy' for the 2 GiB "
                         "calibration copy)")
    ap.add_argument("--opt", action="append", default=[], metavar="KEY=VALUE",
                    help="with --only: set a measurement knob of sws_dev.h first (A/B profiles), e.g. conv2d_variant=2")
    return ap.parse_args()


def slide_bytes(rows, length, w):
    return 4 * (rows * length + rows * (length - w + 1))


def read_traffic(name):
    """HBM bytes per launch measured offline with rocprofv3 counters (profiles/), or None."""
    path = os.path.join(ROOT, "profiles", name)
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    return float(line.split(":", 1)[1])
    except OSError:
        pass
    return None


def time_launches(torch, fn, iters, warm=8):
    """Mean duration in ms of `fn` (one launch): `iters` back-to-back launches between two events on
    the current stream.  An event recorded after every launch keeps the next kernel from starting
    until the event has been written (measured: 3.7 us per launch on a 35 us kernel), so only the
    two ends are marked."""
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / iters


def ops_table(torch, B, workloads, iters=40):
    """Each operator of configurations 1-4 on its own.  These tensors fit in the 256 MB
    last-level cache, so besides the warm figure a cold one is taken by rotating through
    enough distinct buffers that more than 512 MB is touched between reuses."""
    out = {}

    def rotate(make_args, nbytes):
        n = max(1, min(64, int(600e6 // max(nbytes, 1)) + 1))
        sets = [make_args() for _ in range(n)]
        state = {"i": 0}

        def pick():
            state["i"] = (state["i"] + 1) % n
            return sets[state["i"]]
        return sets[0], pick, sets

    def graph_ms(launch, args, n=20, replays=5, sets=None):
        """Mean duration of one launch inside a HIP graph of n back-to-back launches: what the
        small operators cost once the host's launch path (about 10 us from Python) is out of the way.
        With `sets` the launches of the graph go round the rotating buffer sets (the cold figure)."""
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            launch(*args)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        if sets is not None:
            n = len(sets) * max(1, (n + len(sets) - 1) // len(sets))
        gr = torch.cuda.CUDAGraph()
        with torch.cuda.graph(gr):
            for i in range(n):
                launch(*(sets[i % len(sets)] if sets is not None else args))
        gr.replay()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(replays):
            gr.replay()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / (n * replays)

    def record(name, launch, make_args, nbytes, flops=0.0, graph=False):
        first, pick, sets = rotate(make_args, nbytes)
        warm = time_launches(torch, lambda: launch(*first), iters)
        cold = time_launches(torch, lambda: launch(*pick()), iters)
        rec = {"ms_warm": round(warm, 5), "ms_cold": round(cold, 5),
               "GBps_cold": round(nbytes / cold / 1e6, 1),
               "frac_hbm_cold": round(nbytes / cold / 1e6 / HBM_PEAK_GBPS, 4)}
        if flops:
            rec["GFLOPs_warm"] = round(flops / warm / 1e6, 1)
            rec["GFLOPs_cold"] = round(flops / cold / 1e6, 1)
            rec["frac_fp32_peak_warm"] = round(flops / warm / 1e6 / FP32_PEAK_GFLOPS, 4)
        if graph:
            rec["ms_in_graph"] = round(graph_ms(launch, first), 5)
            rec["GBps_in_graph"] = round(nbytes / rec["ms_in_graph"] / 1e6, 1)
            if len(sets) > 1:                          # cold and in a graph: rotating buffers, no host launch path
                rec["ms_cold_in_graph"] = round(graph_ms(launch, first, sets=sets), 5)
                rec["GBps_cold_in_graph"] = round(nbytes / rec["ms_cold_in_graph"] / 1e6, 1)
                rec["frac_hbm_cold_in_graph"] = round(nbytes / rec["ms_cold_in_graph"] / 1e6 / HBM_PEAK_GBPS, 4)
            if flops:
                rec["GFLOPs_in_graph"] = round(flops / rec["ms_in_graph"] / 1e6, 1)
        out[name] = rec

    g = lambda a: torch.from_numpy(a).cuda()
    # cfg1: one sequence of 1,048,576, w = 5
    x1, t1 = workloads.make(1)
    x1, t1 = g(x1), g(t1)
    mk = lambda: (x1.clone(), torch.empty(1, 1, 1048572, device="cuda"))
    nb = slide_bytes(1, 1048576, 5)
    record("cfg1_slide_add_w5", lambda x, y: B.sws_slide1d(0, x, 5, 0.2, y=y), mk, nb, graph=True)
    record("cfg1_slide_max_w5", lambda x, y: B.sws_slide1d(1, x, 5, 1.0, y=y), mk, nb, graph=True)
    record("cfg1_corr_k5", lambda x, y: B.sws_conv1d(x, t1, y=y), mk, nb + 20, 2.0 * 5 * 1048572, graph=True)
    del x1
    # cfg2: [16,64,4096], pool w=3 and conv1d [64,64,3]
    x2, w2 = workloads.make(2)
    x2, w2 = g(x2), g(w2)
    mk = lambda: (x2.clone(), torch.empty(16, 64, 4094, device="cuda"))
    nb = slide_bytes(1024, 4096, 3)
    record("cfg2_avgpool_w3", lambda x, y: B.sws_slide1d(0, x, 3, 1 / 3, y=y), mk, nb, graph=True)
    record("cfg2_maxpool_w3", lambda x, y: B.sws_slide1d(1, x, 3, 1.0, y=y), mk, nb, graph=True)
    record("cfg2_conv1d_64x64x3", lambda x, y: B.sws_conv1d(x, w2, y=y), mk, nb + 4 * 64 * 64 * 3,
           2.0 * 16 * 64 * 4094 * 64 * 3, graph=True)
    del x2
    # cfg3: [32,64,112,112] 3x3 pad 1, stride 1 and 2
    x3, _ = workloads.make(3)
    x3 = g(x3)
    for s, ho in ((1, 112), (2, 56)):
        mk = lambda: (x3.clone(), torch.empty(32, 64, ho, ho, device="cuda"))
        nb = 4 * (2048 * 112 * 112 + 2048 * ho * ho)
        record("cfg3_maxpool3x3_s%d" % s, lambda x, y: B.sws_pool2d(1, x, 3, 3, s, s, 1, 1, 1.0, y=y), mk, nb, graph=True)
        record("cfg3_avgpool3x3_s%d" % s, lambda x, y: B.sws_pool2d(0, x, 3, 3, s, s, 1, 1, 1 / 9, y=y), mk, nb, graph=True)
    # the ceiling for an operator of this size: a plain copy of the same tensor, timed the same ways
    mk = lambda: (x3.clone(), torch.empty(32, 64, 112, 112, device="cuda"))
    record("cfg3_sized_copy", lambda x, y: B.sws_copy(x, y), mk, 2 * 4 * 2048 * 112 * 112, graph=True)
    del x3
    # cfg4: conv2d [32,64,56,56] x [64,64,3,3], pad 1
    x4, w4 = workloads.make(4)
    x4, w4 = g(x4), g(w4)
    mk = lambda: (x4.clone(), torch.empty(32, 64, 56, 56, device="cuda"))
    nb = 4 * (2 * 32 * 64 * 56 * 56 + 64 * 64 * 9)
    fl4 = 2.0 * 32 * 64 * 56 * 56 * 64 * 9
    record("cfg4_conv2d_3x3", lambda x, y: B.sws_conv2d(x, w4, 1, 1, 1, 1, y=y), mk, nb, fl4, graph=True)
    # The library's choice for this layer evaluates every fp32 product as six bf16 products on the bf16
    # matrix cores (operands split exactly into three bf16 pieces): GFLOPs above count the layer's 2*MACs
    # once ("fp32-equivalent"); the matrix cores execute six times as many, priced against the bf16 peak.
    r4 = out["cfg4_conv2d_3x3"]
    r4["arithmetic"] = "fp32 operands split exactly into 3 bf16 pieces, 6 products per term on bf16 MFMA, fp32 accumulation"
    r4["executed_bf16_GFLOPs_cold"] = round(6 * fl4 / r4["ms_cold"] / 1e6, 1)
    r4["frac_bf16_mfma_peak_cold"] = round(6 * fl4 / r4["ms_cold"] / 1e6 / BF16_PEAK_GFLOPS, 4)
    # the same layer on the fp32 matrix instructions (the streaming kernel's first form)
    B.sws_set_option("conv2d_variant", 17)
    try:
        record("cfg4_conv2d_3x3_fp32_mfma", lambda x, y: B.sws_conv2d(x, w4, 1, 1, 1, 1, y=y), mk, nb, fl4, graph=True)
    finally:
        B.sws_set_option("conv2d_variant", 0)
    del x4
    torch.cuda.empty_cache()
    return out


def sweeps_table(torch, B, workloads, iters=20):
    """The shapes of the paper's two experiments (Experiments section): 1-D convolution of
    single-channel sequences over the filter sizes of its first figure, and a 51-tap kernel with
    dilation 8 at the output sizes of its second figure (one sequence: launch-latency bound;
    plus a batched depthwise form that fills the device).  GB/s on algorithmic bytes, TFLOP/s on
    2*k FLOP per output; the vector-ALU peak without packed fp32 is 78.6 TFLOP/s."""
    g = lambda a: torch.from_numpy(a).cuda()
    out = {"filter_sweep": {}, "dilated_single": {}, "dilated_batched": {}, "pair_operator": {}, "same_size_pooling": {},
           "long_windows": {}, "storage_16bit": {}, "short_rows": {}, "adjoints": {}}
    c6 = workloads.CONFIGS[6]
    rows, length = c6.x_shape[0], c6.x_shape[2]
    x6 = g(workloads.make(6)[0])
    for k in workloads.FILTER_SIZES:
        taps = g(workloads.make(6, x_shape=(1,), wgt_shape=(1, 1, k))[1])
        lo = length - k + 1
        y = torch.empty(rows, 1, lo, device="cuda")
        ms = time_launches(torch, lambda: B.sws_conv1d(x6, taps, y=y), iters)
        nb, fl = 4 * rows * (length + lo) + 4 * k, 2.0 * k * rows * lo
        out["filter_sweep"]["k%d" % k] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                          "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4),
                                          "TFLOPs": round(fl / ms / 1e9, 2)}
        del y
    del x6
    torch.cuda.empty_cache()
    k, d = workloads.DILATED_K, workloads.DILATED_D
    for q in workloads.DILATED_OUTPUT_SIZES:
        x7, taps = workloads.make(7, x_shape=(1, 1, q + (k - 1) * d), wgt_shape=(1, 1, k))
        x7, taps = g(x7), g(taps)
        y = torch.empty(1, 1, q, device="cuda")
        ms = time_launches(torch, lambda: B.sws_conv1d(x7, taps, 1, 0, d, 1, y=y), iters)
        out["dilated_single"]["q%d" % q] = {"us": round(ms * 1e3, 2), "GFLOPs": round(2.0 * k * q / ms / 1e6, 1)}
    c7 = workloads.CONFIGS[7]
    ch, length = c7.x_shape[1], c7.x_shape[2]
    x7, taps = workloads.make(7)
    x7, taps = g(x7), g(taps)
    lo = length - (k - 1) * d
    y = torch.empty(1, ch, lo, device="cuda")
    ms = time_launches(torch, lambda: B.sws_conv1d(x7, taps, 1, 0, d, ch, y=y), iters)
    nb, fl = 4 * ch * (length + lo) + 4 * ch * k, 2.0 * k * ch * lo
    out["dilated_batched"]["dwconv_k51_d8"] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                               "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4),
                                               "TFLOPs": round(fl / ms / 1e9, 2),
                                               "frac_valu_peak": round(fl / ms / 1e9 / 78.6, 4)}
    del x7, y
    torch.cuda.empty_cache()
    # the dense form of the same scenario: 15 -> 15 channels, batch 64 (every output channel sums over
    # the input channels on the vector ALU; the matrix-core kernel would leave most of its tile idle)
    xd = g(workloads.make(7, x_shape=(64, 15, 100000 + (k - 1) * d), wgt_shape=(15, 15, k))[0])
    wd = g(workloads.make(7, x_shape=(1,), wgt_shape=(15, 15, k))[1])
    yd = torch.empty(64, 15, 100000, device="cuda")
    ms = time_launches(torch, lambda: B.sws_conv1d(xd, wd, 1, 0, d, 1, y=yd), iters)
    fl = 2.0 * 64 * 15 * 100000 * 15 * k
    out["dilated_batched"]["dense_15x15_k51_d8_q100000_b64"] = {
        "ms": round(ms, 4), "TFLOPs": round(fl / ms / 1e9, 2), "frac_valu_peak": round(fl / ms / 1e9 / 78.6, 4)}
    del xd, yd
    torch.cuda.empty_cache()
    # sliding window sum under the pair operator (Section 2.4, Eq. 8): 16 algorithmic bytes per output
    u, v = workloads.make_pairs()
    u, v = g(u), g(v)
    rows, length = u.shape
    for w in (16, 255):
        lo = length - w + 1
        yu, yv = torch.empty(rows, lo, device="cuda"), torch.empty(rows, lo, device="cuda")
        ms = time_launches(torch, lambda: B.sws_slide1d_pair(u, v, w, yu=yu, yv=yv), iters)
        nb = 8 * rows * (length + lo)
        out["pair_operator"]["w%d" % w] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                           "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        del yu, yv
    # one output per input: rows extended by (w-1)/2 mirrored elements at both ends (boundary rules, Section 3)
    for op, opn in ((0, "avg"), (1, "max")):
        for w in (15, 255):
            y = torch.empty_like(u)
            ms = time_launches(torch, lambda: B.sws_slide1d_padded(op, u, w, w // 2, w // 2, B.SWS_PAD_MIRROR, 1.0 / w, y=y),
                               iters)
            nb = 8 * u.numel()
            out["same_size_pooling"]["%s_w%d_mirror" % (opn, w)] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                                                    "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
            del y
    del u, v
    torch.cuda.empty_cache()
    # windows longer than a wave tile (one pass: suffix sums of the tile, one shared middle reduction, prefix sums
    # where the windows end) on a quarter of configuration 5's rows
    xl = torch.rand(8192, LEN5, device="cuda")
    for op, opn in ((0, "avg"), (1, "max")):
        for w in (512, 1024, 2048, 8192):
            y = torch.empty(8192, LEN5 - w + 1, device="cuda")
            ms = time_launches(torch, lambda: B.sws_slide1d(op, xl, w, 1.0 / w, y=y), iters)
            nb = 4 * (xl.numel() + y.numel())
            out["long_windows"]["%s_w%d" % (opn, w)] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                                        "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
            del y
    del xl
    torch.cuda.empty_cache()
    # configuration 5's depthwise layer with 15 mirrored elements at both ends of every row (sws_conv1d_padded)
    x5, t5 = workloads.make(5)
    x5, t5 = g(x5), g(t5)
    y = torch.empty_like(x5)
    ms = time_launches(torch, lambda: B.sws_conv1d_padded(x5, t5, 1, K5 // 2, K5 // 2, 1, CH5, B.SWS_PAD_MIRROR, y=y), iters)
    nb = 8 * x5.numel()
    out["same_size_pooling"]["dwconv_k31_mirror"] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                                     "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    del x5, y
    torch.cuda.empty_cache()
    # the same in two dimensions: configuration 3's planes extended by k/2 mirrored rows and columns on every side
    x3 = g(workloads.make(3)[0])
    for op, opn in ((0, "avg"), (1, "max")):
        for k, st in ((3, 1), (3, 2), (7, 1)):
            ho = (112 + 2 * (k // 2) - k) // st + 1
            y = torch.empty(32, 64, ho, ho, device="cuda")
            ms = time_launches(torch, lambda: B.sws_pool2d_padded(op, x3, k, k, st, st, (k // 2,) * 4, B.SWS_PAD_MIRROR,
                                                                  1.0 / (k * k), y=y), iters)
            nb = 4 * (x3.numel() + y.numel())
            out["same_size_pooling"]["cfg3_%s_%dx%d_s%d_mirror" % (opn, k, k, st)] = {
                "ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
            del y
    # larger centred windows on the same planes (plain and mirrored), warm like the rows above
    for opn, op, k, mode in (("avg", 0, 9, None), ("avg", 0, 13, None), ("max", 1, 13, None), ("avg", 0, 13, B.SWS_PAD_MIRROR)):
        y = torch.empty(32, 64, 112, 112, device="cuda")
        if mode is None:
            fn = lambda: B.sws_pool2d(op, x3, k, k, 1, 1, k // 2, k // 2, 1.0 / (k * k), y=y)
        else:
            fn = lambda: B.sws_pool2d_padded(op, x3, k, k, 1, 1, (k // 2,) * 4, mode, 1.0 / (k * k), y=y)
        ms = time_launches(torch, fn, iters)
        nb = 4 * (x3.numel() + y.numel())
        out["same_size_pooling"]["cfg3_%s_%dx%d_s1%s" % (opn, k, k, "" if mode is None else "_mirror")] = {
            "ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        del y
    del x3
    torch.cuda.empty_cache()
    # planes wider than a wavefront's 256 columns and rows that are not a multiple of 4 long (strips), and the adjoints
    # of 2 x 2 stride-2 pooling
    out["wide_planes"] = {}
    xw = torch.empty(8, 16, 512, 512, device="cuda").uniform_(-1, 1)
    yw = torch.empty_like(xw)
    gxw = torch.empty_like(xw)
    nb2 = 8.0 * xw.numel()
    for name, fn, nb in (("512x512_avg_3x3_s1", lambda: B.sws_pool2d(0, xw, 3, 3, 1, 1, 1, 1, 1 / 9, y=yw), nb2),
                         ("512x512_max_7x7_s1", lambda: B.sws_pool2d(1, xw, 7, 7, 1, 1, 3, 3, 1.0, y=yw), nb2),
                         ("512x512_avg_3x3_s1_mirror",
                          lambda: B.sws_pool2d_padded(0, xw, 3, 3, 1, 1, (1, 1, 1, 1), B.SWS_PAD_MIRROR, 1 / 9, y=yw), nb2),
                         ("512x512_maxpool3x3_s1_grad", lambda: B.sws_maxpool2d_grad(xw, yw, 3, 3, 1, 1, 1, 1, gx=gxw), 1.5 * nb2)):
        ms = time_launches(torch, fn, iters)
        out["wide_planes"][name] = {"us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1),
                                    "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    del xw, yw, gxw
    xr_ = torch.empty(32, 64, 111, 111, device="cuda").uniform_(-1, 1)
    yr_ = torch.empty_like(xr_)
    ms = time_launches(torch, lambda: B.sws_pool2d(1, xr_, 3, 3, 1, 1, 1, 1, 1.0, y=yr_), iters)
    out["wide_planes"]["111x111_max_3x3_s1"] = {"us": round(ms * 1e3, 2), "GBps": round(8.0 * xr_.numel() / ms / 1e6, 1),
                                                "frac_hbm": round(8.0 * xr_.numel() / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    gyr_ = torch.empty(32, 64, 56, 56, device="cuda").normal_()
    gxr_ = torch.empty_like(xr_)
    for name, fn, nb in (("111x111_maxpool3x3_s1_grad", lambda: B.sws_maxpool2d_grad(xr_, yr_, 3, 3, 1, 1, 1, 1, gx=gxr_),
                          12.0 * xr_.numel()),
                         ("111x111_maxpool3x3_s2_grad", lambda: B.sws_maxpool2d_grad(xr_, gyr_, 3, 3, 2, 2, 1, 1, gx=gxr_),
                          4.0 * (2 * xr_.numel() + gyr_.numel()))):
        ms = time_launches(torch, fn, iters)
        out["wide_planes"][name] = {"us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1),
                                    "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    del xr_, yr_, gyr_, gxr_
    x3b = torch.empty(32, 64, 112, 112, device="cuda").uniform_(-1, 1)
    gy3b = torch.empty(32, 64, 56, 56, device="cuda").normal_()
    gx3b = torch.empty_like(x3b)
    for name, fn, nb in (("cfg3_maxpool2x2_s2_grad", lambda: B.sws_maxpool2d_grad(x3b, gy3b, 2, 2, 2, 2, 0, 0, gx=gx3b),
                          4.0 * (2 * x3b.numel() + gy3b.numel())),
                         ("cfg3_avgpool2x2_s2_grad", lambda: B.sws_avgpool2d_grad(gy3b, 112, 112, 2, 2, 2, 2, 0, 0, 0, 0.25, gx=gx3b),
                          4.0 * (x3b.numel() + gy3b.numel()))):
        ms = time_launches(torch, fn, iters)
        out["wide_planes"][name] = {"us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1),
                                    "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
    del x3b, gy3b, gx3b
    torch.cuda.empty_cache()
    # configuration 5's sliding sums on 16-bit storage (fp32 arithmetic, one rounding): half the bytes
    x16 = g(workloads.make(5)[0]).to(torch.bfloat16)
    for dt, dn in ((torch.bfloat16, "bf16"), (torch.float16, "f16")):
        xs = x16 if dt == torch.bfloat16 else x16.to(dt)
        for op, opn in ((0, "add"), (1, "max")):
            for w in (3, 9) + tuple(WINDOWS5) if dn == "bf16" else (64,):
                y = torch.empty(256, 128, LEN5 - w + 1, device="cuda", dtype=dt)
                ms = time_launches(torch, lambda: B.sws_slide1d_16(op, xs, w, 1.0 / w, y=y), iters)
                nb = slide_bytes(ROWS5, LEN5, w) // 2
                out["storage_16bit"]["%s_%s_w%d" % (dn, opn, w)] = {
                    "ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4),
                    "Gelem_per_s": round(ROWS5 * (LEN5 - w + 1) / ms / 1e6, 1)}
                del y
        del xs
    # configuration 5's depthwise layer on bf16 storage (fp32 taps and arithmetic, one rounding)
    taps = g(workloads.make(5, x_shape=(1, 128, 64))[1])
    k5 = taps.shape[-1]
    x16 = x16.view(256, 128, LEN5)
    y = torch.empty(256, 128, LEN5 - k5 + 1, device="cuda", dtype=torch.bfloat16)
    ms = time_launches(torch, lambda: B.sws_conv1d_16(x16, taps, groups=128, y=y), iters)
    nb = slide_bytes(ROWS5, LEN5, k5) // 2
    out["storage_16bit"]["bf16_depthwise_conv_k%d" % k5] = {
        "ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4),
        "Gelem_per_s": round(ROWS5 * (LEN5 - k5 + 1) / ms / 1e6, 1)}
    del y, taps
    del x16
    torch.cuda.empty_cache()
    x3 = g(workloads.make(3)[0]).to(torch.bfloat16)       # configuration 3's pooling on bf16 storage
    for st, ho in ((1, 112), (2, 56)):
        y = torch.empty(32, 64, ho, ho, device="cuda", dtype=torch.bfloat16)
        nb = 2 * 2048 * (112 * 112 + ho * ho)
        for op, opn in ((1, "max"), (0, "avg")):
            ms = time_launches(torch, lambda: B.sws_pool2d_16(op, x3, 3, 3, st, st, 1, 1, 1.0 / 9, y=y), iters)
            out["storage_16bit"]["bf16_%spool3x3_s%d" % (opn, st)] = {
                "us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        del y
    del x3
    torch.cuda.empty_cache()
    # rows far shorter than a wave tile (the rows of configuration 3's and 4's planes as a 1-D problem)
    for rows, ln in ((262144, 56), (65536, 224)):
        xs = g(workloads.make(5, x_shape=(rows, ln), wgt_shape=(1, 1, 1))[0])
        for dt, dn in ((torch.float32, "f32"), (torch.bfloat16, "bf16")):
            xd = xs.to(dt)
            for w in (3, 16):
                y = torch.empty(rows, ln - w + 1, device="cuda", dtype=dt)
                fn = (lambda: B.sws_slide1d(1, xd, w, 1.0, y=y)) if dt == torch.float32 else \
                     (lambda: B.sws_slide1d_16(1, xd, w, 1.0, y=y))
                ms = time_launches(torch, fn, iters)
                nb = xd.element_size() * rows * (2 * ln - w + 1)
                out["short_rows"]["%s_max_w%d_%dx%d" % (dn, w, rows, ln)] = {
                    "us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
                del y
            del xd
        del xs
    # planes of a few dozen elements, thousands of channels (a network's last stages)
    for shape, geoms in (((32, 2048, 7, 7), ((7, 7, 1, 0), (3, 3, 1, 1))), ((32, 1024, 14, 14), ((3, 3, 2, 1), (2, 2, 2, 0)))):
        xs = g(workloads.make(3, x_shape=shape)[0])
        for k, _, st, pd in geoms:
            ho = (shape[2] + 2 * pd - k) // st + 1
            y = torch.empty(shape[0], shape[1], ho, ho, device="cuda")
            for op, opn in ((1, "max"), (0, "avg")):
                ms = time_launches(torch, lambda: B.sws_pool2d(op, xs, k, k, st, st, pd, pd, 1.0 / (k * k), y=y), iters)
                nb = 4 * shape[0] * shape[1] * (shape[2] * shape[3] + ho * ho)
                out["short_rows"]["f32_%spool%dx%d_s%d_%dx%dx%dx%d" % ((opn, k, k, st) + shape)] = {
                    "us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1), "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
            del y
        del xs
    torch.cuda.empty_cache()
    # the adjoints of the sliding dot product (training): configuration 5's depthwise layer (HBM-bound:
    # grad-input moves what the forward pass moves, grad-weight reads x and gy) and configuration 2's
    # dense layer (matrix cores; 2*Cin*k FLOP per output element for either adjoint)
    x5, t5 = workloads.make(5)
    x5, t5 = g(x5), g(t5)
    lo = LEN5 - K5 + 1
    gy5 = torch.empty(256, 128, lo, device="cuda").uniform_(-1, 1)
    gx5 = torch.empty_like(x5)
    gw5 = torch.empty_like(t5)
    nb, fl = slide_bytes(ROWS5, LEN5, K5) + 4 * CH5 * K5, 2.0 * ROWS5 * lo * K5
    for name, fn in (("dwconv_k31_grad_input", lambda: B.sws_conv1d_grad_input(gy5, t5, LEN5, groups=CH5, gx=gx5)),
                     ("dwconv_k31_grad_weight", lambda: B.sws_conv1d_grad_weight(x5, gy5, K5, groups=CH5, gw=gw5))):
        ms = time_launches(torch, fn, iters)
        out["adjoints"][name] = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1),
                                 "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4), "TFLOPs": round(fl / ms / 1e9, 2)}
    del x5, gy5, gx5
    torch.cuda.empty_cache()
    x2, w2 = workloads.make(2)
    x2, w2 = g(x2), g(w2)
    gy2 = torch.empty(16, 64, 4094, device="cuda").normal_()
    gx2, gw2 = torch.empty_like(x2), torch.empty_like(w2)
    fl = 2.0 * 16 * 64 * 4094 * 64 * 3
    for name, fn in (("cfg2_conv1d_grad_input", lambda: B.sws_conv1d_grad_input(gy2, w2, 4096, gx=gx2)),
                     ("cfg2_conv1d_grad_weight", lambda: B.sws_conv1d_grad_weight(x2, gy2, 3, gw=gw2))):
        ms = time_launches(torch, fn, iters)
        out["adjoints"][name] = {"us": round(ms * 1e3, 2), "TFLOPs": round(fl / ms / 1e9, 2),
                                 "frac_fp32_mfma_peak": round(fl / ms / 1e9 / 157.3, 4)}
    x3 = g(workloads.make(3)[0])                          # configuration 3's max pooling: gradients routed to the maxima
    gx3 = torch.empty_like(x3)
    for st, ho in ((1, 112), (2, 56)):
        gy3 = torch.empty(32, 64, ho, ho, device="cuda").normal_()
        nb = 4 * 2048 * (2 * 112 * 112 + ho * ho)
        ms = time_launches(torch, lambda: B.sws_maxpool2d_grad(x3, gy3, 3, 3, st, st, 1, 1, gx=gx3), iters)
        out["adjoints"]["cfg3_maxpool3x3_s%d_grad" % st] = {"us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1),
                                                           "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        nb = 4 * 2048 * (112 * 112 + ho * ho)
        ms = time_launches(torch, lambda: B.sws_avgpool2d_grad(gy3, 112, 112, 3, 3, st, st, 1, 1, 0, 1 / 9, gx=gx3), iters)
        out["adjoints"]["cfg3_avgpool3x3_s%d_grad" % st] = {"us": round(ms * 1e3, 2), "GBps": round(nb / ms / 1e6, 1),
                                                           "frac_hbm": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        del gy3
    del x3, gx3
    torch.cuda.empty_cache()
    x4, w4 = workloads.make(4)
    x4, w4 = g(x4), g(w4)
    gy4 = torch.empty(32, 64, 56, 56, device="cuda").normal_()
    gx4, gw4 = torch.empty_like(x4), torch.empty_like(w4)
    fl = 7398752256.0
    for name, fn in (("cfg4_conv2d_grad_input", lambda: B.sws_conv2d_grad_input(gy4, w4, 56, 56, 1, 1, 1, 1, gx=gx4)),
                     ("cfg4_conv2d_grad_weight", lambda: B.sws_conv2d_grad_weight(x4, gy4, 3, 3, 1, 1, 1, 1, gw=gw4))):
        ms = time_launches(torch, fn, iters)
        out["adjoints"][name] = {"us": round(ms * 1e3, 2), "TFLOPs": round(fl / ms / 1e9, 2),
                                 "frac_fp32_mfma_peak": round(fl / ms / 1e9 / 157.3, 4)}
    del x4, gy4, gx4
    xr = torch.empty(32, 256, 3136, device="cuda").normal_()
    gr = torch.empty(32, 256, 3136, device="cuda").normal_()
    wr = torch.empty(256, 256, 3, device="cuda").normal_()
    gxr, gwr = torch.empty_like(xr), torch.empty_like(wr)
    fl = 2.0 * 32 * 3136 * 256 * 256 * 3
    for name, fn in (("dense_256x256_k3_b32_l3136_grad_input", lambda: B.sws_conv1d_grad_input(gr, wr, 3136, 1, 1, gx=gxr)),
                     ("dense_256x256_k3_b32_l3136_grad_weight", lambda: B.sws_conv1d_grad_weight(xr, gr, 3, 1, 1, gw=gwr))):
        ms = time_launches(torch, fn, iters)
        out["adjoints"][name] = {"ms": round(ms, 4), "TFLOPs": round(fl / ms / 1e9, 2),
                                 "frac_fp32_mfma_peak": round(fl / ms / 1e9 / 157.3, 4)}
    del xr, gr, gxr
    torch.cuda.empty_cache()
    # a down-sampling layer (3 x 3, stride 2, 128 -> 128 channels on 56 x 56 planes) and a late layer with short
    # rows (3 x 3, 256 -> 256 channels on 14 x 14 planes), 32 images: forward and both adjoints
    for tag, ch, hh, st in (("s2_3x3_128ch_56x56", 128, 56, 2), ("s1_3x3_256ch_14x14", 256, 14, 1)):
        ho = (hh + 2 - 3) // st + 1
        xs = torch.empty(32, ch, hh, hh, device="cuda").normal_()
        ws = torch.empty(ch, ch, 3, 3, device="cuda").normal_(0, 0.03)
        ys = torch.empty(32, ch, ho, ho, device="cuda")
        gs = torch.empty(32, ch, ho, ho, device="cuda").normal_()
        gxs, gws = torch.empty_like(xs), torch.empty_like(ws)
        fl = 2.0 * 32 * ch * ch * 9 * ho * ho
        for name, fn in (("forward", lambda: B.sws_conv2d(xs, ws, st, st, 1, 1, y=ys)),
                         ("grad_input", lambda: B.sws_conv2d_grad_input(gs, ws, hh, hh, st, st, 1, 1, gx=gxs)),
                         ("grad_weight", lambda: B.sws_conv2d_grad_weight(xs, gs, 3, 3, st, st, 1, 1, gw=gws))):
            ms = time_launches(torch, fn, iters)
            out["adjoints"]["layer_%s_%s" % (tag, name)] = {"us": round(ms * 1e3, 2), "TFLOPs": round(fl / ms / 1e9, 2),
                                                             "frac_fp32_mfma_peak": round(fl / ms / 1e9 / 157.3, 4)}
        del xs, ws, ys, gs, gxs, gws
    torch.cuda.empty_cache()
    return out


def run_only(torch, B, workloads, name, steps, cold=False):
    """Launch one operator `steps` times (for rocprofv3 runs that should see a single kernel)."""
    g = lambda a: torch.from_numpy(a).cuda()

    def rotating(x, y):
        """fn(launch) -> a call that goes round copies of (x, y): more than 600 MB between reuses if cold."""
        nbytes = x.numel() * x.element_size() + y.numel() * y.element_size()
        n = int(600e6 // nbytes) + 1 if cold else 1
        sets = [(x, y)] + [(x.clone(), torch.empty_like(y)) for _ in range(n - 1)]
        state = {"i": 0}

        def wrap(launch):
            def call():
                state["i"] = (state["i"] + 1) % n
                launch(*sets[state["i"]])
            return call
        return wrap
    if name == "copy":
        src = torch.rand(ROWS5, LEN5, device="cuda")
        dst = torch.empty_like(src)
        fn = lambda: B.sws_copy(src, dst)
    elif name in ("grad_input_dwconv_k31", "grad_weight_dwconv_k31"):
        x, taps = workloads.make(5)
        x, taps = g(x), g(taps)
        gy = torch.empty(256, 128, LEN5 - K5 + 1, device="cuda").uniform_(-1, 1)
        if name.startswith("grad_input"):
            gx = torch.empty_like(x)
            fn = lambda: B.sws_conv1d_grad_input(gy, taps, LEN5, groups=CH5, gx=gx)
        else:
            gw = torch.empty_like(taps)
            fn = lambda: B.sws_conv1d_grad_weight(x, gy, K5, groups=CH5, gw=gw)
    elif name in ("grad_input_cfg2", "grad_weight_cfg2"):
        x2, w2 = workloads.make(2)
        x2, w2 = g(x2), g(w2)
        gy = torch.empty(16, 64, 4094, device="cuda").normal_()
        if name.startswith("grad_input"):
            gx = torch.empty_like(x2)
            fn = lambda: B.sws_conv1d_grad_input(gy, w2, 4096, gx=gx)
        else:
            gw = torch.empty_like(w2)
            fn = lambda: B.sws_conv1d_grad_weight(x2, gy, 3, gw=gw)
    elif name.startswith("gw2d_"):                        # gw2d_<n>x<cin>x<h>x<w>_<cout>_k<kh>x<kw>_p<ph>x<pw>: any stride-1 layer's grad-weight
        _, shp, co, kk, pp = name.split("_")
        n, ci, h, w = (int(v) for v in shp.split("x"))
        kh, kw = (int(v) for v in kk[1:].split("x"))
        ph, pw = (int(v) for v in pp[1:].split("x"))
        xs = torch.empty(n, ci, h, w, device="cuda").normal_()
        gs = torch.empty(n, int(co), h + 2 * ph - kh + 1, w + 2 * pw - kw + 1, device="cuda").normal_()
        gws = torch.empty(int(co), ci, kh, kw, device="cuda")
        fn = lambda: B.sws_conv2d_grad_weight(xs, gs, kh, kw, 1, 1, ph, pw, gw=gws)
    elif name in ("grad_input_dense256", "grad_weight_dense256"):   # the 256 -> 256 channel 1-D layer of the adjoints table
        xr = torch.empty(32, 256, 3136, device="cuda").normal_()
        gr = torch.empty(32, 256, 3136, device="cuda").normal_()
        if name.startswith("grad_input"):
            wr = torch.empty(256, 256, 3, device="cuda").normal_()
            fn = lambda: B.sws_conv1d_grad_input(gr, wr, 3136, 1, 1, gx=xr)
        else:
            gwr = torch.empty(256, 256, 3, device="cuda")
            fn = lambda: B.sws_conv1d_grad_weight(xr, gr, 3, 1, 1, gw=gwr)
    elif name in ("grad_input_cfg4", "grad_weight_cfg4"):
        x4, w4 = workloads.make(4)
        x4, w4 = g(x4), g(w4)
        gy = torch.empty(32, 64, 56, 56, device="cuda").normal_()
        if name.startswith("grad_input"):
            gx = torch.empty_like(x4)
            fn = lambda: B.sws_conv2d_grad_input(gy, w4, 56, 56, 1, 1, 1, 1, gx=gx)
        else:
            gw = torch.empty_like(w4)
            fn = lambda: B.sws_conv2d_grad_weight(x4, gy, 3, 3, 1, 1, 1, 1, gw=gw)
    elif name.startswith("short_rows_"):                  # short_rows_<f32|bf16>_<add|max>_w<w>_<rows>x<len>
        _, _, dn, opn, wn, shp = name.split("_")
        w = int(wn[1:])
        rows, ln = (int(v) for v in shp.split("x"))
        dt = {"f32": torch.float32, "bf16": torch.bfloat16}[dn]
        xd = g(workloads.make(5, x_shape=(rows, ln), wgt_shape=(1, 1, 1))[0]).to(dt)
        y = torch.empty(rows, ln - w + 1, device="cuda", dtype=dt)
        op = 0 if opn == "add" else 1
        fn = (lambda: B.sws_slide1d(op, xd, w, 1.0, y=y)) if dn == "f32" else (lambda: B.sws_slide1d_16(op, xd, w, 1.0, y=y))
    elif name.startswith("slide16_"):                     # slide16_<bf16|f16>_<add|max>_w<w>
        _, dn, opn, wn = name.split("_")
        w = int(wn[1:])
        dt = torch.bfloat16 if dn == "bf16" else torch.float16
        x = g(workloads.make(5)[0]).to(dt)
        y = torch.empty(256, 128, LEN5 - w + 1, device="cuda", dtype=dt)
        fn = lambda: B.sws_slide1d_16(0 if opn == "add" else 1, x, w, 1.0 / w, y=y)
    elif name == "dwconv16_k31":                          # the depthwise layer on bf16 storage
        x_host, taps_host = workloads.make(5)
        x = g(x_host).to(torch.bfloat16)
        taps = g(taps_host)
        y = torch.empty(256, 128, LEN5 - K5 + 1, device="cuda", dtype=torch.bfloat16)
        fn = lambda: B.sws_conv1d_16(x, taps, groups=CH5, y=y)
    elif name.startswith("dwconv_k31_"):                  # dwconv_k31_<mirror|periodic|edge>: one output per input
        mode = {"mirror": B.SWS_PAD_MIRROR, "periodic": B.SWS_PAD_PERIODIC, "edge": B.SWS_PAD_EDGE}[name.split("_")[2]]
        x_host, taps_host = workloads.make(5)
        x, taps = g(x_host), g(taps_host)
        y = torch.empty(256, 128, LEN5, device="cuda")
        fn = lambda: B.sws_conv1d_padded(x, taps, 1, K5 // 2, K5 // 2, 1, CH5, mode, y=y)
    elif name.startswith("long_"):                        # long_<add|max>_w<w>: 8192 rows of 16384, windows longer than a tile
        _, opn, wn = name.split("_")
        w = int(wn[1:])
        xl = torch.rand(8192, LEN5, device="cuda")
        y = torch.empty(8192, LEN5 - w + 1, device="cuda")
        fn = lambda: B.sws_slide1d(0 if opn == "add" else 1, xl, w, 1.0 / w, y=y)
    elif name.startswith("slide_") or name == "dwconv_k31":
        x_host, taps_host = workloads.make(5)
        x = g(x_host)
        if name == "dwconv_k31":
            taps = g(taps_host)
            y = torch.empty(256, 128, LEN5 - K5 + 1, device="cuda")
            fn = lambda: B.sws_conv1d(x, taps, groups=CH5, y=y)
        else:
            _, opn, wn = name.split("_")
            w = int(wn[1:])
            y = torch.empty(256, 128, LEN5 - w + 1, device="cuda")
            fn = lambda: B.sws_slide1d(0 if opn == "add" else 1, x, w, 1.0 / w, y=y)
    elif name.startswith("cfg1_"):
        x1, t1 = workloads.make(1)
        x1, t1 = g(x1), g(t1)
        y = torch.empty(1, 1, 1048572, device="cuda")
        if name == "cfg1_corr_k5":
            fn = lambda: B.sws_conv1d(x1, t1, y=y)
        else:
            op = 1 if "max" in name else 0
            fn = lambda: B.sws_slide1d(op, x1, 5, 0.2, y=y)
    elif name in ("cfg2_avgpool_w3", "cfg2_maxpool_w3"):
        x2 = g(workloads.make(2)[0])
        y = torch.empty(16, 64, 4094, device="cuda")
        op = 1 if "max" in name else 0
        fn = rotating(x2, y)(lambda xx, yy: B.sws_slide1d(op, xx, 3, 1 / 3, y=yy))
    elif name.startswith("layer_"):                       # layer_<s2_3x3_128ch_56x56|s1_3x3_256ch_14x14>_<forward|grad_input|grad_weight>
        tag, what = (name[6:].rsplit("_", 2)[0], "_".join(name.rsplit("_", 2)[1:])) if name.endswith(("grad_input", "grad_weight")) else (name[6:].rsplit("_", 1)[0], "forward")
        ch, hh, st = {"s2_3x3_128ch_56x56": (128, 56, 2), "s1_3x3_256ch_14x14": (256, 14, 1)}[tag]
        ho = (hh + 2 - 3) // st + 1
        xs = torch.empty(32, ch, hh, hh, device="cuda").normal_()
        ws = torch.empty(ch, ch, 3, 3, device="cuda").normal_(0, 0.03)
        ys = torch.empty(32, ch, ho, ho, device="cuda")
        gs = torch.empty(32, ch, ho, ho, device="cuda").normal_()
        gxs, gws = torch.empty_like(xs), torch.empty_like(ws)
        fn = {"forward": lambda: B.sws_conv2d(xs, ws, st, st, 1, 1, y=ys),
              "grad_input": lambda: B.sws_conv2d_grad_input(gs, ws, hh, hh, st, st, 1, 1, gx=gxs),
              "grad_weight": lambda: B.sws_conv2d_grad_weight(xs, gs, 3, 3, st, st, 1, 1, gw=gws)}[what]
    elif name in ("grad_cfg3_avgpool_s1", "grad_cfg3_avgpool_s2"):
        s = int(name[-1])
        ho = 112 if s == 1 else 56
        gy = torch.empty(32, 64, ho, ho, device="cuda").normal_()
        gx = torch.empty(32, 64, 112, 112, device="cuda")
        fn = lambda: B.sws_avgpool2d_grad(gy, 112, 112, 3, 3, s, s, 1, 1, 0, 1 / 9, gx=gx)
    elif name.startswith("poolgrad_"):                    # poolgrad_<max|avg>_<planes>x<h>x<w>_k<k>_s<s>_p<p>: any pooling adjoint
        _, opn, shp, kn, sn, pn = name.split("_")
        pl_, h_, w_ = (int(v) for v in shp.split("x"))
        k, st, pd = int(kn[1:]), int(sn[1:]), int(pn[1:])
        ho_, wo_ = (h_ + 2 * pd - k) // st + 1, (w_ + 2 * pd - k) // st + 1
        xw = torch.empty(1, pl_, h_, w_, device="cuda").uniform_(-1, 1)
        gyw = torch.empty(1, pl_, ho_, wo_, device="cuda").normal_()
        gxw = torch.empty_like(xw)
        if opn == "max":
            fn = lambda: B.sws_maxpool2d_grad(xw, gyw, k, k, st, st, pd, pd, gx=gxw)
        else:
            fn = lambda: B.sws_avgpool2d_grad(gyw, h_, w_, k, k, st, st, pd, pd, 0, 1.0 / (k * k), gx=gxw)
    elif name.startswith("widegrad_"):                    # widegrad_<max|avg>_s<s>: adjoints of 3 x 3 pad 1 pooling on x[8,16,512,512]
        _, opn, sn = name.split("_")
        st = int(sn[1:])
        ho = 512 if st == 1 else 256
        xw = torch.empty(8, 16, 512, 512, device="cuda").uniform_(-1, 1)
        gyw = torch.empty(8, 16, ho, ho, device="cuda").normal_()
        gxw = torch.empty_like(xw)
        if opn == "max":
            fn = lambda: B.sws_maxpool2d_grad(xw, gyw, 3, 3, st, st, 1, 1, gx=gxw)
        else:
            fn = lambda: B.sws_avgpool2d_grad(gyw, 512, 512, 3, 3, st, st, 1, 1, 0, 1 / 9, gx=gxw)
    elif name in ("grad_cfg3_maxpool_s1", "grad_cfg3_maxpool_s2"):
        x3 = g(workloads.make(3)[0])
        s = int(name[-1])
        ho = 112 if s == 1 else 56
        gy = torch.empty(32, 64, ho, ho, device="cuda").normal_()
        gx = torch.empty_like(x3)
        fn = lambda: B.sws_maxpool2d_grad(x3, gy, 3, 3, s, s, 1, 1, gx=gx)
    elif name.startswith("padded_cfg3_"):                 # padded_cfg3_<avg|max>_<mirror|periodic|edge>_k<k>_s<s>
        _, _, opn, mn, kn, sn = name.split("_")
        k, st = int(kn[1:]), int(sn[1:])
        mode = {"mirror": B.SWS_PAD_MIRROR, "periodic": B.SWS_PAD_PERIODIC, "edge": B.SWS_PAD_EDGE}[mn]
        x3 = g(workloads.make(3)[0])
        ho = (112 + 2 * (k // 2) - k) // st + 1
        y = torch.empty(32, 64, ho, ho, device="cuda")
        op = 1 if opn == "max" else 0
        fn = rotating(x3, y)(lambda xx, yy: B.sws_pool2d_padded(op, xx, k, k, st, st, (k // 2,) * 4, mode, 1.0 / (k * k), y=yy))
    elif name.startswith("widepad_"):                     # widepad_<avg|max>_<mirror|periodic|edge>_k<k>: x[8,16,512,512], stride 1, pad k // 2
        _, opn, mn, kn = name.split("_")
        k = int(kn[1:])
        mode = {"mirror": B.SWS_PAD_MIRROR, "periodic": B.SWS_PAD_PERIODIC, "edge": B.SWS_PAD_EDGE}[mn]
        xw = torch.empty(8, 16, 512, 512, device="cuda").uniform_(-1, 1)
        y = torch.empty(8, 16, 512, 512, device="cuda")
        op = 1 if opn == "max" else 0
        fn = rotating(xw, y)(lambda xx, yy: B.sws_pool2d_padded(op, xx, k, k, 1, 1, (k // 2,) * 4, mode, 1.0 / (k * k), y=yy))
    elif name.startswith("pool_"):                        # pool_<planes>x<h>x<w>_<avg|max>_k<k>_s<s>_p<p>: any plain 2-D pooling
        _, shp, opn, kn, sn, pn = name.split("_")
        pl_, h_, w_ = (int(v) for v in shp.split("x"))
        k, st, pd = int(kn[1:]), int(sn[1:]), int(pn[1:])
        xw = torch.empty(1, pl_, h_, w_, device="cuda").uniform_(-1, 1)
        y = torch.empty(1, pl_, (h_ + 2 * pd - k) // st + 1, (w_ + 2 * pd - k) // st + 1, device="cuda")
        op = 1 if opn == "max" else 0
        fn = rotating(xw, y)(lambda xx, yy: B.sws_pool2d(op, xx, k, k, st, st, pd, pd, 1.0 / (k * k), y=yy))
    elif name.startswith("wide_"):                        # wide_<avg|max>_k<k>_s<s>: x[8,16,512,512], pad k // 2 (0 for k = 2)
        _, opn, kn, sn = name.split("_")
        k, st = int(kn[1:]), int(sn[1:])
        pd = 0 if k == 2 else k // 2
        xw = torch.empty(8, 16, 512, 512, device="cuda").uniform_(-1, 1)
        ho = (512 + 2 * pd - k) // st + 1
        y = torch.empty(8, 16, ho, ho, device="cuda")
        op = 1 if opn == "max" else 0
        fn = rotating(xw, y)(lambda xx, yy: B.sws_pool2d(op, xx, k, k, st, st, pd, pd, 1.0 / (k * k), y=yy))
    elif name.startswith("cfg3_"):
        x3 = g(workloads.make(3)[0])
        s = int(name[-1])
        ho = 112 if s == 1 else 56
        y = torch.empty(32, 64, ho, ho, device="cuda")
        op = 1 if "max" in name else 0
        fn = rotating(x3, y)(lambda xx, yy: B.sws_pool2d(op, xx, 3, 3, s, s, 1, 1, 1 / 9, y=yy))
    elif name == "cfg4_conv2d_3x3":
        x4, w4 = workloads.make(4)
        x4, w4 = g(x4), g(w4)
        y = torch.empty(32, 64, 56, 56, device="cuda")
        fn = rotating(x4, y)(lambda xx, yy: B.sws_conv2d(xx, w4, 1, 1, 1, 1, y=yy))
    elif name.startswith("cfg4_conv2d_3x3_"):             # cfg4_conv2d_3x3_<mirror|periodic|edge>
        mode = {"mirror": B.SWS_PAD_MIRROR, "periodic": B.SWS_PAD_PERIODIC, "edge": B.SWS_PAD_EDGE}[name.split("_")[3]]
        x4, w4 = workloads.make(4)
        x4, w4 = g(x4), g(w4)
        y = torch.empty(32, 64, 56, 56, device="cuda")
        fn = rotating(x4, y)(lambda xx, yy: B.sws_conv2d_padded(xx, w4, 1, 1, (1, 1, 1, 1), mode, y=yy))
    elif name == "cfg2_conv1d_64x64x3":
        x2, w2 = workloads.make(2)
        x2, w2 = g(x2), g(w2)
        y = torch.empty(16, 64, 4094, device="cuda")
        fn = rotating(x2, y)(lambda xx, yy: B.sws_conv1d(xx, w2, y=yy))
    elif name == "exp_dwconv_k51_d8":
        x7, taps = workloads.make(7)
        x7, taps = g(x7), g(taps)
        k, d = workloads.DILATED_K, workloads.DILATED_D
        y = torch.empty(1, x7.shape[1], x7.shape[2] - (k - 1) * d, device="cuda")
        fn = lambda: B.sws_conv1d(x7, taps, 1, 0, d, x7.shape[1], y=y)
    elif name.startswith("exp_pair_w"):
        w = int(name[len("exp_pair_w"):])
        u, v = workloads.make_pairs()
        u, v = g(u), g(v)
        yu = torch.empty(u.shape[0], u.shape[1] - w + 1, device="cuda")
        yv = torch.empty_like(yu)
        fn = lambda: B.sws_slide1d_pair(u, v, w, yu=yu, yv=yv)
    elif name.startswith("exp_conv1d_k"):
        k = int(name[len("exp_conv1d_k"):])
        x6 = g(workloads.make(6)[0])
        taps = g(workloads.make(6, x_shape=(1,), wgt_shape=(1, 1, k))[1])
        y = torch.empty(x6.shape[0], 1, x6.shape[2] - k + 1, device="cuda")
        fn = lambda: B.sws_conv1d(x6, taps, y=y)
    else:
        raise SystemExit("bench.py --only: unknown operator %r" % name)
    ms = time_launches(torch, fn, steps, warm=2)
    print(json.dumps({"only": name, "launches": steps, "cold": bool(cold), "ms_per_launch": round(ms, 5)}))


def cpu_baseline(x_host, taps_host):
    """The oracle, as it stands, on the whole of configuration 5 (all 32768 rows, the same seven
    operators), in slabs of 8192 rows to bound its fp64 outputs.  GB/s on the same
    algorithmic-byte basis as the GPU figure."""
    import oracle
    slab = 8192
    xs_all = x_host.reshape(ROWS5, LEN5)
    t0 = time.perf_counter()
    nbytes = 0
    for r0 in range(0, ROWS5, slab):
        xs = xs_all[r0:r0 + slab]
        for w in WINDOWS5:
            oracle.slide1d(oracle.OP_ADD, xs, w)
            oracle.slide1d(oracle.OP_MAX, xs, w)
            nbytes += 2 * slide_bytes(slab, LEN5, w)
        oracle.conv1d(xs.reshape(slab // CH5, CH5, LEN5), taps_host, groups=CH5)
        nbytes += slide_bytes(slab, LEN5, K5) + 4 * CH5 * K5
    dt = time.perf_counter() - t0
    cores = oracle.threads()
    # per-core figure: the same seven operators on 1/64 of the rows with one thread
    one = ROWS5 // 64
    xs = xs_all[:one]
    oracle.set_threads(1)
    t1 = time.perf_counter()
    nb1 = 0
    for w in WINDOWS5:
        oracle.slide1d(oracle.OP_ADD, xs, w)
        oracle.slide1d(oracle.OP_MAX, xs, w)
        nb1 += 2 * slide_bytes(one, LEN5, w)
    oracle.conv1d(xs.reshape(one // CH5, CH5, LEN5), taps_host, groups=CH5)
    nb1 += slide_bytes(one, LEN5, K5) + 4 * CH5 * K5
    dt1 = time.perf_counter() - t1
    oracle.set_threads(cores)
    return {"value": round(nbytes / dt / 1e9, 4), "unit": "GB/s", "cores": cores, "kind": "oracle",
            "seconds": round(dt, 3),
            "sample": "all 32768 rows of cfg5, all seven operators, i.e. one whole step "
                      "(fp64 naive O(w*N), OpenMP over rows)",
            "single_core_GBps": round(nb1 / dt1 / 1e9, 4), "single_core_seconds": round(dt1, 3),
            "single_core_sample": "first 512 rows, one thread"}


def main():
    args = parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU (rows / planes / images are independent, so more "
              "GPUs would each take a slice with no communication); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_2305_16513_amd import binding as B, workloads
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    B.lib()                                       # fail loudly if the HIP library is missing
    if args.only:
        for kv in args.opt:
            key, _, val = kv.partition("=")
            B.sws_set_option(key, int(val))
        run_only(torch, B, workloads, args.only, args.steps, args.cold)
        return

    x_host, taps_host = workloads.make(5)
    x = torch.from_numpy(x_host).cuda()
    taps = torch.from_numpy(taps_host).cuda()
    outs = {w: torch.empty(256, 128, LEN5 - w + 1, device="cuda") for w in WINDOWS5}
    y_conv = torch.empty(256, 128, LEN5 - K5 + 1, device="cuda")

    launches = []                                  # (name, fn, algorithmic bytes, flops)
    for w in WINDOWS5:
        nb = slide_bytes(ROWS5, LEN5, w)
        launches.append(("slide_add_w%d" % w, (lambda w=w: B.sws_slide1d(0, x, w, 1.0 / w, y=outs[w])), nb, 0.0))
        launches.append(("slide_max_w%d" % w, (lambda w=w: B.sws_slide1d(1, x, w, 1.0, y=outs[w])), nb, 0.0))
    launches.append(("dwconv_k31", lambda: B.sws_conv1d(x, taps, groups=CH5, y=y_conv),
                     slide_bytes(ROWS5, LEN5, K5) + 4 * CH5 * K5, 2.0 * ROWS5 * (LEN5 - K5 + 1) * K5))
    step_bytes = sum(l[2] for l in launches)

    def step(events=None):
        for i, (_, fn, _, _) in enumerate(launches):
            fn()
            if events is not None:
                events[i].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    ev0 = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps)]
    evs = [[torch.cuda.Event(enable_timing=True) for _ in launches] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        ev0[k].record()
        step(evs[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0

    samples = [[] for _ in launches]               # ms per launch, one sample per step
    for k in range(args.steps):
        prev = ev0[k]
        for i in range(len(launches)):
            samples[i].append(prev.elapsed_time(evs[k][i]))
            prev = evs[k][i]
    per = [sum(v) / len(v) for v in samples]       # mean ms per launch
    ms_step = wall * 1e3 / args.steps

    # the ceiling of a one-read-one-write kernel on this device: a plain copy of the same 2 GiB
    y_copy = outs[WINDOWS5[0]].view(-1)
    n_copy = y_copy.numel()
    copy_ms = time_launches(torch, lambda: B.sws_copy(x.view(-1)[:n_copy], y_copy), max(5, args.steps))
    copy_gbps = 8.0 * n_copy / copy_ms / 1e6
    # and what HBM gives the finest-grained copy (one 1 KB strip per single-wavefront workgroup), which
    # the 4 KB tiles of the scans cannot imitate: the distance between the two is the price of the tile
    B.sws_set_option("copy_variant", 4)
    try:
        fine_ms = time_launches(torch, lambda: B.sws_copy(x.view(-1)[:n_copy], y_copy), max(5, args.steps))
    finally:
        B.sws_set_option("copy_variant", 0)
    fine_gbps = 8.0 * n_copy / fine_ms / 1e6

    kernels = {}
    for (name, _, nb, fl), ms in zip(launches, per):
        rec = {"ms": round(ms, 4), "GBps": round(nb / ms / 1e6, 1), "frac_hbm_peak": round(nb / ms / 1e6 / HBM_PEAK_GBPS, 4)}
        v = sorted(samples[len(kernels)])
        rec["ms_median"] = round(v[len(v) // 2], 4)
        rec["ms_min"] = round(v[0], 4)
        rec["frac_copy_ceiling"] = round(nb / ms / 1e6 / copy_gbps, 4)
        if fl:
            rec["GFLOPs"] = round(fl / ms / 1e6, 1)
        kernels[name] = rec

    # dominant kernel: the one the step spends most time in.  The six sliding-sum launches run the scan kernel
    # (slide_scan_kernel; on inputs of this size with streamed loads for w = 16 and 64), the depthwise convolution
    # the thin-channel kernel.
    scan = list(range(6))
    for i, l in enumerate(launches):
        kernels[l[0]]["kernel"] = "slide_scan_kernel" if i in scan else "conv1d_thin_kernel"
    scan_ms = sum(per[i] for i in scan)
    slide_ms = sum(per[:6])
    if scan_ms >= per[6]:
        dom_name = "slide_scan_kernel (sws_slide1d, w in {16,64,255}, add and max)"
        dom_bytes = sum(launches[i][2] for i in scan) / len(scan)
        dom_ms = scan_ms / len(scan)
        ts = [read_traffic("slide_scan_cfg5_w%d_hbm_traffic.txt" % w) for w in (16, 64, 255)]
        traffic = sum(ts) / 3.0 if all(ts) else None
    else:
        dom_name = "depthwise conv kernel (sws_conv1d, k=31, groups=128)"
        dom_bytes = launches[6][2]
        dom_ms = per[6]
        traffic = read_traffic("dwconv_cfg5_hbm_traffic.txt")
    achieved = dom_bytes / dom_ms / 1e6
    pool_bytes = sum(l[2] for l in launches[:6])
    result = {
        "metric": "sliding pool GB/s (% HBM peak); sliding conv GFLOP/s (% roofline)",
        "value": round(step_bytes / ms_step / 1e6, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "cfg5_large_window_1d: x[256,128,16384] fp32 U[-1,1]; sliding add+max w in {16,64,255}; "
                               "depthwise conv k=31; 7 launches per step",
                   "algorithmic_bytes_per_step": step_bytes},
        "pool_GBps": round(pool_bytes / slide_ms / 1e6, 1),
        "pool_frac_hbm_peak": round(pool_bytes / slide_ms / 1e6 / HBM_PEAK_GBPS, 4),
        "dwconv_GFLOPs": kernels["dwconv_k31"]["GFLOPs"],
        "copy_ceiling": {"GBps": round(copy_gbps, 1), "frac_hbm_peak": round(copy_gbps / HBM_PEAK_GBPS, 4),
                         "what": "sws_copy of 2 GiB -> 2 GiB, the same 128-bit strips with no arithmetic",
                         "fine_grained_copy_GBps": round(fine_gbps, 1), "fine_grained_frac_hbm_peak": round(fine_gbps / HBM_PEAK_GBPS, 4),
                         "fine_grained_what": "the same copy as one 1 KB strip per single-wavefront workgroup (copy_variant 4)"},
        "roofline": {"bound": "hbm", "kernel": dom_name, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS,
                     "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBPS, 4),
                     "avg_launch_ms": round(dom_ms, 4), "algorithmic_bytes_per_launch": dom_bytes,
                     "frac_of_copy_ceiling": round(achieved / copy_gbps, 4), "traffic": traffic},
        "kernels": kernels,
    }
    del outs, y_conv
    torch.cuda.empty_cache()
    if not args.no_ops:
        result["ops"] = ops_table(torch, B, workloads)
        result["experiments"] = sweeps_table(torch, B, workloads)
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(x_host, taps_host)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
