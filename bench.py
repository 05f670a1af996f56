#!/usr/bin/env python3
"""Benchmark of the binarized conv / GEMM path on one MI355X.

A "step" is one pass of the whole hot path over one batch of synthetic input.  The
default workload is the binarized VGG-small stack at batch 256: real-valued first layer
with sign-packed output, six binarized 3x3 convolutions as implicit XOR-popcount GEMMs over
packed NHWC activations (pool + scale/bias + sign + pack in the GEMM epilogue), the binarized
FC layer with fp32 epilogue and the fp32 classifier.  `--stack unfused` runs the same network
through bnn_conv2d (sign-encode, packed operands, int32 NCHW maps, separate glue kernels).
Inputs and pre-encoded weights are resident in HBM before the timed region.  Prints ONE JSON
line; the other configurations, the streaming kernels and the MFMA ablation ride along in it.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload cfg4|cfg2|cfg3|cfg5a|cfg5b]

The defaults (200 warm-up + 1000 timed steps, about a third of a second of GPU time) matter: a
GPU that was idle reaches its sustained clocks only after about 35 ms of continuous work (the
step falls from 0.303 to 0.277 ms over the first 80 steps and stays there), so a run of 5 + 20
steps of this 0.28 ms step, 7 ms in all, reads 9 % slower than the sustained rate.  Such a run
prints the 200 + 1000 figure beside its own, as `sustained`.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np

# Published MI355X figures used as roofline denominators.
HBM_PEAK_GBS = 8000.0
# Vector-ALU ceiling of the method's instruction pair, derived from the chip's unit counts and clock
# (256 compute units x 4 SIMDs, 2.4 GHz).  A wave64 v_xor_b32 issues in 2 clocks on a SIMD, a wave64
# v_bcnt_u32_b32 (popcount-accumulate) in 4: one pair = 2 x 64 lane-operations per 6 clocks per SIMD.
#   1024 SIMDs x 128 lane-ops / 6 clk x 2.4 GHz = 52.43 T lane-ops/s   <- the roofline's `peak`
# The figure with every instruction at 4 clocks (16 lanes per clock and SIMD, half of the chip's
# 157.3 TFLOP/s fp32 vector rate, which counts 2 flops per fma and packed fp32) is kept beside it as
# `peak_nominal_4clk`, and the register-only probe of the GEMM's own row statements, timed in the same
# run, as `peak_measured`.
N_SIMD = 256 * 4
CLOCK_HZ = 2.4e9
VALU_PEAK_TLANEOPS = N_SIMD * 128 / 6.0 * CLOCK_HZ / 1e12  # 52.43
VALU_PEAK_NOMINAL_4CLK = N_SIMD * 16 * CLOCK_HZ / 1e12     # 39.32
BOPS_PER_LANEOP = 32.0  # 2 lane-instructions (xor, popcount-accumulate) per 32 bit-MACs = 64 binary ops

# HBM bytes per launch of xnor_gemm_kernel from rocprofv3 counters, valid for the default workload only
# (profiles/xnor_gemm_cfg4_fused_stack_b256.md, average of the five launches of a step).  Reads: the
# L2's read requests by size class, 128 B x a + 64 B x b = 2751 KiB (exact: the same counters read
# 1 GiB for a 1 GiB copy); writes: WRITE_SIZE 972.8 KiB.  The FETCH_SIZE metric scaled by the copy
# kernel's factor (x 2.00) over-prices this kernel's 64-byte requests and would give 4.83e6.
GEMM_TRAFFIC_BYTES = 3.81e6
GEMM_TRAFFIC_BYTES_FETCH_SIZE_SCALED = 4.83e6


NO_GRAPHS = False


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=1000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--workload", default="cfg4", choices=["cfg4", "cfg2", "cfg3", "cfg5a", "cfg5b"])
    ap.add_argument("--reading", default="A", choices=["A", "B"])
    ap.add_argument("--stack", default="fused", choices=["fused", "unfused"],
                    help="cfg4 only: activations packed between layers (fused) or fp32/int32 NCHW maps (unfused)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-kernel side measurements")
    ap.add_argument("--no-graphs", action="store_true",
                    help="time short kernels with eager launches instead of HIP-graph replays (for runs under rocprofv3 "
                         "--pmc, whose counter collection does not survive a graph replay; the times are then not "
                         "meaningful, the counters are)")
    ap.add_argument("--no-sustained", action="store_true", help="skip the extra 200 + 1000 step run that a short --steps adds")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="target CPU time of the oracle sample")
    return ap.parse_args()


def gemm_laneops(M, N, K):
    return 2.0 * M * N * ((K + 31) // 32)


def time_steps(fn, steps, warmup):
    import torch
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for _ in range(steps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    return e0.elapsed_time(e1) / 1e3, wall


def graph_time(fn, n=20, reps=20, warm=5):
    """GPU seconds per call of fn: n calls captured into one HIP graph (the library neither allocates
    nor synchronises, so the graph holds exactly the calls' kernels), replayed `reps` times between one
    event pair.  Unlike an event pair around every launch (2-3 us on a 10 us kernel) and unlike eager
    launches through the Python binding (the host cannot submit faster than one call per ~8 us), this
    reads what the GPU needs for a short kernel sequence; an empty kernel reads ~3.3 us here."""
    import torch
    if NO_GRAPHS:
        s, _ = time_steps(fn, 20, 5)
        return s / 20
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        fn()
        fn()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        for _ in range(n):
            fn()
    for _ in range(warm):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / 1e3 / (reps * n)


def kernel_times(fn, reps):
    """Per-kernel seconds per step from the library's HIP-event hook (same stream)."""
    import torch
    from paper_1911_04477_amd import binding as B
    B.prof_enable(True)
    try:
        fn()
        torch.cuda.synchronize()
        tot = {}
        cnt = {}
        for _ in range(reps):
            B.prof_reset()
            fn()
            torch.cuda.synchronize()
            for name, ms in B.prof_records():
                tot[name] = tot.get(name, 0.0) + ms / 1e3
                cnt[name] = cnt.get(name, 0) + 1
        return {k: v / reps for k, v in tot.items()}, {k: v // reps for k, v in cnt.items()}
    finally:
        B.prof_enable(False)


def gemm_launches(fn, shapes, reps):
    """Per-launch (kernel name, seconds, lane-ops) of the step's GEMM launches, in launch order.

    The library records one HIP-event pair per launch on the launch stream; the GEMM launches of a
    step come in the order of `shapes`."""
    import torch
    from paper_1911_04477_amd import binding as B
    B.prof_enable(True)
    try:
        fn()
        torch.cuda.synchronize()
        acc = None
        for _ in range(reps):
            B.prof_reset()
            fn()
            torch.cuda.synchronize()
            rec = [(n, ms / 1e3) for n, ms in B.prof_records() if n.startswith("xnor_gemm")]
            assert len(rec) == len(shapes), (len(rec), len(shapes))
            if acc is None:
                acc = [[n, 0.0] for n, _ in rec]
            for a, (_, t) in zip(acc, rec):
                a[1] += t
        return [(n, t / reps, gemm_laneops(*sh)) for (n, t), sh in zip(acc, shapes)]
    finally:
        B.prof_enable(False)


def replay_launches(calls, reps=50, warm=10):
    """Seconds per launch of each closure: `reps` back-to-back launches between ONE pair of HIP events
    on the launch stream, so the few microseconds an event pair adds around a single short launch
    are spread over `reps` launches."""
    out = []
    for call in calls:
        s, _ = time_steps(call, reps, warm)
        out.append(s / reps)
    return out


def build_workload(name, args):
    """Returns dict(fn, bops, gemm_shapes, label, oracle_fn(sample) -> (bops_done, seconds))."""
    import torch
    from paper_1911_04477_amd import binding as B
    from paper_1911_04477_amd import inputs
    dev = "cuda:0"

    def up(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(dev)

    if name == "cfg4":
        from paper_1911_04477_amd.stack import VggStack, VggStackFused
        batch = 256
        d = inputs.cfg4(batch=batch, reading=args.reading)
        net = (VggStackFused if args.stack == "fused" else VggStack)(d["layers"], d["params"], batch=batch, device=dev)
        x = up(d["x"])
        shapes = []
        for L in d["layers"]:
            if L.kind == "bconv":
                shapes.append((L.cout, batch * L.hw * L.hw, L.cin * 9))
            elif L.kind == "bfc":
                shapes.append((batch, L.cout, L.cin))
        bit_macs = inputs.stack_bit_macs(d["layers"], batch)

        def oracle_sample(seconds):
            import oracle
            t0 = time.perf_counter()
            oracle.vgg_stack(d["x"][:1], d["layers"], d["params"])
            t1 = time.perf_counter() - t0
            n = int(max(1, min(batch, seconds / max(t1, 1e-3))))
            t0 = time.perf_counter()
            oracle.vgg_stack(d["x"][:n], d["layers"], d["params"])
            dt = time.perf_counter() - t0
            return 2.0 * inputs.stack_bit_macs(d["layers"], n), dt, f"{n} of {batch} images through the whole stack"

        replay = None
        if args.stack == "fused":
            net.forward(x)  # fills the inter-layer buffers the per-layer closures launch on
            torch.cuda.synchronize()
            replay = net.conv_launches()
        split = None
        if args.stack == "fused":
            from paper_1911_04477_amd.stack import SplitBatch
            sb = SplitBatch(d["layers"], d["params"], batch=batch, parts=2, device=dev)
            split = sb
        return dict(fn=lambda: net.forward(x), bops=2.0 * bit_macs, gemm_shapes=shapes, replay=replay, split=split, split_input=x,
                    label=f"cfg4_vgg_small_stack_b{batch}_reading{args.reading}_{args.stack}", oracle=oracle_sample,
                    extra={"batch": batch, "reading": args.reading, "activations": "packed 1-bit NHWC between layers"
                           if args.stack == "fused" else "fp32 / int32 NCHW maps between layers"})

    if name == "cfg2":
        d = inputs.cfg2()
        s = inputs.CFG2
        act, wp = up(d["act"]), B.bnn_encode(up(d["wt"]))
        sc, bi = up(d["scale"]), up(d["bias"])
        ap = torch.empty((s.M, B.packed_words(s.K)), dtype=torch.int64, device=dev)

        yout = torch.empty((s.M, s.N), dtype=torch.float32, device=dev)

        def fn():
            B.bnn_encode(act, ap)
            B.bnn_xnor_gemm_epilogue(ap, wp, s.K, sc, bi, B.CH_COL, out_y=yout)

        def gemm_fn():
            B.bnn_xnor_gemm_epilogue(ap, wp, s.K, sc, bi, B.CH_COL, out_y=yout)

        def oracle_sample(seconds):
            import oracle
            rows = 16
            t0 = time.perf_counter()
            oracle.scale_bias(oracle.gemm_pm1(d["act"][:rows], d["wt"]), d["scale"], d["bias"], "col")
            t1 = time.perf_counter() - t0
            n = int(max(rows, min(s.M, rows * seconds / max(t1, 1e-3))))
            t0 = time.perf_counter()
            oracle.scale_bias(oracle.gemm_pm1(d["act"][:n], d["wt"]), d["scale"], d["bias"], "col")
            return 2.0 * n * s.N * s.K, time.perf_counter() - t0, f"{n} of {s.M} activation rows"

        return dict(fn=fn, gemm_fn=gemm_fn, bops=2.0 * s.M * s.N * s.K, gemm_shapes=[(s.M, s.N, s.K)],
                    label="cfg2_binarized_fc_256x4096x4096", oracle=oracle_sample, extra={})

    shape = {"cfg3": inputs.CFG3, "cfg5a": inputs.CFG5A, "cfg5b": inputs.CFG5B}[name]
    d = {"cfg3": inputs.cfg3, "cfg5a": inputs.cfg5a, "cfg5b": inputs.cfg5b}[name]()
    x, wp = up(d["x"]), B.bnn_pack_conv_weight(up(d["w"]))
    st, pd = (shape.sH, shape.sW), (shape.pH, shape.pW)
    ws = torch.empty(B.conv2d_workspace_bytes(x.shape, shape.kH, shape.kW, st, pd), dtype=torch.uint8, device=dev)
    out = torch.empty((shape.N, shape.D, shape.OH, shape.OW), dtype=torch.int32, device=dev)

    def fn():
        B.bnn_conv2d(x, wp, shape.D, shape.kH, shape.kW, st, pd, want_int=True, workspace=ws, out_i32=out)

    # the GEMM alone: the same convolution on the packed image the encode left in the workspace
    fn()
    if shape.kH == 1:
        img = ws[:shape.P * B.packed_words(shape.C) * 8].view(torch.int64).view(shape.N, shape.OH, shape.OW, -1)
        gst = (1, 1)
    else:
        img = ws[:shape.N * shape.H * shape.W * B.packed_words(shape.C) * 8].view(torch.int64).view(shape.N, shape.H,
                                                                                                   shape.W, -1)
        gst = st

    def gemm_fn():
        B.bnn_conv2d_packed(img, wp, shape.C, shape.D, shape.kH, shape.kW, gst, pd, out="i32", out_buf=out)

    def oracle_sample(seconds):
        import oracle
        t0 = time.perf_counter()
        oracle.conv2d_pm1(d["x"][:1], d["w"], st, pd)
        t1 = time.perf_counter() - t0
        n = int(max(1, min(shape.N, seconds / max(t1, 1e-3))))
        t0 = time.perf_counter()
        oracle.conv2d_pm1(d["x"][:n], d["w"], st, pd)
        return 2.0 * shape.bit_macs * n / shape.N, time.perf_counter() - t0, f"{n} of {shape.N} images"

    return dict(fn=fn, gemm_fn=gemm_fn, bops=2.0 * shape.bit_macs, gemm_shapes=[(shape.D, shape.P, shape.K)],
                label=f"{name}_binarized_conv_{shape.N}x{shape.C}x{shape.H}x{shape.W}_to_{shape.D}_k{shape.kH}s{shape.sH}p{shape.pH}",
                oracle=oracle_sample, extra={})


def side_measurements():
    """Streaming kernels against the HBM roof, the VALU probe, and the other configurations."""
    import torch
    from paper_1911_04477_amd import binding as B
    from paper_1911_04477_amd import inputs
    dev = "cuda:0"
    res = {}

    def t(fn, reps=100, warm=100):
        # memory-bound kernels also need tens of milliseconds of continuous work to reach their sustained rate
        s, _ = time_steps(fn, reps, warm)
        return s / reps

    def kt_warm(fn, reps=20, warm=30):
        for _ in range(warm):
            fn()
        return kernel_times(fn, reps)[0]

    # plain copy: the achievable-HBM yardstick (1 GiB read + 1 GiB written)
    n = 1 << 30
    a = torch.empty(n, dtype=torch.uint8, device=dev).random_(0, 255)
    b = torch.empty(n, dtype=torch.uint8, device=dev)
    dt = t(lambda: B.bnn_copy_probe(a, b))
    res["copy_probe_GBs"] = round(2 * n / dt / 1e9, 1)
    del b
    # row-major encode, 1 GiB of fp32 (streams from HBM) and the cfg2 weight matrix (64 MiB)
    src = a.view(torch.float32).view(-1, 4096)
    dst = torch.empty((src.shape[0], 64), dtype=torch.int64, device=dev)
    dt = t(lambda: B.bnn_encode(src, dst))
    res["encode_1GiB_GBs"] = round((src.numel() * 4 + dst.numel() * 8) / dt / 1e9, 1)
    w = src[:4096]
    dt = t(lambda: B.bnn_encode(w, dst[:4096]))
    res["encode_cfg2_weights_GBs"] = round((w.numel() * 4 + 4096 * 64 * 8) / dt / 1e9, 1)
    del src, dst, a
    # input encode + packed im2col at the conv configurations: the whole bnn_im2col_packed call (one or
    # two kernels) by graph replay, its kernels by the event hook, and a plain copy moving the same
    # number of bytes beside it
    for name, shape in (("cfg3", inputs.CFG3), ("cfg5a", inputs.CFG5A), ("cfg5b", inputs.CFG5B)):
        x = torch.randn((shape.N, shape.C, shape.H, shape.W), device=dev)
        st, pd = (shape.sH, shape.sW), (shape.pH, shape.pW)
        Cw = B.packed_words(shape.C)
        Kw = B.conv_kwords(shape.C, shape.kH, shape.kW)
        cols = torch.empty((shape.P, Kw), dtype=torch.int64, device=dev)
        wsb = torch.empty(max(16, B.im2col_workspace_bytes(x.shape, shape.kH, shape.kW, st, pd)), dtype=torch.uint8,
                          device=dev)
        fn = lambda: B.bnn_im2col_packed(x, shape.kH, shape.kW, st, pd, cols=cols, workspace=wsb)
        tot = graph_time(fn)
        kt = kt_warm(fn)
        # algorithmic bytes: the fp32 values the convolution uses + the patch matrix written
        used = x.numel() * 4 * (0.25 if shape.sH == 2 else 1.0)
        byts = used + shape.P * Kw * 8
        res[f"{name}_im2col_total_GBs"] = round(byts / tot / 1e9, 1)
        res[f"{name}_im2col_total_us"] = round(tot * 1e6, 2)
        half = int(byts // 32) * 16
        ca = torch.empty(half, dtype=torch.uint8, device=dev)
        cb = torch.empty(half, dtype=torch.uint8, device=dev)
        res[f"{name}_copy_same_bytes_us"] = round(graph_time(lambda: B.bnn_copy_probe(ca, cb)) * 1e6, 2)
        if "encode_nchw" in kt:
            eb = (shape.P * shape.C * 4 + shape.P * Cw * 8) if shape.kH == 1 else (x.numel() * 4 + shape.N * shape.H * shape.W * Cw * 8)
            res[f"{name}_encode_nchw_GBs_event_hook"] = round(eb / kt["encode_nchw"] / 1e9, 1)
        if "im2col_gather" in kt:
            gb = shape.P * Kw * 8 + shape.N * shape.H * shape.W * Cw * 8
            res[f"{name}_im2col_gather_GBs_event_hook"] = round(gb / kt["im2col_gather"] / 1e9, 1)
        del x, cols, wsb, ca, cb
    # the same two kernels on an input several times larger than the 256 MB last-level cache:
    # encode 822 MB in / 26 MB out; gather 26 MB in / 231 MB out
    x = torch.randn((256, 256, 56, 56), device=dev)
    kt = kt_warm(lambda: B.bnn_im2col_packed(x, 3, 3, (1, 1), (1, 1)))
    pix = 256 * 56 * 56
    res["encode_nchw_822MB_with_gather_between_GBs"] = round((x.numel() * 4 + pix * 4 * 8) / kt["encode_nchw"] / 1e9, 1)
    res["im2col_gather_231MB_GBs"] = round((pix * 4 * 8 + pix * 36 * 8) / kt["im2col_gather"] / 1e9, 1)
    kt = kt_warm(lambda: B.bnn_im2col_packed(x, 1, 1, (1, 1), (0, 0)))  # pointwise: the encode alone
    res["encode_nchw_822MB_GBs"] = round((x.numel() * 4 + pix * 4 * 8) / kt["encode_nchw"] / 1e9, 1)
    del x
    return res


def valu_probes():
    """Register-only yardsticks (no loads): T lane-ops/s of independent xor + popcount pairs as the
    compiler schedules them, and of the GEMM's own row statements (4 and 2 column groups per lane)."""
    import torch
    from paper_1911_04477_amd import binding as B
    blocks, iters = 256 * 16, 2000
    sink = torch.empty(blocks * 256, dtype=torch.int32, device="cuda:0")
    out = {}
    for name, kind in (("independent_pairs", 0), ("gemm_rows_tn4", 4), ("gemm_rows_tn2", 2)):
        s, _ = time_steps(lambda: B.bnn_valu_peak_probe(sink, blocks, iters, kind), 20, 10)
        out[name] = round(blocks * 256 * iters * 128 / (s / 20) / 1e12, 2)
    return out


def small_batch_latency(args):
    """One pass of the fused stack at small batch sizes, launched eagerly (eight launches through
    the Python binding) and as one replay of a captured HIP graph: a pass at these sizes is
    shorter than its launches take to submit."""
    import torch
    from paper_1911_04477_amd import inputs
    from paper_1911_04477_amd.stack import VggStackFused
    out = {}
    for batch in (1, 8, 32):
        d = inputs.cfg4(batch=batch, reading=args.reading)
        net = VggStackFused(d["layers"], d["params"], batch=batch, device="cuda:0")
        x = torch.from_numpy(d["x"]).to("cuda:0")
        net.capture(x)
        res = {}
        for name, fn in (("eager", lambda: net.forward(x)), ("graph", net.replay)):
            for _ in range(200):
                fn()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(500):
                fn()
            torch.cuda.synchronize()
            res[name + "_us"] = round((time.perf_counter() - t0) / 500 * 1e6, 1)
        res["images_per_s_graph"] = round(batch / (res["graph_us"] * 1e-6))
        out[f"batch{batch}"] = res
    return out


def mfma_ablation():
    """The MFMA ablations beside the VALU GEMM on the GEMM view of cfg 5a and cfg 3: int8 and fp4 with the
    bits expanded on the fly, and fp4 on operands kept expanded in memory (the expansion timed apart)."""
    import torch
    from paper_1911_04477_amd import binding as B
    dev = "cuda:0"
    out = {}
    for name, (M, N, K) in (("cfg5a_gemm_256x200704x2304", (256, 200704, 2304)),
                            ("cfg3_gemm_128x131072x1152", (128, 131072, 1152))):
        Kw = (K + 63) // 64
        A = torch.randint(-2**62, 2**62, (M, Kw), dtype=torch.int64, device=dev)
        Bm = torch.randint(-2**62, 2**62, (N, Kw), dtype=torch.int64, device=dev)
        C = torch.empty((M, N), dtype=torch.int32, device=dev)
        C2 = torch.empty((M, N), dtype=torch.int32, device=dev)
        C3 = torch.empty((M, N), dtype=torch.int32, device=dev)
        C4 = torch.empty((M, N), dtype=torch.int32, device=dev)
        A4, B4 = B.bnn_expand_fp4(A, K), B.bnn_expand_fp4(Bm, K)
        tv, _ = time_steps(lambda: B.bnn_xnor_gemm(A, Bm, K, C), 200, 100)
        tm, _ = time_steps(lambda: B.bnn_xnor_gemm_mfma_i8(A, Bm, K, C2), 200, 100)
        t4, _ = time_steps(lambda: B.bnn_xnor_gemm_mfma_fp4(A, Bm, K, C3), 200, 100)
        tx, _ = time_steps(lambda: B.bnn_xnor_gemm_mfma_fp4_expanded(A4, B4, K, C4), 200, 100)
        te, _ = time_steps(lambda: B.bnn_expand_fp4(Bm, K, out=B4), 200, 100)
        bops = 2.0 * M * N * K
        moved = A4.numel() + B4.numel() + 4 * M * N   # bytes the expanded form reads and writes once
        out[name] = {"valu_TBOPS": round(bops / (tv / 200) / 1e12, 1), "mfma_i8_TBOPS": round(bops / (tm / 200) / 1e12, 1),
                     "mfma_fp4_TBOPS": round(bops / (t4 / 200) / 1e12, 1),
                     "mfma_fp4_expanded_TBOPS": round(bops / (tx / 200) / 1e12, 1),
                     "bit_identical": bool((C == C2).all().item() and (C == C3).all().item()
                                           and (C == C4).all().item()),
                     "mfma_i8_frac_of_int8_dense_peak": round(bops / (tm / 200) / 5.0e15, 4),
                     "mfma_fp4_frac_of_fp4_dense_peak": round(bops / (t4 / 200) / 10.1e15, 4),
                     "mfma_fp4_expanded_frac_of_fp4_dense_peak": round(bops / (tx / 200) / 10.1e15, 4),
                     "mfma_fp4_expanded_GBs": round(moved / (tx / 200) / 1e9, 1),
                     "expand_B_us": round(te / 200 * 1e6, 1),
                     "expand_B_GBs": round((Bm.numel() * 8 + B4.numel()) / (te / 200) / 1e9, 1)}
        del A, Bm, C, C2, C3, C4, A4, B4
    # the same ablation as a convolution: patches gathered inside the GEMM from a 4-bit NHWC image,
    # beside the VALU convolution from the 1-bit image (both int32 NCHW out, images already in their format)
    for name, (N, Cc, H, W, D) in (("cfg5a_conv_64x256x56x56_to_256", (64, 256, 56, 56, 256)),
                                   ("cfg3_conv_128x128x32x32_to_128", (128, 128, 32, 32, 128))):
        Cw = Cc // 64
        xp = torch.randint(-2**62, 2**62, (N, H, W, Cw), dtype=torch.int64, device=dev)
        wp = torch.randint(-2**62, 2**62, (D, 9 * Cw), dtype=torch.int64, device=dev)
        x4 = B.bnn_expand_fp4(xp.view(N * H * W, Cw), Cc).view(N, H, W, Cc // 2)
        w4 = B.bnn_expand_fp4(wp, 9 * Cc)
        o1 = torch.empty((N, D, H, W), dtype=torch.int32, device=dev)
        o2 = torch.empty((N, D, H, W), dtype=torch.int32, device=dev)
        tv, _ = time_steps(lambda: B.bnn_conv2d_packed(xp, wp, Cc, D, 3, 3, (1, 1), (1, 1), out="i32", out_buf=o1), 200, 100)
        tx, _ = time_steps(lambda: B.bnn_conv2d_mfma_fp4_expanded(x4, w4, Cc, D, 3, 3, (1, 1), (1, 1), out=o2), 200, 100)
        te = graph_time(lambda: B.bnn_expand_fp4(xp.view(N * H * W, Cw), Cc, out=x4.view(N * H * W, Cc // 2)))
        bops = 2.0 * N * H * W * D * 9 * Cc
        out[name] = {"valu_TBOPS": round(bops / (tv / 200) / 1e12, 1),
                     "mfma_fp4_expanded_TBOPS": round(bops / (tx / 200) / 1e12, 1),
                     "bit_identical": bool((o1 == o2).all().item()),
                     "mfma_fp4_expanded_frac_of_fp4_dense_peak": round(bops / (tx / 200) / 10.1e15, 4),
                     "expand_image_us": round(te * 1e6, 1)}
        del xp, wp, x4, w4, o1, o2
    return out


def control_group():
    """The paper's float control group on this machine: the same convolution as an fp32 MFMA GEMM on
    sign(x), sign(w) (implicit GEMM, no patch matrix) beside the Xnor-Bitcount path (bnn_conv2d)."""
    import torch
    from paper_1911_04477_amd import binding as B
    from paper_1911_04477_amd import inputs
    dev = "cuda:0"
    out = {}
    for name, shape in (("cfg3", inputs.CFG3), ("cfg5a", inputs.CFG5A)):
        x = torch.randn((shape.N, shape.C, shape.H, shape.W), device=dev)
        w = torch.randn((shape.D, shape.C, shape.kH, shape.kW), device=dev)
        st, pd = (shape.sH, shape.sW), (shape.pH, shape.pW)
        yf = torch.empty((shape.N, shape.D, shape.OH, shape.OW), dtype=torch.float32, device=dev)
        yi = torch.empty((shape.N, shape.D, shape.OH, shape.OW), dtype=torch.int32, device=dev)
        wp = B.bnn_pack_conv_weight(w)
        ws = torch.empty(B.conv2d_workspace_bytes(x.shape, shape.kH, shape.kW, st, pd), dtype=torch.uint8, device=dev)
        tc, _ = time_steps(lambda: B.bnn_control_conv2d_f32(x, w, st, pd, yf), 30, 10)
        tb, _ = time_steps(lambda: B.bnn_conv2d(x, wp, shape.D, shape.kH, shape.kW, st, pd, want_int=True, workspace=ws,
                                               out_i32=yi), 300, 100)
        tc, tb = tc / 30, tb / 300
        flops = 2.0 * shape.bit_macs
        out[name] = {"control_fp32_ms": round(tc * 1e3, 4), "control_TFLOPs": round(flops / tc / 1e12, 1),
                     "control_frac_of_fp32_mfma_peak": round(flops / tc / 157.3e12, 4),
                     "xnor_ms": round(tb * 1e3, 4), "speedup": round(tc / tb, 2),
                     "speedup_vs_fp32_mfma_peak": round(flops / 157.3e12 / tb, 2),
                     "same_result": bool((yf == yi.to(torch.float32)).all().item())}
        del x, w, yf, yi, ws
    return out


def unfused_stack(args):
    """The same network through bnn_conv2d and the glue kernels (sign-encode, implicit GEMM with int32 /
    fp32 NCHW maps, separate max-pool): every step of the path as its own kernel."""
    import torch
    from paper_1911_04477_amd import inputs
    from paper_1911_04477_amd.stack import VggStack
    d = inputs.cfg4(batch=256, reading=args.reading)
    net = VggStack(d["layers"], d["params"], batch=256, device="cuda:0")
    x = torch.from_numpy(np.ascontiguousarray(d["x"])).to("cuda:0")
    s, _ = time_steps(lambda: net.forward(x), 300, 100)
    kt, _ = kernel_times(lambda: net.forward(x), 10)
    per = s / 300
    return {"ms_per_step": round(per * 1e3, 4),
            "TBOPS": round(2.0 * inputs.stack_bit_macs(d["layers"], 256) / per / 1e12, 2),
            "kernels_ms": {k: round(v * 1e3, 4) for k, v in kt.items()}}


def other_configs(args):
    """The other configurations: whole call and GEMM alone, GPU time per call from graph replays (these
    kernels last 10-200 us; see graph_time), and the per-kernel split from the library's event hook."""
    out = {}
    for name in ("cfg2", "cfg3", "cfg5a", "cfg5b"):
        wl = build_workload(name, args)
        per = graph_time(wl["fn"])
        g = graph_time(wl["gemm_fn"])
        kt, _ = kernel_times(wl["fn"], 10)
        lane = sum(gemm_laneops(*sh) for sh in wl["gemm_shapes"])
        out[name] = {"TBOPS_end_to_end": round(wl["bops"] / per / 1e12, 2), "ms": round(per * 1e3, 4),
                     "gemm_ms": round(g * 1e3, 4), "TBOPS_gemm_only": round(wl["bops"] / g / 1e12, 2),
                     "gemm_frac_valu_peak": round(lane / g / 1e12 / VALU_PEAK_TLANEOPS, 4),
                     "kernels_ms_event_hook": {k: round(v * 1e3, 4) for k, v in kt.items()}}
        if name == "cfg5b":
            sh = inputs_shape("cfg5b")
            out[name]["gemm_store_GBs"] = round(sh.D * sh.P * 4 / g / 1e9, 1)
        del wl
    return out


def inputs_shape(name):
    from paper_1911_04477_amd import inputs
    return {"cfg3": inputs.CFG3, "cfg5a": inputs.CFG5A, "cfg5b": inputs.CFG5B}[name]


def reading_b_step(args):
    """Config 4 under its second reading (six binarized convolutions after the real-valued one)."""
    import torch
    from paper_1911_04477_amd import inputs
    from paper_1911_04477_amd.stack import VggStackFused
    d = inputs.cfg4(batch=256, reading="B")
    net = VggStackFused(d["layers"], d["params"], batch=256, device="cuda:0")
    x = torch.from_numpy(np.ascontiguousarray(d["x"])).to("cuda:0")
    s, _ = time_steps(lambda: net.forward(x), 500, 200)
    per = s / 500
    bops = 2.0 * inputs.stack_bit_macs(d["layers"], 256)
    return {"ms_per_step": round(per * 1e3, 4), "TBOPS": round(bops / per / 1e12, 2), "GBOP_per_step": round(bops / 1e9, 1)}


def main():
    global NO_GRAPHS
    args = parse_args()
    NO_GRAPHS = args.no_graphs
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no collectives, no sharding); --gpus must be 1", file=sys.stderr)
        sys.exit(2)
    import torch
    from paper_1911_04477_amd import binding as B
    B.lib()  # fail loudly if the HIP library is missing
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)

    wl = build_workload(args.workload, args)
    secs, _wall = time_steps(wl["fn"], args.steps, args.warmup)
    per_step = secs / args.steps
    value = wl["bops"] / per_step / 1e12

    # dominant kernel: the XOR-popcount GEMM kernel that takes most of the step, timed per launch with
    # HIP events on the launch stream
    reps = max(3, min(args.steps, 10))
    kt, kc = kernel_times(wl["fn"], reps)
    launches = gemm_launches(wl["fn"], wl["gemm_shapes"], reps)
    by_name = {}
    for n, t, ops in launches:
        e = by_name.setdefault(n, [0.0, 0.0, 0])
        e[0] += t
        e[1] += ops
        e[2] += 1
    dom = max(by_name, key=lambda n: by_name[n][0])
    dom_s, dom_ops, dom_n = by_name[dom]
    gemm_s = sum(t for _, t, _ in launches)
    method = "one HIP-event pair around each launch inside a pass of the stack (library hook)"
    per_launch = [{"kernel": n, "ms": round(t * 1e3, 4), "frac": round(ops / t / 1e12 / VALU_PEAK_TLANEOPS, 4)}
                  for n, t, ops in launches]
    if wl.get("replay"):
        # the stack's xnor_gemm_kernel launches, each replayed back to back between one event pair
        idx = [i for i, (n, _, _) in enumerate(launches) if n == dom]
        assert len(idx) == len(wl["replay"]), (len(idx), len(wl["replay"]))
        rt = replay_launches(wl["replay"])
        dom_s = sum(rt)
        gemm_s = gemm_s - sum(launches[i][1] for i in idx) + dom_s
        for i, t in zip(idx, rt):
            per_launch[i]["ms_replayed"] = round(t * 1e3, 4)
            per_launch[i]["frac"] = round(launches[i][2] / t / 1e12 / VALU_PEAK_TLANEOPS, 4)
        method = "each launch of the step replayed 50x back to back between one HIP-event pair on the launch stream"
    achieved = dom_ops / dom_s / 1e12
    default_wl = args.workload == "cfg4" and args.reading == "A" and args.stack == "fused"
    probes = valu_probes()
    fracs = [achieved / VALU_PEAK_TLANEOPS] + [e["frac"] for e in per_launch]
    if max(fracs) > 1.0:
        print(f"bench.py: WARNING roofline fraction above 1 ({max(fracs):.4f}): the derived peak is not a ceiling",
              file=sys.stderr)
    roofline = {
        "kernel": {"xnor_gemm": "xnor_gemm_kernel", "xnor_gemm_small": "xnor_gemm_direct_kernel / 32x64 tiles"}.get(dom, dom),
        "bound": "alu", "achieved": round(achieved, 3), "peak": round(VALU_PEAK_TLANEOPS, 2),
        "unit": "Tlaneop/s", "frac": round(achieved / VALU_PEAK_TLANEOPS, 4),
        "peak_nominal_4clk": round(VALU_PEAK_NOMINAL_4CLK, 2),
        "peak_measured": probes["gemm_rows_tn4"], "frac_of_peak_measured": round(achieved / probes["gemm_rows_tn4"], 4),
        "valu_probes_Tlaneops": probes,
        "all_fracs_le_1": bool(max(fracs) <= 1.0),
        "traffic": GEMM_TRAFFIC_BYTES if default_wl else None,
        "traffic_fetch_size_x2": GEMM_TRAFFIC_BYTES_FETCH_SIZE_SCALED if default_wl else None,
        "launches_per_step": dom_n, "avg_launch_ms": round(dom_s / dom_n * 1e3, 4),
        "per_launch": per_launch,
        "gemm_only_TBOPS": round(wl["bops"] / gemm_s / 1e12, 2),
        "timing": method,
        "note": "achieved = 2*M*N*ceil(K/32) lane-ops of the dominant kernel's launches in one step / their summed "
                "duration; peak = 1024 SIMDs x (2 x 64 lane-ops per xor+popcount pair) / (2 + 4 clocks) x 2.4 GHz: the issue "
                "ceiling of the method's instruction pair; peak_nominal_4clk = 16 lanes per clock and SIMD; peak_measured = "
                "the GEMM's row statements from registers, no loads, timed in this run; traffic = HBM bytes per launch of that kernel (rocprofv3: read requests by size class + WRITE_SIZE; "
                "traffic_fetch_size_x2 = FETCH_SIZE scaled by the copy kernel's factor + WRITE_SIZE, an over-estimate here)",
    }

    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        done, dt, what = wl["oracle"](args.cpu_seconds)
        cpu = {"value": round(done / dt / 1e12, 6), "unit": "TBOPS", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": what, "seconds": round(dt, 2)}

    line = {
        "metric": "binary_ops_per_sec", "value": round(value, 3), "unit": "TBOPS", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(per_step * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "u32", "data": "synthetic",
        "config": dict({"workload": wl["label"]}, **wl["extra"]),
        "roofline": roofline, "cpu_baseline": cpu,
        "kernels_ms_per_step": {k: round(v * 1e3, 4) for k, v in kt.items()},
    }
    if wl.get("split"):
        # throughput mode: every batch as two half batches on two streams, successive batches free to
        # overlap (images are independent); fork before the first step, join after the last
        sb = wl["split"]
        xin = wl["split_input"]
        for _ in range(args.warmup):
            sb.forward(xin)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        sb.fork()
        for _ in range(args.steps):
            sb.forward(xin, sync=False)
        sb.join()
        e1.record()
        torch.cuda.synchronize()
        s2 = e0.elapsed_time(e1) / 1e3
        line["two_half_batches_on_two_streams"] = {"ms_per_step": round(s2 / args.steps * 1e3, 4),
                                                   "TBOPS": round(wl["bops"] / (s2 / args.steps) / 1e12, 3)}
    def side(name, fn):
        # a side measurement must never cost the line its headline figures
        try:
            line[name] = fn()
        except Exception as e:  # noqa: BLE001
            line[name] = {"error": f"{type(e).__name__}: {e}"[:300]}
            print(f"bench.py: side measurement {name} failed: {e}", file=sys.stderr)

    if (args.steps < 200 or args.warmup < 100) and not args.no_sustained:
        # the same step after the clocks have settled (a few hundred steps of continuous work)
        def sustained():
            s3, _ = time_steps(wl["fn"], 1000, 200)
            return {"steps": 1000, "warmup": 200, "ms_per_step": round(s3 / 1000 * 1e3, 4),
                    "value": round(wl["bops"] / (s3 / 1000) / 1e12, 3)}
        side("sustained", sustained)
    if not args.no_extras:
        side("streaming", side_measurements)
        line["hbm_peak_GBs"] = HBM_PEAK_GBS
        if args.workload == "cfg4" and args.stack == "fused":
            side("unfused_stack", lambda: unfused_stack(args))
            if args.reading == "A":
                side("reading_B_fused_stack", lambda: reading_b_step(args))
            if not args.no_graphs:
                side("small_batch_latency", lambda: small_batch_latency(args))
        side("other_configs", lambda: other_configs(args))
        side("mfma_ablation", mfma_ablation)
        side("control_group", control_group)
    print(json.dumps(line), flush=True)


if __name__ == "__main__":
    main()
