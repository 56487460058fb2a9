#!/usr/bin/env python3
"""Benchmark of the Bolt hot path on one MI355X.

A "step" is one pass over the whole hot path on resident synthetic inputs:
  config 1 (GEMM+bias+ReLU), config 2 (3x3 conv), config 3 (fused b2b GEMM), config 4 (fused b2b
  conv) and config 5 (the 53 conv layers of a ResNet-50-shaped stack at batch 32, the stem reading its
  3-channel input unpadded through the first-layer kernel), every kernel with the template parameters
  bolt_tune picked for its shape (tuning happens before the timed region).
value = useful FP16 FLOPs of one step / time of one step, in TFLOP/s.

Prints ONE JSON line.  Besides the contract fields it carries
  roofline     -- the dominant kernel (the implicit-GEMM conv template over the 54 conv launches of
                  a step): algorithmic FLOPs / average launch duration against the FP16 MFMA peak
  cpu_baseline -- the CPU oracle timed on this machine's host cores on a bounded sample
  shapes       -- per-shape TFLOP/s, fraction of MFMA / HBM roofline and the chosen template
  b2b          -- fused vs unfused-pair time for configs 3 and 4
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

MFMA_PEAK_TFLOPS = 2500.0   # MI355X FP16 dense
HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the oracle timing (profiling runs)")
    ap.add_argument("--reps", type=int, default=50, help="launches per shape for the per-shape table")
    ap.add_argument("--tune-cache", default=None, help="JSON file of tuned configs: loaded if present, else written")
    ap.add_argument("--eager-timing", action="store_true",
                    help="time the per-shape tables with eager launch loops instead of graph replays")
    ap.add_argument("--graph", action="store_true",
                    help="replay two captured HIP graphs per step instead of launching every op eagerly "
                         "(measured: no faster on MI355X, the default stays eager)")
    ap.add_argument("--no-cold", action="store_true", help="skip the cold (rotating buffer sets) column of the HBM-bound rows")
    ap.add_argument("--large-only", action="store_true",
                    help="profiling runs: only the large-shape table (8192^3, 4096^3, the FFN GEMM, the batch-128 conv)")
    ap.add_argument("--steps-only", action="store_true",
                    help="profiling runs: only warm-up + timed steps (no per-shape table, no probes, no oracle)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path would shard by batch, "
              "weights replicated, with no collective)" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    import paper_2110_15238_amd as bolt
    import workloads as wl

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    stream = torch.cuda.current_stream()

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).cuda()

    def empty(*shape):
        return torch.empty(shape, dtype=torch.float16, device="cuda")

    REPS_MEDIAN = 5

    def timed(fn, reps):
        """GPU ms per call of fn: the median of REPS_MEDIAN repetitions, each `reps` calls enqueued back to back on
        the launch stream between two events (Section 4's protocol of averaged repeated runs; the median of
        five repetitions rejects the occasional slow one).

        The calls are captured into a HIP graph once and every repetition is one replay: issuing a call from
        Python costs ~5 us of host time, as much as the shortest kernels run, so an eager loop would time the
        interpreter for them and flatter "fused vs unfused" (the unfused side pays two calls).  Nothing the library
        enqueues is a memset or an allocation, so every captured call is a chain of plain kernel nodes.
        --eager-timing times eager loops instead."""
        for _ in range(3):
            fn()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        g = None
        if not args.eager_timing:
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for _ in range(reps):
                    fn()
            g.replay()  # warm
        times = []
        for _ in range(REPS_MEDIAN):
            e0.record(stream)
            if g is None:
                for _ in range(reps):
                    fn()
            else:
                g.replay()
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_time(e1) / reps)
        return float(np.median(times))

    def timed_cold(make_run, set_bytes, reps):
        """GPU ms per call on inputs and outputs no cache holds: enough distinct buffer sets (at least 5, together more
        than the 256 MB memory-side cache plus the L2s) are visited round-robin, so every launch finds its
        activations, weights and output lines evicted by the launches since its set's previous turn.  One graph
        replay is one pass over the sets; median of REPS_MEDIAN replays."""
        nsets = max(5, int(np.ceil(320e6 / max(set_bytes, 1))))
        nsets = min(nsets, 64)
        runs = [make_run() for _ in range(nsets)]
        for r in runs:
            r()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for r in runs:
                r()
        g.replay()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        times = []
        for _ in range(REPS_MEDIAN):
            e0.record(stream)
            g.replay()
            e1.record(stream)
            e1.synchronize()
            times.append(e0.elapsed_time(e1) / nsets)
        del g, runs
        return float(np.median(times)), nsets

    ws = torch.empty(64 << 20, dtype=torch.uint8, device="cuda")  # split-K workspace shared by all ops

    cache = {}
    if args.tune_cache and os.path.exists(args.tune_cache):
        cache = json.load(open(args.tune_cache))

    def tuned(name, op, d0, d1, tensors, workspace=None):
        """bolt_tune, or the config stored under `name` by an earlier run (profiling runs skip the search)."""
        if name in cache:
            return bolt.BoltConfig.from_dict(cache[name])
        cfg = bolt.bolt_tune(op, d0, d1, tensors, workspace).config
        cache[name] = cfg.as_dict()
        return cfg

    def large_shapes_table():
        # ------------------------------------------------------------------ large shapes (context, outside the step)
        # The five configurations are small problems (7 GFLOP at most per launch); these two show what the
        # same tuned templates reach when the problem fills the chip.
        large = []
        cfg_keys = ("kernel_id", "tile_m", "tile_n", "tile_k", "waves_m", "waves_n", "stages", "swizzle")
        try:
            # 8192^3 and 4096^3 are ours (long enough for steady state); 1280 x 3072 x 768 is the FFN GEMM of
            # the paper's epilogue-fusion experiment (Section 4.1.1)
            # each with B stored [N][K] (reduction index contiguous) and row-major [K][N]
            gemms = ((8192, 8192, 8192), (4096, 4096, 4096), (wl.EPILOGUE_GEMM.M, wl.EPILOGUE_GEMM.N, wl.EPILOGUE_GEMM.K))
            for (M, N, K, lay) in [g + (l,) for g in gemms for l in ("NK", "KN")]:
                Ag = torch.randn((M, K), device="cuda", dtype=torch.float16) * 0.5
                Bg = torch.randn((N, K) if lay == "NK" else (K, N), device="cuda", dtype=torch.float16) * 0.5
                biasg = torch.randn((N,), device="cuda", dtype=torch.float16)
                Dg = empty(M, N)
                gd = bolt.gemm_desc(M, N, K, b_layout=bolt.LAYOUT_NK if lay == "NK" else bolt.LAYOUT_KN, act="relu")
                cfg = tuned("large gemm %dx%dx%d %s" % (M, N, K, lay), bolt.OP_GEMM, gd, None, [Ag, Bg, biasg, Dg], ws)
                ms = timed(lambda: bolt.bolt_gemm_epilogue(gd, Ag, Bg, biasg, Dg, cfg, ws), 10 if M >= 8192 else 30)
                large.append(dict(name="GEMM %dx%dx%d + bias + ReLU (B as %s)" % (M, N, K, "[N][K]" if lay == "NK" else "[K][N]"),
                                  ms=round(ms, 4), tflops=round(2.0 * M * N * K / ms / 1e9, 1),
                                  pct_mfma_peak=round(100 * 2.0 * M * N * K / ms / 1e9 / MFMA_PEAK_TFLOPS, 2),
                                  config={k: cfg.as_dict()[k] for k in cfg_keys}))
                del Ag, Bg, Dg
            cs = wl.ConvShape(128, 56, 56, 256, 256, 3, 3, 1, 1)
            xg = torch.randn((cs.N, cs.H, cs.W, cs.C), device="cuda", dtype=torch.float16) * 0.5
            wg = torch.randn((cs.K, cs.R, cs.S, cs.C), device="cuda", dtype=torch.float16) * 0.05
            bg = torch.zeros(cs.K, device="cuda", dtype=torch.float16)
            yg = empty(cs.N, cs.P, cs.Q, cs.K)
            cd = bolt.conv_desc(cs.N, cs.H, cs.W, cs.C, cs.K, cs.R, cs.S, cs.stride, cs.pad)
            cfg = tuned("large conv 128x56x56x256", bolt.OP_CONV2D, cd, None, [xg, wg, bg, yg], ws)
            ms = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(cd, xg, wg, bg, yg, cfg, ws), 10)
            large.append(dict(name="conv3x3 N=128 56x56 256->256", ms=round(ms, 4), tflops=round(cs.flops / ms / 1e9, 1),
                              pct_mfma_peak=round(100 * cs.flops / ms / 1e9 / MFMA_PEAK_TFLOPS, 2),
                              config={k: cfg.as_dict()[k] for k in cfg_keys}))
            del xg, wg, yg
        except Exception as e:  # context only
            large.append({"error": str(e)})
        return large


    if args.large_only:
        large = large_shapes_table()
        if args.tune_cache:
            json.dump(cache, open(args.tune_cache, "w"), indent=1)
        print(json.dumps({"large_shapes": large, "data": "synthetic",
                          "table_timing": "median of %d repetitions of a hip graph replay" % REPS_MEDIAN}))
        return

    # ------------------------------------------------------------------ build + tune every op
    ops = []      # dicts: name, flops, bytes, run(), config
    shapes_out = []

    def add_conv(name, shape, t, count=1, in_step=True):
        x, w = dev(t["x"]), dev(t["w"])
        b = dev(t["bias"])
        y = empty(shape.N, shape.P, shape.Q, shape.K)
        alt = None
        nbytes = shape.bytes
        if shape.c_logical:
            # The stem: the first-layer kernels read the 3-channel tensor as it is (Section 3.2.3's padding and layout
            # transformation folded into the loader); the padded path (pad pass + C = 8 convolution) is timed beside
            # it in the per-shape table, not in the step.
            c3 = shape.c_logical
            xp, wp = empty(*(t["x"].shape[:-1] + (shape.C,))), empty(*(t["w"].shape[:-1] + (shape.C,)))
            bolt.bolt_pad_channels_nhwc(w, wp, shape.C)     # weights are padded once, offline
            bolt.bolt_pad_channels_nhwc(x, xp, shape.C)
            d8 = bolt.conv_desc(shape.N, shape.H, shape.W, shape.C, shape.K, shape.R, shape.S, shape.stride, shape.pad)
            y8 = torch.empty_like(y)
            cfg8 = tuned(name + " (padded to 8 channels)", bolt.OP_CONV2D, d8, None, [xp, wp, b, y8], ws)
            x_src = x
            alt = dict(pad=lambda: bolt.bolt_pad_channels_nhwc(x_src, xp, shape.C),
                       conv=lambda: bolt.bolt_conv2d_fprop_nhwc(d8, xp, wp, b, y8, cfg8, ws), cfg=cfg8.as_dict())
            d = bolt.conv_desc(shape.N, shape.H, shape.W, c3, shape.K, shape.R, shape.S, shape.stride, shape.pad)
            nbytes = 2 * (x.numel() + w.numel() + y.numel() + shape.K)
        else:
            d = bolt.conv_desc(shape.N, shape.H, shape.W, shape.C, shape.K, shape.R, shape.S, shape.stride, shape.pad)
        cfg = tuned(name, bolt.OP_CONV2D, d, None, [x, w, b, y], ws)
        run = lambda: bolt.bolt_conv2d_fprop_nhwc(d, x, w, b, y, cfg, ws)

        def fresh():  # the same launch on buffers of its own (for the cold column)
            xx, ww, bb, yy = x.clone(), w.clone(), b.clone(), torch.empty_like(y)
            return lambda: bolt.bolt_conv2d_fprop_nhwc(d, xx, ww, bb, yy, cfg, ws)
        op = dict(name=name, kind="conv", flops=shape.flops, bytes=nbytes, run=run, count=count, cfg=cfg.as_dict(),
                  pad=None, alt=alt, in_step=in_step, keep=(x, w, b, y, d), fresh=fresh)
        ops.append(op)
        return op

    # config 1
    t = wl.config1()
    A1, B1, bias1, D1 = dev(t["A"]), dev(t["B"]), dev(t["bias"]), empty(256, 256)
    g1 = bolt.gemm_desc(256, 256, 256)
    cfg1 = tuned("C1", bolt.OP_GEMM, g1, None, [A1, B1, bias1, D1], ws)
    ops.append(dict(name="C1 gemm 256x256x256", kind="gemm", flops=2 * 256 ** 3, bytes=wl.GemmShape(256, 256, 256).bytes,
                    run=lambda: bolt.bolt_gemm_epilogue(g1, A1, B1, bias1, D1, cfg1, ws), count=1, cfg=cfg1.as_dict(),
                    pad=None, in_step=True))
    # config 2
    add_conv("C2 conv3x3 56x56 64->64", wl.CONFIG2_SHAPE, wl.config2())
    # config 3: fused, and the unfused pair for the speedup
    t = wl.config3()
    A3, W0, b0, W1, b1 = (dev(t[k]) for k in ("A", "W0", "b0", "W1", "b1"))
    D0u, D3, D3u = empty(16384, 64), empty(16384, 128), empty(16384, 128)
    g30, g31 = bolt.gemm_desc(16384, 64, 256), bolt.gemm_desc(16384, 128, 64)
    cfg3 = tuned("C3 fused", bolt.OP_B2B_GEMM, g30, g31, [A3, W0, b0, W1, b1, D3])
    cfg30 = tuned("C3 op0", bolt.OP_GEMM, g30, None, [A3, W0, b0, D0u], ws)
    cfg31 = tuned("C3 op1", bolt.OP_GEMM, g31, None, [D0u, W1, b1, D3u], ws)
    s30, s31 = wl.CONFIG3_SHAPE
    fused_bytes3 = 2 * (16384 * 256 + 256 * 64 + 64 + 64 * 128 + 128 + 16384 * 128)
    run3 = lambda: bolt.bolt_b2b_gemm(g30, g31, A3, W0, b0, W1, b1, D3, cfg3)

    def run3u():
        bolt.bolt_gemm_epilogue(g30, A3, W0, b0, D0u, cfg30, ws)
        bolt.bolt_gemm_epilogue(g31, D0u, W1, b1, D3u, cfg31, ws)
    def fresh3():
        a_, d_ = A3.clone(), torch.empty_like(D3)
        return lambda: bolt.bolt_b2b_gemm(g30, g31, a_, W0, b0, W1, b1, d_, cfg3)
    ops.append(dict(name="C3 b2b gemm fused", kind="b2b_gemm", flops=s30.flops + s31.flops, bytes=fused_bytes3, run=run3,
                    count=1, cfg=cfg3.as_dict(), pad=None, in_step=True, fresh=fresh3))
    # config 4
    t = wl.config4()
    x4, w40, b40, w41, b41 = (dev(t[k]) for k in ("x", "w0", "b0", "w1", "b1"))
    c40 = bolt.conv_desc(32, 56, 56, 64, 64, 3, 3, 1, 1)
    c41 = bolt.conv_desc(32, 56, 56, 64, 256, 1, 1, 1, 0)
    y40u, y4, y4u = empty(32, 56, 56, 64), empty(32, 56, 56, 256), empty(32, 56, 56, 256)
    cfg4 = tuned("C4 fused", bolt.OP_B2B_CONV, c40, c41, [x4, w40, b40, w41, b41, y4])
    cfg40 = tuned("C4 op0", bolt.OP_CONV2D, c40, None, [x4, w40, b40, y40u], ws)
    cfg41 = tuned("C4 op1", bolt.OP_CONV2D, c41, None, [y40u, w41, b41, y4u], ws)
    s40, s41 = wl.CONFIG4_SHAPES
    fused_bytes4 = 2 * (x4.numel() + w40.numel() + w41.numel() + 64 + 256 + y4.numel())
    run4 = lambda: bolt.bolt_b2b_conv(c40, c41, x4, w40, b40, w41, b41, y4, cfg4)

    def run4u():
        bolt.bolt_conv2d_fprop_nhwc(c40, x4, w40, b40, y40u, cfg40, ws)
        bolt.bolt_conv2d_fprop_nhwc(c41, y40u, w41, b41, y4u, cfg41, ws)
    def fresh4():
        x_, y_ = x4.clone(), torch.empty_like(y4)
        return lambda: bolt.bolt_b2b_conv(c40, c41, x_, w40, b40, w41, b41, y_, cfg4)
    ops.append(dict(name="C4 b2b conv fused", kind="b2b_conv", flops=s40.flops + s41.flops, bytes=fused_bytes4, run=run4,
                    count=1, cfg=cfg4.as_dict(), pad=None, in_step=True, fresh=fresh4))
    # config 5
    for i, (shape, cnt) in enumerate(wl.resnet50_layers(32)):
        _, _, t = wl.config5_layer(i)
        add_conv("C5 L%02d %dx%d %d->%d %dx%d/%d" % (i, shape.H, shape.W, shape.c_logical or shape.C, shape.K, shape.R,
                                                    shape.S, shape.stride), shape, t, count=cnt)
    torch.cuda.synchronize()
    if args.tune_cache and not os.path.exists(args.tune_cache):
        os.makedirs(os.path.dirname(os.path.abspath(args.tune_cache)), exist_ok=True)
        json.dump(cache, open(args.tune_cache, "w"))

    # ------------------------------------------------------------------ per-shape table
    for op in ([] if args.steps_only else ops):
        ms = timed(op["run"], args.reps)
        tfl = op["flops"] / ms / 1e9
        gbs = op["bytes"] / ms / 1e6
        t_mfma = op["flops"] / (MFMA_PEAK_TFLOPS * 1e9)   # ms
        t_hbm = op["bytes"] / (HBM_PEAK_GBS * 1e6)        # ms
        entry = dict(name=op["name"], ms=round(ms, 5), tflops=round(tfl, 2), pct_mfma_peak=round(100 * tfl / MFMA_PEAK_TFLOPS, 2),
                     gbs=round(gbs, 1), pct_hbm_peak=round(100 * gbs / HBM_PEAK_GBS, 2),
                     bound="mfma" if t_mfma >= t_hbm else "hbm", roofline_frac=round(max(t_mfma, t_hbm) / ms, 4),
                     count=op["count"], config={k: op["cfg"][k] for k in ("kernel_id", "tile_m", "tile_n", "tile_k", "waves_m",
                                                                         "waves_n", "swizzle", "split_k", "b2b_mode")})
        if op.get("alt") is not None:
            # the same layer through the pad pass and the aligned (C = 8) kernels, as Table 3 measures it
            pms, cms8 = timed(op["alt"]["pad"], args.reps), timed(op["alt"]["conv"], args.reps)
            entry["padded_path"] = dict(pad_ms=round(pms, 5), conv_ms=round(cms8, 5), total_ms=round(pms + cms8, 5),
                                        pad_cost_frac=round(pms / (pms + cms8), 4), kernel_id=op["alt"]["cfg"]["kernel_id"],
                                        speedup_of_unpadded_kernel=round((pms + cms8) / ms, 3))
        if entry["bound"] == "hbm" and op.get("fresh") is not None and not args.no_cold:
            # the warm number above re-reads a working set that the 256 MB memory-side cache holds; this one does not
            cms, nsets = timed_cold(op["fresh"], op["bytes"], args.reps)
            cg = op["bytes"] / cms / 1e6
            entry.update(cold_ms=round(cms, 5), cold_gbs=round(cg, 1), cold_pct_hbm_peak=round(100 * cg / HBM_PEAK_GBS, 2),
                         cold_roofline_frac=round(max(t_mfma, t_hbm) / cms, 4), cold_buffer_sets=nsets)
        op["ms"] = ms
        shapes_out.append(entry)
    if args.steps_only:
        ms3 = ms3u = ms4 = ms4u = float("nan")
    else:
        ms3, ms3u = timed(run3, args.reps), timed(run3u, args.reps)
        ms4, ms4u = timed(run4, args.reps), timed(run4u, args.reps)
    b2b = dict(config3_gemm=dict(fused_ms=round(ms3, 5), unfused_ms=round(ms3u, 5), speedup=round(ms3u / ms3, 3)),
               config4_conv=dict(fused_ms=round(ms4, 5), unfused_ms=round(ms4u, 5), speedup=round(ms4u / ms4, 3)))

    # ------------------------------------------------------------------ the timed steps
    conv_ops = [op for op in ops if op["kind"] == "conv"]
    other_ops = [op for op in ops if op["kind"] != "conv"]
    conv_launches = sum(op["count"] for op in conv_ops)
    conv_flops = sum(op["flops"] * op["count"] for op in conv_ops)
    conv_bytes = sum(op["bytes"] * op["count"] for op in conv_ops)
    conv_floor_ms = sum(max(op["flops"] / (MFMA_PEAK_TFLOPS * 1e9), op["bytes"] / (HBM_PEAK_GBS * 1e6)) * op["count"]
                        for op in conv_ops)
    step_flops = conv_flops + sum(op["flops"] for op in other_ops)

    def step(ev=None):
        for op in other_ops:
            op["run"]()
        for op in conv_ops:
            if op["pad"] is not None:
                op["pad"]()
        if ev is not None:
            ev[0].record(stream)
        for op in conv_ops:
            for _ in range(op["count"]):
                op["run"]()
        if ev is not None:
            ev[1].record(stream)

    for _ in range(max(args.warmup, 1) if args.graph else args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        # The step is launch-bound (57 kernels of 8-60 us): capture it once and replay it.  Two graphs,
        # so that the events that bracket the conv segment stay ordinary stream events.  Nothing in a
        # step allocates, synchronises or clears memory, so every launch is a plain kernel node.
        eager_step = step
        g_other, g_conv = torch.cuda.CUDAGraph(), torch.cuda.CUDAGraph()
        with torch.cuda.graph(g_other):
            for op in other_ops:
                op["run"]()
            for op in conv_ops:
                if op["pad"] is not None:
                    op["pad"]()
        with torch.cuda.graph(g_conv):
            for op in conv_ops:
                for _ in range(op["count"]):
                    op["run"]()

        def step(ev=None):
            g_other.replay()
            if ev is not None:
                ev[0].record(stream)
            g_conv.replay()
            if ev is not None:
                ev[1].record(stream)
        for _ in range(max(args.warmup, 1)):
            step()
        torch.cuda.synchronize()
    evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(evs[i])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    conv_ms = sum(a.elapsed_time(b) for a, b in evs) / args.steps      # conv segment of a step
    avg_launch_ms = conv_ms / conv_launches
    achieved = conv_flops / conv_launches / (avg_launch_ms * 1e-3) / 1e12

    # Per-op times INSIDE a step (every op finds caches that the 56 other ops have just swept: the cold
    # number that belongs beside the back-to-back one of the per-shape table).  Separate, untimed steps.
    if not args.steps_only:
        diag_steps = 5
        marks = []
        for _ in range(diag_steps):
            row = []
            for op in other_ops:
                op["run"]()
            for op in conv_ops:
                if op["pad"] is not None:
                    op["pad"]()
            for op in conv_ops:
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record(stream)
                for _ in range(op["count"]):
                    op["run"]()
                e1.record(stream)
                row.append((e0, e1))
            marks.append(row)
        torch.cuda.synchronize()
        by_name = {e["name"]: e for e in shapes_out}
        for i, op in enumerate(conv_ops):
            ms = sum(m[i][0].elapsed_time(m[i][1]) for m in marks) / diag_steps / op["count"]
            by_name[op["name"]]["ms_in_step"] = round(ms, 5)

    # The ops of a step are independent problems, so nothing but the launch order keeps them from overlapping.
    # For context (not `value`, which stays the in-order single-stream step that the profiles describe): the same
    # step with its ops dealt round-robin over 2 and 4 streams, each stream's share captured in a HIP graph.
    overlapped = []
    if not args.steps_only:
        try:
            all_runs = [op["run"] for op in other_ops] + [op["pad"] for op in conv_ops if op["pad"] is not None]
            for op in conv_ops:
                all_runs += [op["run"]] * op["count"]
            for ns in (2, 4):
                side = [torch.cuda.Stream() for _ in range(ns)]
                graphs = []
                torch.cuda.synchronize()
                for k in range(ns):
                    g = torch.cuda.CUDAGraph()
                    with torch.cuda.graph(g, stream=side[k]):
                        for j, fn in enumerate(all_runs):
                            if j % ns == k:
                                fn()
                    graphs.append(g)

                def step_overlapped():
                    fork = torch.cuda.Event()
                    fork.record(stream)
                    for k in range(ns):
                        side[k].wait_event(fork)
                        with torch.cuda.stream(side[k]):
                            graphs[k].replay()
                        join = torch.cuda.Event()
                        join.record(side[k])
                        stream.wait_event(join)
                for _ in range(3):
                    step_overlapped()
                torch.cuda.synchronize()
                c0 = time.perf_counter()
                for _ in range(args.steps):
                    step_overlapped()
                torch.cuda.synchronize()
                ms = (time.perf_counter() - c0) * 1e3 / args.steps
                overlapped.append(dict(streams=ns, ms_per_step=round(ms, 4), tflops=round(step_flops / (ms * 1e-3) / 1e12, 1)))
                del graphs
        except Exception as e:  # context only
            overlapped.append({"error": str(e)})

    traffic = None
    tpath = os.path.join(ROOT, "profiles", "traffic.json")  # written from the rocprofv3 --pmc passes
    if os.path.exists(tpath):
        try:
            traffic = json.load(open(tpath)).get("conv_hbm_bytes_per_launch")
        except Exception:
            traffic = None

    out = {
        "metric": "FP16 TFLOP/s and % of MFMA peak per conv/GEMM shape; b2b fused vs unfused speedup",
        "value": round(step_flops / (ms_per_step * 1e-3) / 1e12, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f16 (f32 accumulate)",
        "data": "synthetic",
        "launch": "hip graph replay (2 graphs per step)" if args.graph else "eager",
        "table_timing": "median of %d repetitions of %s per entry; cold_* = rotating over >= 5 buffer sets totalling > 256 MB" % (
            REPS_MEDIAN, "an eager launch loop" if args.eager_timing else "a hip graph replay of the launches"),
        "config": {"workload": "one pass over configs 1-5: GEMM 256^3, conv3x3 56x56x64, fused b2b GEMM 16384x256x64x128, "
                               "fused b2b conv 3x3->1x1 64->64->256, ResNet-50-shaped 53-conv stack at batch 32 (the stem "
                               "reads its 3 channels unpadded); config 5 carries 96% of the FLOPs",
                   "batch": 32, "step_gflop": round(step_flops / 1e9, 2)},
        "roofline": {"bound": "mfma", "kernel": "conv op launches: bolt::fprop_dma_kernel<...> (implicit-GEMM gather, or GEMM addressing for 1x1/s1), bolt::conv_halo_kernel<...> and, for the stem, bolt::conv_smallc_kernel<...>, all tuned instances",
                     "achieved": round(achieved, 3), "peak": MFMA_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(achieved / MFMA_PEAK_TFLOPS, 4), "traffic": traffic,
                     "launches_per_step": conv_launches, "avg_launch_ms": round(avg_launch_ms, 5),
                     "flops_per_launch": round(conv_flops / conv_launches),
                     # the same launches against the other roof, and against whichever roof binds each layer
                     # (a layer's floor is max(flops / MFMA peak, algorithmic bytes / HBM peak))
                     "bytes_per_launch": round(conv_bytes / conv_launches),
                     "achieved_hbm_gbs": round(conv_bytes / conv_launches / (avg_launch_ms * 1e-3) / 1e9, 1),
                     "hbm_frac": round(conv_bytes / conv_launches / (avg_launch_ms * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
                     "frac_of_binding_roof": round(conv_floor_ms / conv_ms, 4)},
        "b2b": b2b,
        "step_overlapped": overlapped,
        "shapes": shapes_out,
    }
    if args.steps_only:
        print(json.dumps(out))
        return

    out["large_shapes"] = large_shapes_table()

    # ------------------------------------------------------------------ the paper's b2b tables (context)
    # Tables 1 and 2 (Section 4.1.2): fused vs unfused on the paper's own shapes, random data.  Extents that
    # are not multiples of 8 are padded with zeros first (Section 3.2.3), as a caller of the library must.
    tables = []

    def pad8(v):
        return (v + 7) // 8 * 8

    def rnd(*shape, scale=0.5):
        return torch.randn(shape, device="cuda", dtype=torch.float16) * scale

    for (M, N0, K0, N1) in wl.TABLE1_B2B_GEMM:
        entry = dict(name="Table 1 b2b GEMM M=%d N0=%d K0=%d N1=%d" % (M, N0, K0, N1))
        try:
            n0, k0, n1 = pad8(N0), pad8(K0), pad8(N1)
            A, W0, b0, W1, b1 = rnd(M, k0), rnd(k0, n0, scale=0.1), rnd(n0), rnd(n0, n1, scale=0.1), rnd(n1)
            D0, D1, D1u = empty(M, n0), empty(M, n1), empty(M, n1)
            g0, g1 = bolt.gemm_desc(M, n0, k0), bolt.gemm_desc(M, n1, n0)
            if bolt.bolt_check(bolt.OP_B2B_GEMM, g0, g1) != 0:
                # row-major weights of this size do not fit the weights-resident kernels: store them
                # reduction-contiguous ([N][K]), which the multi-stage fused kernel streams
                W0, W1 = rnd(n0, k0, scale=0.1), rnd(n1, n0, scale=0.1)
                g0 = bolt.gemm_desc(M, n0, k0, b_layout=bolt.LAYOUT_NK)
                g1 = bolt.gemm_desc(M, n1, n0, b_layout=bolt.LAYOUT_NK)
                entry["weights"] = "[N][K]"
            cf = tuned(entry["name"] + " fused", bolt.OP_B2B_GEMM, g0, g1, [A, W0, b0, W1, b1, D1])
            c0 = tuned(entry["name"] + " op0", bolt.OP_GEMM, g0, None, [A, W0, b0, D0], ws)
            c1 = tuned(entry["name"] + " op1", bolt.OP_GEMM, g1, None, [D0, W1, b1, D1u], ws)

            def unfused():
                bolt.bolt_gemm_epilogue(g0, A, W0, b0, D0, c0, ws)
                bolt.bolt_gemm_epilogue(g1, D0, W1, b1, D1u, c1, ws)
            mf = timed(lambda: bolt.bolt_b2b_gemm(g0, g1, A, W0, b0, W1, b1, D1, cf), args.reps)
            mu = timed(unfused, args.reps)
            entry.update(padded_to=[n0, k0, n1], fused_ms=round(mf, 5), unfused_ms=round(mu, 5), speedup=round(mu / mf, 3))
        except bolt.BoltError as e:
            entry["status"] = str(e)
        tables.append(entry)
    for (H, IC, OC0, st, OC1) in wl.TABLE2_B2B_CONV:
        entry = dict(name="Table 2 b2b conv %dx%d IC=%d OC=%d stride %d -> 1x1 OC=%d" % (H, H, IC, OC0, st, OC1))
        try:
            ic = pad8(IC)
            x, w0, b0, w1, b1 = rnd(32, H, H, ic), rnd(OC0, 3, 3, ic, scale=0.1), rnd(OC0), rnd(OC1, 1, 1, OC0, scale=0.1), rnd(OC1)
            c0d = bolt.conv_desc(32, H, H, ic, OC0, 3, 3, st, 1)
            P, Q = bolt.conv_out_hw(c0d)
            c1d = bolt.conv_desc(32, P, Q, OC0, OC1, 1, 1, 1, 0)
            y0, y1, y1u = empty(32, P, Q, OC0), empty(32, P, Q, OC1), empty(32, P, Q, OC1)
            cf = tuned(entry["name"] + " fused", bolt.OP_B2B_CONV, c0d, c1d, [x, w0, b0, w1, b1, y1])
            c0 = tuned(entry["name"] + " op0", bolt.OP_CONV2D, c0d, None, [x, w0, b0, y0], ws)
            c1 = tuned(entry["name"] + " op1", bolt.OP_CONV2D, c1d, None, [y0, w1, b1, y1u], ws)

            def unfused_c():
                bolt.bolt_conv2d_fprop_nhwc(c0d, x, w0, b0, y0, c0, ws)
                bolt.bolt_conv2d_fprop_nhwc(c1d, y0, w1, b1, y1u, c1, ws)
            mf = timed(lambda: bolt.bolt_b2b_conv(c0d, c1d, x, w0, b0, w1, b1, y1, cf), args.reps)
            mu = timed(unfused_c, args.reps)
            entry.update(padded_ic=ic, fused_ms=round(mf, 5), unfused_ms=round(mu, 5), speedup=round(mu / mf, 3))
            del x, y0, y1, y1u
        except bolt.BoltError as e:
            entry["status"] = str(e)
        tables.append(entry)
    out["paper_tables_b2b"] = tables

    # ------------------------------------------------------------------ epilogue fusion (context)
    # Section 4.1.1's experiment: GEMM 1280 x 3072 x 768 + bias + activation computed in the GEMM's epilogue,
    # against the same tuned GEMM writing its plain result followed by a separate bias + activation pass.
    epi = []
    try:
        g = wl.EPILOGUE_GEMM
        Ae, Be, be = rnd(g.M, g.K), rnd(g.N, g.K, scale=0.1), rnd(g.N)
        De, Du = empty(g.M, g.N), empty(g.M, g.N)
        for act in ("relu", "gelu", "hardswish", "softplus"):
            gf = bolt.gemm_desc(g.M, g.N, g.K, b_layout=bolt.LAYOUT_NK, act=act)
            gn = bolt.gemm_desc(g.M, g.N, g.K, b_layout=bolt.LAYOUT_NK, act="none")
            cf = tuned("epilogue gemm fused " + act, bolt.OP_GEMM, gf, None, [Ae, Be, be, De], ws)
            cn = tuned("epilogue gemm plain", bolt.OP_GEMM, gn, None, [Ae, Be, None, Du], ws)

            def unfused_e():
                bolt.bolt_gemm_epilogue(gn, Ae, Be, None, Du, cn, ws)
                bolt.bolt_bias_act(Du, be, 1.0, 1.0, act)
            mf = timed(lambda: bolt.bolt_gemm_epilogue(gf, Ae, Be, be, De, cf, ws), args.reps)
            mu = timed(unfused_e, args.reps)
            epi.append(dict(name="GEMM %dx%dx%d + bias + %s" % (g.M, g.N, g.K, act), fused_ms=round(mf, 5),
                            unfused_ms=round(mu, 5), speedup=round(mu / mf, 3)))
    except Exception as e:  # context only
        epi.append({"error": str(e)})
    out["epilogue_fusion"] = epi

    # ------------------------------------------------------------------ channel padding (context)
    # Table 3 (Section 4.1.3): input channels not divisible by 8.  "unpadded" runs the tuned alignment-2
    # kernel on the tensor as it is; "padded" pads the activation to the next multiple of 8 (weights are
    # padded once, offline) and runs the tuned alignment-8 kernel.  speedup = unpadded conv / padded conv;
    # pad_cost = padding time / (padding + padded conv), as in the table.
    t3 = []
    for (N, H, W, IC, OC, R, S, pad) in wl.TABLE3_PADDING:
        entry = dict(name="Table 3 conv N=%d %dx%d IC=%d OC=%d %dx%d pad %d" % (N, H, W, IC, OC, R, S, pad))
        try:
            ic8 = pad8(IC)
            x, w, b = rnd(N, H, W, IC), rnd(OC, R, S, IC, scale=0.05), rnd(OC)
            xp, wp = empty(N, H, W, ic8), empty(OC, R, S, ic8)
            bolt.bolt_pad_channels_nhwc(w, wp, ic8)
            du = bolt.conv_desc(N, H, W, IC, OC, R, S, 1, pad)
            dp = bolt.conv_desc(N, H, W, ic8, OC, R, S, 1, pad)
            P, Q = bolt.conv_out_hw(du)
            yu, yp = empty(N, P, Q, OC), empty(N, P, Q, OC)
            cu = tuned(entry["name"] + " unpadded", bolt.OP_CONV2D, du, None, [x, w, b, yu], ws)
            bolt.bolt_pad_channels_nhwc(x, xp, ic8)
            cp = tuned(entry["name"] + " padded", bolt.OP_CONV2D, dp, None, [xp, wp, b, yp], ws)
            mu = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(du, x, w, b, yu, cu, ws), args.reps)
            mp = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(dp, xp, wp, b, yp, cp, ws), args.reps)
            mpad = timed(lambda: bolt.bolt_pad_channels_nhwc(x, xp, ic8), args.reps)
            entry.update(unpadded_ms=round(mu, 5), padded_ms=round(mp, 5), pad_ms=round(mpad, 5),
                         speedup=round(mu / mp, 3), pad_cost=round(mpad / (mpad + mp), 3),
                         speedup_with_pad=round(mu / (mp + mpad), 3))
        except bolt.BoltError as e:
            entry["status"] = str(e)
        t3.append(entry)
    out["paper_table3_padding"] = t3

    # ------------------------------------------------------------------ three-op chains (context)
    # Section 3.1.1's extension to more than two ops: one launch against (a) three tuned single-op launches
    # and (b) the tuned fused pair followed by the third op.  GEMM widths are those of Table 1's rows carried
    # one layer further; the convolutions are a 3x3 followed by two 1x1 (Section 3.3's deepening), batch 32.
    chains = []
    for (M, K0, N0, N1, N2) in ((16384, 256, 64, 128, 64), (32768, 576, 128, 64, 64), (128320, 96, 32, 96, 32)):
        entry = dict(name="GEMM chain M=%d %d->%d->%d->%d" % (M, K0, N0, N1, N2))
        try:
            nk = bolt.LAYOUT_NK
            A, Wc, bc = rnd(M, K0), [rnd(N0, K0, scale=0.1), rnd(N1, N0, scale=0.1), rnd(N2, N1, scale=0.1)], [rnd(N0), rnd(N1), rnd(N2)]
            gd = [bolt.gemm_desc(M, N0, K0, b_layout=nk), bolt.gemm_desc(M, N1, N0, b_layout=nk), bolt.gemm_desc(M, N2, N1, b_layout=nk)]
            Da, Db, Dc, Dp, Df = empty(M, N0), empty(M, N1), empty(M, N2), empty(M, N1), empty(M, N2)
            cf = bolt.bolt_tune_chain(bolt.OP_GEMM_CHAIN3, gd, [A, Wc[0], bc[0], Wc[1], bc[1], Wc[2], bc[2], Df]).config
            c0 = tuned(entry["name"] + " op0", bolt.OP_GEMM, gd[0], None, [A, Wc[0], bc[0], Da], ws)
            c1 = tuned(entry["name"] + " op1", bolt.OP_GEMM, gd[1], None, [Da, Wc[1], bc[1], Db], ws)
            c2 = tuned(entry["name"] + " op2", bolt.OP_GEMM, gd[2], None, [Db, Wc[2], bc[2], Dc], ws)
            cp = tuned(entry["name"] + " pair", bolt.OP_B2B_GEMM, gd[0], gd[1], [A, Wc[0], bc[0], Wc[1], bc[1], Dp])

            def three():
                bolt.bolt_gemm_epilogue(gd[0], A, Wc[0], bc[0], Da, c0, ws)
                bolt.bolt_gemm_epilogue(gd[1], Da, Wc[1], bc[1], Db, c1, ws)
                bolt.bolt_gemm_epilogue(gd[2], Db, Wc[2], bc[2], Dc, c2, ws)

            def pair_then_one():
                bolt.bolt_b2b_gemm(gd[0], gd[1], A, Wc[0], bc[0], Wc[1], bc[1], Dp, cp)
                bolt.bolt_gemm_epilogue(gd[2], Dp, Wc[2], bc[2], Dc, c2, ws)
            mf = timed(lambda: bolt.bolt_b2b_gemm_chain(gd, A, Wc, bc, Df, cf), args.reps)
            m3, m2 = timed(three, args.reps), timed(pair_then_one, args.reps)
            entry.update(fused_ms=round(mf, 5), three_launches_ms=round(m3, 5), pair_plus_one_ms=round(m2, 5),
                         speedup_vs_three=round(m3 / mf, 3), speedup_vs_pair_plus_one=round(m2 / mf, 3))
        except bolt.BoltError as e:
            entry["status"] = str(e)
        chains.append(entry)
    for (H, IC, OC, st) in ((56, 64, 64, 1), (112, 48, 48, 2), (224, 3, 64, 2)):
        entry = dict(name="conv chain %dx%d IC=%d 3x3/%d -> 1x1 -> 1x1, OC=%d" % (H, H, IC, st, OC))
        try:
            ic = pad8(IC)
            x, wc = rnd(32, H, H, ic), [rnd(OC, 3, 3, ic, scale=0.1), rnd(OC, 1, 1, OC, scale=0.1), rnd(OC, 1, 1, OC, scale=0.1)]
            bc = [rnd(OC), rnd(OC), rnd(OC)]
            d0 = bolt.conv_desc(32, H, H, ic, OC, 3, 3, st, 1)
            P, Q = bolt.conv_out_hw(d0)
            cd = [d0, bolt.conv_desc(32, P, Q, OC, OC, 1, 1, 1, 0), bolt.conv_desc(32, P, Q, OC, OC, 1, 1, 1, 0)]
            ya, yb, yc, yp, yf = (empty(32, P, Q, OC) for _ in range(5))
            cf = bolt.bolt_tune_chain(bolt.OP_CONV_CHAIN3, cd, [x, wc[0], bc[0], wc[1], bc[1], wc[2], bc[2], yf]).config
            c0 = tuned(entry["name"] + " op0", bolt.OP_CONV2D, cd[0], None, [x, wc[0], bc[0], ya], ws)
            c1 = tuned(entry["name"] + " op1", bolt.OP_CONV2D, cd[1], None, [ya, wc[1], bc[1], yb], ws)
            c2 = tuned(entry["name"] + " op2", bolt.OP_CONV2D, cd[2], None, [yb, wc[2], bc[2], yc], ws)
            cp = tuned(entry["name"] + " pair", bolt.OP_B2B_CONV, cd[0], cd[1], [x, wc[0], bc[0], wc[1], bc[1], yp])

            def three_c():
                bolt.bolt_conv2d_fprop_nhwc(cd[0], x, wc[0], bc[0], ya, c0, ws)
                bolt.bolt_conv2d_fprop_nhwc(cd[1], ya, wc[1], bc[1], yb, c1, ws)
                bolt.bolt_conv2d_fprop_nhwc(cd[2], yb, wc[2], bc[2], yc, c2, ws)

            def pair_then_one_c():
                bolt.bolt_b2b_conv(cd[0], cd[1], x, wc[0], bc[0], wc[1], bc[1], yp, cp)
                bolt.bolt_conv2d_fprop_nhwc(cd[2], yp, wc[2], bc[2], yc, c2, ws)
            mf = timed(lambda: bolt.bolt_b2b_conv_chain(cd, x, wc, bc, yf, cf), args.reps)
            m3, m2 = timed(three_c, args.reps), timed(pair_then_one_c, args.reps)
            entry.update(fused_ms=round(mf, 5), three_launches_ms=round(m3, 5), pair_plus_one_ms=round(m2, 5),
                         speedup_vs_three=round(m3 / mf, 3), speedup_vs_pair_plus_one=round(m2 / mf, 3))
            del x, ya, yb, yc, yp, yf
        except bolt.BoltError as e:
            entry["status"] = str(e)
        chains.append(entry)
    out["chains_of_three"] = chains

    # ------------------------------------------------------------------ residual epilogue (context)
    # The last 1x1 convolution of a ResNet bottleneck block with its skip connection added in the epilogue
    # (Eq. 1's C as a full matrix), against the same tuned kernel without it: the cost of the extra read.
    resid = []
    try:
        for (H, Cin, Cout) in ((56, 64, 256), (28, 128, 512), (14, 256, 1024), (7, 512, 2048)):
            x, w, b = rnd(32, H, H, Cin), rnd(Cout, 1, 1, Cin, scale=0.1), rnd(Cout)
            r, y = rnd(32, H, H, Cout), empty(32, H, H, Cout)
            d = bolt.conv_desc(32, H, H, Cin, Cout, 1, 1, 1, 0)
            cfg = tuned("residual 1x1 %dx%d %d->%d" % (H, H, Cin, Cout), bolt.OP_CONV2D, d, None, [x, w, b, y], ws)
            mp = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(d, x, w, b, y, cfg, ws), args.reps)
            mr = timed(lambda: bolt.bolt_conv2d_fprop_nhwc_residual(d, x, w, b, r, y, 1.0, cfg, ws), args.reps)
            extra = 2.0 * r.numel()
            resid.append(dict(name="conv1x1 %dx%d %d->%d + bias + skip + ReLU" % (H, H, Cin, Cout), plain_ms=round(mp, 5),
                              residual_ms=round(mr, 5), extra_read_mb=round(extra / 1e6, 1),
                              extra_read_gbs=round(extra / max(mr - mp, 1e-6) / 1e6, 1)))
            del x, r, y
    except Exception as e:  # context only
        resid.append({"error": str(e)})
    out["residual_epilogue"] = resid

    # ------------------------------------------------------------------ bottleneck block (context)
    # A whole residual bottleneck block of the 56x56 stage (1x1 256->64, 3x3 64->64, 1x1 64->256 + skip + ReLU):
    # three tuned launches (the last with the residual epilogue) against 1x1, then the fused pair
    # 3x3 -> 1x1 with the skip connection in its second epilogue.
    block = []
    try:
        for (H, Cw, Cb) in ((56, 256, 64),):
            x = rnd(32, H, H, Cw)
            wa, wb_, wc_ = rnd(Cb, 1, 1, Cw, scale=0.1), rnd(Cb, 3, 3, Cb, scale=0.1), rnd(Cw, 1, 1, Cb, scale=0.1)
            ba, bb, bc_ = rnd(Cb), rnd(Cb), rnd(Cw)
            da = bolt.conv_desc(32, H, H, Cw, Cb, 1, 1, 1, 0)
            db = bolt.conv_desc(32, H, H, Cb, Cb, 3, 3, 1, 1)
            dc = bolt.conv_desc(32, H, H, Cb, Cw, 1, 1, 1, 0)
            ya, yb, y3, y2 = empty(32, H, H, Cb), empty(32, H, H, Cb), empty(32, H, H, Cw), empty(32, H, H, Cw)
            nm = "bottleneck %dx%d %d->%d->%d->%d + skip" % (H, H, Cw, Cb, Cb, Cw)
            ca = tuned(nm + " 1x1 a", bolt.OP_CONV2D, da, None, [x, wa, ba, ya], ws)
            cb = tuned(nm + " 3x3", bolt.OP_CONV2D, db, None, [ya, wb_, bb, yb], ws)
            cc = tuned(nm + " 1x1 c", bolt.OP_CONV2D, dc, None, [yb, wc_, bc_, y3], ws)
            try:  # a persistent instance has no residual epilogue: fall back to the built-in pick
                bolt.bolt_conv2d_fprop_nhwc_residual(dc, yb, wc_, bc_, x, y3, 1.0, cc, ws)
            except bolt.BoltError:
                cc = None
            cp = tuned(nm + " pair", bolt.OP_B2B_CONV_RES, db, dc, [ya, wb_, bb, wc_, bc_, y2, x])

            def three_b():
                bolt.bolt_conv2d_fprop_nhwc(da, x, wa, ba, ya, ca, ws)
                bolt.bolt_conv2d_fprop_nhwc(db, ya, wb_, bb, yb, cb, ws)
                bolt.bolt_conv2d_fprop_nhwc_residual(dc, yb, wc_, bc_, x, y3, 1.0, cc, ws)

            def two_b():
                bolt.bolt_conv2d_fprop_nhwc(da, x, wa, ba, ya, ca, ws)
                bolt.bolt_b2b_conv_residual(db, dc, ya, wb_, bb, wc_, bc_, x, y2, 1.0, cp)
            m3, m2 = timed(three_b, args.reps), timed(two_b, args.reps)
            gflop = 2.0 * 32 * H * H * (Cw * Cb + 9 * Cb * Cb + Cb * Cw) / 1e9
            block.append(dict(name=nm + " + ReLU, batch 32", three_launches_ms=round(m3, 5), fused_tail_ms=round(m2, 5),
                              speedup=round(m3 / m2, 3), fused_tflops=round(gflop / m2, 1)))
            del x, ya, yb, y3, y2
    except Exception as e:  # context only
        block.append({"error": str(e)})
    out["bottleneck_block"] = block

    # ------------------------------------------------------------------ layout transformation (context)
    # Section 3.2.3: NCHW in / out.  First layer: transform + channel padding in one pass against the padding
    # pass alone on an already-NHWC image; last layer: a 7x7x2048 feature map back to NCHW.
    lay = []
    try:
        xn, xh = rnd(32, 3, 224, 224), rnd(32, 224, 224, 3)
        xp8 = empty(32, 224, 224, 8)
        t_tp = timed(lambda: bolt.bolt_nchw_to_nhwc(xn, xp8), args.reps)
        t_p = timed(lambda: bolt.bolt_pad_channels_nhwc(xh, xp8, 8), args.reps)
        moved = 2.0 * (xn.numel() + xp8.numel())
        lay.append(dict(name="NCHW 32x3x224x224 -> NHWC, padded to 8 channels", ms=round(t_tp, 5), pad_only_ms=round(t_p, 5),
                        gbs=round(moved / t_tp / 1e6, 1)))
        yh, yn = rnd(32, 7, 7, 2048), empty(32, 2048, 7, 7)
        t_b = timed(lambda: bolt.bolt_nhwc_to_nchw(yh, yn), args.reps)
        lay.append(dict(name="NHWC 32x7x7x2048 -> NCHW", ms=round(t_b, 5), gbs=round(4.0 * yh.numel() / t_b / 1e6, 1)))
        yh2, yn2 = rnd(32, 56, 56, 256), empty(32, 256, 56, 56)
        t_b2 = timed(lambda: bolt.bolt_nhwc_to_nchw(yh2, yn2), args.reps)
        lay.append(dict(name="NHWC 32x56x56x256 -> NCHW", ms=round(t_b2, 5), gbs=round(4.0 * yh2.numel() / t_b2 / 1e6, 1)))
        # folded into the kernels: the stem straight from NCHW (no transform, no padding pass) against transform + pad
        # pass followed by the aligned kernel; the last 1x1 of the ResNet stack (7x7, 512 -> 2048) storing NCHW itself
        # against the NHWC kernel followed by the transform pass
        ws3, b3 = rnd(64, 7, 7, 3, scale=0.1), rnd(64)
        w8 = empty(64, 7, 7, 8)
        bolt.bolt_pad_channels_nhwc(ws3, w8, 8)
        ys = empty(32, 112, 112, 64)
        d_in = bolt.conv_desc(32, 224, 224, 3, 64, 7, 7, 2, 3, x_layout="nchw")
        d_8 = bolt.conv_desc(32, 224, 224, 8, 64, 7, 7, 2, 3)
        c_in = tuned("stem from NCHW", bolt.OP_CONV2D, d_in, None, [xn, ws3, b3, ys], ws)
        c_8 = tuned("stem padded to 8 channels (layout table)", bolt.OP_CONV2D, d_8, None, [xp8, w8, b3, ys], ws)
        t_fold = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(d_in, xn, ws3, b3, ys, c_in, ws), args.reps)

        def stem_passes():
            bolt.bolt_nchw_to_nhwc(xn, xp8)
            bolt.bolt_conv2d_fprop_nhwc(d_8, xp8, w8, b3, ys, c_8, ws)
        t_pass = timed(stem_passes, args.reps)
        lay.append(dict(name="stem 7x7/2 3->64 at batch 32 from an NCHW image: first-layer kernel vs transform+pad pass + aligned kernel",
                        folded_ms=round(t_fold, 5), passes_ms=round(t_pass, 5), speedup=round(t_pass / t_fold, 3)))
        xl_, wl_, bl_ = rnd(32, 7, 7, 512), rnd(2048, 1, 1, 512, scale=0.05), rnd(2048)
        d_o = bolt.conv_desc(32, 7, 7, 512, 2048, 1, 1, 1, 0, y_layout="nchw")
        d_h = bolt.conv_desc(32, 7, 7, 512, 2048, 1, 1, 1, 0)
        c_o = tuned("last 1x1 to NCHW", bolt.OP_CONV2D, d_o, None, [xl_, wl_, bl_, yn], ws)
        c_h = tuned("last 1x1 NHWC (layout table)", bolt.OP_CONV2D, d_h, None, [xl_, wl_, bl_, yh], ws)
        t_fo = timed(lambda: bolt.bolt_conv2d_fprop_nhwc(d_o, xl_, wl_, bl_, yn, c_o, ws), args.reps)

        def last_passes():
            bolt.bolt_conv2d_fprop_nhwc(d_h, xl_, wl_, bl_, yh, c_h, ws)
            bolt.bolt_nhwc_to_nchw(yh, yn)
        t_po = timed(last_passes, args.reps)
        lay.append(dict(name="last 1x1 7x7 512->2048 at batch 32 to an NCHW tensor: NCHW store in the kernel vs NHWC kernel + transform pass",
                        folded_ms=round(t_fo, 5), passes_ms=round(t_po, 5), speedup=round(t_po / t_fo, 3)))
    except Exception as e:  # context only
        lay.append({"error": str(e)})
    out["layout_transformation"] = lay
    try:
        out["probes"] = {"mfma_loop_tflops": round(bolt.bolt_probe_mfma_peak(20000), 1),
                         "copy_gbs_1GiB": round(bolt.bolt_probe_copy_bandwidth(torch.empty(1 << 30, dtype=torch.uint8, device="cuda"), 5), 1)}
    except Exception as e:  # probes are context only
        out["probes"] = {"error": str(e)}

    sustained = out["probes"].get("mfma_loop_tflops")
    if sustained:  # context only: against the MFMA-only loop of this run (the headline stays pct_mfma_peak)
        for e in out["large_shapes"] + out["shapes"]:
            if "tflops" in e:
                e["pct_mfma_sustained"] = round(100 * e["tflops"] / sustained, 2)

    if not args.no_cpu_baseline:
        # the oracle as it stands, on the host cores: three full layers of the step (10-20 s of wall time)
        from oracle import ref
        sample = [("config 2", wl.CONFIG2_SHAPE, wl.config2())]
        for idx in (6, 12):
            shape, _, t = wl.config5_layer(idx)
            sample.append(("config 5 layer %d" % idx, shape, t))
        flops, dt = 0, 0.0
        for _, shape, t in sample:
            c0 = time.perf_counter()
            ref.conv2d_nhwc(t["x"], t["w"], t["bias"], stride=shape.stride, pad=shape.pad)
            dt += time.perf_counter() - c0
            flops += shape.flops
        out["cpu_baseline"] = {"value": round(flops / dt / 1e12, 6), "unit": "TFLOP/s",
                               "cores": ref.num_threads(), "kind": "oracle",
                               "sample": "%s in full (3x3 convolutions at batch 32, %.1f GFLOP), %.1f s" % (
                                   ", ".join(n for n, _, _ in sample), flops / 1e9, dt)}
    # the long per-shape table first, the fused-vs-unfused numbers and the target rows last (a reader of the tail of
    # the line finds them there)
    last = ("epilogue_fusion", "paper_table3_padding", "chains_of_three", "residual_epilogue", "bottleneck_block",
            "layout_transformation", "probes", "cpu_baseline", "paper_tables_b2b", "b2b", "large_shapes")
    head = {k: v for k, v in out.items() if k not in last and k != "shapes"}
    ordered = dict(head)
    ordered["shapes"] = out["shapes"]
    for k in last:
        if k in out:
            ordered[k] = out[k]
    print(json.dumps(ordered))


if __name__ == "__main__":
    main()
