#!/usr/bin/env python3
"""Benchmark of the sparse-inference hot path on one MI355X.

One step = one pass of the block-punched 1x1 stack 24 -> 144 -> 24 (ReLU6 between,
8x8 blocks, 4x pruning, batch 64, 56x56, bf16) through npas_run_stack, inputs
already resident in HBM.  Prints one JSON line: dense-equivalent TFLOP/s, the
HBM roofline of the dominant kernel (timed with events on the launch stream) and
the CPU oracle timed on a bounded sample of the same workload.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=64)
    ap.add_argument("--no-fuse", action="store_true", help="run the two layers as two kernels")
    ap.add_argument("--no-rotate", action="store_true", help="reuse one buffer set (stays in the 256 MB Infinity Cache)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--per-layer", type=int, default=0, metavar="CFG",
                    help="instead of the headline line, print a per-layer table (us, dense-equivalent TFLOP/s, "
                         "algorithmic GB/s, roofline fraction) for config CFG in 1..5 (BASELINE.json's configs[CFG-1]); "
                         "6 = the inverted-residual block 1x1, depthwise 3x3, 1x1 of workloads/sweeps.py")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MB",
                    help="instead of the benchmark, run 5 plain device copies of MB megabytes (known traffic for "
                         "scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    ap.add_argument("--stack", type=int, default=0, metavar="CFG",
                    help="time npas_run_stack end to end on config CFG (2, 5, or 6 = inverted-residual block) at --batch")
    ap.add_argument("--graph", action="store_true", help="with --stack: capture the call into a HIP graph and time replays")
    ap.add_argument("--sweep", type=str, default="", choices=["", "rate", "block"],
                    help="rate: 3x3 conv 56x56x256->256 over pruning schemes and rates; block: residual stack over block sizes at 6x")
    ap.add_argument("--only", type=str, default="", help="with --per-layer: comma-separated layer indices to run")
    ap.add_argument("--reps", type=int, default=20, help="with --per-layer: timed launches per layer")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    import paper_2012_00596_amd as npas
    from tests import helpers
    from workloads import configs

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        n = args.copy_calibration * 2**20
        src = torch.arange(n // 4, dtype=torch.int32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(5):
            dst.copy_(src)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1) / 5
        e0.record()
        for _ in range(5):
            dst.zero_()
        e1.record()
        torch.cuda.synchronize()
        ms_w = e0.elapsed_time(e1) / 5
        e0.record()
        for _ in range(5):
            src.sum()
        e1.record()
        torch.cuda.synchronize()
        ms_r = e0.elapsed_time(e1) / 5
        print(json.dumps({"copy_calibration_bytes_read": n, "copy_calibration_bytes_written": n, "launches": 10,
                          "copy_GBps": 2 * n / ms / 1e6, "fill_GBps": n / ms_w / 1e6, "read_sum_GBps": n / ms_r / 1e6}))
        return
    if args.per_layer:
        return per_layer(args, torch, npas, helpers, configs)
    if args.stack:
        return stack_mode(args, torch, npas, helpers, configs)
    if args.sweep:
        return sweep_mode(args, torch, npas, helpers)
    w = configs.config2(batch=args.batch)
    N, H, W, C = w.x_shape
    npx = N * H * W
    packed = [helpers.pack_layer(npas, L, w.dtype) for L in w.layers]
    flags = 0 if args.no_fuse else npas.STACK_FUSE_POINTWISE
    st = npas.Stack(helpers.stack_descs(npas, w.layers, packed), H, W, flags)
    wsb = st.workspace_bytes(N)
    launches = st.num_launches()

    F1, F2 = w.layers[0].F, w.layers[1].F
    x_bytes, mid_bytes, y_bytes = npx * C * 2, npx * F1 * 2, npx * F2 * 2
    meta_bytes = sum(p.info()["device_bytes"] for p in packed)
    set_bytes = x_bytes + y_bytes + wsb
    nsets = 1 if args.no_rotate else max(2, -(-640 * 2**20 // set_bytes))
    xs = [helpers.to_dev(w.x_store, torch) for _ in range(nsets)]
    ys = [helpers.new_dev((N, H, W, F2), w.dtype, torch, fill=0) for _ in range(nsets)]
    wss = [torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
    stream = torch.cuda.current_stream().cuda_stream

    def step(i):
        k = i % nsets
        st.run(xs[k], ys[k], N, wss[k], wsb, stream)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    dt = (time.perf_counter() - t0) / args.steps

    # per-step device time with events on the launch stream (excludes host launch gaps only if the
    # queue stays full; reported next to the wall-clock figure)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.steps):
        step(i)
    e1.record()
    torch.cuda.synchronize()
    dev_ms = e0.elapsed_time(e1) / args.steps

    dense_flop = 2.0 * w.dense_macs()
    # dominant kernel: fused -> the only kernel (reads x, writes y); per-layer -> either layer moves
    # x/mid (read) + mid/y (write) = 67.4 MB, the slower one is timed
    if launches == 1:
        alg_bytes = x_bytes + y_bytes + meta_bytes
        kern_ms = dev_ms
        kname = "pointwise_pair_fused"
    else:
        alg_bytes = x_bytes + mid_bytes + packed[0].info()["device_bytes"]
        mids = [helpers.new_dev((N, H, W, F1), w.dtype, torch, fill=0) for _ in range(nsets)]
        per = []
        for li, L in enumerate(w.layers):
            e0.record()
            for i in range(args.steps):
                k = i % nsets
                if li == 0:
                    npas.conv2d_sparse(packed[0], xs[k], mids[k], N, H, W, 1, 0, None, None, L.act, stream)
                else:
                    npas.conv2d_sparse(packed[1], mids[k], ys[k], N, H, W, 1, 0, None, None, L.act, stream)
            e1.record()
            torch.cuda.synchronize()
            per.append(e0.elapsed_time(e1) / args.steps)
        kern_ms = max(per)
        kname = "%s (layer %d of 2)" % (npas.conv2d_kernel_name(packed[per.index(kern_ms)], N, H, W, 1, 0), per.index(kern_ms) + 1)
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    # HBM bytes per launch of the fused kernel as measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE scaled by a
    # plain copy); only valid for the default workload and launch configuration
    traffic = None
    tfile = os.path.join(ROOT, "profiles", "fused_pointwise_pair_cfg2_hbm_traffic.md")
    if launches == 1 and N == 64 and os.path.exists(tfile):
        for line in open(tfile):
            if line.startswith("traffic_bytes_per_launch:"):
                traffic = int(line.split(":")[1])

    out = {
        "metric": "dense-equivalent TFLOP/s and per-layer us for block-punched sparse conv at 1 GPU",
        "value": dense_flop / dt / 1e12,
        "unit": "TFLOP/s (dense-equivalent)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "device_ms_per_step": dev_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "configs[1]: 1x1 stack 24->144->24, batch %d, 56x56, bf16 NHWC, 8x8 blocks, 4x pruning, ReLU6"
                               % N, "launches_per_step": launches, "buffer_sets": nsets,
                   "dense_equiv_gflop_per_step": dense_flop / 1e9},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": traffic, "kernel": kname,
                     "algorithmic_bytes_per_launch": alg_bytes, "kernel_ms": kern_ms},
    }

    if not args.no_cpu:
        import oracle
        sample_px = 2 * H * W                      # two images' worth of pixels
        xsub = w.x_exact.reshape(npx, C)[:sample_px].reshape(1, 1, sample_px, C)
        t0 = time.perf_counter()
        reps = 0
        while time.perf_counter() - t0 < 10.0:
            oracle.run_stack(xsub, w.layers, w.dtype)
            reps += 1
        cdt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": dense_flop * (sample_px / npx) / cdt / 1e12,
                               "unit": "TFLOP/s (dense-equivalent)", "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%d of %d pixels of the same stack, %d repetitions" % (sample_px, npx, reps)}
    print(json.dumps(out))


def time_stack(w, reps, torch, npas, helpers, fuse=True, graph=False):
    """(us per npas_run_stack call, launches, workspace bytes) for workload w.  graph: the call is
    captured once into a HIP graph (the library allocates nothing and sets nothing during a run) and
    the replays are timed: what a serving loop at small batch would do about the launch gaps."""
    N, H, W, C = w.x_shape
    packed = [helpers.pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w.layers]
    st = npas.Stack(helpers.stack_descs(npas, w.layers, packed), H, W,
                    npas.STACK_FUSE_POINTWISE | npas.STACK_FUSE_INVERTED_RESIDUAL | npas.STACK_FUSE_CONV_MAXPOOL if fuse else 0)
    wsb = st.workspace_bytes(N)
    x = helpers.to_dev(w.x_store, torch)
    shapes = {0: w.x_shape}
    for i, L in enumerate(w.layers):
        shapes[i + 1] = helpers.out_shape(L, shapes[L.src])
    y = helpers.new_dev(shapes[len(w.layers)], w.dtype, torch, fill=0)
    ws = torch.empty(max(wsb, 256), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        st.run(x, y, N, ws, wsb, stream)
    torch.cuda.synchronize()
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            st.run(x, y, N, ws, wsb, torch.cuda.current_stream().cuda_stream)
        for _ in range(3):
            g.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(reps):
            g.replay()
        e1.record()
    else:
        e0.record()
        for _ in range(reps):
            st.run(x, y, N, ws, wsb, stream)
        e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps, st.num_launches(), wsb


def stack_mode(args, torch, npas, helpers, configs):
    """npas_run_stack end to end: one call runs every layer of the config on one stream."""
    cfg = args.stack
    from workloads import sweeps
    w = {2: lambda: configs.config2(batch=args.batch), 5: lambda: configs.config5(batch=args.batch),
         6: lambda: sweeps.inverted_residual_block(batch=args.batch)}[cfg]()
    us, launches, wsb = time_stack(w, args.reps, torch, npas, helpers, fuse=not args.no_fuse, graph=args.graph)
    flop = 2.0 * w.dense_macs()
    print("# config %d %s batch %d: npas_run_stack%s %.1f us per call, %d launches, workspace %.1f MB, %.1f TFLOP/s dense-equivalent, %.1f images/s"
          % (cfg, w.name, w.x_shape[0], " (HIP graph replay)" if args.graph else "", us, launches, wsb / 2**20, flop / us / 1e6,
             w.x_shape[0] / us * 1e6))


def sweep_mode(args, torch, npas, helpers):
    """The paper's two design-space sweeps (section 4) on synthetic layers: latency only."""
    from workloads import sweeps
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.sweep == "block":
        print("# residual stack, every pruned layer at 6x, batch %d: npas_run_stack per call" % args.batch)
        print("%-9s %10s %12s" % ("Bf x Bc", "us", "images/s"))
        for Bf, Bc in sweeps.BLOCK_SIZES:
            w = sweeps.block_sweep_stack(Bf, Bc, batch=args.batch)
            us, _, _ = time_stack(w, args.reps, torch, npas, helpers)
            print("%-9s %10.1f %12.1f" % ("%dx%d" % (Bf, Bc), us, args.batch / us * 1e6), flush=True)
        return
    print("# 3x3 conv 56x56x256 -> 256, stride 1, batch %d, bf16; us per launch (dense-equivalent TFLOP/s of the unpruned layer)" % args.batch)
    print("%-14s" % "scheme" + "".join("%22s" % ("%gx" % r) for r in sweeps.RATES))
    dense_flop = 2.0 * args.batch * 56 * 56 * 256 * 256 * 9
    for scheme in sweeps.RATE_SCHEMES:
        cells, kerns = [], set()
        for r in sweeps.RATES:
            if scheme == "pattern" and r < 2.25:
                cells.append("%22s" % "-")
                continue
            w = sweeps.rate_sweep_layer(scheme, r, batch=args.batch)
            L = w.layers[0]
            packed = helpers.pack_layer(npas, L, w.dtype)
            N, H, W_, C = w.x_shape
            x = helpers.to_dev(w.x_store, torch)
            y = helpers.new_dev((N, H, W_, L.F), w.dtype, torch, fill=0)
            for _ in range(3):
                npas.conv2d_sparse(packed, x, y, N, H, W_, 1, 1, None, None, 0, stream)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(args.reps):
                npas.conv2d_sparse(packed, x, y, N, H, W_, 1, 1, None, None, 0, stream)
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / args.reps
            kerns.add(npas.conv2d_kernel_name(packed, N, H, W_, 1, 1).replace("conv_", ""))
            cells.append("%22s" % ("%.1f (%.0f)" % (us, dense_flop / us / 1e6)))
            del packed, x, y
        print("%-14s" % scheme + "".join(cells) + "   " + ",".join(sorted(kerns)), flush=True)


def per_layer(args, torch, npas, helpers, configs):
    """Per-layer timing of one config, every layer on its own buffers (rotated when small)."""
    MFMA_PEAK, HBM_PEAK = 2500.0, 8000.0           # TFLOP/s (bf16 dense), GB/s
    cfg = args.per_layer
    from workloads import sweeps
    w = {1: configs.config1, 2: lambda: configs.config2(batch=args.batch), 3: configs.config3, 4: configs.config4,
         5: lambda: configs.config5(batch=args.batch), 6: lambda: sweeps.inverted_residual_block(batch=args.batch)}[cfg]()
    stream = torch.cuda.current_stream().cuda_stream
    shapes = {0: w.x_shape}
    rows = []
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    tot_us = tot_flop = tot_bytes = 0.0
    only = set(int(t) for t in args.only.split(",") if t)
    for i, L in enumerate(w.layers):
        ishape = shapes[L.src]
        oshape = helpers.out_shape(L, ishape)
        shapes[i + 1] = oshape
        if only and i not in only:
            continue
        esz = 4 if w.dtype == 0 else 2
        nin, nout = int(np.prod(ishape)), int(np.prod(oshape))
        packed = helpers.pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None
        wbytes = packed.info()["device_bytes"] if packed else 0
        if L.kind == "dwconv":
            wbytes = L.C * 9 * 2
        nin_alg = nin
        if L.kind == "conv" and L.KH == 1 and L.KW == 1 and L.stride > 1:
            nin_alg = nout // L.F * L.C  # a strided 1x1 layer needs only the input pixels it samples
        abytes = (nin_alg + nout + (nout if L.res >= 0 else 0)) * esz + wbytes
        nsets = max(1, min(8, -(-600 * 2**20 // max(1, (nin + nout) * esz))))
        td = torch.float32 if w.dtype == 0 else torch.int16
        xs = [torch.randint(-3, 3, (nin,), device="cuda").to(td) if w.dtype else torch.randn(nin, device="cuda")
              for _ in range(nsets)]
        if w.dtype == 1:   # small finite bf16 values
            xs = [(torch.randn(nin, device="cuda") ).to(torch.bfloat16).view(torch.int16) for _ in range(nsets)]
        ys = [torch.empty(nout, dtype=td, device="cuda") for _ in range(nsets)]
        rs = [torch.zeros(nout, dtype=td, device="cuda") for _ in range(nsets)] if L.res >= 0 else None

        def run(k):
            if L.kind == "conv":
                N, H, W_, _ = ishape
                npas.conv2d_sparse(packed, xs[k], ys[k], N, H, W_, L.stride, L.pad, None, rs[k] if rs else None, L.act, stream)
            elif L.kind == "fc":
                npas.fc_sparse(packed, xs[k], ys[k], ishape[0], None, L.act, stream)
            elif L.kind == "dwconv":
                N, H, W_, _ = ishape
                npas.depthwise3x3(packed, xs[k], ys[k], N, H, W_, L.stride, None, rs[k] if rs else None, L.act, stream)
            elif L.kind == "maxpool":
                N, H, W_, C = ishape
                npas.maxpool3x3s2(xs[k], ys[k], N, H, W_, C, w.dtype, stream)
            else:
                N, H, W_, C = ishape
                npas.global_avgpool(xs[k], ys[k], N, H, W_, C, w.dtype, stream)
        reps = args.reps
        for k in range(3):
            run(k % nsets)
        torch.cuda.synchronize()
        e0.record()
        for k in range(reps):
            run(k % nsets)
        e1.record()
        torch.cuda.synchronize()
        us = e0.elapsed_time(e1) * 1e3 / reps
        macs = 0
        if L.kind == "conv":
            macs = oshape[0] * oshape[1] * oshape[2] * L.F * L.C * L.KH * L.KW
        elif L.kind == "fc":
            macs = ishape[0] * L.F * L.C
        elif L.kind == "dwconv":
            macs = oshape[0] * oshape[1] * oshape[2] * L.C * 9
        flop = 2.0 * macs
        peak = 157.3 if (w.dtype == 0 or L.kind == "dwconv") else MFMA_PEAK    # fp32 and depthwise layers run on the vector ALUs
        t_hbm, t_mfma = abytes / (HBM_PEAK * 1e9) * 1e6, flop / (peak * 1e12) * 1e6
        bound = "hbm" if t_hbm >= t_mfma else ("alu" if (w.dtype == 0 or L.kind == "dwconv") else "mfma")
        frac = max(t_hbm, t_mfma) / us
        if L.kind == "conv":
            kern = npas.conv2d_kernel_name(packed, ishape[0], ishape[1], ishape[2], L.stride, L.pad)
        elif L.kind == "fc":
            kern = npas.conv2d_kernel_name(packed, ishape[0], 1, 1, 1, 0)
        else:
            kern = L.kind
        rows.append((i, L.name or L.kind, "x".join(map(str, ishape)), "x".join(map(str, oshape)), L.KH, L.stride, L.rate,
                     kern.replace("conv_", ""), us, flop / us / 1e6, abytes / us / 1e3, bound, frac))
        tot_us += us; tot_flop += flop; tot_bytes += abytes
        del xs, ys, rs
        torch.cuda.empty_cache()
    print("# config %d  %s  (us per launch; TFLOP/s dense-equivalent; GB/s algorithmic; frac = roofline floor / measured)" % (cfg, w.name))
    print("%3s %-12s %-18s %-18s %2s %1s %4s %-14s %9s %9s %9s %5s %6s" % ("i", "layer", "in", "out", "k", "s", "rate", "kernel", "us", "TFLOP/s", "GB/s", "bound", "frac"))
    for r in rows:
        print("%3d %-12s %-18s %-18s %2d %1d %4.1f %-14s %9.2f %9.2f %9.1f %5s %6.3f" % r)
    print("# total %.1f us  %.1f TFLOP/s dense-equivalent  %.1f GB/s algorithmic" % (tot_us, tot_flop / tot_us / 1e6, tot_bytes / tot_us / 1e3))


if __name__ == "__main__":
    main()
