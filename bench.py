#!/usr/bin/env python3
"""Benchmark of the sparse-inference hot path on one MI355X.

Default: one step = one npas_run_stack call on configs[4] of the benchmark definition at batch 128 (the 50-layer
bottleneck residual stack, every conv block-punched 8x4 at a per-layer rate from {2, 3, 5}, block-based
FC), bf16, inputs resident in HBM.  Prints ONE JSON line: dense-equivalent TFLOP/s of the whole stack
(value), median / min per step, the roofline of the stack (sum of per-layer floors / measured) and of the
kernel that takes most of its time, the launch floor measured in the same run, batch-1 latency, the
configs[1] fused-pair figure, and the CPU oracle timed on a bounded sample.

Other modes (tables for profiles/): --per-layer, --stack, --sweep, --copy-calibration.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # GB/s
MFMA_PEAK_TFLOPS = 2500.0      # bf16 / fp16 dense
VALU_PEAK_TFLOPS = 157.3       # fp32 vector
ALL_FUSIONS = 7                # STACK_FUSE_POINTWISE | _INVERTED_RESIDUAL | _CONV_MAXPOOL


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--batch", type=int, default=0, help="batch size (default: 128 for the headline stack, 64 for config 2)")
    ap.add_argument("--headline", type=int, default=5, choices=[2, 5],
                    help="which config the JSON line's value is quoted on: 5 = configs[4] (default), 2 = configs[1]")
    ap.add_argument("--no-fuse", action="store_true", help="no stack fusion flags (one launch per layer)")
    ap.add_argument("--no-rotate", action="store_true", help="reuse one buffer set")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-extras", action="store_true", help="skip the batch-1, configs[1] and per-layer legs of the headline run")
    ap.add_argument("--no-small", action="store_true", help="skip the batch-1 and configs[1] legs of the headline run (profiling: only batch-128 launches remain)")
    ap.add_argument("--per-layer", type=int, default=0, metavar="CFG",
                    help="instead of the headline line, print a per-layer table (us, dense-equivalent TFLOP/s, "
                         "algorithmic GB/s, roofline fraction) for config CFG in 1..5 (configs[CFG-1] of the benchmark definition); "
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
    ap.add_argument("--ir", type=str, default="", choices=["", "s2", "bias", "s2bias"],
                    help="config 6 (inverted-residual block): depthwise stride 2 and / or a bias on every layer")
    ap.add_argument("--reps", type=int, default=20, help="with --per-layer / --stack / --sweep: timed launches")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2012_00596_amd as npas
    from workloads import configs, harness

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    if args.copy_calibration:
        return copy_calibration(args, torch)
    if args.per_layer:
        return per_layer(args, torch, npas, harness, configs)
    if args.stack:
        return stack_mode(args, torch, npas, harness, configs)
    if args.sweep:
        return sweep_mode(args, torch, npas, harness)
    return headline(args, torch, npas, harness, configs)


# ---- shared pieces ---------------------------------------------------------------------------------------------

class StackRunner:
    """A packed workload as an npas_stack plus rotating device buffer sets."""

    def __init__(self, w, torch, npas, harness, flags, nsets):
        self.w, self.torch, self.npas = w, torch, npas
        self.N, self.H, self.W = w.x_shape[0], w.x_shape[1], w.x_shape[2]
        self.packed = [harness.pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w.layers]
        self.biases = harness.bias_tensors(w.layers, torch)   # device tensors the stack's layers point at
        self.st = npas.Stack(harness.stack_descs(npas, w.layers, self.packed, self.biases), self.H, self.W, flags)
        self.wsb = self.st.workspace_bytes(self.N)
        shapes = {0: w.x_shape}
        for i, L in enumerate(w.layers):
            shapes[i + 1] = harness.out_shape(L, shapes[L.src])
        self.shapes = shapes
        self.xs = [harness.to_dev(w.x_store, torch) for _ in range(nsets)]
        self.ys = [harness.new_dev(shapes[len(w.layers)], w.dtype, torch, fill=0) for _ in range(nsets)]
        self.wss = [torch.empty(max(self.wsb, 256), dtype=torch.uint8, device="cuda") for _ in range(nsets)]
        self.nsets = nsets
        self.stream = torch.cuda.current_stream().cuda_stream
        self.ptrs = [(x.data_ptr(), y.data_ptr(), ws.data_ptr()) for x, y, ws in zip(self.xs, self.ys, self.wss)]

    def step(self, i):
        xp, yp, wp = self.ptrs[i % self.nsets]
        self.st.run(xp, yp, self.N, wp, self.wsb, self.stream)

    def timed_graph(self, replays, warmup=5):
        """Device microseconds per step with one pass over all buffer sets captured in a HIP graph and replayed: for
        steps of a few microseconds, where the host cannot issue calls as fast as the device finishes them
        (npas_run_stack allocates and clears nothing, so it can be captured)."""
        torch = self.torch
        g = torch.cuda.CUDAGraph()
        keep = self.stream
        with torch.cuda.graph(g):
            self.stream = torch.cuda.current_stream().cuda_stream
            for k in range(self.nsets):
                self.step(k)
        self.stream = keep
        for _ in range(warmup):
            g.replay()
        torch.cuda.synchronize()
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(replays + 1)]
        ev[0].record()
        for i in range(replays):
            g.replay()
            ev[i + 1].record()
        torch.cuda.synchronize()
        return np.array([ev[i].elapsed_time(ev[i + 1]) * 1e3 / self.nsets for i in range(replays)])

    def timed(self, steps, warmup, chunk=1):
        """(wall seconds per step over all steps, per-step device milliseconds from events on the launch stream).
        chunk > 1: an event every `chunk` steps and their mean per step (an event between two launches of a few
        microseconds costs about as much as the launch)."""
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        steps = steps // chunk * chunk
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps // chunk + 1)]
        t0 = time.perf_counter()
        ev[0].record()
        for i in range(steps):
            self.step(i)
            if (i + 1) % chunk == 0:
                ev[(i + 1) // chunk].record()
        torch.cuda.synchronize()
        wall = (time.perf_counter() - t0) / steps
        per = np.array([ev[i].elapsed_time(ev[i + 1]) / chunk for i in range(steps // chunk)])
        return wall, per


def layer_costs(w, packed, harness):
    """Per layer: dense-equivalent and kept FLOPs, algorithmic bytes (activations in and out once, residual once,
    the canonical compact weights and their index: 4 bytes per list entry and per group), and the roofline floor."""
    esz = 4 if w.dtype == 0 else 2
    shapes = {0: w.x_shape}
    rows = []
    for i, L in enumerate(w.layers):
        ishape = shapes[L.src]
        oshape = harness.out_shape(L, ishape)
        shapes[i + 1] = oshape
        nin, nout = int(np.prod(ishape)), int(np.prod(oshape))
        macs = kept = 0
        wbytes = 0
        if L.kind in ("conv", "fc"):
            npix = nout // L.F
            macs = npix * L.F * L.C * L.KH * L.KW
            kept = npix * int(L.mask.sum())
            info = packed[i].info()
            wbytes = info["compact_weight_bytes"] + 4 * info["K_total"] + 4 * (info["G"] + 1)
        elif L.kind == "dwconv":
            macs = kept = nout * 9
            wbytes = L.C * 9 * esz
        nin_alg = nin
        if L.kind == "conv" and L.KH == 1 and L.KW == 1 and L.stride > 1:
            nin_alg = nout // L.F * L.C          # a strided 1x1 layer needs only the input pixels it samples
        abytes = (nin_alg + nout + (nout if L.res >= 0 else 0)) * esz + wbytes
        vec = w.dtype == 0 or L.kind == "dwconv"  # fp32 and depthwise layers run on the vector ALUs
        peak = VALU_PEAK_TFLOPS if vec else MFMA_PEAK_TFLOPS
        t_hbm, t_mm = abytes / (HBM_PEAK_GBS * 1e9) * 1e6, 2.0 * macs / (peak * 1e12) * 1e6
        rows.append(dict(i=i, L=L, ishape=ishape, oshape=oshape, nin=nin, nout=nout, flop=2.0 * macs, kept_flop=2.0 * kept,
                         abytes=abytes, wbytes=wbytes, t_hbm=t_hbm, t_mm=t_mm, floor_us=max(t_hbm, t_mm),
                         bound="hbm" if t_hbm >= t_mm else ("alu" if vec else "mfma")))
    return rows


def stack_floor_us(rows, fused_conv_pool=True):
    """Sum of the per-launch floors.  A conv whose max pool runs in the same launch neither writes the conv output
    nor reads it back: its floor is taken on input + pooled output."""
    total = 0.0
    skip = set()
    for k, r in enumerate(rows):
        if k in skip:
            continue
        L = r["L"]
        nxt = rows[k + 1] if k + 1 < len(rows) else None
        if fused_conv_pool and L.kind == "conv" and L.C < 8 and nxt is not None and nxt["L"].kind == "maxpool" and nxt["L"].src == k + 1:
            esz = 2
            b = (r["nin"] + nxt["nout"]) * esz + r["wbytes"]
            total += max(b / (HBM_PEAK_GBS * 1e9) * 1e6, r["t_mm"])
            skip.add(k + 1)
            continue
        total += r["floor_us"]
    return total


def time_layers(w, packed, rows, torch, npas, reps, only=()):
    """Times every layer on its own seeded-size buffers (rotated so that small layers do not sit in the cache);
    fills rows[i]['us'] and rows[i]['kernel']."""
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    esz = 4 if w.dtype == 0 else 2
    for r in rows:
        i, L, ishape, oshape = r["i"], r["L"], r["ishape"], r["oshape"]
        if only and i not in only:
            continue
        nin, nout = r["nin"], r["nout"]
        p = packed[i]
        nsets = max(1, min(8, -(-600 * 2**20 // max(1, (nin + nout) * esz))))
        td = torch.float32 if w.dtype == 0 else torch.int16
        if w.dtype == 0:
            xs = [torch.randn(nin, device="cuda") for _ in range(nsets)]
        elif w.dtype == 1:
            xs = [torch.randn(nin, device="cuda").to(torch.bfloat16).view(torch.int16) for _ in range(nsets)]
        else:
            xs = [torch.randn(nin, device="cuda").to(torch.float16).view(torch.int16) for _ in range(nsets)]
        ys = [torch.empty(nout, dtype=td, device="cuda") for _ in range(nsets)]
        rs = [torch.zeros(nout, dtype=td, device="cuda") for _ in range(nsets)] if L.res >= 0 else None
        bias = None if getattr(L, "bias", None) is None else torch.from_numpy(np.ascontiguousarray(L.bias, dtype=np.float32)).cuda()

        def run(k):
            if L.kind == "conv":
                N, H, W_, _ = ishape
                npas.conv2d_sparse(p, xs[k], ys[k], N, H, W_, L.stride, L.pad, bias, rs[k] if rs else None, L.act, stream)
            elif L.kind == "fc":
                npas.fc_sparse(p, xs[k], ys[k], ishape[0], bias, L.act, stream)
            elif L.kind == "dwconv":
                N, H, W_, _ = ishape
                npas.depthwise3x3(p, xs[k], ys[k], N, H, W_, L.stride, bias, rs[k] if rs else None, L.act, stream)
            elif L.kind == "maxpool":
                N, H, W_, C = ishape
                npas.maxpool3x3s2(xs[k], ys[k], N, H, W_, C, w.dtype, stream)
            else:
                N, H, W_, C = ishape
                npas.global_avgpool(xs[k], ys[k], N, H, W_, C, w.dtype, stream)
        for k in range(3):
            run(k % nsets)
        torch.cuda.synchronize()
        e0.record()
        for k in range(reps):
            run(k % nsets)
        e1.record()
        torch.cuda.synchronize()
        r["us"] = e0.elapsed_time(e1) * 1e3 / reps
        if L.kind == "conv":
            r["kernel"] = npas.conv2d_kernel_name(p, ishape[0], ishape[1], ishape[2], L.stride, L.pad)
        elif L.kind == "fc":
            r["kernel"] = npas.conv2d_kernel_name(p, ishape[0], 1, 1, 1, 0)
        else:
            r["kernel"] = L.kind
        del xs, ys, rs
        torch.cuda.empty_cache()


def launch_floor_us(torch, npas, n=2000):
    """Launch-to-launch time of an empty kernel on the stream the benchmark uses, measured now."""
    stream = torch.cuda.current_stream().cuda_stream
    npas.launch_empty(200, stream)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    npas.launch_empty(n, stream)
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / n


def graph_replay_floor_us(torch, npas, per_graph=55, replays=200):
    """The same floor with the empty launches captured in a HIP graph (per_graph launches per replay)."""
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        npas.launch_empty(per_graph, torch.cuda.current_stream().cuda_stream)
    for _ in range(5):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(replays):
        g.replay()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / (replays * per_graph)


def stored_traffic(layer_ids):
    """Mean measured HBM bytes per launch of the given layers of configs[4] at batch 128, from the committed counter
    summary (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, one run each; counters cannot be read from inside this process).
    None when the table is not there or lacks a layer."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "cfg5_batch128_hbm_traffic_per_layer.md")
    try:
        rows = {}
        for line in open(path):
            f = [c.strip() for c in line.split("|")]
            if len(f) >= 8 and f[1].isdigit():
                rows[int(f[1])] = (float(f[5]) + float(f[6])) * 1e6
        return float(np.mean([rows[i] for i in layer_ids]))
    except (OSError, KeyError, ValueError):
        return None


# ---- the headline line -----------------------------------------------------------------------------------------

def headline(args, torch, npas, harness, configs):
    cfg = args.headline
    batch = args.batch or (128 if cfg == 5 else 64)
    flags = 0 if args.no_fuse else ALL_FUSIONS
    w = configs.config5(batch=batch) if cfg == 5 else configs.config2(batch=batch)
    # buffer sets: the stack's working set at batch 128 (several hundred MB of intermediates) is far beyond the
    # 256 MB Infinity Cache on its own; two sets keep even the input and output cold.  configs[1] is 19 MB: rotate
    # through enough sets to exceed the cache.
    probe = StackRunner(w, torch, npas, harness, flags, 1)
    set_bytes = probe.wsb + sum(t.numel() * t.element_size() for t in (probe.xs[0], probe.ys[0]))
    nsets = 1 if args.no_rotate else max(2, min(64, -(-640 * 2**20 // set_bytes)))
    del probe
    torch.cuda.empty_cache()
    run = StackRunner(w, torch, npas, harness, flags, nsets)
    wall, per = run.timed(args.steps, args.warmup)
    launches = run.st.num_launches()
    dense_flop = 2.0 * w.dense_macs()
    rows = layer_costs(w, run.packed, harness)
    kept_flop = sum(r["kept_flop"] for r in rows)
    floor_us = stack_floor_us(rows, fused_conv_pool=bool(flags & 4))
    med_ms, min_ms = float(np.median(per)), float(per.min())

    name = ("configs[4]: 50-layer bottleneck residual stack, 224x224x3, batch %d, bf16 NHWC, every conv block-punched 8x4 at a "
            "per-layer rate from {2,3,5}, block-based 16x32 FC 2048->1000" % batch) if cfg == 5 else \
           ("configs[1]: 1x1 stack 24->144->24, batch %d, 56x56, bf16 NHWC, 8x8 blocks, 4x pruning, ReLU6" % batch)
    out = {
        "metric": "dense-equivalent TFLOP/s and per-layer us for block-punched sparse conv at 1 GPU",
        "value": dense_flop / wall / 1e12,
        "unit": "TFLOP/s (dense-equivalent)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3,
        "device_ms_per_step": {"median": med_ms, "min": min_ms, "mean": float(per.mean())},
        "kept_TFLOPs": kept_flop / wall / 1e12,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": name, "launches_per_step": launches, "buffer_sets": nsets, "images_per_s": batch / wall,
                   "workspace_MB": run.wsb / 2**20, "dense_equiv_gflop_per_step": dense_flop / 1e9,
                   "kept_gflop_per_step": kept_flop / 1e9,
                   "executed_gflop_per_step_note": "the MFMA kernels of this stack multiply every position of a 16-filter "
                   "tile that any of its filter groups keeps; at these rates that is the dense count (dense_equiv)"},
    }

    # roofline: the stack as a whole (sum of per-launch floors over the measured median), and the kernel that takes
    # most of the stack's time, from a per-layer timing pass of the same run
    roof = {"stack_floor_ms": floor_us / 1e3, "stack_frac": floor_us / 1e3 / med_ms,
            "stack_floor_note": "sum over launches of max(algorithmic bytes / 8 TB/s, dense-equivalent FLOP / 2.5 PFLOP/s); "
                                "bytes = activations in + out (+ residual) once + compact weights + 4 B per list entry"}
    if not args.no_extras:
        time_layers(w, run.packed, rows, torch, npas, max(5, min(20, args.steps // 5)))
        per_kernel = {}
        for r in rows:
            k = per_kernel.setdefault(r["kernel"], dict(launches=0, us=0.0, bytes=0.0, flop=0.0, floor_us=0.0))
            k["launches"] += 1; k["us"] += r["us"]; k["bytes"] += r["abytes"]; k["flop"] += r["flop"]; k["floor_us"] += r["floor_us"]
        for k in per_kernel.values():
            k["frac"] = k["floor_us"] / k["us"]
            k["GBps"] = k["bytes"] / k["us"] / 1e3
            k["TFLOPs_dense_equiv"] = k["flop"] / k["us"] / 1e6
        dom = max(per_kernel, key=lambda n: per_kernel[n]["us"])
        d = per_kernel[dom]
        hbm_rows = [r for r in rows if r["kernel"] == dom and r["bound"] == "hbm"]
        mm_rows = [r for r in rows if r["kernel"] == dom and r["bound"] != "hbm"]
        hbm_us, mm_us = sum(r["us"] for r in hbm_rows), sum(r["us"] for r in mm_rows)
        if hbm_us >= mm_us:      # the dominant kernel's launches are mostly HBM-bound ones: quote it on those
            ach = sum(r["abytes"] for r in hbm_rows) / hbm_us / 1e3
            roof.update(bound="hbm", achieved=ach, peak=HBM_PEAK_GBS, unit="GB/s", frac=ach / HBM_PEAK_GBS,
                        launches_counted=len(hbm_rows), avg_launch_us=hbm_us / len(hbm_rows),
                        algorithmic_bytes_per_launch=sum(r["abytes"] for r in hbm_rows) / len(hbm_rows))
        else:
            ach = sum(r["flop"] for r in mm_rows) / mm_us / 1e6
            roof.update(bound="mfma", achieved=ach, peak=MFMA_PEAK_TFLOPS, unit="TFLOP/s", frac=ach / MFMA_PEAK_TFLOPS,
                        launches_counted=len(mm_rows), avg_launch_us=mm_us / len(mm_rows),
                        algorithmic_flop_per_launch=sum(r["flop"] for r in mm_rows) / len(mm_rows))
        counted = hbm_rows if hbm_us >= mm_us else mm_rows
        stored = stored_traffic([r["i"] for r in counted]) if cfg == 5 and batch == 128 else None
        roof.update(kernel=dom, traffic=stored,
                    traffic_note=("STORED figure, not measured in this run: mean HBM bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain "
                                  "copy) of the same launches, read from profiles/cfg5_batch128_hbm_traffic_per_layer.md" if stored is not None else
                                  "not measured inside this run; rocprofv3 --pmc figures per layer are in profiles/"),
                    kernel_share_of_stack_time=d["us"] / sum(k["us"] for k in per_kernel.values()))
        out["per_kernel"] = {n: {a: (round(b, 4) if isinstance(b, float) else b) for a, b in k.items() if a not in ("bytes", "flop")}
                             for n, k in per_kernel.items()}
        out["per_layer_sum_ms"] = sum(r["us"] for r in rows) / 1e3
        floor = launch_floor_us(torch, npas)
        out["launch_floor_us"] = {"empty_kernel": floor, "times_launches": floor * launches,
                                  "empty_kernel_in_graph_replay": graph_replay_floor_us(torch, npas, launches)}
    else:
        roof.update(bound="hbm", achieved=None, peak=HBM_PEAK_GBS, unit="GB/s", frac=floor_us / 1e3 / med_ms, traffic=None)
    out["roofline"] = roof

    if not args.no_extras and not args.no_small and cfg == 5:
        # the same stack at batch 1 (latency), and the configs[1] fused pair
        del run
        torch.cuda.empty_cache()
        w1 = configs.config5(batch=1)
        r1 = StackRunner(w1, torch, npas, harness, flags, 4)
        _, p1 = r1.timed(200, 20, chunk=10)
        out["batch1"] = {"workload": "configs[4] at batch 1", "timing": "means over 10 consecutive steps", "median_us": float(np.median(p1)) * 1e3, "min_us": float(p1.min()) * 1e3,
                         "launches": r1.st.num_launches(), "floor_us": stack_floor_us(layer_costs(w1, r1.packed, harness)),
                         "launch_floor_us": out["launch_floor_us"]["empty_kernel"] * r1.st.num_launches()}
        del r1
        w2 = configs.config2(batch=64)
        x2 = int(np.prod(w2.x_shape)) * 2
        r2 = StackRunner(w2, torch, npas, harness, flags, max(2, -(-640 * 2**20 // (2 * x2))))
        _, p2h = r2.timed(1000, 50, chunk=50)
        p2 = r2.timed_graph(40) / 1e3   # ms per launch
        b2 = 2 * x2 + sum(4 * p.info()["K_total"] + p.info()["compact_weight_bytes"] for p in r2.packed)
        med2 = float(np.median(p2)) * 1e3
        out["config2_fused_pair"] = {"workload": "configs[1]: 24->144->24, batch 64, 56x56, one fused launch",
                                     "timing": "one pass over the rotating buffer sets captured in a HIP graph, 40 replays, mean per launch of a replay",
                                     "host_issued_median_us": float(np.median(p2h)) * 1e3, "median_us": med2,
                                     "min_us": float(p2.min()) * 1e3, "launches": r2.st.num_launches(),
                                     "algorithmic_bytes": b2, "GBps": b2 / med2 / 1e3, "hbm_frac": b2 / med2 / 1e3 / HBM_PEAK_GBS,
                                     "TFLOPs_dense_equiv": 2.0 * w2.dense_macs() / med2 / 1e6}
        del r2
        r2w = StackRunner(w2, torch, npas, harness, flags, 1)   # one buffer set: input and output stay in the Infinity Cache
        r2w.ptrs = r2w.ptrs * 32   # the same set 32 times per replay
        r2w.nsets = 32
        out["config2_fused_pair"]["warm_median_us"] = float(np.median(r2w.timed_graph(40)))
        del r2w
        torch.cuda.empty_cache()

    if not args.no_cpu:
        import oracle
        nimg = min(2, batch) if cfg == 5 else 1
        if cfg == 5:
            xsub = w.x_exact[:nimg]
            frac = nimg / batch
            what = "%d of %d images of the same stack" % (nimg, batch)
        else:
            npx = int(np.prod(w.x_shape[:3]))
            spx = 2 * w.x_shape[1] * w.x_shape[2]
            xsub = w.x_exact.reshape(npx, -1)[:spx].reshape(1, 1, spx, -1)
            frac = spx / npx
            what = "%d of %d pixels of the same stack" % (spx, npx)
        t0 = time.perf_counter()
        reps = 0
        while reps < 1 or time.perf_counter() - t0 < 10.0:
            oracle.run_stack(xsub, w.layers, w.dtype)
            reps += 1
        cdt = (time.perf_counter() - t0) / reps
        out["cpu_baseline"] = {"value": dense_flop * frac / cdt / 1e12, "unit": "TFLOP/s (dense-equivalent)",
                               "cores": oracle.num_threads(), "kind": "oracle",
                               "sample": "%s, %d repetition(s), %.2f s each, scaled to the unit" % (what, reps, cdt)}
    print(json.dumps(out))


# ---- tables ----------------------------------------------------------------------------------------------------

def copy_calibration(args, torch):
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


def time_stack(w, reps, torch, npas, harness, fuse=True, graph=False):
    """(us per npas_run_stack call, launches, workspace bytes) for workload w.  graph: the call is
    captured once into a HIP graph (the library allocates nothing and sets nothing during a run) and
    the replays are timed: what a serving loop at small batch would do about the launch gaps."""
    run = StackRunner(w, torch, npas, harness, ALL_FUSIONS if fuse else 0, 1)
    x, y, ws, N = run.xs[0], run.ys[0], run.wss[0], run.N
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for _ in range(5):
        run.step(0)
    torch.cuda.synchronize()
    if graph:
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            run.st.run(x, y, N, ws, run.wsb, torch.cuda.current_stream().cuda_stream)
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
            run.step(0)
        e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e3 / reps, run.st.num_launches(), run.wsb


def stack_mode(args, torch, npas, harness, configs):
    """npas_run_stack end to end: one call runs every layer of the config on one stream."""
    cfg = args.stack
    from workloads import sweeps
    batch = args.batch or 64
    w = {2: lambda: configs.config2(batch=batch), 5: lambda: configs.config5(batch=batch),
         6: lambda: sweeps.inverted_residual_block(batch=batch, stride=2 if "s2" in args.ir else 1, bias="bias" in args.ir)}[cfg]()
    us, launches, wsb = time_stack(w, args.reps, torch, npas, harness, fuse=not args.no_fuse, graph=args.graph)
    flop = 2.0 * w.dense_macs()
    print("# config %d %s batch %d: npas_run_stack%s %.1f us per call, %d launches, workspace %.1f MB, %.1f TFLOP/s dense-equivalent, %.1f images/s"
          % (cfg, w.name, w.x_shape[0], " (HIP graph replay)" if args.graph else "", us, launches, wsb / 2**20, flop / us / 1e6,
             w.x_shape[0] / us * 1e6))


def sweep_mode(args, torch, npas, harness):
    """The paper's two design-space sweeps (section 4) on synthetic layers: latency only."""
    from workloads import sweeps
    batch = args.batch or 64
    stream = torch.cuda.current_stream().cuda_stream
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    if args.sweep == "block":
        print("# residual stack, every pruned layer at 6x, batch %d: npas_run_stack per call" % batch)
        print("%-9s %10s %12s" % ("Bf x Bc", "us", "images/s"))
        for Bf, Bc in sweeps.BLOCK_SIZES:
            w = sweeps.block_sweep_stack(Bf, Bc, batch=batch)
            us, _, _ = time_stack(w, args.reps, torch, npas, harness)
            print("%-9s %10.1f %12.1f" % ("%dx%d" % (Bf, Bc), us, batch / us * 1e6), flush=True)
        return
    print("# 3x3 conv 56x56x256 -> 256, stride 1, batch %d, bf16; us per launch (dense-equivalent TFLOP/s of the unpruned layer)" % batch)
    print("%-14s" % "scheme" + "".join("%22s" % ("%gx" % r) for r in sweeps.RATES))
    dense_flop = 2.0 * batch * 56 * 56 * 256 * 256 * 9
    for scheme in sweeps.RATE_SCHEMES:
        cells, kerns = [], set()
        for r in sweeps.RATES:
            if scheme == "pattern" and r < 2.25:
                cells.append("%22s" % "-")
                continue
            w = sweeps.rate_sweep_layer(scheme, r, batch=batch)
            L = w.layers[0]
            packed = harness.pack_layer(npas, L, w.dtype)
            N, H, W_, C = w.x_shape
            x = harness.to_dev(w.x_store, torch)
            y = harness.new_dev((N, H, W_, L.F), w.dtype, torch, fill=0)
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


def per_layer(args, torch, npas, harness, configs):
    """Per-layer timing of one config, every layer on its own buffers (rotated when small)."""
    cfg = args.per_layer
    from workloads import sweeps
    batch = args.batch or (128 if cfg == 5 else 64)
    w = {1: configs.config1, 2: lambda: configs.config2(batch=batch), 3: configs.config3, 4: configs.config4,
         5: lambda: configs.config5(batch=batch),
         6: lambda: sweeps.inverted_residual_block(batch=batch, stride=2 if "s2" in args.ir else 1, bias="bias" in args.ir)}[cfg]()
    packed = [harness.pack_layer(npas, L, w.dtype) if L.kind in ("conv", "fc", "dwconv") else None for L in w.layers]
    rows = layer_costs(w, packed, harness)
    only = set(int(t) for t in args.only.split(",") if t)
    time_layers(w, packed, rows, torch, npas, args.reps, only)
    rows = [r for r in rows if "us" in r]
    print("# config %d  %s  (us per launch; TFLOP/s dense-equivalent; GB/s algorithmic, weights counted in compact form + index; "
          "frac = roofline floor / measured)" % (cfg, w.name))
    print("%3s %-12s %-18s %-18s %2s %1s %4s %-14s %9s %9s %9s %5s %6s" % ("i", "layer", "in", "out", "k", "s", "rate", "kernel", "us", "TFLOP/s", "GB/s", "bound", "frac"))
    for r in rows:
        L = r["L"]
        print("%3d %-12s %-18s %-18s %2d %1d %4.1f %-14s %9.2f %9.2f %9.1f %5s %6.3f"
              % (r["i"], L.name or L.kind, "x".join(map(str, r["ishape"])), "x".join(map(str, r["oshape"])), L.KH, L.stride, L.rate,
                 r["kernel"].replace("conv_", ""), r["us"], r["flop"] / r["us"] / 1e6, r["abytes"] / r["us"] / 1e3, r["bound"],
                 r["floor_us"] / r["us"]))
    tot_us = sum(r["us"] for r in rows)
    print("# total %.1f us  %.1f TFLOP/s dense-equivalent  %.1f GB/s algorithmic  sum of floors %.1f us (%.3f of the total)"
          % (tot_us, sum(r["flop"] for r in rows) / tot_us / 1e6, sum(r["abytes"] for r in rows) / tot_us / 1e3,
             sum(r["floor_us"] for r in rows), sum(r["floor_us"] for r in rows) / tot_us))


if __name__ == "__main__":
    main()
