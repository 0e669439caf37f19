#!/usr/bin/env python3
"""Benchmark of direct sparse convolution on one MI355X.

A step is one pass of the hot path over one batch: the sparse convolution of
every layer of the workload on its resident (already in HBM) input.  Prints one
JSON line: effective GFLOP/s = 2 * stored weights * E * F * N / time, the
roofline position of the tile kernel, per-layer figures and the CPU oracle
timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

from paper_2011_06295_amd.roofs import (HBM_PEAK, LDS_PEAK, VALU_PEAK_FMA, MEASURED_LDS_B_PER_CLK_PER_CU,  # noqa: E402
                                        MEASURED_TRAFFIC_BYTES_PER_LAUNCH,
                                        MEASURED_COPY_BYTES_PER_S, CUS, CLOCK_HZ, PROFILE as ROOF_PROFILE)

# what the default run reports beside the headline (configs 2, 4, 5 and 1 of the benchmark list)
CONFIG_LINES = ("vgg16_f16", "sweep90", "sweep95", "sweep99", "sweep90r", "lenet5", "config1")


def make_workload(name: str):
    from paper_2011_06295_amd import workloads as wl
    if name == "vgg16_f32":
        return wl.vgg16(128, "f32"), None
    if name == "vgg16_f16":
        return wl.vgg16(256, "f16"), None
    if name == "lenet5":
        return wl.lenet5(64), None
    if name == "config1":
        return wl.config1(), None
    for base, fn in (("resnet1x1", wl.resnet_1x1), ("densenet1x1", wl.densenet_1x1), ("cnn1d", wl.cnn_1d),
                     ("vgg16_224", wl.vgg16_imagenet)):
        if name in (base, base + "_f16"):
            return fn(128, "f16" if name.endswith("_f16") else "f32"), None
    if name.startswith("sweep"):      # sweep90, sweep95r (r = ragged rows)
        ragged = name.endswith("r")
        s = int(name[5:].rstrip("r")) * 100
        return wl.sweep_layer(s, ragged), [wl.sweep_layer_index(s, ragged)]
    raise SystemExit(f"unknown workload {name}")


def layer_roofs(run, N, b):
    s = run.spec
    macs = run.macs(N)
    hbm_bytes = N * s.C * s.H * s.W * b + N * s.K * s.E * s.F * b + run.nnz * (b + 4) + (s.K + 1) * 4
    return {
        "macs": macs,
        "hbm_bytes": hbm_bytes,
        "lds_bytes": macs * b,
        "t_hbm": hbm_bytes / HBM_PEAK,
        "t_lds": macs * b / LDS_PEAK,
        "t_valu": macs / VALU_PEAK_FMA,
    }


def oracle_leg(net, work, budget_s=12.0, npts=2000, time_it=True):
    """The CPU oracle leg, after the timed region: (1) sampled outputs of every layer, as the timed launches
    left them in the first buffer set, against the oracle's exact-order double sums of the same operands;
    (2) the oracle itself (float accumulation, one thread) timed on the first n images of every layer."""
    import oracle
    tol = 2e-3 if work.dtype == "f16" else 1e-5
    worst, checked = 0.0, 0
    for li, (r, (w, m)) in enumerate(zip(net.runs, net.host_weights)):
        s = r.spec
        x = r.x.float().cpu().numpy()
        y = r.y.float().cpu().numpy()
        rng = np.random.default_rng(4242 + li)
        pool = 2 if getattr(r, "fused_pool", False) else 1      # fused store: sampled windows instead of sampled elements
        pts = np.stack([rng.integers(0, x.shape[0], npts), rng.integers(0, s.K, npts),
                        rng.integers(0, s.E // pool, npts), rng.integers(0, s.F // pool, npts)], 1).astype(np.int32)
        rowptr, colidx, values = oracle.csr_encode(w, m)
        if net.unified:
            rowptr, colidx, values = r.layer.csr()
            values = values if work.dtype != "f16" else values.view(np.float16).astype(np.float32)
        if work.dtype == "f16":
            values, x = oracle.round_through_f16(values), oracle.round_through_f16(x)
        if pool == 2:
            ref = None
            for di in (0, 1):
                for dj in (0, 1):
                    q = pts.copy()
                    q[:, 2], q[:, 3] = 2 * pts[:, 2] + di, 2 * pts[:, 3] + dj
                    v = oracle.sparse_conv_points((rowptr, colidx, values), x, s.K, s.R, s.S, s.stride, s.pad, q)
                    ref = v if ref is None else np.maximum(ref, v)
        else:
            ref = oracle.sparse_conv_points((rowptr, colidx, values), x, s.K, s.R, s.S, s.stride, s.pad, pts)
        if getattr(r, "fused_relu", False):
            ref = np.maximum(ref, 0.0)
        got = y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]].astype(np.float64)
        scale = float(np.abs(ref).max()) or 1.0
        worst = max(worst, float(np.abs(got - ref).max()) / scale)
        checked += npts
    parity = {"checked": checked, "max_rel": worst, "tolerance": tol, "ok": bool(worst <= tol),
              "rule": "max |gpu - oracle| / max |oracle| per layer, sampled outputs of the timed launches"}
    return parity, (cpu_baseline(oracle, net, work, budget_s) if time_it else None)


def cpu_baseline(oracle, net, work, budget_s=12.0):
    """The oracle (float accumulation, one thread) on the first n images of every layer."""
    # operands exactly as the GPU saw them
    ins = [r.x.float().cpu().numpy() for r in net.runs]

    def run_sample(n):
        t0 = time.perf_counter()
        macs = 0
        for r, (w, m), x in zip(net.runs, net.host_weights, ins):
            csr = oracle.csr_encode(w, m)
            oracle.sparse_conv(csr, x[:n], r.spec.K, r.spec.R, r.spec.S, r.spec.stride, r.spec.pad, acc="f32")
            macs += r.macs(n)
        return time.perf_counter() - t0, macs

    t1, m1 = run_sample(1)
    n = int(max(1, min(work.N, budget_s / max(t1, 1e-6))))
    if n > 1:
        t, macs = run_sample(n)
    else:
        t, macs = t1, m1
    return {
        "value": 2.0 * macs / t / 1e9, "unit": "GFLOP/s", "cores": 1, "cores_available": os.cpu_count(),
        "kind": "oracle",
        "sample": f"first {n} of {work.N} images through all {len(net.runs)} layers "
                  f"({macs:.3g} MACs in {t:.1f} s, float accumulation, single thread: 1 of {os.cpu_count()} cores)",
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="vgg16_f32",
                    help="vgg16_f32 (default: VGG-16 for 32x32 images, batch 128), vgg16_f16 (batch 256), lenet5, config1, "
                         "sweepNN / sweepNNr (256->256 14x14 layer at NN %% sparsity, unified / ragged rows), "
                         "resnet1x1, densenet1x1, cnn1d, vgg16_224 (each also with _f16)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle leg (sampled comparison and baseline timing)")
    ap.add_argument("--configs", type=int, default=1,
                    help="1: the default workload's line also carries `configs`, the other benchmark configurations "
                         "(vgg16_f16, the 14x14 layer at 90/95/99 %% and with ragged rows, lenet5, config1), each tuned and "
                         "timed by the same protocol; 0: the one workload only")
    ap.add_argument("--codebook", action="store_true",
                    help="cluster-quantised layers: weights given as 4-bit centroid numbers into 16 binary16 centroids "
                         "(the device entries are 4 bytes instead of 8)")
    ap.add_argument("--tuning-table", default="",
                    help="JSON file keyed by layer geometry (dtype,N,C,H,W,K,R,S,stride,pad,nnz): if it exists and knows "
                         "every layer, their launch configurations (and dense/sparse routes) are pinned from it instead of "
                         "being measured again; after the run the table is written back with what was used")
    ap.add_argument("--probe", action="store_true",
                    help="measure the roofs instead of a workload: LDS read rate of the gather's access pattern and the "
                         "rate of a plain copy, with the library's probe kernels; prints one JSON line")
    ap.add_argument("--launch", default="", help="comma separated launch override applied to every layer")
    ap.add_argument("--autotune", type=int, default=12,
                    help="before the warm-up, let every layer measure this many of its best-ranked launch "
                         "configurations and keep the fastest (0: the cost estimate's first choice)")
    ap.add_argument("--compare-dense", action="store_true",
                    help="also time the platform's dense convolution (torch / MIOpen) per layer and report which "
                         "of the two a dispatcher would pick")
    ap.add_argument("--buffer-mib", type=int, default=512,
                    help="the timed steps go round copies of the resident activations that together hold at least "
                         "this much (at most 16 copies), so that the last-level cache cannot serve them; 0: one set")
    ap.add_argument("--refine-top", type=int, default=12,
                    help="best-ranked candidates the second look times beside the measured choice")
    ap.add_argument("--unify", action="store_true",
                    help="create the layers with the unify flag (rows padded with explicit zeros to the fullest row's "
                         "count): `value` then counts the stored entries, `useful_value` the kept weights only")
    ap.add_argument("--refine", type=int, default=1,
                    help="1: after the measured launch choice, time each layer's choice, the cost estimate's first choice "
                         "and both kinds of output store inside a pass and keep the fastest (0: skip)")
    ap.add_argument("--fused", action="store_true",
                    help="the ReLU and the 2 x 2 maximum that follow a layer in the workload are done in its store step "
                         "(the pooled layers then write a quarter of the output)")
    ap.add_argument("--graph", type=int, default=1,
                    help="1: also record the K timed steps into one HIP graph and report its replay per step (0: skip)")
    ap.add_argument("--copy-probe-mib", type=int, default=0,
                    help="after the timed steps, copy a device buffer of this size once (a kernel of known "
                         "traffic that calibrates rocprofv3's FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (the path shards by batch with no exchange "
                         "step; no multi-GPU figure is produced). Use --gpus 1.")

    import torch
    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (there is no CPU fallback of the product path)")
    if args.probe:
        print(json.dumps(probe_roofs()))
        return
    out = run_workload(args.workload, args, args.steps, args.warmup, brief=False)
    if args.configs and args.workload == "vgg16_f32" and not args.launch and not args.unify and not args.codebook and not args.fused:
        # the other benchmark configurations, each tuned and timed by the same protocol (fewer steps, no
        # per-layer table, no CPU timing; the sampled comparison with the oracle stays)
        out["configs"] = []
        for name in CONFIG_LINES:
            r = run_workload(name, args, min(args.steps, 20), min(args.warmup, 5), brief=True)
            line = {"workload": name, "batch": r["config"]["batch"], "dtype": r["dtype"], "ms_per_step": r["ms_per_step"],
                    "graph_ms_per_step": r["graph_ms_per_step"],
                    "value": r["value"], "unit": r["unit"], "bound": r["roofline"]["bound"],
                    "roofline_frac": r["roofline"]["frac"], "lds_frac": r["roofline"]["lds_frac"],
                    "launches_per_step": r["roofline"]["launches_per_step"]}
            if "parity" in r:
                line["parity"] = {k: r["parity"][k] for k in ("checked", "max_rel", "ok")}
            out["configs"].append(line)
    print(json.dumps(out))


def probe_roofs():
    """Measured roofs: the LDS read rate of the gather's access pattern and the rate of a plain copy."""
    import torch
    from paper_2011_06295_amd import binding as B
    stream = torch.cuda.current_stream().cuda_stream
    out = {"clock_hz_assumed": CLOCK_HZ, "cus": CUS}
    wgs, iters = CUS * 4, 4000
    sink = torch.empty(wgs * 1024, dtype=torch.float32, device="cuda")
    B.sparse_conv_probe_lds_read(sink.data_ptr(), wgs, 50, stream)
    torch.cuda.synchronize()
    best = None
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        nbytes = B.sparse_conv_probe_lds_read(sink.data_ptr(), wgs, iters, stream)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3
        best = t if best is None else min(best, t)
    out["lds_read_TBs"] = nbytes / best / 1e12
    out["lds_B_per_clk_per_CU"] = nbytes / best / CUS / CLOCK_HZ
    out["lds_frac_of_published"] = nbytes / best / LDS_PEAK
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    B.sparse_conv_probe_copy(dst.data_ptr(), src.data_ptr(), n, stream)
    torch.cuda.synchronize()
    best = None
    for _ in range(5):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        B.sparse_conv_probe_copy(dst.data_ptr(), src.data_ptr(), n, stream)
        e1.record()
        torch.cuda.synchronize()
        t = e0.elapsed_time(e1) * 1e-3
        best = t if best is None else min(best, t)
    assert torch.equal(dst, src)
    out["copy_GiB"] = n >> 30
    out["copy_read_plus_write_GBs"] = 2 * n / best / 1e9
    out["copy_frac_of_published_hbm"] = 2 * n / best / HBM_PEAK
    return out


def run_workload(name, args, steps, warmup, brief):
    import torch
    from paper_2011_06295_amd import harness, workloads as wl

    work, layer_ids = make_workload(name)
    net = harness.Network(work, unify=args.unify, layer_ids=layer_ids, codebook=args.codebook, fuse=args.fused)
    if args.launch:
        for r in net.runs:
            r.layer.set_launch([int(v) for v in args.launch.split(",")])
    net.run_chain(wl.make_input(work))
    N = work.N
    b = 2 if work.dtype == "f16" else 4
    pinned = [int(v) for v in args.launch.split(",")] if args.launch else []
    tune = args.autotune > 0 and not all(pinned[:4] + [len(pinned) >= 4])   # a launch shape given in full is taken as it is
    known = 0
    if args.tuning_table and os.path.exists(args.tuning_table) and not args.launch:
        known = net.load_table(args.tuning_table)      # launches (and routes) measured by an earlier run
        tune = tune and known < len(net.runs)
    if tune:
        net.autotune(args.autotune)

    # Buffer sets: the timed steps go round copies of the resident activations that together exceed
    # the last-level cache (256 MB), so that no step finds its operands left there by the one before;
    # the same loop on a single set is reported beside it as the cache-hot figure.
    nsets = net.make_buffer_sets(args.buffer_mib << 20) if args.buffer_mib > 0 else 1
    if tune and args.refine:
        net.refine_in_context(top=args.refine_top)

    runners = net.prepare_steps()   # one per buffer set: the step's calls, checked and marshalled beforehand

    def timed(rotate):
        for i in range(warmup):
            runners[i % nsets if rotate else 0]()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record()
        for i in range(steps):
            runners[i % nsets if rotate else 0]()
        e1.record()
        torch.cuda.synchronize()
        return time.perf_counter() - t0, e0.elapsed_time(e1)

    hot_wall = timed(False)[0] if not brief else 0.0
    wall, gpu_ms = timed(True)
    ms_per_step = wall * 1e3 / steps

    # The same K steps recorded once into a HIP graph (on a stream of their own) and replayed: what the step
    # costs when the host issues one graph launch instead of a launch per layer.  The launches record no
    # memset nodes and allocate nothing once every geometry has run.
    graph_ms = None
    if args.graph:
        side = torch.cuda.Stream()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.stream(side):
            recorded = net.prepare_steps()
            with torch.cuda.graph(graph, stream=side):
                for i in range(steps):
                    recorded[i % nsets]()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        best = None
        for _ in range(3):
            t0 = time.perf_counter()
            graph.replay()
            torch.cuda.synchronize()
            t = time.perf_counter() - t0
            best = t if best is None else min(best, t)
        graph_ms = best * 1e3 / steps
        del graph

    # per-layer durations, in the order and cache state of a step: events between the launches of
    # further (untimed) steps on the launch stream
    reps = 0 if brief else max(10, min(steps, 50))
    # (an event between two launches keeps them apart by a few microseconds, which a step does not have: what the
    # intervals of a pass add up to beyond the duration of a timed step is taken off the layers in equal shares)
    marks = [[torch.cuda.Event(enable_timing=True) for _ in range(len(net.runs) + 1)] for _ in range(reps)]
    for j, ev in enumerate(marks):
        calls = runners[j % nsets].calls
        ev[0].record()
        for i, enqueue in enumerate(calls):
            enqueue()
            ev[i + 1].record()
    torch.cuda.synchronize()
    raw = [sum(ev[i].elapsed_time(ev[i + 1]) for ev in marks) * 1e-3 / reps for i in range(len(net.runs))] if reps else []
    event_gap = max(0.0, (sum(raw) - gpu_ms * 1e-3 / steps) / len(net.runs)) if reps else 0.0
    layers = []
    for i, r in enumerate(net.runs):
        if brief:
            break
        t_raw = raw[i]
        t = max(t_raw - event_gap, 0.25 * t_raw)
        roofs = layer_roofs(r, N, b)
        bound = max(("hbm", roofs["t_hbm"]), ("lds", roofs["t_lds"]), ("alu", roofs["t_valu"]), key=lambda kv: kv[1])
        layers.append({
            "name": r.spec.name, "shape": f"{r.spec.C}x{r.spec.H}x{r.spec.W}->{r.spec.K}",
            "nnz": r.nnz, "us": round(t * 1e6, 2), "us_between_events": round(t_raw * 1e6, 2),
            "gflops": round(2 * roofs["macs"] / t / 1e9, 1),
            "bound": bound[0], "roof_frac": round(bound[1] / t, 4),
            "hbm_GBs": round(roofs["hbm_bytes"] / t / 1e9, 1), "lds_GBs": round(roofs["lds_bytes"] / t / 1e9, 1),
            "launch": {k: v for k, v in r.layer.get_launch(N, r.spec.H, r.spec.W, r.spec.stride, r.spec.pad).items()
                       if k in ("V", "WP", "WK", "KW", "Cc", "LP", "kblocks", "store", "lanes", "csplit", "grid", "lds_bytes", "threads")},
        })

    if args.copy_probe_mib > 0:
        src = torch.empty(args.copy_probe_mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)      # reads and writes copy_probe_mib MiB
        torch.cuda.synchronize()
        del src, dst

    total_macs = net.total_macs()
    roofs = [layer_roofs(r, N, b) for r in net.runs]
    nl = len(net.runs)
    avg_launch_s = gpu_ms * 1e-3 / (steps * nl)
    sums = {k: sum(rf[k] for rf in roofs) for k in ("t_hbm", "t_lds", "t_valu", "lds_bytes", "hbm_bytes")}
    # the binding roof is the largest of the three times (fp32: the LDS read rate and the non-packed multiply-add
    # rate tie, reported as LDS; fp16: half the LDS bytes per multiply-add, so the multiply-add rate binds)
    if sums["t_valu"] > sums["t_lds"] and sums["t_valu"] >= sums["t_hbm"]:
        roofline = {"bound": "alu", "achieved": 2.0 * total_macs / nl / avg_launch_s / 1e12,
                    "peak": 2.0 * VALU_PEAK_FMA / 1e12, "unit": "TFLOP/s"}
    elif sums["t_lds"] >= sums["t_hbm"]:
        roofline = {"bound": "lds", "achieved": sums["lds_bytes"] / nl / avg_launch_s / 1e9, "peak": LDS_PEAK / 1e9,
                    "unit": "GB/s"}
    else:
        roofline = {"bound": "hbm", "achieved": sums["hbm_bytes"] / nl / avg_launch_s / 1e9, "peak": HBM_PEAK / 1e9,
                    "unit": "GB/s"}
    roofline["frac"] = roofline["achieved"] / roofline["peak"]
    # the LDS fraction whatever binds, and the same against the read rate measured on this machine (bench.py --probe)
    roofline["lds_frac"] = sums["lds_bytes"] / nl / avg_launch_s / LDS_PEAK
    roofline["lds_frac_of_measured_read_rate"] = (sums["lds_bytes"] / nl / avg_launch_s /
                                                  (MEASURED_LDS_B_PER_CLK_PER_CU * CUS * CLOCK_HZ))
    roofline["measured_roofs"] = {"lds_B_per_clk_per_CU": MEASURED_LDS_B_PER_CLK_PER_CU,
                                  "copy_bytes_per_s": MEASURED_COPY_BYTES_PER_S, "source": ROOF_PROFILE}
    # HBM-side bytes per launch come from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs (profiles/); a bench run
    # does not count them, it quotes the profile of the same workload in its default configuration
    measured = MEASURED_TRAFFIC_BYTES_PER_LAUNCH.get(name) if not (args.launch or args.unify or args.codebook or args.fused) else None
    roofline["traffic"] = measured[0] if measured else None
    if measured:
        roofline["traffic_source"] = measured[1]
        roofline["traffic_over_algorithmic"] = measured[0] / (sums["hbm_bytes"] / nl)
    roofline["kernel"] = "sc::tile_kernel"
    roofline["avg_launch_us"] = avg_launch_s * 1e6
    roofline["launches_per_step"] = nl
    roofline["hbm_frac"] = sums["hbm_bytes"] / nl / avg_launch_s / HBM_PEAK
    roofline["alu_frac"] = total_macs / nl / avg_launch_s / VALU_PEAK_FMA

    out = {
        "metric": "effective GFLOP/s (2*nnz*E*F*N over the sparse conv layers of the workload)",
        "value": 2.0 * total_macs / (ms_per_step * 1e-3) / 1e9,
        "unit": "GFLOP/s",
        "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms_per_step, "gpu_ms_per_step": gpu_ms / steps,
        "cache_hot_ms_per_step": hot_wall * 1e3 / steps, "buffer_sets": nsets,
        "graph_ms_per_step": graph_ms, "event_gap_us": round(event_gap * 1e6, 2),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": work.dtype, "data": "synthetic" + (", cluster-quantised weights (4-bit numbers, 16 centroids)" if args.codebook else "") +
                (", ReLU and 2x2 maximum in the store step" if args.fused else ""),
        "config": {"workload": f"{work.name}, batch {N}, {nl} sparse conv layer(s), conv only, inputs resident in HBM, {nsets} buffer set(s) in rotation",
                   "layers": nl, "batch": N, "total_macs": total_macs,
                   "launch": ((f"override {args.launch}; " if args.launch else "") +
                              (f"measured best of {args.autotune} ranked candidates per layer" + (", re-checked inside a pass" if args.refine else "") if tune
                               else f"pinned from {args.tuning_table}" if known else "cost estimate"))},
        "roofline": roofline,
        "layers": layers,
    }
    if args.unify:
        useful = sum(int(m.sum()) * r.spec.E * r.spec.F * N for (_, m), r in zip(net.host_weights, net.runs))
        out["useful_value"] = 2.0 * useful / (ms_per_step * 1e-3) / 1e9
        out["config"]["stored_entries"] = sum(r.nnz for r in net.runs)
        out["config"]["kept_weights"] = sum(int(m.sum()) for _, m in net.host_weights)
    if args.compare_dense:
        rows = net.compare_with_dense()
        # the routed pass is run and timed as one loop, like the all-sparse one beside it
        out["dense_comparison"] = {"layers": rows,
                                   "sparse_us": round(sum(r["sparse_us"] for r in rows), 1),
                                   "dense_us": round(sum(r["dense_us"] for r in rows), 1),
                                   "routes": list(net.route),
                                   "sparse_pass_us": round(net.time_pass(False), 1),
                                   "dispatched_pass_us": round(net.time_pass(True), 1)}
    if args.tuning_table:
        net.save_table(args.tuning_table)
        out["config"]["tuning_table"] = args.tuning_table
    if not args.no_cpu:
        # the outputs the oracle looks at are those of a pass with the timed launches over the first buffer set
        for r in net.runs:
            r.y.fill_(float("nan"))
        net.step(0)
        torch.cuda.synchronize()
        parity, cpu = oracle_leg(net, work, npts=500 if brief else 2000, time_it=not brief)
        out["parity"] = parity
        if cpu is not None:
            out["cpu_baseline"] = cpu
    net.close()
    del net
    torch.cuda.empty_cache()
    return out


if __name__ == "__main__":
    main()
