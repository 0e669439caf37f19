"""Runs a synthetic workload (a stack of pruned conv layers) through the library.

Only the convolutions are the library's; ReLU and 2x2 max-pool between layers
(section 3 of the paper: bias/activation follow the convolution and are not
part of the sparse kernel of section 8) are plain torch ops on the same stream.
"""
from __future__ import annotations

import json
import os
from typing import Dict, List, Optional

import numpy as np

from . import binding as B
from . import workloads as wl


class LayerRun:
    def __init__(self, spec: wl.LayerSpec, layer: B.SparseConv, nnz: int):
        self.spec = spec
        self.layer = layer
        self.nnz = nnz
        self.x = None   # resident device input  [N][C][H][W]
        self.y = None   # resident device output [N][K][E][F]

    def macs(self, N: int) -> int:
        return self.nnz * self.spec.E * self.spec.F * N


class Network:
    """Handles of all layers of a workload plus their resident activations."""

    def __init__(self, work: wl.Workload, unify: bool = False, layer_ids: Optional[List[int]] = None,
                 codebook: bool = False, fuse: bool = False):
        """fuse: the ReLU and the 2 x 2 maximum that follow a layer in the workload are done in that layer's
        store step (where the library can plan it; elsewhere they stay torch ops between the layers)."""
        self.work = work
        self.fuse = fuse
        self.layer_ids = layer_ids
        self.unified = unify
        self.runs: List[LayerRun] = []
        self.host_weights = []
        for li, spec in enumerate(work.layers, 1):
            lid = layer_ids[li - 1] if layer_ids else li
            m = wl.make_mask(work.config, lid, spec)
            if codebook:   # cluster-quantised stand-in: 4-bit centroid numbers, 16 binary16 centroids
                index, centroids = wl.make_codebook(work.config, lid, spec, with_zero=unify)
                layer = B.SparseConv.from_codebook(index, centroids, m, dtype=work.dtype, unify=unify)
                w = centroids.astype(np.float16).astype(np.float32)[index]     # the weights the layer stands for
            else:
                w = wl.make_weights(work.config, lid, spec)
                layer = B.SparseConv(w, m, dtype=work.dtype, unify=unify)
            rowptr = layer.csr()[0]
            self.runs.append(LayerRun(spec, layer, int(rowptr[-1])))
            self.runs[-1].fused_relu = self.runs[-1].fused_pool = False
            if fuse and (spec.relu_after or spec.pool_after):
                layer.set_epilogue(None, relu=spec.relu_after, maxpool=spec.pool_after)
                try:
                    layer.get_launch(work.N, spec.H, spec.W, spec.stride, spec.pad)
                    self.runs[-1].fused_pool = spec.pool_after
                except B.SparseConvError:       # no tiles of whole row pairs for this map: pooling stays outside
                    layer.set_epilogue(None, relu=spec.relu_after, maxpool=False)
                self.runs[-1].fused_relu = spec.relu_after
            self.host_weights.append((w, m))
        # per layer: "sparse" (this library) or "dense" (the platform's dense convolution on the masked weights);
        # filled by compare_with_dense or load_table, honoured by step(dispatch=True) / run_chain(dispatch=True)
        self.route: List[str] = ["sparse"] * len(self.runs)
        self._dense_w = [None] * len(self.runs)
        self._dense_out = [None] * len(self.runs)
        self.timings: Dict[int, dict] = {}

    def torch_dtype(self):
        import torch
        return torch.float16 if self.work.dtype == "f16" else torch.float32

    def glue(self, spec: wl.LayerSpec, y, run=None):
        """What the workload does between this layer and the next, less what the layer's store step did already
        (ReLU and maximum are both monotonic, so their order does not matter)."""
        import torch.nn.functional as F
        relu = spec.relu_after and not (run is not None and run.fused_relu)
        pool = spec.pool_after and not (run is not None and run.fused_pool)
        if pool and spec.pool_before_relu:
            y = F.max_pool2d(y, 2)
        if relu:
            y = F.relu(y)
        if pool and not spec.pool_before_relu:
            y = F.max_pool2d(y, 2)
        return y.contiguous()

    # ------------------------------------------------------------ routing (the paper's Algorithm 2)

    def _dense_weights(self, li: int):
        import torch
        if self._dense_w[li] is None:
            w, m = self.host_weights[li]
            self._dense_w[li] = torch.from_numpy(w * m).cuda().to(self.torch_dtype())
        return self._dense_w[li]

    def forward_layer(self, li: int, x, y=None, dispatch: bool = False):
        """One layer on x: the sparse kernel (into y if given), or, with dispatch and a "dense" route, the
        platform's dense convolution on the masked weights (its own output tensor)."""
        import torch.nn.functional as F
        run = self.runs[li]
        s = run.spec
        if dispatch and self.route[li] == "dense":
            self._dense_out[li] = F.conv2d(x, self._dense_weights(li), None, s.stride, s.pad)
            return self._dense_out[li]
        return run.layer.forward(x, s.stride, s.pad, out=y)

    def table_key(self, li: int) -> str:
        s = self.runs[li].spec
        return ",".join(str(v) for v in (self.work.dtype, self.work.N, s.C, s.H, s.W, s.K, s.R, s.S, s.stride, s.pad,
                                         self.runs[li].nnz))

    def save_table(self, path: str) -> dict:
        """Writes (merging with what the file holds) per layer geometry: the route the comparison picked, the
        launch configuration in force, and the measured times.  Key: dtype,N,C,H,W,K,R,S,stride,pad,nnz."""
        table = {}
        if os.path.exists(path):
            with open(path) as f:
                table = json.load(f)
        for li, run in enumerate(self.runs):
            s = run.spec
            d = run.layer.get_launch(self.work.N, s.H, s.W, s.stride, s.pad)
            entry = {"route": self.route[li],
                     "launch": [d["V"], d["WP"], d["WK"], d["KW"], d["Cc"], 0, d["LP"], d["kblocks"], d["store"], d["lanes"],
                                d["csplit"]]}
            entry.update(self.timings.get(li, {}))
            table[self.table_key(li)] = entry
        with open(path, "w") as f:
            json.dump(table, f, indent=1, sort_keys=True)
        return table

    def load_table(self, path: str) -> int:
        """Pins route and launch configuration of every layer the table knows; returns how many it knew."""
        with open(path) as f:
            table = json.load(f)
        known = 0
        for li, run in enumerate(self.runs):
            entry = table.get(self.table_key(li))
            if entry is None:
                continue
            run.layer.set_launch(entry["launch"])
            self.route[li] = entry.get("route", "sparse")
            known += 1
        return known

    def run_chain(self, x0: np.ndarray, dispatch: bool = False):
        """Pushes x0 through every layer once, keeping each layer's input and output on the device
        (dispatch: every layer through the implementation its route names)."""
        import torch
        self._prepared = {}   # calls prepared by step() refer to the buffers replaced here
        x = torch.from_numpy(x0).cuda().to(self.torch_dtype()).contiguous()
        for li, run in enumerate(self.runs, 1):
            if not self.work.chain and li > 1:   # independent layers: each has its own seeded input
                lid = self.layer_ids[li - 1] if self.layer_ids else li
                xi = wl.make_layer_input(self.work.config, lid, run.spec, self.work.N, self.work.input_dist)
                x = torch.from_numpy(xi).cuda().to(self.torch_dtype()).contiguous()
            run.x = x
            run.y = self.forward_layer(li - 1, x, None, dispatch)
            x = self.glue(run.spec, run.y, None if (dispatch and self.route[li - 1] == "dense") else run)
        torch.cuda.synchronize()
        return x

    def autotune(self, max_candidates: int = 0):
        """Tunes every layer's launch configuration on its resident buffers (after run_chain)."""
        return [run.layer.autotune(run.x, run.spec.stride, run.spec.pad, out=run.y, max_candidates=max_candidates)
                for run in self.runs]

    def refine_in_context(self, steps: int = 8, top: int = 4):
        """Second look at every layer's launch choice, inside a pass: sparse_conv_autotune times a
        layer repeated on the same buffers (which stay in the last-level cache if they fit), and
        that flatters some configurations.  Per layer the measured choice and the `top` candidates
        the planner ranks first are run in pass order (going round the buffer sets if there are
        any) with events around that layer only, briefly; the three fastest are then timed for
        `steps` passes each, the two fastest of those once more with the other kind of output
        store, and the fastest of all is pinned."""
        import torch

        def geom(run):
            return (self.work.N, run.spec.H, run.spec.W, run.spec.stride, run.spec.pad)

        def time_layer(li, launch, passes):
            try:
                self.runs[li].layer.set_launch(launch)
                self.runs[li].layer.get_launch(*geom(self.runs[li]))
            except B.SparseConvError:
                return float("inf")          # a candidate this geometry cannot run
            t = 0.0
            for j in range(2 + passes):
                sets = getattr(self, "sets", None)
                bufs = sets[j % len(sets)] if sets else [(r.x, r.y) for r in self.runs]
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                for i, (r, (x, y)) in enumerate(zip(self.runs, bufs)):
                    if i == li:
                        e0.record()
                    r.layer.forward(x, r.spec.stride, r.spec.pad, out=y)
                    if i == li:
                        e1.record()
                torch.cuda.synchronize()
                if j >= 2:
                    t += e0.elapsed_time(e1)
            return t / passes

        # short passes are timed more often: about 3 ms of timed passes per candidate, 8 to 64 passes
        t0, t1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        self.step(0)
        t0.record()
        self.step(0)
        t1.record()
        torch.cuda.synchronize()
        steps = max(steps, min(64, int(3.0 / max(t0.elapsed_time(t1), 1e-3))))

        for li, run in enumerate(self.runs):
            d = run.layer.get_launch(*geom(run))
            tuned = [d["V"], d["WP"], d["WK"], d["KW"], d["Cc"], 0, d["LP"], d["kblocks"], d["store"], d["lanes"], d["csplit"]]
            run.layer.set_launch([])                 # back to the estimate (this discards the measured choice)
            cands = [tuned]
            for c in run.layer.rank_launches(*geom(run), max_candidates=top):
                if c[:8] + c[9:] not in [k[:8] + k[9:] for k in cands]:
                    cands.append(c)
            if len(cands) > 3:
                brief = sorted((time_layer(li, c, max(2, steps // 3)), i) for i, c in enumerate(cands))
                cands = [cands[i] for _, i in brief[:3]]
            timed = sorted(((time_layer(li, c, steps), i, c) for i, c in enumerate(cands)), key=lambda e: e[:2])
            for t, i, c in list(timed[:2]):
                other = c[:8] + [3 - c[8]] + c[9:]
                timed.append((time_layer(li, other, steps), len(timed), other))
            run.layer.set_launch(min(timed, key=lambda e: e[:2])[2])
        return [run.layer.get_launch(*geom(run)) for run in self.runs]

    def make_buffer_sets(self, min_bytes: int = 512 << 20, max_sets: int = 16) -> int:
        """Further copies of every layer's resident input (and outputs of their own) at other
        addresses, until all sets together hold min_bytes: passes that go round the sets do not
        find their operands in the 256 MB last-level cache.  Returns the number of sets."""
        import torch
        per_set = sum(r.x.numel() * r.x.element_size() + r.y.numel() * r.y.element_size() for r in self.runs)
        nsets = max(1, min(max_sets, -(-min_bytes // per_set)))
        self._prepared = {}
        self.sets = [[(r.x, r.y) for r in self.runs]]
        for _ in range(nsets - 1):
            self.sets.append([(r.x.clone(), torch.empty_like(r.y)) for r in self.runs])
        torch.cuda.synchronize()
        return nsets

    def prepare_steps(self):
        """One function per buffer set that enqueues a pass of the hot path on that set, on the stream that is
        current now, with every call checked and marshalled beforehand (step() does the same lookup per call;
        for launch-bound workloads even that shows)."""
        sets = getattr(self, "sets", None) or [[(r.x, r.y) for r in self.runs]]
        runners = []
        for bufs in sets:
            calls = tuple(run.layer.prepare(x, run.spec.stride, run.spec.pad, out=y) for run, (x, y) in zip(self.runs, bufs))

            def run_set(calls=calls):
                for enqueue in calls:
                    enqueue()

            run_set.calls = calls
            runners.append(run_set)
        return runners

    def step(self, which: int = 0, dispatch: bool = False):
        """One pass of the hot path: every layer's convolution on its resident input
        (buffer set `which`, modulo the number of sets, once make_buffer_sets has run).
        dispatch: layers routed to the dense implementation run there instead."""
        sets = getattr(self, "sets", None)
        bufs = sets[which % len(sets)] if sets else [(r.x, r.y) for r in self.runs]
        if not dispatch:
            import torch
            # the calls of a buffer set are checked and marshalled once per stream, then only enqueued
            key = (which % len(sets) if sets else 0, torch.cuda.current_stream().cuda_stream)
            if not hasattr(self, "_prepared"):
                self._prepared = {}
            calls = self._prepared.get(key)
            if calls is None:
                calls = self._prepared[key] = [run.layer.prepare(x, run.spec.stride, run.spec.pad, out=y)
                                               for run, (x, y) in zip(self.runs, bufs)]
            for enqueue in calls:
                enqueue()
            return
        for li, (x, y) in enumerate(bufs):
            self.forward_layer(li, x, y, True)

    def compare_with_dense(self, reps: int = 20):
        """Per layer: time of the sparse kernel and of the platform's dense convolution
        (torch.nn.functional.conv2d, i.e. MIOpen) on the same masked weights and resident input,
        and which of the two a dispatcher would pick (the paper's Algorithm 2 compares the
        layers' efficiency once and routes each layer to the faster implementation).
        Returns a list of dicts: name, sparse_us, dense_us, choice, max_abs_diff."""
        import torch
        import torch.nn.functional as F
        out = []
        for li, ((w, m), run) in enumerate(zip(self.host_weights, self.runs)):
            s = run.spec
            wd = self._dense_weights(li)
            yd = F.conv2d(run.x, wd, None, s.stride, s.pad)
            ys = run.layer.forward(run.x, s.stride, s.pad, out=run.y)
            diff = float((yd.float() - ys.float()).abs().max())
            times = {}
            for name, fn in (("sparse", lambda: run.layer.forward(run.x, s.stride, s.pad, out=run.y)),
                             ("dense", lambda: F.conv2d(run.x, wd, None, s.stride, s.pad))):
                for _ in range(3):
                    fn()
                a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                a.record()
                for _ in range(reps):
                    fn()
                z.record()
                torch.cuda.synchronize()
                times[name] = a.elapsed_time(z) * 1e3 / reps
            choice = "sparse" if times["sparse"] <= times["dense"] else "dense"
            self.route[li] = choice
            self.timings[li] = {"sparse_us": round(times["sparse"], 2), "dense_us": round(times["dense"], 2)}
            out.append({"name": s.name, "sparsity": s.sparsity_bp / 100.0, "sparse_us": round(times["sparse"], 2),
                        "dense_us": round(times["dense"], 2), "choice": choice, "max_abs_diff": diff})
            del yd
        return out

    def time_pass(self, dispatch: bool, steps: int = 20, warmup: int = 3) -> float:
        """us per pass over the buffer sets in rotation, every layer through its route (dispatch) or all sparse."""
        import torch
        runners = None if dispatch else self.prepare_steps()
        one = (lambda i: self.step(i, True)) if dispatch else (lambda i: runners[i % len(runners)]())
        for i in range(max(warmup, len(runners) if runners else 0)):
            one(i)
        torch.cuda.synchronize()
        a, z = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for i in range(steps):
            one(i)
        z.record()
        torch.cuda.synchronize()
        return a.elapsed_time(z) * 1e3 / steps

    def total_macs(self) -> int:
        return sum(r.macs(self.work.N) for r in self.runs)

    def close(self):
        for r in self.runs:
            r.layer.close()
