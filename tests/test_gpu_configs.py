"""GPU parity on the five benchmark configurations.  Small cases are compared element by
element; at full batch size the oracle evaluates sampled output coordinates one by one
(exact-order double sums of the same operands the GPU layer received), once with the launch
the cost estimate picks and once with the launches bench.py times (measured choice of 12
candidates per layer, re-checked inside a pass over rotating buffer sets)."""
import numpy as np
import pytest

import oracle
from helpers import TOL, assert_close

pytestmark = pytest.mark.gpu


def _net(work, layer_ids=None):
    from paper_2011_06295_amd import harness
    return harness.Network(work, layer_ids=layer_ids)


def _oracle_operands(w, m, x, dtype):
    rowptr, colidx, values = oracle.csr_encode(w, m)
    if dtype == "f16":
        values = oracle.round_through_f16(values)
        x = oracle.round_through_f16(x)
    return (rowptr, colidx, values), x


def check_layer_full(run, wm, dtype, what):
    """Whole output of one layer against the oracle fed with the layer's own device input."""
    import torch
    w, m = wm
    s = run.spec
    x = run.x.float().cpu().numpy()
    csr, xo = _oracle_operands(w, m, x, dtype)
    ref = oracle.sparse_conv(csr, xo, s.K, s.R, s.S, s.stride, s.pad)
    got = run.y.float().cpu().numpy()
    return assert_close(got, ref, TOL[dtype], what)


def check_layer_sampled(run, wm, dtype, what, npts=3000, seed=0):
    """Sampled output coordinates at full size; tolerance scale from the sampled references."""
    w, m = wm
    s = run.spec
    x = run.x.float().cpu().numpy()
    N = x.shape[0]
    rng = np.random.default_rng(seed)
    pts = np.stack([rng.integers(0, N, npts), rng.integers(0, s.K, npts),
                    rng.integers(0, s.E, npts), rng.integers(0, s.F, npts)], 1).astype(np.int32)
    # always include the corners of the index space (first/last image, channel, pixel)
    corners = np.array([[n, k, i, j] for n in (0, N - 1) for k in (0, s.K - 1)
                        for i in (0, s.E - 1) for j in (0, s.F - 1)], dtype=np.int32)
    pts = np.concatenate([corners, pts])
    csr, xo = _oracle_operands(w, m, x, dtype)
    ref = oracle.sparse_conv_points(csr, xo, s.K, s.R, s.S, s.stride, s.pad, pts)
    y = run.y.float().cpu().numpy()
    got = y[pts[:, 0], pts[:, 1], pts[:, 2], pts[:, 3]]
    return assert_close(got, ref, TOL[dtype], what)


def test_config2_lenet_chain_full():
    from paper_2011_06295_amd import workloads as wl
    work = wl.lenet5(64)
    net = _net(work)
    x0 = wl.make_input(work)
    net.run_chain(x0)
    for li, run in enumerate(net.runs):
        print("lenet", run.spec.name, run.layer.get_launch(work.N, run.spec.H, run.spec.W, run.spec.stride, run.spec.pad), flush=True)
        check_layer_full(run, net.host_weights[li], "f32", f"lenet-{run.spec.name}")
    # the oracle's own chain (its ReLU and max-pool) from the same input
    a = x0
    for li, run in enumerate(net.runs):
        w, m = net.host_weights[li]
        s = run.spec
        y = oracle.sparse_conv(oracle.csr_encode(w, m), a, s.K, s.R, s.S, s.stride, s.pad)
        assert_close(run.y.float().cpu().numpy(), y, 5e-5, f"lenet-chain-{s.name}")
        if s.pool_after and s.pool_before_relu:
            y = oracle.maxpool2(y)
        if s.relu_after:
            y = oracle.relu(y)
        if s.pool_after and not s.pool_before_relu:
            y = oracle.maxpool2(y)
        a = y
    net.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_vgg_small_batch_every_element(dtype):
    """All 13 layers at batch 6 (one full and one partial image group), every output element."""
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(6, dtype)
    net = _net(work)
    net.run_chain(wl.make_input(work))
    for li, run in enumerate(net.runs):
        err = check_layer_full(run, net.host_weights[li], dtype, f"vgg6-{dtype}-{run.spec.name}")
        print(f"vgg batch 6 {dtype} {run.spec.name}: max err / max|ref| = {err:.3g}", flush=True)
    net.close()


@pytest.mark.parametrize("dtype,N", [("f32", 128), ("f16", 256)])
def test_config3_4_vgg_full_batch_sampled(dtype, N):
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(N, dtype)
    net = _net(work)
    out = net.run_chain(wl.make_input(work))
    assert np.isfinite(out.float().cpu().numpy()).all()
    for li, run in enumerate(net.runs):
        err = check_layer_sampled(run, net.host_weights[li], dtype, f"vgg{N}-{dtype}-{run.spec.name}", seed=li)
        print(f"vgg batch {N} {dtype} {run.spec.name}: max err / max|ref| = {err:.3g}", flush=True)
    net.close()


@pytest.mark.parametrize("ragged", [False, True], ids=["unified", "ragged"])
@pytest.mark.parametrize("sparsity_bp", [5000, 7000, 8000, 9000, 9500, 9900])
def test_config5_sweep_sampled(sparsity_bp, ragged):
    from paper_2011_06295_amd import workloads as wl
    work = wl.sweep_layer(sparsity_bp, ragged, 256)
    net = _net(work, layer_ids=[wl.sweep_layer_index(sparsity_bp, ragged)])
    net.run_chain(wl.make_input(work))
    run = net.runs[0]
    err = check_layer_sampled(run, net.host_weights[0], "f32", f"sweep-{sparsity_bp}-{ragged}", npts=2000, seed=sparsity_bp)
    print(f"sweep {sparsity_bp} ragged={ragged}: nnz {run.nnz} max err / max|ref| = {err:.3g}", flush=True)
    net.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("which", ["resnet_1x1", "densenet_1x1", "cnn_1d"])
def test_1x1_and_1d_layers(which, dtype):
    """The paper's 1x1 bottleneck and 1-D text-model layers: every element at batch 5, sampled at batch 128."""
    from paper_2011_06295_amd import workloads as wl
    for N, full in ((5, True), (128, False)):
        work = getattr(wl, which)(N, dtype)
        net = _net(work)
        net.run_chain(wl.make_input(work))
        for li, run in enumerate(net.runs):
            what = f"{which}-{dtype}-N{N}-{run.spec.name}"
            if full:
                err = check_layer_full(run, net.host_weights[li], dtype, what)
            else:
                err = check_layer_sampled(run, net.host_weights[li], dtype, what, npts=1500, seed=li)
            print(f"{what}: {run.layer.get_launch(N, run.spec.H, run.spec.W, 1, 0)} max err / max|ref| = {err:.3g}", flush=True)
        net.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_imagenet_sized_vgg_layers_sampled(dtype):
    """The paper's nine 224-pixel VGG layer shapes at batch 6 (banded tiles, partial last image group)."""
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16_imagenet(6, dtype)
    net = _net(work)
    net.run_chain(wl.make_input(work))
    for li, run in enumerate(net.runs):
        what = f"vgg224-{dtype}-{run.spec.name}"
        err = check_layer_sampled(run, net.host_weights[li], dtype, what, npts=1500, seed=li)
        print(f"{what}: {run.layer.get_launch(6, run.spec.H, run.spec.W, 1, 1)} max err / max|ref| = {err:.3g}", flush=True)
    net.close()


def test_largest_tensors_sampled_images():
    """Input and output just under 2^31 elements (the kernels' index range): 65550 images of 181x181,
    one channel in, one out.  Whole images are compared with the oracle at both ends of the batch and
    around the 2^30-element and 2^31-byte marks."""
    import torch
    from paper_2011_06295_amd import binding as B, workloads as wl
    N, H, W = 65550, 181, 181
    assert N * H * W < 2 ** 31 <= (N + 1) * H * W
    w = np.array([[0.5, -1.0, 0.25], [2.0, 1.0, -0.5], [0.125, -2.0, 4.0]], np.float32).reshape(1, 1, 3, 3)
    m = np.array([[1, 0, 1], [1, 1, 0], [0, 1, 1]], np.uint8).reshape(1, 1, 3, 3)
    layer = B.SparseConv(w, m, "f32")
    idx = torch.arange(N * H * W, dtype=torch.int64, device="cuda")
    x = wl.pattern_value(idx).to(torch.float32).reshape(N, 1, H, W)
    del idx
    y = layer.forward(x, 1, 1)
    torch.cuda.synchronize()
    csr = oracle.csr_encode(w, m)
    per_image = H * W
    picks = sorted({0, 1, 2, 3, N - 1, N - 2, N - 3, N - 4, 2 ** 30 // per_image, 2 ** 30 // per_image + 1,
                    2 ** 29 // per_image, 2 ** 29 // per_image + 1, N // 2, 12345})
    for n in picks:
        xi = wl.pattern_value(np.arange(n * per_image, (n + 1) * per_image, dtype=np.int64)).astype(np.float32)
        assert np.array_equal(xi, x[n].reshape(-1).cpu().numpy())
        ref = oracle.sparse_conv(csr, xi.reshape(1, 1, H, W), 1, 3, 3, 1, 1)
        assert_close(y[n:n + 1].cpu().numpy(), ref, TOL["f32"], f"largest-image{n}")
    layer.close()


def test_dense_comparison_routes_every_layer():
    """The dense platform convolution on the masked weights gives the same numbers, and the
    dispatcher names one of the two implementations per layer."""
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(8, "f32")
    net = _net(work)
    net.run_chain(wl.make_input(work))
    rows = net.compare_with_dense(reps=3)
    assert len(rows) == 13
    for r, run in zip(rows, net.runs):
        scale = float(run.y.abs().max())
        assert r["choice"] in ("sparse", "dense") and r["sparse_us"] > 0 and r["dense_us"] > 0
        assert r["max_abs_diff"] <= 2e-5 * max(scale, 1.0), r
    net.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_dispatched_chain_runs_every_layer_through_its_route(dtype, tmp_path):
    """Algorithm 2's routing, run: a chain in which every layer goes through the implementation its route
    names (forced to alternate here, so that both are exercised whatever the timings say), every layer's
    output against the oracle on the layer's own input; then the table (route + launch per geometry) is
    written, read back into a fresh network, and the routed pass gives the same outputs again.
    The dense route is the platform's convolution, not this library's kernel: its algorithm choice is not
    ours, so it is held to a looser bound (1e-4 / 4e-3 of max|ref|)."""
    import torch
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(8, dtype)
    net = _net(work)
    x0 = wl.make_input(work)
    net.run_chain(x0)
    rows = net.compare_with_dense(reps=2)
    measured = list(net.route)
    assert [r["choice"] for r in rows] == measured
    net.route = ["dense" if li % 2 else "sparse" for li in range(len(net.runs))]
    net.run_chain(x0, dispatch=True)
    outs = []
    for li, run in enumerate(net.runs):
        if net.route[li] == "sparse":
            check_layer_full(run, net.host_weights[li], dtype, f"routed-{dtype}-{run.spec.name}-sparse")
        else:
            w, m = net.host_weights[li]
            csr, xo = _oracle_operands(w, m, run.x.float().cpu().numpy(), dtype)
            ref = oracle.sparse_conv(csr, xo, run.spec.K, run.spec.R, run.spec.S, run.spec.stride, run.spec.pad)
            assert_close(run.y.float().cpu().numpy(), ref, {"f32": 1e-4, "f16": 4e-3}[dtype], f"routed-{dtype}-{run.spec.name}-dense")
        outs.append(run.y.clone())
    path = str(tmp_path / "table.json")
    table = net.save_table(path)
    assert len(table) == len({net.table_key(li) for li in range(len(net.runs))})
    fresh = _net(work)
    assert fresh.load_table(path) == len(fresh.runs) and fresh.route == net.route
    fresh.run_chain(x0, dispatch=True)
    for li, run in enumerate(fresh.runs):
        d = run.layer.get_launch(work.N, run.spec.H, run.spec.W, run.spec.stride, run.spec.pad)
        e = net.runs[li].layer.get_launch(work.N, run.spec.H, run.spec.W, run.spec.stride, run.spec.pad)
        assert d == e
        # (the platform's dense convolution need not give the same bits in a second instance, and what follows it inherits that)
        assert_close(run.y.float().cpu().numpy(), outs[li].float().cpu().numpy(), {"f32": 2e-4, "f16": 8e-3}[dtype],
                     f"layer {li} after the table round trip")
    # the routed pass over resident buffers, as the bench times it
    fresh.step(0, dispatch=True)
    torch.cuda.synchronize()
    assert fresh.time_pass(True, steps=2, warmup=1) > 0
    net.close()
    fresh.close()


def test_buffer_sets_in_rotation_give_the_same_outputs():
    """The copies of the activations that the timed steps of bench.py go round hold the same
    inputs at other addresses; a pass over any of them leaves the same outputs as the first."""
    import torch
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(8, "f32")
    net = _net(work)
    net.run_chain(wl.make_input(work))
    first = [r.y.clone() for r in net.runs]
    nsets = net.make_buffer_sets(3 * sum(r.x.numel() * 4 + r.y.numel() * 4 for r in net.runs))
    assert nsets == 3 and len(net.sets) == 3
    for which in (1, 2, 3):
        for _, y in net.sets[which % 3]:
            y.fill_(float("nan"))
        net.step(which)
        torch.cuda.synchronize()
        for li, (x, y) in enumerate(net.sets[which % 3]):
            assert which % 3 == 0 or x.data_ptr() != net.runs[li].x.data_ptr()
            assert torch.equal(y, first[li]), (which, li)
    net.close()


def test_launch_choice_rechecked_inside_a_pass_keeps_the_results():
    """harness.Network.refine_in_context pins, per layer, the fastest of the measured choice, the
    estimate's first choice and both kinds of output store: whatever it pins, the outputs stay right."""
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(6, "f32")
    net = _net(work)
    net.run_chain(wl.make_input(work))
    net.autotune(3)
    net.make_buffer_sets(2 * sum(r.x.numel() * 4 + r.y.numel() * 4 for r in net.runs))
    chosen = net.refine_in_context(steps=2)
    assert len(chosen) == 13 and all(c["store"] in (1, 2) for c in chosen)
    for r in net.runs:
        r.y.fill_(float("nan"))
    net.step(0)
    for li in (0, 1, 6, 12):
        check_layer_full(net.runs[li], net.host_weights[li], "f32", f"refined-{net.runs[li].spec.name}")
    net.close()


def _tune_as_bench_does(net):
    """The launch selection of bench.py's default run, step by step."""
    net.autotune(12)
    net.make_buffer_sets(512 << 20)
    return net.refine_in_context(top=12)


@pytest.mark.parametrize("dtype,N", [("f32", 128), ("f16", 256)])
def test_vgg_full_batch_in_the_launches_the_bench_times(dtype, N):
    """Configs 3 and 4 at full batch with the measured, re-checked launch of every layer (what
    bench.py times): all 13 layers against the oracle on sampled outputs, after a pass over
    the second buffer set as well as the first."""
    import torch
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(N, dtype)
    net = _net(work)
    net.run_chain(wl.make_input(work))
    chosen = _tune_as_bench_does(net)
    for which in (0, 1):
        for _, y in net.sets[which % len(net.sets)]:
            y.fill_(float("nan"))
        net.step(which)
        torch.cuda.synchronize()
        for li, run in enumerate(net.runs):
            x, y = net.sets[which % len(net.sets)][li]
            run_view = type("View", (), {"spec": run.spec, "x": x, "y": y})
            err = check_layer_sampled(run_view, net.host_weights[li], dtype, f"timed-vgg{N}-{dtype}-{run.spec.name}",
                                      npts=2000, seed=100 + li)
            if which == 0:
                print(f"timed launch vgg batch {N} {dtype} {run.spec.name}: {chosen[li]} max err / max|ref| = {err:.3g}",
                      flush=True)
    net.close()


@pytest.mark.parametrize("sparsity_bp", [9000, 9500, 9900])
def test_sweep_layer_in_the_launch_the_bench_times(sparsity_bp):
    import torch
    from paper_2011_06295_amd import workloads as wl
    work = wl.sweep_layer(sparsity_bp, False, 256)
    net = _net(work, layer_ids=[wl.sweep_layer_index(sparsity_bp, False)])
    net.run_chain(wl.make_input(work))
    chosen = _tune_as_bench_does(net)
    net.runs[0].y.fill_(float("nan"))
    net.step(0)
    torch.cuda.synchronize()
    err = check_layer_sampled(net.runs[0], net.host_weights[0], "f32", f"timed-sweep-{sparsity_bp}", npts=2000, seed=sparsity_bp)
    print(f"timed launch sweep {sparsity_bp}: {chosen[0]} max err / max|ref| = {err:.3g}", flush=True)
    net.close()


def test_config5_unify_flag_matches_plain_rows():
    """Ragged rows padded to a unified count with explicit zeros give the same numbers."""
    import torch
    from paper_2011_06295_amd import binding as B, workloads as wl
    work = wl.sweep_layer(9000, True, 8)
    spec = work.layers[0]
    lid = wl.sweep_layer_index(9000, True)
    w, m = wl.make_weights(5, lid, spec), wl.make_mask(5, lid, spec)
    x = torch.from_numpy(wl.make_input(work)).cuda()
    plain = B.SparseConv(w, m, "f32", unify=False)
    unified = B.SparseConv(w, m, "f32", unify=True)
    rp = unified.csr()[0]
    assert len(set(np.diff(rp).tolist())) == 1
    ya = plain.forward(x, 1, 1).cpu().numpy()
    yb = unified.forward(x, 1, 1).cpu().numpy()
    assert_close(yb, ya, 1e-6, "unify-vs-plain")
    csr = oracle.csr_encode(w, m)
    ref = oracle.sparse_conv(csr, x.cpu().numpy(), spec.K, 3, 3, 1, 1)
    assert_close(ya, ref, TOL["f32"], "sweep-ragged-full")
    plain.close()
    unified.close()


def test_steps_replayed_from_a_hip_graph_match_eager_steps():
    """bench.py also records its timed steps into one HIP graph.  A graph of two steps (one per buffer set;
    some layers with their channels dealt over two workgroups, i.e. with partial sums and arrival counters
    that every launch has to leave at zero) is replayed three times, with eager steps and synchronisations
    in between: after every replay all outputs equal, bit for bit, those of the eager steps."""
    import torch
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(8, "f32")
    net = _net(work)
    for li in (5, 8, 11):      # 256x8x8, 512x4x4, 512x2x2
        net.runs[li].layer.set_launch([0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 2])
    net.run_chain(wl.make_input(work))
    for li in (5, 8, 11):
        s = net.runs[li].spec
        assert net.runs[li].layer.get_launch(work.N, s.H, s.W, s.stride, s.pad)["csplit"] == 2
    eager = [r.y.clone() for r in net.runs]
    assert net.make_buffer_sets(2 * sum(r.x.numel() * 4 + r.y.numel() * 4 for r in net.runs)) == 2
    net.step(0)
    net.step(1)                # every geometry has run: nothing is built or uploaded under capture
    torch.cuda.synchronize()
    side, graph = torch.cuda.Stream(), torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        recorded = net.prepare_steps()
        with torch.cuda.graph(graph, stream=side):
            recorded[0]()
            recorded[1]()
    torch.cuda.synchronize()
    for replay in range(3):
        for bufs in net.sets:
            for _, y in bufs:
                y.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for which, bufs in enumerate(net.sets):
            for li, (_, y) in enumerate(bufs):
                assert torch.equal(y, eager[li]), (replay, which, li)
        net.step(replay)       # the program's own eager work between replays
        torch.cuda.synchronize()
        for li, (_, y) in enumerate(net.sets[replay % 2]):
            assert torch.equal(y, eager[li]), ("eager", replay, li)
    del graph
    net.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_chain_with_relu_and_pooling_in_the_store_step_equals_the_chain_with_them_between_layers(dtype):
    """The 32-pixel VGG chain at N = 8, once with ReLU and the 2 x 2 maximum as operations between the
    layers and once with both in the store step of the layer before them.  Layer by layer, on the same
    input, the fused layer's output is what the plain layer's output becomes after the two operations
    (to the tolerance: a fused layer may get another tile shape and with it another order of summation),
    every pooled layer writes a quarter, and the chains end in the same values."""
    import torch
    from paper_2011_06295_amd import harness, workloads as wl
    work = wl.vgg16(8, dtype)
    plain = harness.Network(work)
    fused = harness.Network(work, fuse=True)
    x0 = wl.make_input(work)
    a = plain.run_chain(x0)
    b = fused.run_chain(x0)
    pooled = [r.spec.name for r in fused.runs if r.fused_pool]
    # (at this batch the smallest maps have too few image groups for output lanes: their maximum stays outside;
    # a host test shows that at the benchmark batches all five pooled layers can take it)
    assert pooled[:2] == ["conv2", "conv4"] and set(pooled) <= {r.spec.name for r in fused.runs if r.spec.pool_after}
    for p, f in zip(plain.runs, fused.runs):
        assert f.fused_relu == f.spec.relu_after
        assert f.y.numel() * (4 if f.fused_pool else 1) == p.y.numel()
        want = plain.glue(p.spec, p.y)                                   # both operations, outside
        got = fused.glue(f.spec, f.layer.forward(p.x, f.spec.stride, f.spec.pad), f)   # the same input; what is left to do outside
        torch.cuda.synchronize()
        assert_close(got.float().cpu().numpy(), want.float().cpu().numpy(), TOL[dtype], f"fused-{dtype}-{f.spec.name}")
    assert_close(b.float().cpu().numpy(), a.float().cpu().numpy(), 20 * TOL[dtype], f"fused-chain-{dtype}")
    plain.close()
    fused.close()
