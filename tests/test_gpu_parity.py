"""GPU parity: the HIP path (through the C ABI) against the CPU oracle,
element by element, on seeded inputs.  fp32 tolerance 1e-5, fp16 2e-3
(|got-ref| <= tol*max|ref|)."""
import numpy as np
import pytest

import oracle
from helpers import TOL, assert_close, rand_layer

pytestmark = pytest.mark.gpu


def _torch():
    import torch
    return torch


def run_gpu(layer, x, stride, pad, dtype):
    torch = _torch()
    xt = torch.from_numpy(x).cuda()
    if dtype == "f16":
        xt = xt.half()
    y = layer.forward(xt.contiguous(), stride, pad)
    torch.cuda.synchronize()
    return y.float().cpu().numpy()


def oracle_ref(w, m, x, stride, pad, dtype, unify=False):
    K, _, R, S = w.shape
    mm = oracle.unify_mask(m)[0] if unify else m
    rowptr, colidx, values = oracle.csr_encode(w, mm)
    if dtype == "f16":   # same binary16-rounded operands, wide accumulation
        values = oracle.round_through_f16(values)
        x = oracle.round_through_f16(x)
    return oracle.sparse_conv((rowptr, colidx, values), x, K, R, S, stride, pad)


def check(w, m, x, stride, pad, dtype, unify=False, launch=None, what=""):
    from paper_2011_06295_amd import binding as B
    layer = B.SparseConv(w, m, dtype=dtype, unify=unify)
    if launch is not None:
        layer.set_launch(launch)
    N, _, H, W = x.shape
    print(what, "launch", layer.get_launch(N, H, W, stride, pad), flush=True)
    got = run_gpu(layer, x, stride, pad, dtype)
    ref = oracle_ref(w, m, x, stride, pad, dtype, unify)
    assert_close(got, ref, TOL[dtype], what)
    layer.close()
    return got


def _shapes():
    rng = np.random.default_rng(77)
    out = []
    for t in range(24):
        R, S = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 3, 5]))
        st, p = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        H, W = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        if H + 2 * p < R or W + 2 * p < S:
            H, W = H + R, W + S
        out.append((int(rng.integers(1, 12)), int(rng.integers(1, 24)), int(rng.integers(1, 40)), R, S, H, W, st, p))
    return out


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("shape", _shapes())
def test_random_small_layers(shape, dtype):
    N, C, K, R, S, H, W, st, p = shape
    rng = np.random.default_rng(abs(hash(shape)) % (2 ** 32))
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=float(rng.choice([0.05, 0.3, 1.0])))
    check(w, m, x, st, p, dtype, what=f"shape{shape}-{dtype}")


LAUNCHES = [
    # V, WP, WK, KW, Cc, lds budget[, positions per lane]
    [1, 1, 1, 1, 0, 0],
    [1, 2, 2, 2, 2, 0],
    [2, 1, 4, 4, 5, 0],
    [4, 2, 2, 16, 3, 0],
    [4, 1, 1, 8, 16, 0],
    [2, 3, 3, 2, 1, 0],
    [4, 4, 4, 1, 0, 40960],
    [0, 8, 2, 2, 7, 0],
    [4, 1, 2, 4, 0, 0, 2],
    [0, 1, 3, 1, 4, 0, 2],
    [2, 2, 1, 8, 5, 0, 2],
    [1, 1, 4, 8, 6, 0, 2],
    [0, 2, 2, 2, 0, 0, 2],
    [4, 1, 3, 4, 0, 0, 1, 5],     # 37 output channels over 5 blocks of 12 slots: 4-5 empty slots a block
    [0, 1, 4, 2, 6, 0, 1, 37],    # one output channel per workgroup
    [4, 2, 2, 4, 0, 0, 1, 0, 2],  # non-temporal output stores
    [0, 0, 0, 0, 0, 0, 2, 0, 2],
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("launch", LAUNCHES, ids=lambda l: "-".join(map(str, l)))
def test_launch_overrides_do_not_change_the_result(launch, dtype):
    """Several tiles, several channel chunks, ragged tails in every dimension."""
    rng = np.random.default_rng(5150)
    N, C, K, R, S, H, W = 11, 13, 37, 3, 3, 13, 11
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.25)
    m[3] = 0     # an output channel without stored weights must still be written (as zeros)
    m[7] = 1     # a full row
    got = check(w, m, x, 1, 1, dtype, launch=launch, what=f"launch{launch}-{dtype}")
    assert not got[:, 3].any()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_degenerate_cases(dtype):
    rng = np.random.default_rng(99)
    # all-zero mask: output exactly zero
    w, m, x = rand_layer(rng, 3, 4, 5, 3, 3, 6, 6)
    got = check(w, m * 0, x, 1, 1, dtype, what="zero-mask")
    assert not got.any()
    # dense mask (0 % sparsity) equals dense convolution
    check(w, np.ones_like(m), x, 1, 1, dtype, what="dense-mask")
    # unify flag: same numbers
    check(w, m, x, 1, 1, dtype, unify=True, what="unify")
    # single pixel output, filter as large as the padded input
    w2, m2, x2 = rand_layer(rng, 2, 3, 4, 5, 5, 3, 3, density=0.5)
    check(w2, m2, x2, 1, 1, dtype, what="filter==padded-input")
    # 1x1 filter, K = C = 1
    w3, m3, x3 = rand_layer(rng, 5, 1, 1, 1, 1, 7, 9, density=1.0)
    check(w3, m3, x3, 2, 0, dtype, what="1x1")


STAGING_CASES = [
    # name, (N, C, K, R, S, H, W, stride, pad), launch override or None
    ("tiny-maps-many-groups-per-tile", (37, 40, 24, 3, 3, 2, 2, 1, 1), [4, 1, 4, 1, 16, 0]),  # whole planes, channel-minor order
    ("tiny-maps-automatic", (37, 40, 24, 3, 3, 2, 2, 1, 1), None),
    ("4x4-maps-two-buffers", (29, 70, 20, 3, 3, 4, 4, 1, 1), [4, 1, 4, 2, 9, 0]),        # 8 chunks, ragged last chunk
    ("rows-tile-spans-three-groups", (23, 12, 16, 3, 3, 8, 8, 1, 1), [4, 1, 3, 2, 5, 0]),
    ("several-staging-passes", (3, 6, 10, 3, 3, 9, 70, 1, 1), [1, 1, 1, 2, 3, 0]),      # 64 threads, wide rows
    ("several-passes-two-buffers-f16-wide", (9, 9, 8, 5, 5, 12, 50, 1, 2), [2, 1, 2, 1, 4, 0]),
    ("one-image-per-element", (5, 7, 9, 3, 3, 10, 10, 1, 1), [1, 2, 2, 2, 0, 0]),
    ("stride-2-pad-2", (6, 5, 12, 3, 3, 11, 13, 2, 2), [2, 1, 5, 1, 2, 0]),
    ("single-chunk-single-buffer", (8, 3, 16, 3, 3, 16, 16, 1, 1), None),
    # maps much wider than a tile: banded tile layout (positions of a tile wrap over lattice rows)
    ("banded-3x3-wide", (3, 5, 7, 3, 3, 9, 150, 1, 1), [4, 1, 2, 2, 2, 0]),
    ("banded-1x1-56x56", (5, 24, 16, 1, 1, 56, 56, 1, 0), None),
    ("banded-5x5-two-position-waves", (2, 4, 6, 5, 5, 40, 300, 1, 2), [2, 2, 2, 1, 3, 0]),
    ("banded-stride-2", (6, 3, 9, 3, 3, 31, 200, 2, 1), [4, 1, 3, 1, 0, 0]),
    ("banded-1d", (7, 20, 10, 1, 3, 1, 500, 1, 0), None),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("case", STAGING_CASES, ids=lambda c: c[0])
def test_staging_modes(case, dtype):
    """Slot orders (rows / whole planes), one or two tile buffers, one or several staging passes."""
    name, (N, C, K, R, S, H, W, st, p), launch = case
    rng = np.random.default_rng(len(name) * 1000 + N)
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.3)
    check(w, m, x, st, p, dtype, launch=launch, what=f"{name}-{dtype}")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_bias_and_relu_in_the_store_step(dtype):
    """Section 3: the sum is added to the channel's bias, then the activation is applied."""
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(404)
    N, C, K, R, S, H, W = 7, 9, 21, 3, 3, 12, 10
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.3)
    bias = rng.standard_normal(K).astype(np.float32)
    conv = oracle_ref(w, m, x, 1, 1, dtype).astype(np.float64)
    layer = B.SparseConv(w, m, dtype=dtype)
    cases = [(None, False, conv), (bias, False, conv + bias[None, :, None, None]),
             (None, True, np.maximum(conv, 0.0)), (bias, True, np.maximum(conv + bias[None, :, None, None], 0.0))]
    for b, relu, ref in cases + cases[:1]:   # and back to the bare sum
        layer.set_epilogue(b, relu)
        got = run_gpu(layer, x, 1, 1, dtype)
        assert_close(got, ref.astype(np.float32), TOL[dtype], f"epilogue-bias{b is not None}-relu{relu}-{dtype}")
        if relu:
            assert (got >= 0).all() and (got == 0).any()
    layer.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_measured_launch_choice_keeps_the_result(dtype):
    """Section 8 fixes the launch shape per layer by experiment: the measured choice is one of the
    ranked candidates, later forwards of that geometry use it, and the result does not change."""
    import torch
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(505)
    N, C, K, R, S, H, W = 9, 24, 40, 3, 3, 14, 14
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.2)
    ref = oracle_ref(w, m, x, 1, 1, dtype)
    layer = B.SparseConv(w, m, dtype=dtype)
    before = run_gpu(layer, x, 1, 1, dtype)
    xt = torch.from_numpy(x).cuda().to(torch.float16 if dtype == "f16" else torch.float32).contiguous()
    us = layer.autotune(xt, 1, 1, max_candidates=6)
    assert us > 0
    tuned = layer.get_launch(N, H, W, 1, 1)
    other = layer.get_launch(N + 1, H, W, 1, 1)          # another geometry keeps the estimate's choice
    assert 64 <= tuned["threads"] <= 1024 and other["threads"] >= 64
    assert tuned["store"] in (1, 2) and other["store"] == 1
    after = run_gpu(layer, x, 1, 1, dtype)
    assert_close(after, ref, TOL[dtype], f"autotuned-{dtype}")
    assert_close(before, ref, TOL[dtype], f"estimated-{dtype}")
    layer.set_launch([tuned["V"], tuned["WP"], tuned["WK"], tuned["KW"], tuned["Cc"], 0, tuned["LP"], tuned["kblocks"],
                      tuned["store"]])   # pinning it by hand gives the same plan
    pinned = layer.get_launch(N, H, W, 1, 1)
    assert pinned == tuned
    layer.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("unify", [False, True])
def test_cluster_quantised_weights(dtype, unify):
    """Sections 6 and 9: weights given as 4-bit centroid numbers; the result is the convolution with the
    binary16 centroids in their place."""
    import oracle
    from paper_2011_06295_amd import binding as B, workloads as wl
    spec = wl.LayerSpec("cb", C=19, K=33, R=3, S=3, H=11, W=9, stride=1, pad=1, sparsity_bp=8000)
    index, centroids = wl.make_codebook(2, 5, spec, with_zero=unify)
    rng = np.random.default_rng(808)
    mask = (rng.random(index.shape) < 0.2).astype(np.uint8)
    x = rng.standard_normal((6, spec.C, spec.H, spec.W)).astype(np.float32)
    omask = oracle.unify_mask(mask)[0] if unify else mask
    rowptr, colidx, _, _, values = oracle.codebook_csr_encode(index, centroids, omask)
    xin = oracle.round_through_f16(x) if dtype == "f16" else x
    ref = oracle.sparse_conv((rowptr, colidx, values), xin, spec.K, 3, 3, 1, 1)
    layer = B.SparseConv.from_codebook(index, centroids, mask, dtype=dtype, unify=unify)
    plain = B.SparseConv(np.zeros(index.shape, np.float32), omask != 0, dtype=dtype)   # same pattern, uncoded
    for launch in ([0], [0, 0, 0, 0, 4, 0, 0, 0, 0, 0, 2], [0, 1, 2, 2, 3, 0, 1, 0, 0, 5, 1], [4, 2, 1, 4, 5, 0, 2, 0, 2, 1, 1]):
        layer.set_launch(launch)
        plain.set_launch(launch)
        info, pinfo = layer.get_launch(6, spec.H, spec.W, 1, 1), plain.get_launch(6, spec.H, spec.W, 1, 1)
        # the device reads one word per entry (LDS offset and the centroid as binary16): half the table of the same
        # pattern as an fp32 layer (binary16 layers have one-word entries whether cluster-quantised or not)
        assert info["entry_bytes"] == 4 and pinfo["entry_bytes"] == (8 if dtype == "f32" else 4)
        assert info["entries"] == pinfo["entries"]
        assert layer.check_plan(6, spec.H, spec.W, 1, 1) == 0
        got = run_gpu(layer, x, 1, 1, dtype)
        assert_close(got, ref, TOL[dtype], f"codebook-{dtype}-unify{unify}-{launch}")
    layer.close()
    plain.close()


_OUTPUT_LANE_CASES = [
    # N, C, K, R, S, H, W, stride, pad: the small maps of the VGG stack, maps that fill 16 lanes with part rows,
    # batches that leave the last super-group part empty, strides, a map wider than a tile
    (37, 24, 20, 3, 3, 2, 2, 1, 1), (128, 40, 24, 3, 3, 4, 4, 1, 1), (21, 12, 33, 3, 3, 8, 8, 1, 1),
    (9, 6, 10, 3, 3, 16, 16, 1, 1), (5, 3, 8, 3, 3, 32, 32, 1, 1), (70, 9, 12, 3, 3, 14, 14, 1, 1),
    (11, 7, 9, 5, 5, 12, 12, 1, 0), (19, 5, 6, 3, 3, 9, 7, 2, 1), (6, 4, 7, 1, 1, 6, 6, 1, 0), (8, 3, 5, 3, 2, 5, 40, 1, 2),
    (33, 10, 6, 2, 3, 7, 3, 3, 2),
]


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("G", [1, 2, 4, 8, 16])
def test_lanes_as_outputs(G, dtype):
    """Lanes that stand for output elements only (G image groups interleaved per LDS element) against
    the oracle, every element, for every G, automatic and pinned workgroup shapes."""
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(500 + G)
    ran = 0
    for ci, (N, C, K, R, S, H, W, st, p) in enumerate(_OUTPUT_LANE_CASES):
        w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.3)
        for launch in ([0, 0, 0, 0, 0, 0, 0, 0, 0, 1 + G], [0, 2, 3, 2, 5, 0, 1, 0, 2, 1 + G], [0, 4, 1, 4, 0, 0, 1, 0, 0, 1 + G]):
            try:
                check(w, m, x, st, p, dtype, launch=launch, what=f"outputs-G{G}-{dtype}-case{ci}-{launch}")
                ran += 1
            except B.SparseConvError as e:
                # a pinned G whose tiles start at too many different places of a super-group (a 43-wide
                # map in tiles of 8 outputs: 301 staging patterns) is refused, never planned unasked
                assert e.code == B.SC_EUNSUPPORTED and (H, W) == (5, 40), (ci, launch, e)
    assert ran >= 27


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("J", [2, 4, 8])
def test_channels_dealt_over_several_workgroups(J, dtype):
    """The input channels of a (tile, channel block) dealt over J workgroups whose partial sums the last one
    to finish adds up: against the oracle, every element; repeated launches give the same bits (the sums are
    added in the order of the parts, and the arrival counters are back at zero after every launch)."""
    torch = _torch()
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(900 + J)
    cases = [(37, 96, 40, 3, 3, 2, 2, 1, 1, [4, 0, 0, 0, 48 // J, 0, 0, 0, 0, 1, J]),     # lattice lanes, two chunks a part
             (70, 64, 24, 3, 3, 4, 4, 1, 1, [4, 1, 3, 2, 32 // J, 0, 1, 0, 0, 9, J]),     # output lanes
             (9, 40, 50, 3, 3, 9, 11, 2, 1, [0, 2, 2, 4, 40 // J, 0, 2, 0, 2, 1, J]),     # two positions per lane, one chunk a part
             (130, 32, 17, 1, 1, 3, 3, 1, 0, [0, 0, 0, 0, 4, 0, 0, 0, 0, 0, J])]    # automatic kind of lanes
    for ci, (N, C, K, R, S, H, W, st, p, launch) in enumerate(cases):
        w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.3)
        layer = B.SparseConv(w, m, dtype=dtype)
        layer.set_launch(launch)
        info = layer.get_launch(N, H, W, st, p)
        print(f"channel parts {J} {dtype} case {ci}: {info}", flush=True)
        assert info["csplit"] == J
        xt = torch.from_numpy(x).cuda()
        xt = (xt.half() if dtype == "f16" else xt).contiguous()
        ref = oracle_ref(w, m, x, st, p, dtype)
        first = None
        for rep in range(3):
            y = layer.forward(xt, st, p)
            torch.cuda.synchronize()
            assert_close(y.float().cpu().numpy(), ref, TOL[dtype], f"parts{J}-{dtype}-case{ci}-rep{rep}")
            first = y.clone() if first is None else first
            assert torch.equal(y, first), f"parts{J}-{dtype}-case{ci}: launch {rep} differs from the first"
        layer.close()


@pytest.mark.parametrize("seed", [7, 11, 23])
def test_random_shapes_with_random_launch_overrides(seed):
    """Random geometry (filters up to 5x5, stride 1..3, pad 0..3, maps up to 40 x 200) crossed with random
    launch overrides, both precisions, unified or not.  Overrides the planner refuses are skipped."""
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(seed)
    ran = 0
    for t in range(40):
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        st, p = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 40)), int(rng.integers(1, 200 if t % 3 == 0 else 70))
        if H + 2 * p < R or W + 2 * p < S:
            continue
        N, C, K = int(rng.integers(1, 20)), int(rng.integers(1, 40)), int(rng.integers(1, 70))
        dtype = str(rng.choice(["f32", "f16"]))
        unify = bool(rng.integers(0, 2))
        w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=float(rng.choice([0.02, 0.1, 0.3, 0.7])))
        vmax = 8 if dtype == "f16" else 4
        launch = [int(rng.choice([0, 1, 2, 4, vmax])), int(rng.choice([0, 1, 2, 3, 4])), int(rng.choice([0, 1, 2, 3, 5, 8])),
                  int(rng.choice([0, 1, 2, 4, 8, 16])), int(rng.choice([0, 0, 1, 2, 3, 7, 16])), 0, int(rng.choice([0, 1, 2])),
                  0, int(rng.choice([0, 1, 2])), int(rng.choice([0, 1, 2, 3, 5, 9, 17])), int(rng.choice([0, 0, 1, 2, 4, 8]))]
        if launch[9] > 1:                 # lanes stand for outputs (G image groups interleaved): one output per lane
            launch[6] = int(rng.choice([0, 1]))
        if rng.integers(0, 3) == 0:
            launch = [0]
        layer = B.SparseConv(w, m, dtype=dtype, unify=unify)
        try:
            layer.set_launch(launch)
            info = layer.get_launch(N, H, W, st, p)
        except B.SparseConvError:
            layer.close()
            continue
        print(f"case {t}: {(N, C, K, R, S, H, W, st, p)} {dtype} unify={unify} launch={launch} -> {info}", flush=True)
        got = run_gpu(layer, x, st, p, dtype)
        assert_close(got, oracle_ref(w, m, x, st, p, dtype, unify), TOL[dtype], f"random-{seed}-{t}")
        layer.close()
        ran += 1
    assert ran >= 20


def test_forward_can_be_captured_in_a_graph():
    """After one eager call (which uploads the plan) a forward is a single kernel launch on the caller's
    stream: captured once and replayed on new input contents it gives what the eager call gives."""
    import torch
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(2718)
    N, C, K, R, S, H, W = 8, 24, 48, 3, 3, 16, 16
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.15)
    layer = B.SparseConv(w, m, dtype="f32")
    layer.set_epilogue(rng.standard_normal(K).astype(np.float32), relu=True)
    xt = torch.from_numpy(x).cuda()
    y = layer.forward(xt, 1, 1)                      # eager: builds and uploads the plan
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        layer.forward(xt, 1, 1, out=y)               # warm-up on the capture stream
        side.synchronize()
        with torch.cuda.graph(graph, stream=side):
            layer.forward(xt, 1, 1, out=y)
    for rep in range(3):
        xt.copy_(torch.from_numpy(rng.standard_normal(x.shape).astype(np.float32)))
        want = layer.forward(xt, 1, 1).clone()       # eager work between the replays
        torch.cuda.synchronize()
        y.zero_()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(y, want), f"replay {rep}"
    layer.close()


def test_hand_examples_on_gpu():
    import json
    import os
    g = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "hand_3x3.json")))
    x = np.array(g["x"], dtype=np.float32).reshape(1, 1, 3, 3)
    for case in g["cases"]:
        w = np.array(case["w"], dtype=np.float32).reshape(1, 1, 3, 3)
        m = np.array(case["mask"], dtype=np.uint8).reshape(1, 1, 3, 3)
        for dtype in ("f32", "f16"):
            got = check(w, m, x, case["stride"], case["pad"], dtype, what=case["name"])
            assert got[0, 0].tolist() == [[float(v) for v in row] for row in case["out"]]


def test_config1_single_layer():
    from paper_2011_06295_amd import workloads as wl
    work = wl.config1()
    spec = work.layers[0]
    w, m = wl.make_weights(1, 1, spec), wl.make_mask(1, 1, spec)
    x = wl.make_input(work)
    check(w, m, x, spec.stride, spec.pad, "f32", what="config1")


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_non_finite_inputs_are_weighted_as_the_definition_says(dtype):
    """Inputs holding +Inf, -Inf and NaN: an output is NaN, +Inf or -Inf exactly where the oracle's is (a
    non-finite element counts only under a stored weight: the zero-weight entries that fill a row's last
    batch read a plane of zeros, not the input), and the finite outputs stay within tolerance.  Lattice
    lanes, output lanes and channels dealt over two workgroups."""
    torch = _torch()
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(4242)
    cases = [(9, 24, 20, 3, 3, 12, 12, 1, 1, []),
             (37, 48, 40, 3, 3, 4, 4, 1, 1, [4, 0, 0, 0, 0, 0, 1, 0, 0, 5, 1]),
             (37, 96, 40, 3, 3, 2, 2, 1, 1, [4, 0, 0, 0, 24, 0, 0, 0, 0, 1, 2]),
             (5, 30, 17, 1, 1, 9, 9, 1, 0, []),
             (6, 16, 33, 5, 3, 11, 14, 2, 2, [])]
    for ci, (N, C, K, R, S, H, W, st, p, launch) in enumerate(cases):
        w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.15)
        flat = x.reshape(-1)
        where = rng.choice(flat.size, size=12, replace=False)
        flat[where[:5]] = np.inf
        flat[where[5:10]] = -np.inf
        flat[where[10:]] = np.nan
        layer = B.SparseConv(w, m, dtype=dtype)
        layer.set_launch(launch)
        print(f"non-finite {dtype} case {ci}: {layer.get_launch(N, H, W, st, p)}", flush=True)
        xt = torch.from_numpy(x).cuda()
        xt = (xt.half() if dtype == "f16" else xt).contiguous()
        with np.errstate(invalid="ignore", over="ignore"):
            ref = oracle_ref(w, m, x, st, p, dtype)
        y = layer.forward(xt, st, p)
        torch.cuda.synchronize()
        got = y.float().cpu().numpy().astype(np.float64)
        assert np.isnan(ref).any() or np.isinf(ref).any()
        assert np.array_equal(np.isnan(got), np.isnan(ref)), f"case {ci}: NaN where the oracle has none (or the reverse)"
        assert np.array_equal(np.isposinf(got), np.isposinf(ref)) and np.array_equal(np.isneginf(got), np.isneginf(ref)), f"case {ci}"
        fin = np.isfinite(ref)
        assert_close(got[fin], ref[fin], TOL[dtype], f"non-finite-{dtype}-case{ci}")
        layer.close()


@pytest.mark.parametrize("H,J", [(2, 8), (4, 4), (8, 2)])
def test_channel_parts_over_many_launches_with_alternating_inputs(H, J):
    """The partial sums of a launch live in a buffer the next launch overwrites.  400 launches of a
    512 -> 512 layer whose channels are dealt over J workgroups, on two inputs in turn: a part that read
    sums left by the launch before (the other input's), or sums not yet written, would show as a
    difference from that input's first result, which is checked against the oracle."""
    torch = _torch()
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(500 + H)
    N, C, K = 128, 512, 512
    w = rng.standard_normal((K, C, 3, 3)).astype(np.float32)
    m = (rng.random((K, C, 3, 3)) < 0.08).astype(np.uint8)
    layer = B.SparseConv(w, m, dtype="f32")
    layer.set_launch([0, 0, 0, 0, 0, 0, 0, 0, 0, 0, J])
    info = layer.get_launch(N, H, H, 1, 1)
    print(f"many launches {H}x{H} J={J}: {info}", flush=True)
    assert info["csplit"] == J
    xs = [torch.from_numpy(rng.standard_normal((N, C, H, H)).astype(np.float32)).cuda() for _ in range(2)]
    first = []
    for x in xs:
        y = layer.forward(x, 1, 1)
        torch.cuda.synchronize()
        sub = np.arange(0, N, 16)
        ref = oracle_ref(w, m, x[::16].cpu().numpy(), 1, 1, "f32")
        assert_close(y[::16].float().cpu().numpy(), ref, TOL["f32"], f"many-{H}-{J}")
        first.append(y.clone())
    outs = [torch.empty_like(first[0]) for _ in range(4)]
    for rep in range(100):
        for i in range(4):
            layer.forward(xs[i & 1], 1, 1, out=outs[i])
        torch.cuda.synchronize()
        for i in range(4):
            assert torch.equal(outs[i], first[i & 1]), (rep, i)
    layer.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_maximum_over_2x2_windows_in_the_store_step(dtype):
    """Section 3's layer sequence: convolution, bias, activation, pooling.  With SC_EPILOGUE_MAXPOOL2 the
    store step writes the E/2 x F/2 map of window maxima: against the oracle's convolution followed by its
    ReLU and 2 x 2 maximum, on the map sizes of the 32-pixel VGG (32 ... 2), with and without bias and ReLU,
    with the channels dealt over several workgroups, after a measured launch choice, and back to the plain store."""
    torch = _torch()
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(808)
    for ci, (N, C, K, H, launch) in enumerate([(9, 12, 20, 32, []), (13, 20, 24, 16, []), (21, 24, 40, 8, []),
                                               (37, 96, 40, 4, [0, 0, 0, 0, 24, 0, 0, 0, 0, 0, 2]),
                                               (70, 64, 24, 2, [0, 0, 0, 0, 16, 0, 0, 0, 0, 0, 4]),
                                               (40, 16, 33, 8, [0, 0, 0, 2, 0, 0, 0, 0, 2, 0, 0])]):
        w, m, x = rand_layer(rng, N, C, K, 3, 3, H, H, density=0.3)
        bias = rng.standard_normal(K).astype(np.float32)
        conv = oracle_ref(w, m, x, 1, 1, dtype).astype(np.float32)
        layer = B.SparseConv(w, m, dtype=dtype)
        layer.set_launch(launch)
        xt = torch.from_numpy(x).cuda()
        xt = (xt.half() if dtype == "f16" else xt).contiguous()
        for b, relu in ((None, False), (bias, True)):
            layer.set_epilogue(b, relu, maxpool=True)
            info = layer.get_launch(N, H, H, 1, 1)
            print(f"pooled {dtype} case {ci} bias {b is not None}: {info}", flush=True)
            assert info["lanes"] > 1 and layer.output_shape(H, H, 1, 1) == (H // 2, H // 2)
            if launch and launch[10]:
                assert info["csplit"] == launch[10]
            full = conv + (b[None, :, None, None] if b is not None else 0.0)
            ref = oracle.maxpool2(oracle.relu(full) if relu else full)
            y = layer.forward(xt, 1, 1)
            torch.cuda.synchronize()
            assert tuple(y.shape) == (N, K, H // 2, H // 2)
            assert_close(y.float().cpu().numpy(), ref, TOL[dtype], f"pooled-{dtype}-case{ci}-bias{b is not None}")
        if ci == 2:
            layer.autotune(xt, 1, 1, max_candidates=6)
            y = layer.forward(xt, 1, 1)
            torch.cuda.synchronize()
            assert_close(y.float().cpu().numpy(), ref, TOL[dtype], f"pooled-tuned-{dtype}")
        ys = layer.forward_static(xt, 1, 1)          # the entry point that allocates nothing takes the same store step
        torch.cuda.synchronize()
        assert torch.equal(ys, layer.forward(xt, 1, 1))
        layer.set_epilogue(None, False)
        y = layer.forward(xt, 1, 1)
        torch.cuda.synchronize()
        assert tuple(y.shape) == (N, K, H, H)
        assert_close(y.float().cpu().numpy(), conv, TOL[dtype], f"unpooled-again-{dtype}-case{ci}")
        layer.close()


def test_pooled_store_refuses_what_it_cannot_do():
    """Odd maps, lattice lanes and strides above 1 have no tiles of whole row pairs: SC_EUNSUPPORTED."""
    from paper_2011_06295_amd import binding as B
    rng = np.random.default_rng(809)
    w, m, _ = rand_layer(rng, 1, 8, 8, 3, 3, 4, 4, density=0.5)
    layer = B.SparseConv(w, m, dtype="f32")
    layer.set_epilogue(None, False, maxpool=True)
    for geom in ((4, 7, 7, 1, 1), (4, 16, 16, 2, 1), (4, 6, 6, 1, 1)):     # odd map, stride 2, rows of 6 (no tile of 64 lanes holds pairs of them)
        with pytest.raises(B.SparseConvError) as e:
            layer.get_launch(*geom)
        assert e.value.code == B.SC_EUNSUPPORTED
    layer.set_launch([0, 0, 0, 0, 0, 0, 0, 0, 0, 1, 0])      # lattice lanes
    with pytest.raises(B.SparseConvError) as e:
        layer.get_launch(4, 8, 8, 1, 1)
    assert e.value.code == B.SC_EUNSUPPORTED
    layer.close()
