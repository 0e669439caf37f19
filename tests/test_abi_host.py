"""CPU-side tests of libsparseconv: the library loads, exports what the header
declares, encodes the CSR of section 7 bit-exactly like the oracle, validates
its arguments and plans launches without a GPU.  No kernel is launched here."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
from paper_2011_06295_amd import binding as B
from helpers import rand_layer

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "sparse_conv.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    declared = set(re.findall(r"\b(sparse_conv_[a-z_0-9]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS)
    lib = C.CDLL(B.LIB_PATH)
    for name in declared:
        assert getattr(lib, name) is not None


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("unify", [False, True])
def test_csr_is_bit_exact_against_the_oracle(seed, dtype, unify):
    rng = np.random.default_rng(300 + seed)
    K, Cc, R, S = int(rng.integers(1, 20)), int(rng.integers(1, 12)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    w, m, _ = rand_layer(rng, 1, Cc, K, R, S, 4, 4, density=float(rng.random()))
    if seed == 0:
        m[0] = 0
    if seed == 1:
        w *= 1e-6   # binary16 subnormals
    if seed == 2:
        w.reshape(-1)[:3] = [0.0, -0.0, 70000.0]
        m.reshape(-1)[:3] = 1
    layer = B.SparseConv(w, m, dtype=dtype, unify=unify)
    rowptr, colidx, values = layer.csr()
    om = oracle.unify_mask(m)[0] if unify else m
    orow, ocol, oval = oracle.csr_encode(w, om)
    assert rowptr.tobytes() == orow.tobytes()
    assert colidx.tobytes() == ocol.tobytes()
    if dtype == "f16":
        assert values.dtype == np.uint16 and values.tobytes() == oracle.f32_to_f16_bits(oval).tobytes()
    else:
        assert values.dtype == np.float32 and values.tobytes() == oval.tobytes()
    layer.close()


def test_config_layers_encode_like_the_oracle():
    from paper_2011_06295_amd import workloads as wl
    for cfg, layer_id, spec in [(1, 1, wl.config1().layers[0]), (2, 2, wl.lenet5().layers[1]), (3, 5, wl.vgg16().layers[4])]:
        w, m = wl.make_weights(cfg, layer_id, spec), wl.make_mask(cfg, layer_id, spec)
        for dtype in ("f32", "f16"):
            layer = B.SparseConv(w, m, dtype=dtype)
            rowptr, colidx, values = layer.csr()
            orow, ocol, oval = oracle.csr_encode(w, m)
            assert rowptr.tobytes() == orow.tobytes() and colidx.tobytes() == ocol.tobytes()
            want = oracle.f32_to_f16_bits(oval) if dtype == "f16" else oval
            assert values.tobytes() == want.tobytes()
            layer.close()


def test_argument_validation_returns_status_codes():
    lib = B.raw_library()
    w = np.ones((2, 3, 3, 3), dtype=np.float32)
    m = np.ones((2, 3, 3, 3), dtype=np.uint8)
    h = C.c_void_p()
    assert lib.sparse_conv_create(None, w.ctypes.data, m.ctypes.data, 2, 3, 3, 3, 0, 0) == B.SC_EINVAL
    assert lib.sparse_conv_create(C.byref(h), None, m.ctypes.data, 2, 3, 3, 3, 0, 0) == B.SC_EINVAL
    assert lib.sparse_conv_create(C.byref(h), w.ctypes.data, m.ctypes.data, 0, 3, 3, 3, 0, 0) == B.SC_EINVAL
    assert lib.sparse_conv_create(C.byref(h), w.ctypes.data, m.ctypes.data, 2, 3, 3, 3, 7, 0) == B.SC_EINVAL
    assert lib.sparse_conv_create(C.byref(h), w.ctypes.data, m.ctypes.data, 2, 3, 3, 3, 0, 8) == B.SC_EINVAL
    assert h.value is None
    assert lib.sparse_conv_create(C.byref(h), w.ctypes.data, m.ctypes.data, 2, 3, 3, 3, 0, 0) == B.SC_OK
    e, f = C.c_int(-7), C.c_int(-7)
    assert lib.sparse_conv_output_shape(h, 2, 2, 1, 0, C.byref(e), C.byref(f)) == B.SC_EINVAL   # filter larger than input
    assert (e.value, f.value) == (-7, -7)
    assert lib.sparse_conv_output_shape(h, 5, 5, 0, 0, C.byref(e), C.byref(f)) == B.SC_EINVAL   # stride < 1
    assert lib.sparse_conv_output_shape(h, 5, 5, 1, -1, C.byref(e), C.byref(f)) == B.SC_EINVAL  # pad < 0
    assert lib.sparse_conv_output_shape(h, 8, 7, 2, 1, C.byref(e), C.byref(f)) == B.SC_OK
    assert (e.value, f.value) == (oracle.output_dim(8, 1, 3, 2), oracle.output_dim(7, 1, 3, 2)) == (4, 4)
    # forward: bad geometry / null buffers are rejected before anything touches a GPU
    assert lib.sparse_conv_forward(h, None, None, 1, 2, 2, 1, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(h, None, None, 1, 8, 8, 1, 1, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(h, None, None, -1, 8, 8, 1, 1, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(None, None, None, 1, 8, 8, 1, 1, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(h, None, None, 0, 8, 8, 1, 1, None) == B.SC_OK               # empty batch: no-op
    bad = (C.c_int * 6)(3, 0, 0, 0, 0, 0)
    assert lib.sparse_conv_set_launch(h, bad, 6) == B.SC_EINVAL                                  # V must be a power of two
    lp3 = (C.c_int * 7)(0, 0, 0, 0, 0, 0, 3)
    assert lib.sparse_conv_set_launch(h, lp3, 7) == B.SC_EINVAL                                  # positions per lane: 1 or 2
    assert lib.sparse_conv_set_launch(h, lp3, 12) == B.SC_EINVAL                                 # at most 11 parameters
    cs = (C.c_int * 11)(0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 3)
    assert lib.sparse_conv_set_launch(h, cs, 11) == B.SC_EINVAL                                  # channel parts: 1, 2, 4 or 8
    cs[10] = 16
    assert lib.sparse_conv_set_launch(h, cs, 11) == B.SC_EINVAL
    cs[10] = 4
    assert lib.sparse_conv_set_launch(h, cs, 11) == B.SC_OK
    ln = (C.c_int * 10)(0, 0, 0, 0, 0, 0, 0, 0, 0, 4)
    assert lib.sparse_conv_set_launch(h, ln, 10) == B.SC_EINVAL                                  # lanes: 0, 1 or 1 + a power of two
    ln[9] = 33
    assert lib.sparse_conv_set_launch(h, ln, 10) == B.SC_EINVAL
    ln[9], ln[6] = 5, 2
    assert lib.sparse_conv_set_launch(h, ln, 10) == B.SC_EINVAL                                  # output lanes hold one output each
    ln[6] = 1
    assert lib.sparse_conv_set_launch(h, ln, 10) == B.SC_OK
    st3 = (C.c_int * 9)(0, 0, 0, 0, 0, 0, 0, 0, 3)
    assert lib.sparse_conv_set_launch(h, st3, 9) == B.SC_EINVAL                                  # kind of output store: 1 or 2
    st3[8] = 2
    assert lib.sparse_conv_set_launch(h, st3, 9) == B.SC_OK
    lp3[6] = 2
    assert lib.sparse_conv_set_launch(h, lp3, 7) == B.SC_OK
    assert lib.sparse_conv_set_launch(h, None, 0) == B.SC_OK
    assert lib.sparse_conv_set_epilogue(None, None, 0) == B.SC_EINVAL
    assert lib.sparse_conv_set_epilogue(h, None, 4) == B.SC_EINVAL                               # unknown epilogue flag
    assert lib.sparse_conv_set_epilogue(h, None, B.SC_EPILOGUE_RELU) == B.SC_OK                  # no bias: nothing to copy, needs no GPU
    # the pooled store halves the reported output shape, refuses odd maps, and is planned on the host like any other
    assert lib.sparse_conv_set_epilogue(h, None, B.SC_EPILOGUE_RELU | B.SC_EPILOGUE_MAXPOOL2) == B.SC_OK
    assert lib.sparse_conv_output_shape(h, 8, 8, 1, 1, C.byref(e), C.byref(f)) == B.SC_OK and (e.value, f.value) == (4, 4)
    assert lib.sparse_conv_output_shape(h, 7, 8, 1, 1, C.byref(e), C.byref(f)) == B.SC_EUNSUPPORTED
    info = (C.c_int * 16)()
    assert lib.sparse_conv_get_launch(h, 8, 8, 8, 1, 1, info) == B.SC_OK and info[13] > 1         # lanes as outputs
    assert (64 * info[1] // (info[13] - 1)) % (2 * 8) == 0                                      # a tile holds whole pairs of rows
    status = C.c_int(-1)
    assert lib.sparse_conv_check_plan(h, 8, 8, 8, 1, 1, C.byref(status)) == B.SC_OK and status.value == 0
    assert lib.sparse_conv_get_launch(h, 8, 7, 7, 1, 1, info) == B.SC_EUNSUPPORTED
    assert lib.sparse_conv_set_epilogue(h, None, 0) == B.SC_OK
    assert lib.sparse_conv_output_shape(h, 8, 8, 1, 1, C.byref(e), C.byref(f)) == B.SC_OK and (e.value, f.value) == (8, 8)
    assert lib.sparse_conv_autotune(None, 8, 16, 1, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL    # arguments are checked before any GPU call
    assert lib.sparse_conv_autotune(h, None, 16, 1, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_autotune(h, 8, 8, 1, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL         # in place
    # partial overlap of input [1][3][4][4] (192 bytes from 4096) and output [1][2][2][2] (32 bytes)
    assert lib.sparse_conv_autotune(h, 4096, 4096 + 188, 1, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_autotune(h, 4096, 4096 - 28, 1, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(h, 4096, 4096 + 188, 1, 4, 4, 1, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward(h, 4096, 4096 - 28, 1, 4, 4, 1, 0, None) == B.SC_EINVAL
    assert lib.sparse_conv_autotune(h, 8, 16, 0, 4, 4, 1, 0, None, 0, None) == B.SC_EINVAL        # needs a batch to time
    assert lib.sparse_conv_autotune(h, 8, 16, 1, 4, 4, 0, 0, None, 0, None) == B.SC_EINVAL        # stride 0
    assert lib.sparse_conv_strerror(B.SC_EINVAL) == b"invalid argument"
    lib.sparse_conv_destroy(h)
    lib.sparse_conv_destroy(None)


def test_launch_plans_fit_the_hardware():
    from paper_2011_06295_amd import workloads as wl
    for work, n in [(wl.vgg16(), 128), (wl.vgg16(dtype="f16"), 256), (wl.lenet5(), 64), (wl.sweep_layer(9000, False), 256)]:
        for li, spec in enumerate(work.layers, 1):
            w, m = wl.make_weights(work.config, li, spec), wl.make_mask(work.config, li, spec)
            layer = B.SparseConv(w, m, dtype=work.dtype)
            p = layer.get_launch(n, spec.H, spec.W, spec.stride, spec.pad)
            assert 64 <= p["threads"] <= 1024 and p["threads"] % 64 == 0
            assert 0 < p["lds_bytes"] <= 160 * 1024
            assert p["grid"] >= 1
            layer.close()


@pytest.mark.parametrize("dtype", ["f32", "f16"])
@pytest.mark.parametrize("unify", [False, True])
def test_codebook_csr_is_the_oracles(dtype, unify):
    """Sections 6 and 9: 4-bit centroid numbers into 16 binary16 centroids; everything stored is bit-exact."""
    from paper_2011_06295_amd import workloads as wl
    spec = wl.LayerSpec("cb", C=7, K=9, R=3, S=3, H=8, W=8, stride=1, pad=1, sparsity_bp=7000)
    index, centroids = wl.make_codebook(1, 3, spec, with_zero=unify)
    rng = np.random.default_rng(31)
    mask = (rng.random(index.shape) < 0.3).astype(np.uint8)
    mask[4] = 0                                   # an empty row
    layer = B.SparseConv.from_codebook(index, centroids, mask, dtype=dtype, unify=unify)
    omask = oracle.unify_mask(mask)[0] if unify else mask
    rowptr, colidx, packed, bits, values = oracle.codebook_csr_encode(index, centroids, omask)
    rp, ci, va = layer.csr()
    codes, cbits = layer.codebook()
    assert np.array_equal(rp, rowptr) and np.array_equal(ci, colidx)
    assert np.array_equal(codes, packed) and np.array_equal(cbits, bits)
    if dtype == "f16":
        assert np.array_equal(va, oracle.f32_to_f16_bits(values))
    else:
        assert np.array_equal(va.view(np.uint32), values.view(np.uint32))
    layer.close()


def test_codebook_argument_checks():
    lib = B.raw_library()
    index = np.zeros((2, 1, 2, 2), np.uint8)
    mask = np.ones((2, 1, 2, 2), np.uint8)
    mask[1, 0, 1, :] = 0
    cen = np.arange(1, 17, dtype=np.float32)      # no zero centroid
    h = C.c_void_p()
    args = (index.ctypes.data, cen.ctypes.data, mask.ctypes.data, 2, 1, 2, 2)
    assert lib.sparse_conv_create_codebook(C.byref(h), None, cen.ctypes.data, mask.ctypes.data, 2, 1, 2, 2, B.SC_F32, 0) == B.SC_EINVAL
    assert lib.sparse_conv_create_codebook(C.byref(h), *args, 7, 0) == B.SC_EINVAL                       # unknown dtype
    assert lib.sparse_conv_create_codebook(C.byref(h), *args, B.SC_F32, B.SC_FLAG_UNIFY_NNZ) == B.SC_EINVAL   # zeros needed, none in the codebook
    assert lib.sparse_conv_create_codebook(C.byref(h), *args, B.SC_F32, 0) == B.SC_OK
    assert lib.sparse_conv_get_codebook(h, None, None) == B.SC_OK
    lib.sparse_conv_destroy(h)
    index[0, 0, 0, 0] = 16
    assert lib.sparse_conv_create_codebook(C.byref(h), *args, B.SC_F32, 0) == B.SC_EINVAL                # index above 15
    index[0, 0, 0, 0] = 200
    mask[0, 0, 0, 0] = 0
    assert lib.sparse_conv_create_codebook(C.byref(h), *args, B.SC_F32, 0) == B.SC_OK                    # not read where the mask is zero
    lib.sparse_conv_destroy(h)
    w = np.ones((2, 1, 2, 2), np.float32)
    plain = B.SparseConv(w, mask)
    assert lib.sparse_conv_get_codebook(plain.handle, None, None) == B.SC_EINVAL                        # no codebook in this handle
    plain.close()


def test_sizes_beyond_the_kernels_index_range_are_refused():
    """Positions and tensor elements are 32-bit in the kernels: larger problems are reported, not run."""
    lib = B.raw_library()
    w = np.ones((2, 1, 3, 3), np.float32)
    m = np.ones((2, 1, 3, 3), np.uint8)
    layer = B.SparseConv(w, m)
    out = (C.c_int * 13)()
    # 2^22 images of 64x64: more than 2^31 lattice positions whatever the interleave
    assert lib.sparse_conv_get_launch(layer.handle, 1 << 22, 64, 64, 1, 1, out) == B.SC_EUNSUPPORTED
    # 70000 images of 181x181: the lattice fits, the input tensor has more than 2^31 elements;
    # refused before the (fake) device pointers are touched
    assert lib.sparse_conv_get_launch(layer.handle, 70000, 181, 181, 1, 1, out) == B.SC_OK
    assert lib.sparse_conv_forward(layer.handle, 256, 512, 70000, 181, 181, 1, 1, None) == B.SC_EUNSUPPORTED
    assert lib.sparse_conv_forward(layer.handle, 256, 512, 65551, 181, 181, 1, 1, None) == B.SC_EUNSUPPORTED   # 2^31 + 32663 elements
    # the largest batch of such images that still fits is accepted by the planner
    assert lib.sparse_conv_get_launch(layer.handle, 65550, 181, 181, 1, 1, out) == B.SC_OK
    assert out[8] % 64 == 0 and 0 < out[7] <= 160 * 1024
    layer.close()


def _plan_ok(layer, N, H, W, st, p, what):
    bad = layer.check_plan(N, H, W, st, p)
    assert bad == 0, f"{what}: plan check {bad} failed, launch {layer.get_launch(N, H, W, st, p)}"


def test_plans_hold_every_stored_weight_once_random_shapes_and_launches():
    """Host side of the geometry plan (section 7: the input offsets are computed before the kernel
    runs): for random layers, geometries and launch overrides the library's own check finds every
    CSR entry exactly once in the plan, with its tap's offset inside the staged tile."""
    from helpers import rand_layer
    rng = np.random.default_rng(31337)
    ran = 0
    for t in range(160):
        R, S = int(rng.integers(1, 6)), int(rng.integers(1, 6))
        st, p = int(rng.integers(1, 4)), int(rng.integers(0, 4))
        H, W = int(rng.integers(1, 40)), int(rng.integers(1, 200 if t % 3 == 0 else 70))
        if H + 2 * p < R or W + 2 * p < S:
            continue
        N, Cn, K = int(rng.integers(1, 300 if t % 5 == 0 else 20)), int(rng.integers(1, 40)), int(rng.integers(1, 70))
        dtype = str(rng.choice(["f32", "f16"]))
        w, m, _ = rand_layer(rng, 1, Cn, K, R, S, H, W, density=float(rng.choice([0.02, 0.1, 0.3, 0.7])))
        vmax = 8 if dtype == "f16" else 4
        launch = [int(rng.choice([0, 1, 2, 4, vmax])), int(rng.choice([0, 1, 2, 3, 4])), int(rng.choice([0, 1, 2, 3, 5, 8])),
                  int(rng.choice([0, 1, 2, 4, 8, 16])), int(rng.choice([0, 0, 1, 2, 3, 7, 16])), 0, int(rng.choice([0, 1, 2])),
                  0, 0, int(rng.choice([0, 0, 1, 2, 3, 5, 9, 17])),     # what a lane stands for (1 + G: outputs)
                  int(rng.choice([0, 0, 1, 2, 4, 8]))]                  # workgroups the channels are dealt over
        if launch[9] > 1:
            launch[6] = int(rng.choice([0, 1]))
        if rng.integers(0, 3) == 0:
            launch = [0]
        layer = B.SparseConv(w, m, dtype=dtype, unify=bool(rng.integers(0, 2)))
        try:
            layer.set_launch(launch)
            layer.get_launch(N, H, W, st, p)
        except B.SparseConvError:
            layer.close()
            continue            # a combination the kernels do not run is refused, not planned
        _plan_ok(layer, N, H, W, st, p, f"case {t} {(N, Cn, K, R, S, H, W, st, p)} {dtype} {launch}")
        ran += 1
        layer.close()
    assert ran > 100


def test_plans_of_the_benchmark_layers_are_consistent():
    """Automatic launch choice at full batch size: VGG (both dtypes), the 224-pixel shapes, the 1x1 and 1-D layers."""
    from paper_2011_06295_amd import workloads as wl
    for work in (wl.vgg16(128, "f32"), wl.vgg16(256, "f16"), wl.lenet5(64), wl.resnet_1x1(128, "f32"),
                 wl.densenet_1x1(128, "f16"), wl.cnn_1d(128, "f32")):
        for li, spec in enumerate(work.layers, 1):
            layer = B.SparseConv(wl.make_weights(work.config, li, spec), wl.make_mask(work.config, li, spec), dtype=work.dtype)
            _plan_ok(layer, work.N, spec.H, spec.W, spec.stride, spec.pad, f"{work.name} {spec.name}")
            layer.close()
    work = wl.vgg16_imagenet(128, "f32")
    for li in (1, 2, 9):
        spec = work.layers[li - 1]
        layer = B.SparseConv(wl.make_weights(work.config, li, spec), wl.make_mask(work.config, li, spec), dtype="f32")
        _plan_ok(layer, work.N, spec.H, spec.W, spec.stride, spec.pad, f"{work.name} {spec.name}")
        layer.close()


def test_ranked_launches_can_be_pinned_and_plan_consistently():
    """sparse_conv_rank_launches lists what the measured choice would time: every candidate is accepted
    by sparse_conv_set_launch as it is, yields the same configuration back, and its plan is consistent."""
    from paper_2011_06295_amd import workloads as wl
    work = wl.vgg16(128, "f32")
    for li in (2, 6, 12):
        spec = work.layers[li - 1]
        layer = B.SparseConv(wl.make_weights(work.config, li, spec), wl.make_mask(work.config, li, spec), dtype="f32")
        geom = (work.N, spec.H, spec.W, spec.stride, spec.pad)
        first = layer.get_launch(*geom)
        cands = layer.rank_launches(*geom, max_candidates=6)
        assert 1 <= len(cands) <= 6 and len({tuple(c) for c in cands}) == len(cands)
        assert [first[k] for k in ("V", "WP", "WK", "KW", "Cc", "LP", "kblocks")] == cands[0][:5] + cands[0][6:8]
        for c in cands:
            layer.set_launch(c)
            got = layer.get_launch(*geom)
            assert [got[k] for k in ("V", "WP", "WK", "KW", "Cc", "LP", "kblocks", "store")] == c[:5] + c[6:9]
            _plan_ok(layer, *geom, f"{spec.name} {c}")
        layer.close()


def test_every_pooled_layer_of_the_benchmark_vgg_can_pool_in_its_store_step():
    """Host only: at the benchmark batches the planner finds tiles of whole row pairs for all five layers
    that are followed by a 2 x 2 maximum, and the plans it makes pass the plan check."""
    from paper_2011_06295_amd import workloads as wl
    for dtype, N in (("f32", 128), ("f16", 256)):
        work = wl.vgg16(N, dtype)
        pooled = 0
        for li, spec in enumerate(work.layers, 1):
            if not spec.pool_after:
                continue
            layer = B.SparseConv(wl.make_weights(work.config, li, spec), wl.make_mask(work.config, li, spec), dtype=dtype)
            layer.set_epilogue(None, relu=True, maxpool=True)
            info = layer.get_launch(N, spec.H, spec.W, spec.stride, spec.pad)
            F = layer.output_shape(spec.H, spec.W, spec.stride, spec.pad)[1] * 2
            assert info["lanes"] > 1 and (64 * info["WP"] // (info["lanes"] - 1)) % (2 * F) == 0
            assert layer.check_plan(N, spec.H, spec.W, spec.stride, spec.pad) == 0
            layer.close()
            pooled += 1
        assert pooled == 5
