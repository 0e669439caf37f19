"""Pins of the CPU oracle against things other than itself.

Each test fixes the oracle to something the paper or the mathematics
determines: hand-worked examples of eq. 1 (section 3), the seven-loop brute
force, closed forms, delta inputs, special cases that reduce to library
routines (torch conv2d, scipy CSR product, numpy float16), and independent
NumPy encoders for the CSR of section 7.  All CPU-only.
"""
import json
import os

import numpy as np
import pytest

import oracle

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def rand_layer(rng, N, C, K, R, S, H, W, density=0.4):
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    m = (rng.random((K, C, R, S)) < density).astype(np.uint8)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    return w, m, x


# ------------------------------------------------------------------ shapes

@pytest.mark.parametrize("H,p,R,st,E", [
    (32, 1, 3, 1, 32), (28, 0, 5, 1, 24), (12, 0, 5, 1, 8), (3, 1, 3, 2, 2), (3, 0, 3, 1, 1),
    (7, 2, 3, 3, 3), (8, 0, 3, 2, 3), (2, 1, 3, 1, 2), (1, 1, 3, 1, 1), (2, 0, 3, 1, -1),
    (14, 1, 3, 1, 14), (300, 0, 2, 1, 299),
])
def test_output_dim(H, p, R, st, E):
    # section 3: E = (H + 2*padding - R)/stride + 1, floor; -1 when the filter does not fit
    assert oracle.output_dim(H, p, R, st) == E


# ------------------------------------------------------------------ hand-worked examples

def _gold_cases():
    with open(os.path.join(GOLD, "hand_3x3.json")) as f:
        g = json.load(f)
    return [(g["x"], c) for c in g["cases"]]


@pytest.mark.parametrize("x,case", _gold_cases(), ids=lambda v: v["name"] if isinstance(v, dict) else "x")
def test_hand_examples(x, case):
    w = np.array(case["w"], dtype=np.float32).reshape(1, 1, 3, 3)
    m = np.array(case["mask"], dtype=np.uint8).reshape(1, 1, 3, 3)
    xx = np.array(x, dtype=np.float32).reshape(1, 1, 3, 3)
    rowptr, colidx, values = oracle.csr_encode(w, m)
    assert rowptr.tolist() == case["rowptr"]
    assert colidx.tolist() == case["colidx"]
    assert values.tolist() == [float(v) for v in case["values"]]
    out = oracle.sparse_conv((rowptr, colidx, values), xx, 1, 3, 3, case["stride"], case["pad"])
    assert out[0, 0].tolist() == [[float(v) for v in row] for row in case["out"]]
    out32 = oracle.sparse_conv((rowptr, colidx, values), xx, 1, 3, 3, case["stride"], case["pad"], acc="f32")
    assert np.array_equal(out, out32)
    pts = [(0, 0, i, j) for i in range(out.shape[2]) for j in range(out.shape[3])]
    pv = oracle.sparse_conv_points((rowptr, colidx, values), xx, 1, 3, 3, case["stride"], case["pad"], pts)
    assert pv.tolist() == [float(v) for row in case["out"] for v in row]
    assert oracle.dense_conv7(w, m, xx, case["stride"], case["pad"])[0, 0].tolist() == out[0, 0].tolist()


# ------------------------------------------------------------------ CSR encoder (section 7)

def numpy_csr(w, m):
    K = w.shape[0]
    w2, m2 = w.reshape(K, -1), m.reshape(K, -1)
    rows, cols = np.nonzero(m2)  # row-major order == ascending column within each row
    rowptr = np.zeros(K + 1, dtype=np.int32)
    np.cumsum(np.bincount(rows, minlength=K), out=rowptr[1:])
    return rowptr, cols.astype(np.int32), w2[rows, cols].astype(np.float32)


@pytest.mark.parametrize("seed", range(6))
def test_csr_matches_numpy_encoder(seed):
    rng = np.random.default_rng(100 + seed)
    K, C, R, S = int(rng.integers(1, 9)), int(rng.integers(1, 7)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    m = (rng.random((K, C, R, S)) < rng.random()).astype(np.uint8)
    if seed == 0:
        m[0] = 0          # an empty row is legal
    if seed == 1:
        m[-1] = 1         # a full row
    a = oracle.csr_encode(w, m)
    b = numpy_csr(w, m)
    for u, v in zip(a, b):
        assert u.dtype == v.dtype and u.tobytes() == v.tobytes()
    rowptr, colidx, _ = a
    assert rowptr[0] == 0
    # rowptr[i+1] - rowptr[i] is the stored count of channel i (section 7)
    assert (np.diff(rowptr) == m.reshape(K, -1).astype(bool).sum(1)).all()
    for k in range(K):
        row = colidx[rowptr[k]:rowptr[k + 1]]
        assert (np.diff(row) > 0).all()


def test_csr_mask_decides_and_bits_are_kept():
    # a kept zero / negative zero / NaN is stored bit for bit, a dropped non-zero is not
    w = np.array([[0.0, -0.0, 5.0, np.nan, np.inf, 1e-45]], dtype=np.float32).reshape(1, 6, 1, 1)
    m = np.array([[1, 1, 0, 1, 1, 1]], dtype=np.uint8).reshape(1, 6, 1, 1)
    rowptr, colidx, values = oracle.csr_encode(w, m)
    assert rowptr.tolist() == [0, 5] and colidx.tolist() == [0, 1, 3, 4, 5]
    assert values.tobytes() == w.reshape(-1)[[0, 1, 3, 4, 5]].tobytes()
    # mask bytes other than 1 also mean "keep"
    m2 = m * 255
    assert oracle.csr_encode(w, m2)[1].tolist() == [0, 1, 3, 4, 5]


def python_unify(mask2d):
    K, L = mask2d.shape
    target = int(mask2d.astype(bool).sum(1).max()) if K else 0
    out = np.zeros((K, L), dtype=np.uint8)
    for k in range(K):
        row = [1 if v else 0 for v in mask2d[k]]
        need = target - sum(row)
        j = 1
        while need > 0 and j < L:
            if row[j] == 0 and row[j - 1] != 0:
                row[j] = 2
                need -= 1
            j += 1
        j = 0
        while need > 0 and j < L:
            if row[j] == 0:
                row[j] = 2
                need -= 1
            j += 1
        out[k] = row
    return out, target


@pytest.mark.parametrize("seed", range(5))
def test_unify_rule_and_invariance(seed):
    rng = np.random.default_rng(200 + seed)
    N, C, K, R, S, H, W = 2, 3, 6, 3, 3, 6, 5
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.3)
    if seed == 0:
        m[2] = 0
    um, target = oracle.unify_mask(m)
    pm, ptarget = python_unify(m.reshape(K, -1))
    assert target == ptarget and np.array_equal(um.reshape(K, -1), pm)
    # kept entries stay kept, only dropped ones become explicit zeros
    assert ((um == 1) == (m != 0)).all()
    rowptr, colidx, values = oracle.csr_encode(w, um)
    assert rowptr.tolist() == [k * target for k in range(K + 1)]        # one unified count
    added = um.reshape(K, -1)[np.repeat(np.arange(K), target), colidx] == 2
    assert (values[added] == 0).all() and not np.signbit(values[added]).any()
    base = oracle.sparse_conv(oracle.csr_encode(w, m), x, K, R, S, 1, 1)
    uni = oracle.sparse_conv((rowptr, colidx, values), x, K, R, S, 1, 1)
    assert np.array_equal(base, uni)                                    # "does not change the result"


def test_unify_worked_rows():
    # L = 8, fullest row has 4.  Row 0: kept {1,5}: the run at 1 grows to 2, then 3.
    # Row 1: kept {7}: nothing to the right, so the lowest free columns 0,1,2 are taken.
    # Row 2: kept {0,1,2,3}: already full.  Row 3: empty: columns 0..3.
    m = np.zeros((4, 8), dtype=np.uint8)
    m[0, [1, 5]] = 1
    m[1, 7] = 1
    m[2, :4] = 1
    um, target = oracle.unify_mask(m.reshape(4, 8, 1, 1))
    assert target == 4
    assert um.reshape(4, 8).tolist() == [
        [0, 1, 2, 2, 0, 1, 0, 0],
        [2, 2, 2, 0, 0, 0, 0, 1],
        [1, 1, 1, 1, 0, 0, 0, 0],
        [2, 2, 2, 2, 0, 0, 0, 0],
    ]


# ------------------------------------------------------------------ binary16

def test_f16_matches_numpy_float16():
    # every binary16 value survives the round trip; conversion equals numpy's RNE cast
    allh = np.arange(65536, dtype=np.uint16)
    f = allh.view(np.float16).astype(np.float32)
    back = oracle.f32_to_f16_bits(f)
    notnan = ~np.isnan(f)
    assert np.array_equal(back[notnan], allh[notnan])
    assert np.isnan(back[~notnan].view(np.float16)).all()
    rng = np.random.default_rng(7)
    parts = [
        rng.standard_normal(20000).astype(np.float32),
        (rng.standard_normal(20000) * 1e-5).astype(np.float32),      # binary16 subnormal range
        (rng.standard_normal(5000) * 1e5).astype(np.float32),        # overflow to inf
        rng.integers(0, 2**32, 50000, dtype=np.uint32).view(np.float32),
    ]
    # exact ties between neighbouring binary16 values
    h = rng.integers(0, 0x7bff, 5000).astype(np.uint16)
    lo = h.view(np.float16).astype(np.float64)
    hi = (h + 1).astype(np.uint16).view(np.float16).astype(np.float64)
    parts.append(((lo + hi) / 2).astype(np.float32))
    v = np.concatenate(parts)
    got = oracle.f32_to_f16_bits(v)
    with np.errstate(over="ignore", invalid="ignore"):
        want = v.astype(np.float16).view(np.uint16)
    nn = ~np.isnan(v)
    assert np.array_equal(got[nn], want[nn])
    rt = oracle.round_through_f16(v[nn])
    with np.errstate(over="ignore"):
        assert np.array_equal(rt, v[nn].astype(np.float16).astype(np.float32))


# ------------------------------------------------------------------ brute force (eq. 1)

def _tiny_shapes():
    rng = np.random.default_rng(31)
    shapes = []
    for _ in range(40):
        R, S = int(rng.choice([1, 2, 3, 5])), int(rng.choice([1, 2, 3, 5]))
        st, p = int(rng.integers(1, 4)), int(rng.integers(0, 3))
        H, W = int(rng.integers(1, 10)), int(rng.integers(1, 10))
        if H + 2 * p < R or W + 2 * p < S:
            continue
        shapes.append((int(rng.integers(1, 4)), int(rng.integers(1, 6)), int(rng.integers(1, 6)), R, S, H, W, st, p))
    return shapes


@pytest.mark.parametrize("shape", _tiny_shapes())
def test_sparse_equals_seven_loop_brute_force(shape):
    N, C, K, R, S, H, W, st, p = shape
    rng = np.random.default_rng(abs(hash(shape)) % (2**32))
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W, density=0.5)
    csr = oracle.csr_encode(w, m)
    a = oracle.sparse_conv(csr, x, K, R, S, st, p)
    b = oracle.dense_conv7(w, m, x, st, p)
    assert a.shape == b.shape == (N, K, oracle.output_dim(H, p, R, st), oracle.output_dim(W, p, S, st))
    assert np.array_equal(a, b)          # same double sums in the same (c,r,s) order
    E, F = a.shape[2:]
    pts = np.stack(np.unravel_index(np.arange(a.size), a.shape), 1)
    pv = oracle.sparse_conv_points(csr, x, K, R, S, st, p, pts)
    assert np.array_equal(pv.astype(np.float32), a.reshape(-1))
    # numpy statement of eq. 1, written independently of both C routines
    xp = np.zeros((N, C, H + 2 * p, W + 2 * p))
    xp[:, :, p:p + H, p:p + W] = x
    wm = w.astype(np.float64) * (m != 0)
    ref = np.zeros((N, K, E, F))
    for r in range(R):
        for s in range(S):
            patch = xp[:, :, r:r + (E - 1) * st + 1:st, s:s + (F - 1) * st + 1:st]
            ref += np.einsum("kc,ncij->nkij", wm[:, :, r, s], patch)
    np.testing.assert_allclose(a, ref, rtol=1e-6, atol=1e-6)
    a32 = oracle.sparse_conv(csr, x, K, R, S, st, p, acc="f32")
    np.testing.assert_allclose(a32, ref, rtol=1e-4, atol=1e-4)


# ------------------------------------------------------------------ invariants

def test_dense_mask_equals_torch_conv2d():
    import torch
    import torch.nn.functional as Fnn
    rng = np.random.default_rng(5)
    for (N, C, K, R, S, H, W, st, p) in [(2, 4, 5, 3, 3, 9, 8, 1, 1), (1, 3, 2, 5, 2, 11, 7, 2, 2), (3, 2, 3, 1, 1, 4, 4, 1, 0)]:
        w, _, x = rand_layer(rng, N, C, K, R, S, H, W)
        m = np.ones_like(w, dtype=np.uint8)
        a = oracle.sparse_conv(oracle.csr_encode(w, m), x, K, R, S, st, p)
        b = Fnn.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(), stride=st, padding=p).numpy()
        np.testing.assert_allclose(a, b, rtol=1e-6, atol=1e-6)
        # and with a random mask, against conv2d of w*mask
        m2 = (rng.random(w.shape) < 0.3).astype(np.uint8)
        a2 = oracle.sparse_conv(oracle.csr_encode(w, m2), x, K, R, S, st, p)
        b2 = Fnn.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w * m2).double(), stride=st, padding=p).numpy()
        np.testing.assert_allclose(a2, b2, rtol=1e-6, atol=1e-6)


def test_all_zero_mask_gives_zero_output():
    rng = np.random.default_rng(6)
    w, m, x = rand_layer(rng, 2, 3, 4, 3, 3, 5, 5)
    m[:] = 0
    csr = oracle.csr_encode(w, m)
    assert csr[0].tolist() == [0] * 5 and csr[1].size == 0
    out = oracle.sparse_conv(csr, x, 4, 3, 3, 1, 1)
    assert out.shape == (2, 4, 5, 5) and not out.any()


def test_linear_in_weights_and_additive_in_mask():
    rng = np.random.default_rng(8)
    N, C, K, R, S, H, W = 2, 3, 4, 3, 2, 6, 7
    w1, m, x = rand_layer(rng, N, C, K, R, S, H, W)
    w2 = rng.standard_normal(w1.shape).astype(np.float32)
    conv = lambda w, mm: oracle.sparse_conv(oracle.csr_encode(w, mm), x, K, R, S, 1, 1).astype(np.float64)
    a, b = 0.75, -2.5
    lhs = conv((a * w1 + b * w2).astype(np.float32), m)
    np.testing.assert_allclose(lhs, a * conv(w1, m) + b * conv(w2, m), rtol=0, atol=2e-5)
    ma = m * (rng.random(m.shape) < 0.5)
    mb = m - ma
    np.testing.assert_allclose(conv(w1, m), conv(w1, ma) + conv(w1, mb), rtol=0, atol=2e-6)


def test_one_by_one_filter_is_a_csr_matrix_product():
    import scipy.sparse as sp
    rng = np.random.default_rng(9)
    N, C, K, H, W = 3, 16, 8, 5, 4
    w, m, x = rand_layer(rng, N, C, K, 1, 1, H, W, density=0.25)
    rowptr, colidx, values = oracle.csr_encode(w, m)
    A = sp.csr_matrix((values.astype(np.float64), colidx, rowptr), shape=(K, C))
    out = oracle.sparse_conv((rowptr, colidx, values), x, K, 1, 1, 1, 0)
    for n in range(N):
        ref = A @ x[n].reshape(C, H * W).astype(np.float64)
        np.testing.assert_allclose(out[n].reshape(K, H * W), ref, rtol=1e-6, atol=1e-6)


# ------------------------------------------------------------------ closed forms

def test_constant_input_gives_row_sums():
    rng = np.random.default_rng(10)
    N, C, K, R, S, H, W = 2, 4, 5, 3, 3, 7, 6
    w, m, _ = rand_layer(rng, N, C, K, R, S, H, W)
    x = np.ones((N, C, H, W), dtype=np.float32)
    rowptr, colidx, values = oracle.csr_encode(w, m)
    out = oracle.sparse_conv((rowptr, colidx, values), x, K, R, S, 1, 0)
    for k in range(K):
        rs = np.float32(values[rowptr[k]:rowptr[k + 1]].astype(np.float64).sum())
        assert (out[:, k] == rs).all()


def test_ones_everywhere_counts_taps():
    C = 3
    w = np.ones((2, C, 3, 3), dtype=np.float32)
    m = np.ones_like(w, dtype=np.uint8)
    x = np.ones((1, C, 5, 6), dtype=np.float32)
    out = oracle.sparse_conv(oracle.csr_encode(w, m), x, 2, 3, 3, 1, 1)
    want = np.full((5, 6), 9.0 * C)
    want[0, :] = want[-1, :] = 6.0 * C
    want[:, 0] = want[:, -1] = 6.0 * C
    for i in (0, -1):
        for j in (0, -1):
            want[i, j] = 4.0 * C
    assert (out[0, 0] == want).all() and (out[0, 1] == want).all()


def test_sum_of_magnitudes_output():
    # The optional second output is sum |w * x| over the stored taps of each output element (the
    # scale a rounding-error bound for eq. 1 is relative to).  Pinned three ways: an independent numpy
    # statement of eq. 1 on the magnitudes (dense einsum over the padded input), the closed form for
    # a constant input without padding (sum of |w| over the row), and |out| <= abs_out with equality
    # where all products have one sign.
    rng = np.random.default_rng(77)
    N, C, K, R, S, H, W, st, p = 2, 3, 4, 3, 2, 6, 5, 2, 1
    w, m, x = rand_layer(rng, N, C, K, R, S, H, W)
    csr = oracle.csr_encode(w, m)
    out, aout = oracle.sparse_conv(csr, x, K, R, S, st, p, want_abs=True)
    E, F = out.shape[2:]
    xp = np.zeros((N, C, H + 2 * p, W + 2 * p))
    xp[:, :, p:p + H, p:p + W] = np.abs(x.astype(np.float64))
    wa = np.abs((w * m).astype(np.float64))
    ref = np.zeros((N, K, E, F))
    for r in range(R):
        for s_ in range(S):
            patch = xp[:, :, r:r + (E - 1) * st + 1:st, s_:s_ + (F - 1) * st + 1:st]
            ref += np.einsum("kc,ncij->nkij", wa[:, :, r, s_], patch)
    np.testing.assert_allclose(aout, ref, rtol=2e-7, atol=0)
    assert (np.abs(out) <= aout * (1 + 1e-6)).all()
    # one sign everywhere: the two outputs coincide
    out2, aout2 = oracle.sparse_conv(oracle.csr_encode(np.abs(w), m), np.abs(x), K, R, S, st, p, want_abs=True)
    assert (out2 == aout2).all() and (aout2 == aout).all()
    # constant input, no padding: sum of |w| over the row
    ones = np.ones((1, C, H, W), dtype=np.float32)
    _, a3 = oracle.sparse_conv(csr, ones, K, R, S, 1, 0, want_abs=True)
    rowptr, _, values = csr
    for k in range(K):
        assert (a3[0, k] == np.float32(np.abs(values[rowptr[k]:rowptr[k + 1]].astype(np.float64)).sum())).all()


@pytest.mark.parametrize("st,p", [(1, 0), (1, 1), (2, 1), (3, 2), (2, 0)])
def test_delta_input_reads_back_the_filter(st, p):
    # x = delta at (c0,y0,x0): Out[k][i][j] = (w*mask)[k][c0][y0 - i*st + p][x0 - j*st + p] where that index exists
    rng = np.random.default_rng(11)
    N, C, K, R, S, H, W = 1, 3, 4, 3, 2, 7, 6
    w, m, _ = rand_layer(rng, N, C, K, R, S, H, W, density=0.6)
    c0, y0, x0 = 1, 3, 2
    x = np.zeros((N, C, H, W), dtype=np.float32)
    x[0, c0, y0, x0] = 1.0
    out = oracle.sparse_conv(oracle.csr_encode(w, m), x, K, R, S, st, p)
    E, F = out.shape[2:]
    wm = w * (m != 0)
    for k in range(K):
        for i in range(E):
            for j in range(F):
                r, s = y0 - i * st + p, x0 - j * st + p
                want = wm[k, c0, r, s] if (0 <= r < R and 0 <= s < S) else 0.0
                assert out[0, k, i, j] == want


# ------------------------------------------------------------------ glue

def test_relu_and_maxpool():
    rng = np.random.default_rng(12)
    x = rng.standard_normal((2, 3, 7, 6)).astype(np.float32)
    assert np.array_equal(oracle.relu(x), np.maximum(x, 0))
    mp = oracle.maxpool2(x)
    ref = x[:, :, :6, :6].reshape(2, 3, 3, 2, 3, 2).max(axis=(3, 5))
    assert np.array_equal(mp, ref)


# ------------------------------------------------------------------ cluster-quantised weights (sections 6, 9)

def _numpy_codebook(index, centroids, mask):
    """Independent statement: stored values are the binary16 centroids picked by the kept indices, row-major."""
    c16 = np.asarray(centroids, dtype=np.float32).astype(np.float16)
    keep = np.asarray(mask).reshape(-1) != 0
    codes = np.asarray(index).reshape(-1)[keep].astype(np.uint8)
    padded = np.concatenate([codes, np.zeros(codes.size % 2, dtype=np.uint8)])
    packed = (padded[0::2] | (padded[1::2] << 4)).astype(np.uint8)
    return c16.view(np.uint16), packed, c16.astype(np.float32)[codes]


@pytest.mark.parametrize("seed", range(6))
def test_codebook_csr_matches_numpy(seed):
    rng = np.random.default_rng(600 + seed)
    K, C, R, S = int(rng.integers(1, 9)), int(rng.integers(1, 7)), int(rng.integers(1, 4)), int(rng.integers(1, 4))
    index = rng.integers(0, 16, (K, C, R, S)).astype(np.uint8)
    centroids = (rng.standard_normal(16) * 10.0 ** rng.integers(-6, 3)).astype(np.float32)   # incl. half subnormals
    mask = (rng.random((K, C, R, S)) < 0.4).astype(np.uint8)
    rowptr, colidx, packed, bits, values = oracle.codebook_csr_encode(index, centroids, mask)
    want_bits, want_packed, want_values = _numpy_codebook(index, centroids, mask)
    assert np.array_equal(bits, want_bits)
    assert np.array_equal(packed, want_packed)
    assert np.array_equal(values.view(np.uint32), want_values.view(np.uint32))
    # rows and columns are those of the plain encoder on any weights with that mask
    r2, c2, _ = oracle.csr_encode(np.ones((K, C, R, S), np.float32), mask)
    assert np.array_equal(rowptr, r2) and np.array_equal(colidx, c2)


def test_codebook_worked_example():
    # two output channels of 1x2x2 weights; centroids 0: -1, 1: 0, 2: 0.5, 3: 2, 4: 0.1 (not a half), rest unused
    centroids = np.zeros(16, np.float32)
    centroids[:5] = [-1.0, 0.0, 0.5, 2.0, 0.1]
    index = np.array([[3, 0, 2, 4], [2, 2, 15, 0]], np.uint8).reshape(2, 1, 2, 2)
    mask = np.array([[1, 0, 1, 1], [0, 1, 0, 1]], np.uint8).reshape(2, 1, 2, 2)
    rowptr, colidx, packed, bits, values = oracle.codebook_csr_encode(index, centroids, mask)
    assert rowptr.tolist() == [0, 3, 5] and colidx.tolist() == [0, 2, 3, 1, 3]
    # codes in stored order 3,2,4,2,0 -> bytes (3 | 2<<4), (4 | 2<<4), (0)
    assert packed.tolist() == [0x23, 0x24, 0x00]
    assert bits[:4].tolist() == [0xBC00, 0x0000, 0x3800, 0x4000]
    assert values.tolist() == [2.0, 0.5, float(np.float16(0.1)), 0.5, -1.0]
    # an explicit zero of the unify step takes the first zero centroid (number 1 here)
    m2 = mask.copy()
    m2[1, 0, 0, 0] = 2
    _, colidx2, packed2, _, values2 = oracle.codebook_csr_encode(index, centroids, m2)
    assert colidx2.tolist() == [0, 2, 3, 0, 1, 3] and packed2.tolist() == [0x23, 0x14, 0x02]
    assert values2.tolist() == [2.0, 0.5, float(np.float16(0.1)), 0.0, 0.5, -1.0]
    with pytest.raises(ValueError):
        oracle.codebook_csr_encode(index, np.arange(1, 17, dtype=np.float32), m2)    # no zero centroid
    bad = index.copy()
    bad[0, 0, 0, 0] = 16
    with pytest.raises(ValueError):
        oracle.codebook_csr_encode(bad, centroids, mask)


def test_codebook_convolution_is_the_convolution_of_the_decoded_weights():
    rng = np.random.default_rng(77)
    N, C, K, R, S, H, W = 2, 5, 6, 3, 3, 7, 6
    index = rng.integers(0, 16, (K, C, R, S)).astype(np.uint8)
    centroids = np.sort(rng.standard_normal(16)).astype(np.float32)
    mask = (rng.random((K, C, R, S)) < 0.3).astype(np.uint8)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    rowptr, colidx, _, _, values = oracle.codebook_csr_encode(index, centroids, mask)
    got = oracle.sparse_conv((rowptr, colidx, values), x, K, R, S, 1, 1)
    dense = centroids.astype(np.float16).astype(np.float32)[index]
    want = oracle.dense_conv7(dense, mask, x, 1, 1)
    assert np.array_equal(got, want)
