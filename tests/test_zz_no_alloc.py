"""The entry point that allocates no device memory (sparse_conv_forward_static) against
sparse_conv_forward, through the C ABI: same kernel, tables read from the GPU's static scratch."""
import ctypes as C

import numpy as np
import pytest

import oracle
from helpers import TOL, assert_close, rand_layer

pytestmark = pytest.mark.gpu


def _raw_forward(lib, fn, handle, x, out, stride, pad):
    import torch
    N, _, H, W = x.shape
    rc = getattr(lib, fn)(handle, x.data_ptr(), out.data_ptr(), N, H, W, stride, pad,
                          torch.cuda.current_stream().cuda_stream or None)
    assert rc == 0, (fn, rc)


@pytest.mark.parametrize("dtype", ["f32", "f16"])
def test_static_entry_point_matches_forward_twice_in_a_row(dtype):
    """Two calls in a row on the shared scratch, the second with a smaller input (other geometry,
    smaller tables: the scratch still holds the tail of the first call's), then the first layer
    again, then a second handle: every output equals sparse_conv_forward's bit for bit and
    matches the oracle."""
    import torch
    from paper_2011_06295_amd import binding as B
    lib = B.raw_library()
    tdt = torch.float16 if dtype == "f16" else torch.float32
    rng = np.random.default_rng(2011)
    w, m, xa = rand_layer(rng, 37, 24, 40, 3, 3, 13, 11, density=0.25)
    layer = B.SparseConv(w, m, dtype=dtype)
    w2, m2, xc = rand_layer(rng, 9, 7, 5, 1, 1, 6, 6, density=0.5)
    other = B.SparseConv(w2, m2, dtype=dtype)
    xb = xa[:5, :, :7, :6].copy()                      # smaller batch and map
    split = B.SparseConv(w, m, dtype=dtype)           # its channels dealt over 4 workgroups: partial sums and counters
    split.set_launch([0, 0, 0, 0, 3, 0, 0, 0, 0, 0, 4])   # live in the scratch as well
    # a cluster-quantised layer: 4-byte entries and the centroids go through the scratch
    cen = np.sort(rng.standard_normal(16)).astype(np.float32)
    index = rng.integers(0, 16, w.shape).astype(np.uint8)
    coded = B.SparseConv.from_codebook(index, cen, m, dtype=dtype)
    wc = cen.astype(np.float16).astype(np.float32)[index]
    calls = [(layer, w, m, xa, 1, 1), (layer, w, m, xb, 2, 1), (coded, wc, m, xa, 1, 1), (layer, w, m, xa, 1, 1),
             (other, w2, m2, xc, 1, 0), (coded, wc, m, xb, 2, 1),
             (layer, w, m, xb, 2, 1), (split, w, m, xa, 1, 1), (split, w, m, xa, 1, 1), (split, w, m, xb, 2, 1),
             (layer, w, m, xa, 1, 1), (split, w, m, xb, 2, 1)]
    for step, (lay, ww, mm, x, stride, pad) in enumerate(calls):
        xt = torch.from_numpy(x).cuda().to(tdt).contiguous()
        E, F = lay.output_shape(x.shape[2], x.shape[3], stride, pad)
        want = torch.full((x.shape[0], lay.K, E, F), float("nan"), dtype=tdt, device="cuda")
        got = torch.full_like(want, float("nan"))
        print(f"static entry point, call {step}: {dtype} input {tuple(x.shape)} stride {stride} pad {pad}", flush=True)
        _raw_forward(lib, "sparse_conv_forward_static", lay.handle, xt, got, stride, pad)
        _raw_forward(lib, "sparse_conv_forward", lay.handle, xt, want, stride, pad)
        torch.cuda.synchronize()
        assert torch.equal(got, want), f"call {step}"
        rowptr, colidx, values = oracle.csr_encode(ww, mm)
        xo = x
        if dtype == "f16":
            values, xo = oracle.round_through_f16(values), oracle.round_through_f16(x)
        ref = oracle.sparse_conv((rowptr, colidx, values), xo, lay.K, lay.R, lay.S, stride, pad)
        assert_close(got.float().cpu().numpy(), ref, TOL[dtype], f"static call {step}")
    layer.close()
    other.close()
    split.close()
    coded.close()


def test_static_entry_point_rejects_tables_beyond_the_scratch():
    """A layer whose tables exceed the 16 MiB array is refused with SC_ETOOBIG before anything is
    enqueued (no GPU memory is touched: the pointers are never dereferenced); the ordinary entry
    point's argument checks apply unchanged."""
    from paper_2011_06295_amd import binding as B
    lib = B.raw_library()
    K, Cc = 1024, 256                                   # 2.36 M stored weights: about 19 MB of tables
    w = np.ones((K, Cc, 3, 3), dtype=np.float32)
    m = np.ones_like(w, dtype=np.uint8)
    layer = B.SparseConv(w, m)
    assert lib.sparse_conv_forward_static(layer.handle, 1 << 20, 1 << 30, 4, 8, 8, 1, 1, None) == B.SC_ETOOBIG
    assert lib.sparse_conv_forward_static(layer.handle, None, 1 << 30, 4, 8, 8, 1, 1, None) == B.SC_EINVAL
    assert lib.sparse_conv_forward_static(layer.handle, 1 << 20, 1 << 30, 0, 8, 8, 1, 1, None) == B.SC_OK
    layer.close()
