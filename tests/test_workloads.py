"""The synthetic workload recipe: shapes, per-row counts and determinism."""
import numpy as np

from paper_2011_06295_amd import workloads as wl


def test_vgg_shapes_and_row_counts():
    v = wl.vgg16()
    assert [l.row_nnz for l in v.layers] == [5, 108, 101, 187, 173, 317, 288, 259, 461, 403, 346, 288, 230]
    assert [l.H for l in v.layers] == [32, 32, 16, 16, 8, 8, 8, 4, 4, 4, 2, 2, 2]
    assert [l.C for l in v.layers] == [3, 64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512]
    assert [l.K for l in v.layers] == [64, 64, 128, 128, 256, 256, 256, 512, 512, 512, 512, 512, 512]
    assert [l.sparsity_bp for l in v.layers][0] == 8000 and v.layers[-1].sparsity_bp == 9500
    assert all(l.E == l.H and l.F == l.W for l in v.layers)
    macs = sum(l.K * l.row_nnz * l.E * l.F * v.N for l in v.layers)
    assert abs(macs - 5.19e9) / 5.19e9 < 0.01


def test_lenet_and_sweep_counts():
    le = wl.lenet5()
    assert [(l.row_nnz, l.E) for l in le.layers] == [(3, 24), (50, 8)]
    assert [wl.nnz_per_row(2304, s) for s in wl.SWEEP_SPARSITIES_BP] == [1152, 691, 461, 230, 115, 23]


def test_masks_have_the_stated_structure():
    spec = wl.vgg16().layers[4]
    m = wl.make_mask(3, 5, spec).reshape(spec.K, -1)
    assert (m.sum(1) == spec.row_nnz).all()
    s = wl.sweep_layer(9000, ragged=True).layers[0]
    mr = wl.make_mask(5, wl.sweep_layer_index(9000, True), s).reshape(s.K, -1)
    assert mr.sum() == s.K * s.row_nnz and mr.sum(1).std() > 10
    c1 = wl.config1().layers[0]
    mb = wl.make_mask(1, 1, c1)
    assert 0.07 < mb.mean() < 0.13 and mb.shape == (32, 16, 3, 3)


def test_generators_are_deterministic():
    spec = wl.lenet5().layers[1]
    assert np.array_equal(wl.make_weights(2, 2, spec), wl.make_weights(2, 2, spec))
    assert np.array_equal(wl.make_mask(2, 2, spec), wl.make_mask(2, 2, spec))
    x = wl.make_input(wl.lenet5())
    assert x.shape == (64, 1, 28, 28) and x.min() >= 0 and x.max() < 1
    assert np.array_equal(x, wl.make_input(wl.lenet5()))


def test_bench_refuses_more_than_one_gpu():
    """bench.py is a one-GPU benchmark: any other --gpus value ends with a message, before touching a GPU."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in (r.stderr + r.stdout)
