"""Shared helpers of the test-suite (comparison rule, layer construction)."""
import numpy as np

TOL = {"f32": 1e-5, "f16": 2e-3}


def assert_close(got, ref, tol, what=""):
    """Element-wise |got - ref| <= tol * max|ref|: the stated relative tolerance against the
    largest reference value (an element-wise ratio is undefined where a sum cancels to nearly
    zero); at the largest elements it is exactly the stated relative tolerance."""
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    scale = float(np.max(np.abs(ref))) if ref.size else 0.0
    err = np.abs(got - ref)
    bound = np.full(err.shape, tol * scale)
    bad = err > bound
    if bad.any():
        idx = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(
            f"{what}: {int(bad.sum())}/{bad.size} outside tolerance {tol}; worst at {idx}: "
            f"got {got[idx]!r} ref {ref[idx]!r} (max|ref| {scale})")
    return float(err.max() / scale) if scale > 0 else 0.0


def rand_layer(rng, N, C, K, R, S, H, W, density=0.3, x_dist="normal"):
    w = rng.standard_normal((K, C, R, S)).astype(np.float32)
    m = (rng.random((K, C, R, S)) < density).astype(np.uint8)
    x = rng.standard_normal((N, C, H, W)) if x_dist == "normal" else rng.random((N, C, H, W))
    return w, m, x.astype(np.float32)
