"""The C oracle against the numpy definition and closed forms (it is used where numpy temporaries would not fit)."""
import numpy as np
import pytest

from cr_inputs import workloads as wl
from oracle import cr_tree, native


def _data(m, d, seed):
    rng = np.random.default_rng(seed)
    X = rng.standard_normal((m, d)).astype(np.float32)
    w = rng.standard_normal(d).astype(np.float32)
    y = rng.standard_normal(m).astype(np.float32)
    return X, y, w


@pytest.mark.parametrize("model", [cr_tree.LINEAR, cr_tree.LOGISTIC])
def test_segment_gradient_matches_definition(model):
    X, y, w = _data(700, 33, seed=1)
    if model == cr_tree.LOGISTIC:
        y = (y > 0).astype(np.float32)
    for b, e in [(0, 700), (13, 14), (100, 613), (5, 5)]:
        g = native.segment_gradient(X, y, w, b, e, model)
        ref = cr_tree.partial_gradient(X, y, w, b, e, model) if e > b else np.zeros(33)
        np.testing.assert_allclose(g, ref, rtol=1e-12, atol=1e-12)
    np.testing.assert_allclose(native.full_gradient(X, y, w, model), cr_tree.full_gradient(X, y, w, model), rtol=1e-12, atol=1e-12)


def test_zero_residual_and_integer_exactness():
    rng = np.random.default_rng(2)
    X = rng.integers(-4, 5, size=(300, 6)).astype(np.float32)
    w = rng.integers(-3, 4, size=6).astype(np.float32)
    y = (X @ w).astype(np.float32)                       # exact: small integers
    assert np.array_equal(native.full_gradient(X, y, w), np.zeros(6))
    y2 = y + 1.0                                         # residual -1 on every row: g = -column sums
    assert np.array_equal(native.full_gradient(X, y2, w), -X.astype(np.float64).sum(0))


def test_bf16_bits_are_widened_exactly():
    X, y, w = _data(257, 16, seed=3)
    bits = wl.to_bf16_bits(X)
    Xr = wl.bf16_bits_to_f32(bits)
    g = native.segment_gradient(bits, y, w, 3, 250, cr_tree.LINEAR)
    np.testing.assert_allclose(g, cr_tree.partial_gradient(Xr, y, w, 3, 250), rtol=1e-12, atol=1e-12)
    # rounding recipe: nearest, ties to even, 8 significant bits
    assert np.max(np.abs(Xr - X) / np.abs(X)) <= 2.0 ** -8
    t = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], dtype=np.float32)
    assert list(wl.bf16_bits_to_f32(wl.to_bf16_bits(t))) == [1.0, 1.0, 1.0 + 2.0 ** -6, -2.5, 0.0]


def test_coded_gradient_with_segments():
    X, y, w = _data(400, 12, seed=4)
    segs = [(0, 100, 0.5), (250, 300, -2.0), (399, 400, 3.0)]
    np.testing.assert_allclose(native.local_coded_gradient(X, y, w, segs), cr_tree.local_coded_gradient(X, y, w, segs), rtol=1e-12, atol=1e-12)
    assert native.num_threads() >= 1
