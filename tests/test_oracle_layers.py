"""Pins for the oracle's depthwise, pooling, ReLU, add and dense layers (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O


# ---------------------------------------------------------------- depthwise

@pytest.mark.parametrize("s,pad", [(1, (1, 1, 1, 1)), (2, (0, 1, 0, 1)), (1, (0, 0, 0, 0))])
def test_depthwise_is_block_diagonal_conv(s, pad):
    """Table 1 row 2: G = I_C, K = 1, F_C = 1 == a convolution whose filter is zero
    off the channel diagonal."""
    rng = np.random.default_rng(5)
    C = 6
    x = rng.integers(-6, 7, (2, C, 8, 7)).astype(np.float32)
    w = rng.integers(-3, 4, (C, 1, 3, 3)).astype(np.float32)
    full = np.zeros((C, C, 3, 3), np.float32)
    for c in range(C):
        full[c, c] = w[c, 0]
    assert np.array_equal(O.dwconv2d(x, w, s, pad), O.conv2d(x, full, s, pad))


def test_depthwise_delta_identity_and_torch():
    rng = np.random.default_rng(6)
    x = rng.standard_normal((1, 4, 6, 6)).astype(np.float32)
    w = np.zeros((4, 1, 3, 3), np.float32)
    w[:, 0, 1, 1] = 1
    assert np.array_equal(O.dwconv2d(x, w, 1, (1, 1, 1, 1)), x)
    w = rng.standard_normal((4, 1, 3, 3)).astype(np.float32)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(w).double(),
                                     padding=1, groups=4).float().numpy()
    np.testing.assert_allclose(O.dwconv2d(x, w, 1, (1, 1, 1, 1)), ref, rtol=0, atol=1e-6)


# ---------------------------------------------------------------- pooling

def test_pool_hand_worked(golden):
    g = golden("pool_4x4.txt")
    x = np.array(g["x"], np.float32).reshape(1, 1, 4, 4)
    assert O.pool2d(x, (2, 2), 2, mode="max").ravel().tolist() == g["max"]
    assert O.pool2d(x, (2, 2), 2, mode="avg").ravel().tolist() == g["avg"]
    m3 = O.pool2d(x, (3, 3), 1, (1, 1, 1, 1), "max")
    assert m3.shape == (1, 1, 4, 4) and m3[0, 0, 0].tolist() == g["max3_row0"]
    a3 = O.pool2d(x, (3, 3), 1, (1, 1, 1, 1), "avg")
    assert a3[0, 0, 0, :2].tolist() == [np.float32(v) for v in g["avg3_00_01"]]


def test_pool_special_cases():
    rng = np.random.default_rng(7)
    x = rng.standard_normal((2, 3, 9, 8)).astype(np.float32)
    assert np.array_equal(O.pool2d(x, (1, 1), 1, mode="max"), x)
    assert np.array_equal(O.pool2d(x, (1, 1), 1, mode="avg"), x)
    c = np.full((1, 2, 6, 6), 0.3, np.float32)
    assert np.array_equal(O.pool2d(c, (3, 3), 2, mode="avg"), np.full((1, 2, 2, 2), 0.3, np.float32))
    ga = O.pool2d(x, (9, 8), 1, mode="avg")
    assert ga.shape == (2, 3, 1, 1)
    assert np.array_equal(ga[:, :, 0, 0], x.astype(np.float64).mean(axis=(2, 3)).astype(np.float32))
    gm = O.pool2d(x, (9, 8), 1, mode="max")
    assert np.array_equal(gm[:, :, 0, 0], x.max(axis=(2, 3)))
    assert O.pool2d(np.zeros((1, 1, 56, 56), np.float32), (3, 3), 2).shape == (1, 1, 27, 27)
    ref = torch.nn.functional.max_pool2d(torch.from_numpy(x), 3, 2).numpy()
    assert np.array_equal(O.pool2d(x, (3, 3), 2, mode="max"), ref)


def test_maxpool_ties_and_nan():
    # first-seen wins ties between +0 and -0 (row-major taps); NaN is never selected
    x = np.array([-0.0, 0.0, 0.0, -0.0], np.float32).reshape(1, 1, 2, 2)
    y = O.pool2d(x, (2, 2), 1)
    assert y[0, 0, 0, 0] == 0 and np.signbit(y[0, 0, 0, 0])
    x = np.array([np.nan, -3.0, np.nan, -5.0], np.float32).reshape(1, 1, 2, 2)
    assert O.pool2d(x, (2, 2), 1)[0, 0, 0, 0] == -3.0


# ---------------------------------------------------------------- single element

def test_relu():
    v = np.array([-np.inf, -2.5, -0.0, 0.0, 1e-45, 3.0, np.inf, np.nan], np.float32)
    y = O.relu(v)
    exp = np.array([0, 0, 0, 0, 1e-45, 3.0, np.inf, 0], np.float32)
    assert np.array_equal(y, exp) and not np.signbit(y[:4]).any() and not np.signbit(y[7])
    rng = np.random.default_rng(8)
    x = rng.standard_normal(1000).astype(np.float32)
    assert np.array_equal(O.relu(x), np.maximum(x, 0))       # Table 2: ReLU's reduction is Max
    assert np.array_equal(O.relu(O.relu(x)), O.relu(x))


def test_add():
    rng = np.random.default_rng(9)
    a = rng.standard_normal(999).astype(np.float32)
    b = rng.standard_normal(999).astype(np.float32)
    assert np.array_equal(O.add(a, b), a + b)


# ---------------------------------------------------------------- dense

def test_dense_is_gemv_and_1x1_conv_and_full_window_conv():
    rng = np.random.default_rng(10)
    x = rng.standard_normal((5, 64, 1, 1)).astype(np.float32)
    w = rng.standard_normal((10, 64, 1, 1)).astype(np.float32)
    y = O.dense(x, w)
    gemv = (x.reshape(5, 64).astype(np.float64) @ w.reshape(10, 64).astype(np.float64).T).astype(np.float32)
    np.testing.assert_allclose(y.reshape(5, 10), gemv, rtol=0, atol=2e-6)
    assert np.array_equal(y, O.conv2d(x, w))                      # "very similar to a 1x1 convolution"
    # Table 1 row 5: F_H = I_H, F_W = I_W, F_C = I_C
    x = rng.standard_normal((2, 3, 4, 5)).astype(np.float32)
    w = rng.standard_normal((7, 3, 4, 5)).astype(np.float32)
    np.testing.assert_allclose(O.dense(x, w), O.conv2d(x, w), rtol=0, atol=2e-6)
