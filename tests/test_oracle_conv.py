"""Pins for the oracle's convolution (definitional O1), CPU only.

Each test checks the oracle against something other than itself: hand-worked
fixtures, closed forms, an independently written sliding-window evaluation, a
library GEMM, and PyTorch's CPU convolution as a third opinion.
"""
import numpy as np
import pytest
import torch

from oracle import oracle as O


def _pad_and_slide(x, w, s, pad):
    """Independent evaluation: materialise the zero-padded input, then take the
    windows as array slices and contract with einsum in fp64."""
    t, b, l, r = pad
    xp = np.pad(x.astype(np.float64), ((0, 0), (0, 0), (t, b), (l, r)))
    N, Ci, Hp, Wp = xp.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = (Hp - kh) // s + 1, (Wp - kw) // s + 1
    y = np.zeros((N, Co, Ho, Wo))
    for oh in range(Ho):
        for ow in range(Wo):
            win = xp[:, :, oh * s:oh * s + kh, ow * s:ow * s + kw]
            y[:, :, oh, ow] = np.einsum("nchw,ochw->no", win, w.astype(np.float64))
    return y.astype(np.float32)


def test_hand_worked(golden):
    g = golden("conv_tiny.txt")
    x = np.array(g["a_x"], np.float32).reshape(1, 1, 3, 3)
    w = np.array(g["a_w"], np.float32).reshape(1, 1, 2, 2)
    assert O.conv2d(x, w).ravel().tolist() == g["a_y"]
    assert O.conv2d(x, w, stride=2, pad=(1, 0, 1, 0)).ravel().tolist() == g["c_y"]
    xb = np.array(g["b_x"], np.float32).reshape(1, 2, 2, 2)
    wb = np.array(g["b_w"], np.float32).reshape(2, 2, 1, 1)
    assert O.conv2d(xb, wb).ravel().tolist() == g["b_y"]


def test_output_size_equation():
    # Section 3.1.2: O = (I - F)/S + 1, extended by padding and floor
    assert O.out_dim(32, 3, 1, 1, 1) == 32
    assert O.out_dim(56, 3, 2, 0, 0) == 27
    assert O.out_dim(49, 10, 2, 4, 5) == 25
    assert O.out_dim(10, 4, 2, 1, 1) == 5
    assert O.out_dim(7, 7, 1, 0, 0) == 1
    assert O.out_dim(2, 3, 1, 0, 0) == 0


@pytest.mark.parametrize("dy,dx", [(0, 0), (1, 1), (2, 0), (0, 2), (1, 2)])
def test_delta_filter_is_a_shift(dy, dx):
    """A filter that is 1 at tap (dy, dx) and pad 1 copies the input shifted by
    (dy-1, dx-1) with a zero border: pins tap orientation (no flip) and pad sides."""
    rng = np.random.default_rng(1)
    x = rng.standard_normal((2, 3, 5, 6)).astype(np.float32)
    w = np.zeros((3, 3, 3, 3), np.float32)
    for c in range(3):
        w[c, c, dy, dx] = 1.0
    y = O.conv2d(x, w, 1, (1, 1, 1, 1))
    exp = np.zeros_like(x)
    H, W = 5, 6
    for h in range(H):
        for ww in range(W):
            ih, iw = h + dy - 1, ww + dx - 1
            if 0 <= ih < H and 0 <= iw < W:
                exp[:, :, h, ww] = x[:, :, ih, iw]
    assert np.array_equal(y, exp)


def test_all_ones_counts_in_range_taps():
    Ci, H, W = 5, 6, 7
    x = np.ones((1, Ci, H, W), np.float32)
    w = np.ones((2, Ci, 3, 3), np.float32)
    y = O.conv2d(x, w, 1, (1, 1, 1, 1))
    rows = np.array([2] + [3] * (H - 2) + [2])
    cols = np.array([2] + [3] * (W - 2) + [2])
    exp = Ci * np.outer(rows, cols)
    assert np.array_equal(y[0, 0], exp) and np.array_equal(y[0, 1], exp)
    # asymmetric padding: only top/left padded
    y2 = O.conv2d(x, w, 1, (2, 0, 1, 0))
    assert y2.shape == (1, 2, H, W - 1)
    assert y2[0, 0, 0, 0] == Ci * 1 * 2 and y2[0, 0, 1, 0] == Ci * 2 * 2 and y2[0, 0, 2, 1] == Ci * 9


def test_1x1_conv_is_a_gemm():
    """Section 3.2: a 1x1 convolution reduces all channels of one pixel."""
    rng = np.random.default_rng(2)
    x = rng.standard_normal((3, 24, 5, 4)).astype(np.float32)
    w = rng.standard_normal((10, 24, 1, 1)).astype(np.float32)
    y = O.conv2d(x, w)
    X = x.transpose(0, 2, 3, 1).reshape(-1, 24).astype(np.float64)
    G = (X @ w.reshape(10, 24).astype(np.float64).T).astype(np.float32)
    assert np.array_equal(y.transpose(0, 2, 3, 1).reshape(-1, 10), G)


@pytest.mark.parametrize("s", [2, 3])
def test_stride_subsamples_stride1(s):
    rng = np.random.default_rng(3)
    x = rng.standard_normal((1, 4, 11, 9)).astype(np.float32)
    w = rng.standard_normal((5, 4, 3, 3)).astype(np.float32)
    y1 = O.conv2d(x, w, 1, (1, 1, 1, 1))
    ys = O.conv2d(x, w, s, (1, 1, 1, 1))
    assert np.array_equal(ys, y1[:, :, ::s, ::s][:, :, :ys.shape[2], :ys.shape[3]])


def test_linearity_exact_on_integers():
    rng = np.random.default_rng(4)
    x = rng.integers(-8, 9, (2, 6, 7, 7)).astype(np.float32)
    w1 = rng.integers(-4, 5, (4, 6, 3, 3)).astype(np.float32)
    w2 = rng.integers(-4, 5, (4, 6, 3, 3)).astype(np.float32)
    p = (1, 1, 1, 1)
    assert np.array_equal(O.conv2d(x, w1 + w2, 1, p), O.conv2d(x, w1, 1, p) + O.conv2d(x, w2, 1, p))


CASES = [  # N, Ci, Co, H, W, kh, kw, s, pad
    (1, 1, 1, 3, 3, 2, 2, 1, (0, 0, 0, 0)),
    (2, 3, 4, 6, 5, 3, 3, 1, (1, 1, 1, 1)),
    (1, 3, 8, 9, 9, 3, 3, 2, (0, 1, 0, 1)),
    (2, 1, 6, 13, 10, 10, 4, 2, (4, 5, 1, 1)),
    (1, 16, 16, 8, 8, 1, 1, 2, (0, 0, 0, 0)),
    (1, 5, 2, 7, 4, 2, 3, 3, (1, 0, 2, 1)),
]


@pytest.mark.parametrize("case", CASES)
def test_against_independent_sliding_window(case):
    N, Ci, Co, H, W, kh, kw, s, pad = case
    rng = np.random.default_rng(hash(case) % 2**31)
    x = rng.standard_normal((N, Ci, H, W)).astype(np.float32)
    w = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    y = O.conv2d(x, w, s, pad)
    ref = _pad_and_slide(x, w, s, pad)
    assert y.shape == ref.shape
    # both are fp64-accumulated and rounded once; summation order differs
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-6 * (np.abs(ref).max() + 1))


@pytest.mark.parametrize("case", CASES)
def test_third_opinion_torch_cpu(case):
    N, Ci, Co, H, W, kh, kw, s, pad = case
    rng = np.random.default_rng(11)
    x = rng.standard_normal((N, Ci, H, W)).astype(np.float32)
    w = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    t, b, l, r = pad
    xp = torch.nn.functional.pad(torch.from_numpy(x).double(), (l, r, t, b))
    ref = torch.nn.functional.conv2d(xp, torch.from_numpy(w).double(), stride=s).float().numpy()
    y = O.conv2d(x, w, s, pad)
    np.testing.assert_allclose(y, ref, rtol=0, atol=1e-6 * (np.abs(ref).max() + 1))
