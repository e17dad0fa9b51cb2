"""Pins for the blocked layouts (Section 'Common Data Format') and for the
Algorithm-1 nest on them (O2 == O1 for every layer class)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O


def test_activation_offsets_closed_form():
    N, C, H, W, Cb = 2, 32, 3, 5, 16
    x = np.arange(N * C * H * W, dtype=np.float32).reshape(N, C, H, W)
    b = O.pack(x, Cb)
    # C_b fastest, then W, then H, then channel block, batch outermost
    v = b.reshape(N, C // Cb, H, W, Cb)
    assert np.array_equal(v, x.reshape(N, C // Cb, Cb, H, W).transpose(0, 1, 3, 4, 2))
    for (n, c, h, w) in [(0, 0, 0, 0), (1, 17, 2, 4), (0, 31, 1, 3), (1, 16, 0, 0)]:
        off = (((n * (C // Cb) + c // Cb) * H + h) * W + w) * Cb + c % Cb
        assert b[off] == x[n, c, h, w]
    assert np.array_equal(O.unpack(b, x.shape, Cb), x)


@pytest.mark.parametrize("C,Cb", [(3, 3), (8, 8), (1, 1), (48, 16), (12, 4)])
def test_pack_roundtrip(C, Cb):
    rng = np.random.default_rng(C)
    x = rng.standard_normal((3, C, 5, 7)).astype(np.float32)
    assert np.array_equal(O.unpack(O.pack(x, Cb), x.shape, Cb), x)
    if C == Cb:   # a single block is NHWC
        assert np.array_equal(O.pack(x, Cb), x.transpose(0, 2, 3, 1).ravel())


def test_filter_offsets_follow_loop_order():
    Co, Ci, kh, kw, Cob, Cib = 32, 48, 3, 2, 16, 16
    w = np.arange(Co * Ci * kh * kw, dtype=np.float32).reshape(Co, Ci, kh, kw)
    b = O.pack_filter(w, Cob, Cib)
    v = b.reshape(Co // Cob, Ci // Cib, kh, kw, Cib, Cob)
    exp = w.reshape(Co // Cob, Cob, Ci // Cib, Cib, kh, kw).transpose(0, 2, 4, 5, 3, 1)
    assert np.array_equal(v, exp)
    co, ci, y, x = 21, 37, 2, 1
    off = ((((co // Cob * (Ci // Cib) + ci // Cib) * kh + y) * kw + x) * Cib + ci % Cib) * Cob + co % Cob
    assert b[off] == w[co, ci, y, x]
    d = np.arange(32 * 9, dtype=np.float32).reshape(32, 1, 3, 3)
    db = O.pack_dw_filter(d, 16).reshape(2, 3, 3, 16)
    assert np.array_equal(db, d.reshape(2, 16, 3, 3).transpose(0, 2, 3, 1))


CONV = [  # N, Ci, Co, H, W, kh, kw, s, pad, Cib, Cob, O_wb
    (2, 32, 32, 7, 9, 3, 3, 1, (1, 1, 1, 1), 16, 16, 6),
    (1, 3, 16, 9, 8, 3, 3, 2, (0, 1, 0, 1), 3, 16, 4),
    (1, 1, 32, 13, 10, 10, 4, 2, (4, 5, 1, 1), 1, 16, 5),
    (2, 16, 32, 8, 8, 1, 1, 2, (0, 0, 0, 0), 16, 16, 3),
    (1, 8, 16, 5, 5, 1, 1, 1, (0, 0, 0, 0), 8, 16, 7),
    (3, 64, 10, 1, 1, 1, 1, 1, (0, 0, 0, 0), 16, 10, 1),
]


@pytest.mark.parametrize("case", CONV)
def test_blocked_nest_conv_equals_definition(case):
    N, Ci, Co, H, W, kh, kw, s, pad, Cib, Cob, Owb = case
    rng = np.random.default_rng(21)
    x = rng.standard_normal((N, Ci, H, W)).astype(np.float32)
    w = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
    yb, (OC, OH, OW) = O.conv2d_blocked(O.pack(x, Cib), O.pack_filter(w, Cob, Cib), N, Ci, Co, H, W,
                                        kh, kw, s, pad, Cib, Cob, Owb)
    ref = O.conv2d(x, w, s, pad)
    assert (N, OC, OH, OW) == ref.shape
    got = O.unpack(yb, ref.shape, Cob)
    # same exact products, fp64 sums in a different order, one rounding: at most 1 ulp apart
    assert np.all(np.abs(got - ref) <= np.spacing(np.abs(ref)))


@pytest.mark.parametrize("C,Cb,s,pad,Owb", [(32, 16, 1, (1, 1, 1, 1), 6), (8, 8, 2, (0, 1, 0, 1), 4),
                                             (48, 16, 2, (1, 1, 1, 1), 5)])
def test_blocked_nest_depthwise_and_pool(C, Cb, s, pad, Owb):
    rng = np.random.default_rng(22)
    N, H, W = 2, 9, 7
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((C, 1, 3, 3)).astype(np.float32)
    yb, shp = O.dwconv2d_blocked(O.pack(x, Cb), O.pack_dw_filter(w, Cb), N, C, H, W, 3, 3, s, pad, Cb, Owb)
    ref = O.dwconv2d(x, w, s, pad)
    assert (N,) + shp == ref.shape
    got = O.unpack(yb, ref.shape, Cb)
    assert np.all(np.abs(got - ref) <= np.spacing(np.abs(ref)))
    for mode in ("max", "avg"):
        yb, shp = O.pool2d_blocked(O.pack(x, Cb), N, C, H, W, 3, 3, s, pad, Cb, mode, Owb)
        ref = O.pool2d(x, (3, 3), s, pad, mode)
        got = O.unpack(yb, ref.shape, Cb)
        if mode == "max":
            assert np.array_equal(got, ref)
        else:
            assert np.all(np.abs(got - ref) <= np.spacing(np.abs(ref)))


def test_fig1_group_shape_and_group_conv(golden):
    """Figure 1: G = 2 overlapping groups (S_C < F_C) of K = 3 filters over F_C = 4 channels,
    9 taps each, give O_C = 6. Disjoint groups (S_C = F_C) equal a library grouped conv."""
    G, K, OC, FC, taps = (int(v) for v in golden("paper_constants.txt")["fig1_G_K_OC_FC_taps"])
    I_C, S_C = 6, 2                      # (6 - 4)/2 + 1 = 2 groups
    assert (I_C - FC) // S_C + 1 == G and K * G == OC and taps == 9
    rng = np.random.default_rng(23)
    x = rng.standard_normal((1, I_C, 5, 5)).astype(np.float32)
    wt = rng.standard_normal((G, K, FC, 3, 3)).astype(np.float32)
    # weight layout [G/G_b][K/K_b][F_C/F_Cb][F_H][F_W][F_Cb][G_b][K_b] with G_b = 1, K_b = 3, F_Cb = 2
    wb = wt.reshape(G, 1, K, 2, 2, 3, 3).transpose(0, 1, 3, 5, 6, 4, 2).reshape(-1)
    wb = np.ascontiguousarray(wb)
    yb, (oc, oh, ow) = O.abstract_layer_blocked("fma", O.pack(x, 2), wb, 1, I_C, 5, 5, 3, 3, FC, 1, 1, S_C, K,
                                                (1, 1, 1, 1), 2, 1, 3, 2, 4)
    assert (oc, oh, ow) == (OC, 5, 5)
    got = O.unpack(yb, (1, OC, 5, 5), 3)
    for g in range(G):
        ref = O.conv2d(x[:, g * S_C:g * S_C + FC], wt[g], 1, (1, 1, 1, 1))
        assert np.all(np.abs(got[:, g * K:(g + 1) * K] - ref) <= np.spacing(np.abs(ref)))
    # disjoint groups against torch
    x = rng.standard_normal((1, 8, 5, 5)).astype(np.float32)
    wt = rng.standard_normal((2, 3, 4, 3, 3)).astype(np.float32)
    wb = np.ascontiguousarray(wt.reshape(2, 1, 3, 1, 4, 3, 3).transpose(0, 1, 3, 5, 6, 4, 2).reshape(-1))
    yb, _ = O.abstract_layer_blocked("fma", O.pack(x, 4), wb, 1, 8, 5, 5, 3, 3, 4, 1, 1, 4, 3,
                                     (1, 1, 1, 1), 4, 1, 3, 4, 5)
    ref = torch.nn.functional.conv2d(torch.from_numpy(x).double(), torch.from_numpy(wt.reshape(6, 4, 3, 3)).double(),
                                     padding=1, groups=2).float().numpy()
    np.testing.assert_allclose(O.unpack(yb, (1, 6, 5, 5), 3), ref, rtol=0, atol=1e-5)
