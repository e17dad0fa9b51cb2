"""Pins of the quantized (uint8) oracle against things other than itself (CPU only)."""
from fractions import Fraction
import math

import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workloads as WL
from oracle import oracle as O
from oracle import oracle_u8 as Q


def _rng(k):
    return np.random.default_rng(1000 + k)


CONV_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad, zx, zw
    (2, 16, 16, 7, 9, 3, 3, 1, (1, 1, 1, 1), 128, 128),
    (1, 3, 8, 8, 8, 3, 3, 2, (0, 1, 0, 1), 0, 255),
    (2, 32, 16, 5, 6, 1, 1, 1, (0, 0, 0, 0), 255, 0),
    (1, 16, 32, 9, 4, 3, 2, 2, (1, 0, 2, 1), 17, 201),
    (3, 1, 4, 11, 5, 10, 4, 2, (4, 5, 1, 1), 3, 130),
    (1, 48, 16, 4, 4, 4, 4, 1, (0, 0, 0, 0), 100, 100),      # dense: window = image
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_accumulators_match_a_library_convolution_of_the_shifted_tensors(case):
    """sum over in-image taps of (x - zx)(w - zw) == zero-padded convolution of (x - zx) with (w - zw);
    every value is an integer below 2^53, so the fp64 library result is exact."""
    N, Ci, Co, H, W, kh, kw, s, pad, zx, zw = case
    r = _rng(1)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    acc = Q.conv2d_acc(x, w, s, pad, zx, zw)
    t, b, l, rr = pad
    xs = F.pad(torch.from_numpy(x.astype(np.float64)) - zx, (l, rr, t, b))
    ref = F.conv2d(xs, torch.from_numpy(w.astype(np.float64)) - zw, stride=s).numpy()
    assert acc.shape == ref.shape and acc.dtype == np.int32
    assert np.array_equal(acc.astype(np.float64), ref)
    assert np.abs(acc).max() > 1000


@pytest.mark.parametrize("case", [(2, 16, 9, 7, 3, 3, 1, (1, 1, 1, 1), 128, 128), (1, 8, 6, 6, 3, 3, 2, (0, 1, 0, 1), 0, 255),
                                  (2, 32, 5, 5, 5, 2, 1, (2, 2, 0, 1), 77, 3)])
def test_depthwise_accumulators_match_a_library_grouped_convolution(case):
    N, Cc, H, W, kh, kw, s, pad, zx, zw = case
    r = _rng(2)
    x, w = WL.u8_codes(r, (N, Cc, H, W)), WL.u8_codes(r, (Cc, 1, kh, kw))
    acc = Q.dwconv2d_acc(x, w, s, pad, zx, zw)
    t, b, l, rr = pad
    xs = F.pad(torch.from_numpy(x.astype(np.float64)) - zx, (l, rr, t, b))
    ref = F.conv2d(xs, torch.from_numpy(w.astype(np.float64)) - zw, stride=s, groups=Cc).numpy()
    assert np.array_equal(acc.astype(np.float64), ref)
    # and it is the block-diagonal case of the full convolution
    wf = np.full((Cc, Cc, kh, kw), zw, np.uint8)
    for c in range(Cc):
        wf[c, c] = w[c, 0]
    assert np.array_equal(acc, Q.conv2d_acc(x, wf, s, pad, zx, zw))


def test_requantization_hand_worked_values():
    """Worked by hand from y = clamp(zy + floor(acc * mult / 2^shift + 1/2), lo, hi)."""
    q = lambda acc, **k: int(Q.requant(np.array([acc], np.int32), Q.Quant(**k))[0])
    # mult / 2^shift = 1/2: 1 -> 0.5 -> 1, -1 -> -0.5 -> 0, -3 -> -1.5 -> -1, 3 -> 1.5 -> 2 (ties go up)
    assert [q(a, zy=10, mult=1, shift=1) for a in (1, -1, -3, 3, 0)] == [11, 10, 9, 12, 10]
    # 3/8: 5 -> 1.875 -> 2; -5 -> -1.875 -> -2; 4 -> 1.5 -> 2; -4 -> -1.5 -> -1
    assert [q(a, zy=100, mult=3, shift=3) for a in (5, -5, 4, -4)] == [102, 98, 102, 99]
    # shift 0: plain product; clamps; ReLU as lo = zy
    assert q(7, zy=1, mult=3, shift=0) == 22 and q(-7, zy=1, mult=3, shift=0) == 0
    assert q(1 << 30, zy=0, mult=(1 << 31) - 1, shift=31) == 255
    assert q(-50, zy=128, mult=1, shift=0, lo=128) == 128 and q(50, zy=128, mult=1, shift=0, lo=128, hi=160) == 160
    # the largest product: |acc| < 2^31, mult < 2^31 -> below 2^62, no overflow
    assert q(-(1 << 31) + 1, zy=255, mult=(1 << 31) - 1, shift=31) == 0


def test_requantization_is_exact_rational_rounding():
    r = _rng(3)
    acc = r.integers(-(1 << 31) + 1, 1 << 31, size=4000, dtype=np.int64).astype(np.int32)
    acc[:200] = r.integers(-300, 300, size=200)
    for mult, shift, zy in ((1, 1, 128), (3, 3, 0), (1518500250, 31, 7), (77, 0, 255), ((1 << 31) - 1, 31, 128), (12345, 20, 64)):
        got = Q.requant(acc, Q.Quant(zy=zy, mult=mult, shift=shift))
        for a, g in zip(acc[:600].tolist(), got[:600].tolist()):
            exact = math.floor(Fraction(a * mult, 1 << shift) + Fraction(1, 2))
            assert g == min(max(exact + zy, 0), 255), (a, mult, shift, zy)
    # multiplier one: the code is the accumulator moved by the zero point
    small = np.arange(-128, 128, dtype=np.int32)
    for sh in (0, 1, 13, 30):
        assert np.array_equal(Q.requant(small, Q.Quant(zy=128, mult=1 << sh, shift=sh)), (small + 128).astype(np.uint8))
    # monotone in the accumulator
    srt = np.sort(acc)
    y = Q.requant(srt, Q.Quant(zy=128, mult=40000, shift=31)).astype(int)
    assert (np.diff(y) >= 0).all() and y.min() == 0 and y.max() == 255


def test_quantized_convolution_tracks_the_real_valued_one():
    """The whole chain against real arithmetic: with real = scale * (code - zero point) the quantized output
    is the real convolution, rounded to the output grid, to within half a step (plus the multiplier's
    own rounding)."""
    r = _rng(4)
    N, Ci, Co, H, W = 2, 16, 16, 6, 6
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, 3, 3))
    sx, sw, sy, zx, zw, zy = 0.02, 0.005, 0.05, 120, 131, 100
    shift = 31
    mult = int(round(sx * sw / sy * (1 << shift)))
    y = Q.conv2d(x, w, 1, (1, 1, 1, 1), Q.Quant(zx=zx, zw=zw, zy=zy, mult=mult, shift=shift))
    real = O.conv2d(sx * (x.astype(np.float32) - zx), sw * (w.astype(np.float32) - zw), 1, (1, 1, 1, 1)).astype(np.float64)
    inside = (y > 0) & (y < 255)
    assert inside.mean() > 0.5
    err = np.abs(sy * (y.astype(np.float64) - zy) - real)[inside]
    assert err.max() <= 0.5 * sy * 1.001 + 1e-4


def test_pooling_and_relu_on_codes_match_the_float_oracle():
    r = _rng(5)
    x = WL.u8_codes(r, (2, 16, 9, 7))
    for k, s, pad in (((3, 3), 2, (0, 0, 0, 0)), ((2, 2), 2, (0, 1, 0, 1)), ((3, 3), 1, (1, 1, 1, 1)), ((9, 7), 1, (0, 0, 0, 0))):
        mx = O.pool2d(x.astype(np.float32), k, s, pad, "max")
        assert np.array_equal(Q.pool2d(x, k, s, pad, "max").astype(np.float32), mx)
        # the mean of n <= 63 codes is never within 1e-3 of a half unless it is exactly one: floor(mean + 1/2) is safe in fp64
        av = O.pool2d(x.astype(np.float32), k, s, pad, "avg").astype(np.float64)
        assert np.array_equal(Q.pool2d(x, k, s, pad, "avg").astype(np.float64), np.floor(av + 0.5))
    for z in (0, 77, 128, 255):
        assert np.array_equal(Q.relu(x, z), np.maximum(x, z))
    # two-tap mean with a tie: (3 + 4) / 2 = 3.5 -> 4
    assert Q.pool2d(np.array([[[[3, 4]]]], np.uint8), (1, 2), 1, (0, 0, 0, 0), "avg")[0, 0, 0, 0] == 4


def test_layouts_follow_the_layout_statement():
    """Activations [N][C/Cb][H][W][Cb]; filters [Co/Cob][Ci/Cib][kh][kw][Cob][Cib] (input channel fastest)."""
    r = _rng(6)
    x = WL.u8_codes(r, (2, 32, 3, 5))
    blk = Q.pack(x, 16)
    assert np.array_equal(blk.reshape(2, 2, 3, 5, 16), x.reshape(2, 2, 16, 3, 5).transpose(0, 1, 3, 4, 2))
    assert np.array_equal(Q.unpack(blk, x.shape, 16), x)
    x3 = WL.u8_codes(r, (1, 3, 4, 4))
    assert np.array_equal(Q.pack(x3, 3).reshape(4, 4, 3), x3[0].transpose(1, 2, 0))
    w = WL.u8_codes(r, (32, 48, 3, 2))
    wb = Q.pack_filter(w, 16, 16).reshape(2, 3, 3, 2, 16, 16)
    for co, ci, ky, kx in ((0, 0, 0, 0), (17, 40, 2, 1), (31, 47, 1, 0), (5, 16, 0, 1)):
        assert wb[co // 16, ci // 16, ky, kx, co % 16, ci % 16] == w[co, ci, ky, kx]
    assert np.array_equal(wb, w.reshape(2, 16, 3, 16, 3, 2).transpose(0, 2, 4, 5, 1, 3))
    # depthwise filters: the closed-form offset of channel c, tap (y, x) in [C/Cb][kh][kw][Cb], on codes that count
    # their own plain position (c * kh + y) * kw + x (mod 251, a prime: neighbouring offsets never share a code by
    # accident), for a square and a non-square window and two block sizes
    for C, kh, kw, Cb in ((32, 3, 3, 16), (48, 2, 5, 16), (24, 3, 1, 8)):
        plain = (np.arange(C * kh * kw) % 251).astype(np.uint8).reshape(C, 1, kh, kw)
        blk = Q.pack_dw_filter(plain, Cb)
        assert blk.shape == (C * kh * kw,)
        for c in range(C):
            for y in range(kh):
                for x in range(kw):
                    off = ((c // Cb * kh + y) * kw + x) * Cb + c % Cb
                    assert blk[off] == ((c * kh + y) * kw + x) % 251, (C, kh, kw, Cb, c, y, x)
    # and the general filter layout with one input channel per filter (F_Cb = 1, G_b = Cb) is the same bytes
    wd = WL.u8_codes(r, (32, 1, 3, 3))
    assert np.array_equal(Q.pack_dw_filter(wd, 16), Q.pack_filter(wd, 16, 1))


def test_multiplier_recipe_spreads_outputs_over_the_code_range():
    r = _rng(7)
    x, w = WL.u8_codes(r, (2, 32, 8, 8)), WL.u8_codes(r, (16, 32, 3, 3))
    mult, shift = WL.u8_multiplier(32 * 9)
    y = Q.conv2d(x, w, 1, (1, 1, 1, 1), Q.Quant(mult=mult, shift=shift))
    assert 20 < y.std() < 70 and (y == 0).mean() < 0.05 and (y == 255).mean() < 0.05


# ------------------------------------------------------------------ addition with two input scales, layer chains

ADD_PARAMS = [  # za, zb, zy, mult_a, mult_b, shift, lo, hi
    (128, 128, 128, 3 << 28, 1 << 29, 30, 0, 255),
    (0, 255, 17, (1 << 31) - 1, 1, 31, 0, 255),
    (200, 3, 100, 12345, 67890, 7, 10, 240),
    (5, 9, 0, 7, 3, 0, 0, 255),                       # shift 0: no rounding term
    (128, 128, 128, 0, 1 << 20, 20, 128, 255),        # one input switched off, ReLU bound
    (255, 0, 255, 1 << 30, 1 << 30, 31, 0, 255),
]


@pytest.mark.parametrize("params", ADD_PARAMS)
def test_add_equals_exact_integer_arithmetic_on_every_pair_of_codes(params):
    """All 65536 (a, b) pairs against floor((acc + half) / 2^shift) in numpy int64 (floor_divide rounds towards
    minus infinity, the sums stay below 2^41) -- written here from the rule, not through the oracle's C code."""
    za, zb, zy, ma, mb, sh, lo, hi = params
    a, b = np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")
    got = Q.add(a, b, Q.QuantAdd(za, zb, zy, ma, mb, sh, lo, hi))
    acc = (a.astype(np.int64) - za) * ma + (b.astype(np.int64) - zb) * mb
    half = (1 << (sh - 1)) if sh > 0 else 0
    ref = np.clip(zy + np.floor_divide(acc + half, 1 << sh), lo, hi)
    assert np.array_equal(got.astype(np.int64), ref)
    # and a handful of pairs in exact rational arithmetic
    for ai, bi in [(0, 0), (255, 255), (za, zb), (1, 254), (77, 200)]:
        v = Fraction((ai - za) * ma + (bi - zb) * mb, 1 << sh)
        r = math.floor(v + Fraction(1, 2)) if sh > 0 else int(v)
        assert got[ai, bi] == min(max(zy + r, lo), hi)


def test_add_with_unit_scales_is_plain_saturating_addition_and_commutes():
    r = _rng(31)
    a, b = WL.u8_codes(r, (3, 16, 5, 7)), WL.u8_codes(r, (3, 16, 5, 7))
    q = Q.QuantAdd(0, 0, 0, 1 << 12, 1 << 12, 12, 0, 255)
    assert np.array_equal(Q.add(a, b, q), np.minimum(a.astype(np.int32) + b, 255).astype(np.uint8))
    q1 = Q.QuantAdd(10, 20, 30, 12345, 54321, 16, 0, 255)
    q2 = Q.QuantAdd(20, 10, 30, 54321, 12345, 16, 0, 255)
    assert np.array_equal(Q.add(a, b, q1), Q.add(b, a, q2))


def test_add_is_within_half_a_step_of_the_real_valued_sum():
    """Codes stand for scale * (code - zero point); with multipliers mult / 2^shift = scale_in / scale_out the result
    is the nearest code of the real sum wherever it is not clamped."""
    r = _rng(32)
    a, b = WL.u8_codes(r, (4096,)), WL.u8_codes(r, (4096,))
    sa, sb, sy, sh = 0.031, 0.012, 0.05, 24
    q = Q.QuantAdd(120, 131, 128, int(round(sa / sy * (1 << sh))), int(round(sb / sy * (1 << sh))), sh, 0, 255)
    y = Q.add(a, b, q).astype(np.float64)
    real = sa * (a.astype(np.float64) - 120) + sb * (b.astype(np.float64) - 131)
    free = (y > 0) & (y < 255)
    assert free.sum() > 2000
    assert np.all(np.abs(sy * (y[free] - 128) - real[free]) <= sy * (0.5 + 1e-4))


def _small_residual_table():
    """conv -> relu -> conv -> add(skip) -> relu -> maxpool -> avgpool -> dense on small tensors: every op of the
    quantized path, a second operand from an older buffer, buffers reused."""
    from workloads.nets import Layer, Network, IN, OUT
    net = Network("u8_chain", 16, 6, 6)
    net.wshapes = [((16, 16, 3, 3), 144), ((16, 1, 3, 3), 9), ((16, 16, 1, 1), 16), ((4, 16, 1, 1), 16)]
    p1, z = (1, 1, 1, 1), (0, 0, 0, 0)
    net.layers = [
        Layer("conv", 16, 16, 6, 6, 3, 3, 1, p1, src=IN, dst=0, w=0),
        Layer("relu", 16, 16, 6, 6, src=0, dst=0),
        Layer("dw", 16, 16, 6, 6, 3, 3, 1, p1, src=0, dst=1, w=1),
        Layer("conv", 16, 16, 6, 6, 1, 1, 1, z, src=1, dst=2, w=2),
        Layer("add", 16, 16, 6, 6, src=2, src2=0, dst=2),
        Layer("relu", 16, 16, 6, 6, src=2, dst=2),
        Layer("maxpool", 16, 16, 6, 6, 2, 2, 2, z, src=2, dst=1),
        Layer("avgpool", 16, 16, 3, 3, 3, 3, 1, z, src=1, dst=0),
        Layer("dense", 16, 4, 1, 1, 1, 1, 1, z, src=0, dst=OUT, w=3),
    ]
    return net


def test_run_network_is_the_composition_of_its_layers():
    net = _small_residual_table()
    x, ws, qs = WL.quantized_network_tensors(net, 3, 777)
    taps = {}
    out = Q.run_network(net, x, ws, qs, taps=taps)
    a = Q.relu(Q.conv2d(x, ws[0], 1, (1, 1, 1, 1), Q.Quant(**qs[0])), 128)
    b = Q.conv2d(Q.dwconv2d(a, ws[1], 1, (1, 1, 1, 1), Q.Quant(**qs[2])), ws[2], 1, (0, 0, 0, 0), Q.Quant(**qs[3]))
    c = Q.relu(Q.add(b, a, Q.QuantAdd(**qs[4])), 128)
    d = Q.pool2d(Q.pool2d(c, (2, 2), 2, mode="max"), (3, 3), 1, mode="avg")
    ref = Q.dense(d, ws[3], Q.Quant(**qs[8]))
    assert out.shape == (3, 4, 1, 1) and np.array_equal(out, ref)
    assert np.array_equal(taps[1], a) and np.array_equal(taps[5], c) and np.array_equal(taps[7], d)
    assert np.array_equal(Q.run_network(net, x, ws, qs, upto=4), Q.add(b, a, Q.QuantAdd(**qs[4])))
    assert len(np.unique(out)) > 4                      # the parameters of the recipe spread the codes


def test_run_network_with_unit_scales_is_the_float_oracle_on_integers():
    """With every multiplier 2^shift (scale 1), weights in {-1, 0, 1} around their zero point and inputs small enough
    that nothing saturates, a chain of quantized layers is exact integer arithmetic: code - zero point must equal the
    float oracle's network on the shifted tensors (all values are small integers, exact in fp32)."""
    from workloads.nets import Layer, Network, IN, OUT
    net = Network("u8_exact", 16, 5, 5)
    net.wshapes = [((16, 16, 3, 3), 144), ((16, 1, 3, 3), 9), ((16, 16, 1, 1), 16)]
    p1, z = (1, 1, 1, 1), (0, 0, 0, 0)
    net.layers = [
        Layer("conv", 16, 16, 5, 5, 3, 3, 1, p1, src=IN, dst=0, w=0),
        Layer("dw", 16, 16, 5, 5, 3, 3, 2, p1, src=0, dst=1, w=1),
        Layer("conv", 16, 16, 3, 3, 1, 1, 1, z, src=1, dst=2, w=2),
        Layer("add", 16, 16, 3, 3, src=2, src2=1, dst=OUT),
    ]
    r = _rng(41)
    x = (100 + r.integers(-1, 2, size=(2, 16, 5, 5))).astype(np.uint8)          # x - zx in {-1, 0, 1}
    ws = [(90 + r.integers(-1, 2, size=shp) * (r.random(shp) < 0.3)).astype(np.uint8) for shp, _ in net.wshapes]
    unit = dict(zw=90, mult=1 << 10, shift=10, lo=0, hi=255)
    qs = [dict(zx=100, zy=128, **unit), dict(zx=128, zy=128, **unit), dict(zx=128, zy=60, **unit),
          dict(za=60, zb=128, zy=128, mult_a=1 << 10, mult_b=1 << 10, shift=10, lo=0, hi=255)]
    taps = {}
    out = Q.run_network(net, x, ws, qs, taps=taps)
    xs, wsf = x.astype(np.float32) - 100, [w.astype(np.float32) - 90 for w in ws]
    _, trace = O.run_network(net, xs, wsf, return_all=True)
    for i, zy in enumerate([128, 128, 60, 128]):
        ref = trace[i]
        assert np.abs(ref).max() >= 3 and np.abs(ref).max() < 60, i                 # not trivial, not clamped
        assert np.array_equal(taps[i].astype(np.int32) - zy, ref.astype(np.int32)), i
    assert np.array_equal(out, taps[3])
