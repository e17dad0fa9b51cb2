"""GPU parity of the quantized (uint8) layers against the integer oracle, through the C ABI: bit-exact."""
import numpy as np
import pytest
import torch

import paper_2303_04769_amd as S
import workloads as WL
from oracle import oracle_u8 as Q
from gpu_util import DEV, Guarded8, dev8

pytestmark = pytest.mark.gpu


def _rng(k):
    return np.random.default_rng(WL.BASE_SEED + 100 + k)


def _quant(K, zx, zw, zy=128, relu=False, **kw):
    mult, shift = WL.u8_multiplier(K)
    q = Q.Quant(zx=zx, zw=zw, zy=zy, mult=mult, shift=shift, lo=zy if relu else 0, hi=255)
    for k, v in kw.items():
        setattr(q, k, v)
    return q


def _quant_for(acc, zx, zw, relu=False):
    """Multiplier and output zero point that keep the codes of these accumulators (the oracle's) off the clamps."""
    mean, std = float(acc.mean()), float(acc.std()) + 1.0
    m = min(40.0 / std, 100.0 / (abs(mean) + 1.0))
    zy = int(min(max(round(128 - mean * m), 0), 255))
    mult = min(max(int(round(m * (1 << 31))), 1), (1 << 31) - 1)
    # relu: a lower clamp in the middle of the code distribution (the mean maps to about 128), so that about
    # half of the outputs sit on it
    return Q.Quant(zx=zx, zw=zw, zy=zy, mult=mult, shift=31, lo=min(zy, 128) if relu else 0, hi=255)


def _same(got, ref, what):
    assert got.shape == ref.shape, (got.shape, ref.shape)
    bad = np.argwhere(got != ref)
    assert bad.size == 0, f"{what}: {len(bad)} of {got.size} codes differ, first at {bad[0]}: gpu {got[tuple(bad[0])]} ref {ref[tuple(bad[0])]}"


@pytest.mark.parametrize("shape,Cb", [((2, 32, 5, 7), 16), ((3, 3, 8, 8), 3), ((1, 8, 9, 2), 8), ((2, 48, 1, 1), 16)])
def test_pack_unpack(shape, Cb):
    x = WL.u8_codes(_rng(0), shape)
    N, C, H, W = shape
    g = Guarded8(x.size)
    S.small_pack_u8(dev8(x), g.t, N, C, H, W, Cb)
    blk = g.check()
    assert np.array_equal(blk, Q.pack(x, Cb))
    g2 = Guarded8(x.size)
    S.small_unpack_u8(dev8(blk), g2.t, N, C, H, W, Cb)
    assert np.array_equal(g2.check().reshape(shape), x)


@pytest.mark.parametrize("Co,Ci,kh,kw,Cob,Cib", [(32, 48, 3, 3, 16, 16), (8, 3, 3, 3, 8, 3), (16, 1, 10, 4, 16, 1), (16, 8, 1, 1, 16, 8)])
def test_pack_filter(Co, Ci, kh, kw, Cob, Cib):
    w = WL.u8_codes(_rng(1), (Co, Ci, kh, kw))
    g = Guarded8(w.size)
    S.small_pack_filter_u8(dev8(w), g.t, Co, Ci, kh, kw, Cob, Cib)
    assert np.array_equal(g.check(), Q.pack_filter(w, Cob, Cib))


def _conv(x, w, stride, pad, q, Cib, Cob, with_sums=False):
    """with_sums: the per-channel sums of the filter's codes come from small_filter_sums_u8 instead of being taken
    inside the convolution."""
    N, Ci, H, W = x.shape
    Co, _, kh, kw = w.shape
    Ho, Wo = Q.out_dim(H, kh, stride, pad[0], pad[1]), Q.out_dim(W, kw, stride, pad[2], pad[3])
    g = Guarded8(N * Co * Ho * Wo)
    wb = dev8(Q.pack_filter(w, Cob, Cib))
    sums = None
    if with_sums:
        sums = torch.full((Co,), -1, dtype=torch.int32, device=DEV)
        S.small_filter_sums_u8(wb, sums, Co, Ci, kh, kw, Cob, Cib)
        torch.cuda.synchronize()
        assert np.array_equal(sums.cpu().numpy(), w.reshape(Co, -1).astype(np.int64).sum(axis=1))
    S.small_conv2d_u8(dev8(Q.pack(x, Cib)), wb, g.t, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, q, sums)
    return Q.unpack(g.check(), (N, Co, Ho, Wo), Cob)


CONV_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad, zx, zw, relu
    (2, 16, 16, 7, 9, 3, 3, 1, (1, 1, 1, 1), 128, 128, False),     # no correction sums; 9 chunks: ragged last step
    (3, 32, 48, 13, 11, 3, 3, 1, (1, 1, 1, 1), 120, 131, True),    # both correction sums, 18 chunks
    (2, 64, 32, 9, 9, 3, 3, 2, (0, 1, 0, 1), 0, 255, False),       # extreme zero points, stride 2
    (5, 16, 16, 5, 5, 1, 1, 1, (0, 0, 0, 0), 255, 0, False),       # one chunk: three idle lane groups
    (1, 48, 16, 10, 6, 3, 2, 2, (1, 0, 1, 1), 17, 200, True),
    (3, 16, 16, 5, 7, 3, 3, 1, (1, 1, 1, 1), 130, 128, False),     # 105 pixels: ragged pixel tile; only the filter sum
    (2, 16, 32, 6, 6, 3, 3, 1, (1, 1, 1, 1), 128, 77, False),      # only the pixel sum
    (4, 32, 16, 4, 4, 4, 4, 1, (0, 0, 0, 0), 100, 150, False),     # window = image (dense over 4 x 4)
    (37, 128, 16, 1, 1, 1, 1, 1, (0, 0, 0, 0), 128, 128, True),    # dense on 1 x 1 images
    (2, 512, 16, 3, 3, 3, 3, 1, (1, 1, 1, 1), 3, 250, False),      # long reduction (K = 4608)
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv_matrix_core(case):
    N, Ci, Co, H, W, kh, kw, s, pad, zx, zw, relu = case
    r = _rng(2)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    q = _quant_for(Q.conv2d_acc(x, w, s, pad, zx, zw), zx, zw, relu)
    ref = Q.conv2d(x, w, s, pad, q)
    _same(_conv(x, w, s, pad, q, 16, 16), ref, f"conv u8 {case}")
    _same(_conv(x, w, s, pad, q, 16, 16, with_sums=True), ref, f"conv u8 with filter sums {case}")
    assert ref.std() > 1.5 and len(np.unique(ref)) > 8


@pytest.mark.parametrize("case", [
    (2, 3, 8, 9, 9, 3, 3, 2, (0, 1, 0, 1), 128, 128, 3, 8),        # first layer of the depthwise-separable CNN
    (2, 1, 16, 13, 10, 10, 4, 2, (4, 5, 1, 1), 5, 140, 1, 16),     # first layer of the audio CNN
    (3, 8, 16, 6, 5, 1, 1, 1, (0, 0, 0, 0), 200, 100, 8, 16),
    (2, 16, 8, 5, 5, 3, 3, 1, (1, 1, 1, 1), 128, 128, 16, 8),
    (1, 32, 32, 4, 4, 3, 3, 1, (1, 1, 1, 1), 1, 2, 32, 32),
])
def test_conv_other_blocks(case):
    N, Ci, Co, H, W, kh, kw, s, pad, zx, zw, Cib, Cob = case
    r = _rng(3)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    q = _quant_for(Q.conv2d_acc(x, w, s, pad, zx, zw), zx, zw)
    ref = Q.conv2d(x, w, s, pad, q)
    _same(_conv(x, w, s, pad, q, Cib, Cob), ref, f"conv u8 generic {case}")
    assert len(np.unique(ref)) > 8


def test_requantization_corner_parameters():
    """shift 0, the largest multiplier, clamps at both ends, ReLU ranges: same codes as the oracle."""
    r = _rng(4)
    x, w = WL.u8_codes(r, (2, 16, 6, 6)), WL.u8_codes(r, (16, 16, 3, 3))
    for kw in (dict(mult=1, shift=0), dict(mult=(1 << 31) - 1, shift=31), dict(mult=0, shift=5), dict(mult=3, shift=3, zy=0),
               dict(mult=12345, shift=20, zy=255), dict(mult=9000, shift=31, lo=100, hi=140, zy=120)):
        q = _quant(144, 128, 128, **kw)
        _same(_conv(x, w, 1, (1, 1, 1, 1), q, 16, 16), Q.conv2d(x, w, 1, (1, 1, 1, 1), q), f"requant {kw}")
    S.small_dense_u8  # exported
    xd, wd = WL.u8_codes(r, (9, 32, 1, 1)), WL.u8_codes(r, (16, 32, 1, 1))
    q = _quant(32, 99, 101)
    g = Guarded8(9 * 16)
    S.small_dense_u8(dev8(Q.pack(xd, 16)), dev8(Q.pack_filter(wd, 16, 16)), g.t, 9, 32, 16, 16, 16, q)
    _same(Q.unpack(g.check(), (9, 16, 1, 1), 16), Q.dense(xd, wd, q), "dense u8")
    # a scale too large for the 32-bit requantization path (one step of the sum is 2^20 codes): wide path
    q = _quant(144, 128, 128, mult=1 << 30, shift=10)
    _same(_conv(x, w, 1, (1, 1, 1, 1), q, 16, 16), Q.conv2d(x, w, 1, (1, 1, 1, 1), q), "requant wide path")
    q = _quant(144, 128, 128, mult=(1 << 31) - 1, shift=0, zy=7)
    _same(_conv(x, w, 1, (1, 1, 1, 1), q, 16, 16), Q.conv2d(x, w, 1, (1, 1, 1, 1), q), "requant largest scale")


def test_conv_full_size_sampled():
    """A sweep-sized layer in the launch configuration the benchmark times (64 pixels per wave); the oracle
    recomputes three images (images are independent)."""
    N, C, H = 64, 64, 56
    r = _rng(5)
    x, w = WL.u8_codes(r, (N, C, H, H)), WL.u8_codes(r, (C, C, 3, 3))
    q = _quant(C * 9, 121, 135, relu=True)
    got = _conv(x, w, 1, (1, 1, 1, 1), q, 16, 16)
    got2 = _conv(x, w, 1, (1, 1, 1, 1), q, 16, 16, with_sums=True)
    assert np.array_equal(got, got2)
    for n in (0, 31, N - 1):
        _same(got[n:n + 1], Q.conv2d(x[n:n + 1], w, 1, (1, 1, 1, 1), q), f"conv u8 64x64x56x56 image {n}")


DW_CASES = [  # N, C, H, W, kh, kw, stride, pad, Cb, zx, zw
    (2, 32, 9, 7, 3, 3, 1, (1, 1, 1, 1), 16, 128, 128),
    (3, 16, 12, 12, 3, 3, 2, (0, 1, 0, 1), 16, 7, 250),
    (2, 8, 6, 6, 3, 3, 1, (1, 1, 1, 1), 8, 100, 60),
    (2, 3, 5, 5, 3, 3, 1, (1, 1, 1, 1), 3, 128, 128),             # one lane per code
    (1, 64, 25, 5, 3, 3, 1, (1, 1, 1, 1), 16, 130, 120),
    (2, 16, 7, 7, 5, 2, 2, (2, 2, 0, 1), 16, 0, 0),
]


@pytest.mark.parametrize("case", DW_CASES)
def test_depthwise(case):
    N, C, H, W, kh, kw, s, pad, Cb, zx, zw = case
    r = _rng(6)
    x, w = WL.u8_codes(r, (N, C, H, W)), WL.u8_codes(r, (C, 1, kh, kw))
    q = _quant_for(Q.dwconv2d_acc(x, w, s, pad, zx, zw), zx, zw, relu=True)
    ref = Q.dwconv2d(x, w, s, pad, q)
    assert len(np.unique(ref)) > 8
    g = Guarded8(ref.size)
    S.small_dwconv2d_u8(dev8(Q.pack(x, Cb)), dev8(Q.pack_dw_filter(w, Cb)), g.t, N, C, H, W, kh, kw, s, pad, Cb, q)
    _same(Q.unpack(g.check(), ref.shape, Cb), ref, f"dw u8 {case}")


@pytest.mark.parametrize("case", [(2, 32, 9, 7, 3, 3, 2, (0, 0, 0, 0), 16), (2, 16, 8, 8, 2, 2, 2, (0, 1, 0, 1), 16),
                                  (3, 64, 5, 5, 5, 5, 1, (0, 0, 0, 0), 16), (2, 3, 7, 7, 3, 3, 1, (1, 1, 1, 1), 3),
                                  (1, 8, 6, 9, 3, 2, 1, (1, 1, 0, 1), 8)])
@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pooling(case, mode):
    N, C, H, W, kh, kw, s, pad, Cb = case
    x = WL.u8_codes(_rng(7), (N, C, H, W))
    ref = Q.pool2d(x, (kh, kw), s, pad, mode)
    g = Guarded8(ref.size)
    S.small_pool2d_u8(dev8(Q.pack(x, Cb)), g.t, N, C, H, W, kh, kw, s, pad, Cb, S.POOL_MAX if mode == "max" else S.POOL_AVG)
    _same(Q.unpack(g.check(), ref.shape, Cb), ref, f"pool u8 {mode} {case}")


@pytest.mark.parametrize("n", [1, 4, 1023, 4096, 100003])
def test_relu(n):
    x = WL.u8_codes(_rng(8), (n,))
    for z in (0, 128, 255):
        g = Guarded8(n)
        S.small_relu_u8(dev8(x), g.t, n, z)
        assert np.array_equal(g.check(), Q.relu(x, z))
    t = dev8(x)
    S.small_relu_u8(t, t, n, 77)       # in place
    torch.cuda.synchronize()
    assert np.array_equal(t.cpu().numpy(), np.maximum(x, 77))


def test_errors_are_raised():
    t = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    o = torch.zeros(4096, dtype=torch.uint8, device=DEV)
    with pytest.raises(S.SmallError) as e:
        S.small_conv2d_u8(t, t, o, 1, 16, 16, 4, 4, 3, 3, 1, (1, 1, 1, 1), 16, 16, Q.Quant(zx=300))
    assert e.value.code == 8
    with pytest.raises(TypeError):
        S.small_relu_u8(torch.zeros(4, device=DEV), o, 4, 0)


@pytest.mark.parametrize("seed", range(32))
def test_conv_random_geometries(seed):
    """Seeded random channel counts, images, windows, strides, paddings and zero points: bit-exact whatever kernel runs."""
    r = np.random.default_rng(7000 + seed)
    Ci = int(r.choice([3, 8, 16, 16, 32, 48, 64, 128]))
    Co = int(r.choice([8, 16, 16, 32, 48, 64]))
    kh = int(r.choice([1, 3, 3, 2, 5]))
    kw = kh if r.random() < 0.6 else int(r.choice([1, 3, 2, 4]))
    s = int(r.choice([1, 1, 2, 3]))
    H, W = int(r.integers(kh, 30)), int(r.integers(kw, 30))
    pad = (int(r.integers(0, kh)), int(r.integers(0, kh)), int(r.integers(0, kw)), int(r.integers(0, kw)))
    N = int(r.integers(1, 5)) if seed % 4 else int(r.integers(20, 50))
    zx, zw = int(r.choice([0, 128, 128, 255, r.integers(0, 256)])), int(r.choice([0, 128, 128, 255, r.integers(0, 256)]))
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    q = _quant_for(Q.conv2d_acc(x, w, s, pad, zx, zw), zx, zw, relu=bool(seed & 1))
    ref = Q.conv2d(x, w, s, pad, q)
    Cib, Cob = min(16, Ci), min(16, Co)
    what = f"conv u8 N={N} {Ci}->{Co} {H}x{W} k={kh}x{kw} s={s} pad={pad} z=({zx},{zw})"
    _same(_conv(x, w, s, pad, q, Cib, Cob, with_sums=bool(seed & 2)), ref, what)


# ------------------------------------------------------------------ vectorised element-wise kernels, add, networks

@pytest.mark.parametrize("n", [16, 4096 * 16, 100000 * 16 + 16])
def test_relu_sixteen_bytes_per_lane(n):
    """Multiples of 16 bytes on aligned buffers take the 16-byte kernel (split even / odd bytes, packed 16-bit max)."""
    x = WL.u8_codes(_rng(9), (n,))
    for z in (0, 1, 127, 128, 200, 255):
        g = Guarded8(n)
        S.small_relu_u8(dev8(x), g.t, n, z)
        assert np.array_equal(g.check(), Q.relu(x, z)), z


@pytest.mark.parametrize("case", [(2, 64, 30, 30, 3, 3, 2, (0, 0, 0, 0)), (3, 16, 9, 7, 3, 3, 1, (1, 1, 1, 1)),
                                  (2, 32, 8, 8, 2, 2, 2, (0, 1, 0, 1)), (5, 48, 5, 5, 5, 5, 1, (0, 0, 0, 0)),
                                  (1, 16, 1, 1, 1, 1, 1, (0, 0, 0, 0)), (4, 256, 56, 56, 3, 3, 2, (0, 0, 0, 0))])
def test_max_pooling_on_16_byte_blocks(case):
    N, C, H, W, kh, kw, s, pad = case
    x = WL.u8_codes(_rng(10), (N, C, H, W))
    x[0, :, 0, 0] = 0                                  # a window of zeros at a padded corner
    ref = Q.pool2d(x, (kh, kw), s, pad, "max")
    g = Guarded8(ref.size)
    S.small_pool2d_u8(dev8(Q.pack(x, 16)), g.t, N, C, H, W, kh, kw, s, pad, 16, S.POOL_MAX)
    _same(Q.unpack(g.check(), ref.shape, 16), ref, f"max pool u8 {case}")


@pytest.mark.parametrize("shape", [(2, 16, 3, 3), (2, 32, 64, 64), (1, 16, 20, 130), (3, 48, 33, 66), (2, 16, 4, 5), (1, 16, 57, 125),
                                   (2, 16, 31, 63), (1, 32, 16, 127), (7, 80, 14, 14)])
def test_max_pooling_3x3_stride_2_by_lane_shifts(shape):
    """The 3x3 / stride 2 / unpadded window on 16-byte blocks: bands of 64 pixels (31 outputs) and strips of 7 output rows,
    at widths of one band, a band and one pixel, several bands, and heights that split into ragged strips."""
    N, C, H, W = shape
    x = WL.u8_codes(_rng(11), (N, C, H, W))
    x[:, :, ::3, ::5] = 255
    x[0, :, :3, :3] = 0
    ref = Q.pool2d(x, (3, 3), 2, (0, 0, 0, 0), "max")
    g = Guarded8(ref.size)
    S.small_pool2d_u8(dev8(Q.pack(x, 16)), g.t, N, C, H, W, 3, 3, 2, (0, 0, 0, 0), 16, S.POOL_MAX)
    _same(Q.unpack(g.check(), ref.shape, 16), ref, f"max pool u8 3x3 s2 {shape}")


WIDE_CONV_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad, zx, zw, relu: input and output channels multiples of 64
    (2, 64, 64, 9, 7, 3, 3, 1, (1, 1, 1, 1), 120, 131, False),     # 63 pixels: a ragged fourth tile
    (3, 64, 128, 20, 18, 3, 3, 1, (1, 1, 1, 1), 128, 128, True),   # no corrections; two groups of output blocks
    (2, 128, 64, 11, 13, 3, 3, 2, (0, 1, 0, 1), 0, 255, False),    # stride 2, extreme zero points
    (1, 64, 64, 33, 40, 3, 3, 1, (1, 1, 1, 1), 17, 128, True),     # only the filter sums
    (2, 64, 64, 8, 8, 2, 4, 1, (0, 1, 2, 1), 128, 200, False),     # an uneven window; only the pixel sums
    (1, 256, 64, 6, 5, 3, 3, 1, (1, 1, 1, 1), 140, 100, False),    # four steps per tap
    (2, 64, 64, 5, 5, 5, 5, 1, (2, 2, 2, 2), 99, 160, True),       # 25 taps: an odd number of steps
    (70, 64, 64, 3, 3, 3, 3, 1, (1, 1, 1, 1), 131, 120, False),    # many images of less than one tile
    (1, 64, 64, 57, 56, 1, 3, 1, (0, 0, 1, 1), 120, 131, False),   # a one-row window
]


POINTWISE_STREAM_CASES = [  # N, Ci, Co, H, W, zx, zw, relu: at least 32768 pixels, 64 or 128 input channels
    (40, 64, 64, 29, 29, 120, 131, True),       # 33640 pixels: a ragged last tile; both correction sums
    (20, 128, 96, 41, 41, 128, 128, False),     # two groups of input blocks, six output blocks, no corrections
    (33000, 64, 32, 1, 1, 7, 128, True),        # one pixel per image; only the filter sums
    (9, 128, 64, 61, 60, 128, 250, False),      # only the pixel sums
]


@pytest.mark.parametrize("case", POINTWISE_STREAM_CASES)
def test_pointwise_conv_streaming(case):
    """1x1 convolutions on 64 or 128 channels with enough pixels for the kernel that keeps the filter in registers and
    walks pixel tiles; with the filter sums given and taken inside, and on the wide requantization path."""
    N, Ci, Co, H, W, zx, zw, relu = case
    r = _rng(21)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, 1, 1))
    pad = (0, 0, 0, 0)
    q = _quant_for(Q.conv2d_acc(x, w, 1, pad, zx, zw), zx, zw, relu)
    ref = Q.conv2d(x, w, 1, pad, q)
    _same(_conv(x, w, 1, pad, q, 16, 16, with_sums=True), ref, f"pointwise u8, sums given {case}")
    _same(_conv(x, w, 1, pad, q, 16, 16), ref, f"pointwise u8 {case}")
    assert len(np.unique(ref)) > 8
    q = _quant(Ci, zx, zw, mult=(1 << 31) - 1, shift=0, zy=9)        # the wide requantization path
    _same(_conv(x, w, 1, pad, q, 16, 16, with_sums=True), Q.conv2d(x, w, 1, pad, q), f"pointwise u8 wide {case}")


@pytest.mark.parametrize("case", WIDE_CONV_CASES)
def test_conv_four_blocks_per_step(case):
    """Layers whose matrix instruction takes one tap of four input blocks, with the filter sums given and taken inside."""
    N, Ci, Co, H, W, kh, kw, s, pad, zx, zw, relu = case
    r = _rng(15)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    q = _quant_for(Q.conv2d_acc(x, w, s, pad, zx, zw), zx, zw, relu)
    ref = Q.conv2d(x, w, s, pad, q)
    _same(_conv(x, w, s, pad, q, 16, 16, with_sums=True), ref, f"conv u8, sums given {case}")
    _same(_conv(x, w, s, pad, q, 16, 16), ref, f"conv u8 {case}")
    assert len(np.unique(ref)) > 8
    q = _quant(Ci * kh * kw, zx, zw, mult=(1 << 31) - 1, shift=0, zy=9)        # the wide requantization path
    _same(_conv(x, w, s, pad, q, 16, 16, with_sums=True), Q.conv2d(x, w, s, pad, q), f"conv u8 wide {case}")


FIRST_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad, zx, zw, Cob
    (3, 3, 16, 32, 32, 3, 3, 1, (1, 1, 1, 1), 128, 128, 16),     # residual CNN's first layer
    (2, 3, 8, 96, 96, 3, 3, 2, (0, 1, 0, 1), 117, 140, 8),       # depthwise-separable CNN's
    (5, 1, 64, 49, 10, 10, 4, 2, (4, 5, 1, 1), 3, 250, 16),      # audio CNN's: four blocks of output channels
    (1, 3, 64, 7, 9, 3, 3, 1, (0, 0, 0, 0), 0, 0, 16),
    (2, 3, 32, 17, 5, 3, 3, 2, (1, 1, 1, 1), 255, 255, 8),
    (9, 1, 8, 12, 6, 10, 4, 1, (5, 4, 2, 1), 128, 1, 8),
    (300, 3, 16, 3, 3, 3, 3, 1, (1, 1, 1, 1), 90, 200, 16),      # more images than pixels per image
    (1, 1, 16, 10, 4, 10, 4, 1, (0, 0, 0, 0), 128, 128, 16),     # a single output pixel
    (3, 8, 16, 24, 24, 1, 1, 1, (0, 0, 0, 0), 131, 120, 16),     # pointwise convolution on the 8-channel block
    (2, 8, 24, 5, 7, 1, 1, 2, (0, 0, 0, 0), 0, 255, 8),
]


@pytest.mark.parametrize("case", FIRST_CASES)
def test_first_convolution(case):
    """First layers on 3 (3x3) or 1 (10x4) input channels: one lane per output pixel around four-byte dot products."""
    N, Ci, Co, H, W, kh, kw, s, pad, zx, zw, Cob = case
    r = _rng(12)
    x, w = WL.u8_codes(r, (N, Ci, H, W)), WL.u8_codes(r, (Co, Ci, kh, kw))
    for relu in (False, True):
        q = _quant_for(Q.conv2d_acc(x, w, s, pad, zx, zw), zx, zw, relu)
        ref = Q.conv2d(x, w, s, pad, q)
        _same(_conv(x, w, s, pad, q, Ci, Cob), ref, f"first conv u8 {case} relu={relu}")
    assert len(np.unique(ref)) > 8
    q = _quant(Ci * kh * kw, zx, zw, mult=(1 << 31) - 1, shift=0, zy=9)        # the wide requantization path
    _same(_conv(x, w, s, pad, q, Ci, Cob), Q.conv2d(x, w, s, pad, q), f"first conv u8 wide {case}")


@pytest.mark.parametrize("shape", [(1, 16, 1, 1), (3, 64, 8, 8), (5, 64, 25, 5), (2, 256, 2, 2), (7, 80, 3, 3), (2, 16, 40, 37), (260, 32, 2, 3)])
def test_global_average_pooling(shape):
    N, C, H, W = shape
    x = WL.u8_codes(_rng(13), (N, C, H, W))
    x[0, :8] = 255
    x[-1, -3:] = 0
    ref = Q.pool2d(x, (H, W), 1, (0, 0, 0, 0), "avg")
    g = Guarded8(ref.size)
    S.small_pool2d_u8(dev8(Q.pack(x, 16)), g.t, N, C, H, W, H, W, 1, (0, 0, 0, 0), 16, S.POOL_AVG)
    _same(Q.unpack(g.check(), ref.shape, 16), ref, f"global average u8 {shape}")


@pytest.mark.parametrize("case", [(1, 16, 2, 2), (256, 64, 10, 10), (7, 256, 2, 2), (300, 64, 12, 12), (5, 128, 24, 12), (3, 48, 15, 5),
                                  (2, 1024, 9, 9)])
def test_small_fully_connected(case):
    """Fewer than 16 outputs per block: a wave per (image, output block), the input blocks split over four parts."""
    N, Ci, Co, Cob = case
    r = _rng(14)
    x, w = WL.u8_codes(r, (N, Ci, 1, 1)), WL.u8_codes(r, (Co, Ci, 1, 1))
    for zx, zw in ((128, 128), (3, 250), (255, 0)):
        q = _quant_for(Q.conv2d_acc(x, w, 1, (0, 0, 0, 0), zx, zw), zx, zw)
        g = Guarded8(N * Co)
        S.small_dense_u8(dev8(Q.pack(x, 16)), dev8(Q.pack_filter(w, Cob, 16)), g.t, N, Ci, Co, 16, Cob, q)
        _same(Q.unpack(g.check(), (N, Co, 1, 1), Cob), Q.dense(x, w, q), f"dense u8 {case} z=({zx},{zw})")


ADD_PARAMS = [(128, 128, 128, 3 << 28, 1 << 29, 30, 0, 255), (0, 255, 17, (1 << 31) - 1, 1, 31, 0, 255),
              (200, 3, 100, 12345, 67890, 7, 10, 240), (5, 9, 0, 7, 3, 0, 0, 255), (255, 0, 255, 1 << 30, 1 << 30, 31, 0, 255),
              (128, 128, 128, (1 << 31) - 1, (1 << 31) - 1, 0, 0, 255)]


@pytest.mark.parametrize("params", ADD_PARAMS)
@pytest.mark.parametrize("n", [1, 15, 65536, 100003])
def test_add_two_scales(params, n):
    """Every pair of codes occurs (n = 65536 is the full 256 x 256 table); odd sizes take the byte kernel."""
    q = Q.QuantAdd(*params)
    if n == 65536:
        a, b = [v.reshape(-1).copy() for v in np.meshgrid(np.arange(256, dtype=np.uint8), np.arange(256, dtype=np.uint8), indexing="ij")]
    else:
        r = _rng(11)
        a, b = WL.u8_codes(r, (n,)), WL.u8_codes(r, (n,))
    ref = Q.add(a, b, q)
    g = Guarded8(n)
    S.small_add_u8(dev8(a), dev8(b), g.t, n, q)
    _same(g.check(), ref, f"add u8 {params} n={n}")
    t = dev8(a)
    S.small_add_u8(t, dev8(b), t, n, q)               # in place on the first operand
    torch.cuda.synchronize()
    _same(t.cpu().numpy(), ref, "add u8 in place")


def _run_u8(net, x, ws, qs):
    pn = S.PackedNetworkU8(net, ws, qs, DEV)
    N = x.shape[0]
    g = Guarded8(pn.out_elems(N))
    pn.run(pn.pack_input(dev8(x)), g.t, N)
    L = net.layers[-1]
    return Q.unpack(g.check(), (N, L.Co, L.Ho, L.Wo), L.Cob)


def _chain_table():
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


def test_network_every_op_and_every_prefix():
    """A table with every op of the quantized path: the whole run and every prefix of it (the prefix's last layer
    redirected to the output buffer) equal the oracle's chain, code for code: this checks each intermediate tensor."""
    import copy
    net = _chain_table()
    x, ws, qs = WL.quantized_network_tensors(net, 5, 4242)
    _same(_run_u8(net, x, ws, qs), Q.run_network(net, x, ws, qs), "u8 chain")
    for upto in range(len(net.layers) - 1):
        if net.layers[upto + 1].op == "relu" and net.layers[upto + 1].src == net.layers[upto].dst:
            continue                                   # the next layer's ReLU is folded only when it is in the table
        sub = copy.deepcopy(net)
        sub.layers = sub.layers[:upto + 1]
        sub.layers[-1].dst = -2
        _same(_run_u8(sub, x, ws, qs[:upto + 1]), Q.run_network(net, x, ws, qs, upto=upto), f"u8 chain prefix {upto}")


def test_network_relu_that_must_not_be_folded():
    """A ReLU into another buffer is a layer of its own: the convolution's result stays as it was for the add."""
    from workloads.nets import Layer, Network, IN, OUT
    net = Network("u8_nofold", 16, 5, 5)
    net.wshapes = [((16, 16, 3, 3), 144)]
    net.layers = [Layer("conv", 16, 16, 5, 5, 3, 3, 1, (1, 1, 1, 1), src=IN, dst=0, w=0),
                  Layer("relu", 16, 16, 5, 5, src=0, dst=1),
                  Layer("add", 16, 16, 5, 5, src=0, src2=1, dst=OUT)]
    x, ws, qs = WL.quantized_network_tensors(net, 3, 4243)
    ref = Q.run_network(net, x, ws, qs)
    assert (Q.run_network(net, x, ws, qs, upto=0) < 128).any()
    _same(_run_u8(net, x, ws, qs), ref, "u8 relu into another buffer")


@pytest.mark.parametrize("name,N", [("residual_cnn", 7), ("residual_cnn", 256), ("audio_cnn", 33), ("dsep_cnn", 3)])
def test_quantized_networks(name, N):
    """The stand-in networks on codes (seeded codes and parameters, every tensor's zero point 128): every image of
    the batch, code for code."""
    net = getattr(WL, name)()
    x, ws, qs = WL.quantized_network_tensors(net, N, WL.BASE_SEED + 300 + N)
    ref = Q.run_network(net, x, ws, qs)
    assert len(np.unique(ref)) > min(8, ref.size // 2), "the recipe's parameters must not collapse or saturate the logits"
    _same(_run_u8(net, x, ws, qs), ref, f"u8 {name} batch {N}")


@pytest.mark.parametrize("name,N", [("dsep_cnn", 256), ("audio_cnn", 1024)])
def test_quantized_networks_full_batch_sampled(name, N):
    """The batches the benchmark times; the oracle recomputes the first and the last sixteen images (images are independent)."""
    net = getattr(WL, name)()
    x, ws, qs = WL.quantized_network_tensors(net, N, WL.BASE_SEED + 300 + N)
    got = _run_u8(net, x, ws, qs)
    for lo in (0, N - 16):
        _same(got[lo:lo + 16], Q.run_network(net, x[lo:lo + 16], ws, qs), f"u8 {name} batch {N}, images {lo}..{lo + 15}")


def test_network_table_errors():
    net = _chain_table()
    x, ws, qs = WL.quantized_network_tensors(net, 2, 4244)
    pn = S.PackedNetworkU8(net, ws, qs, DEV)
    pn.table[3].Ci = 32                                 # block / channel mismatch with the tensor in its source buffer
    with pytest.raises(S.SmallError) as e:
        pn.workspace(2)
    assert e.value.code == 7
    pn = S.PackedNetworkU8(net, ws, qs, DEV)
    pn.table[4].qa.shift = 40
    with pytest.raises(S.SmallError) as e:
        pn.workspace(2)
    assert e.value.code == 8
    pn = S.PackedNetworkU8(net, ws, qs, DEV)
    pn.table[0].op = 7                                  # batch normalization has no quantized layer
    with pytest.raises(S.SmallError) as e:
        pn.workspace(2)
    assert e.value.code == 7


DW_LANES_U8_CASES = [  # N, C, H, W, zx, zw: 3x3, stride 1, padding 1, 16-byte blocks
    (3, 64, 56, 56, 120, 131),          # four bands of 14 columns, eight row strips
    (5, 128, 28, 28, 128, 128),
    (9, 256, 14, 14, 0, 255),           # one band; zero points at the ends of the code range
    (11, 512, 7, 7, 255, 0),            # two planes side by side in a row of 16 lanes
    (3, 16, 5, 5, 17, 201),             # ... an odd number of planes
    (5, 48, 7, 3, 130, 120),
    (1, 16, 1, 1, 128, 128),
    (2, 32, 1, 40, 100, 60),
    (4, 48, 61, 63, 7, 250),
    (7, 32, 33, 17, 128, 128),
    (2, 32, 70, 100, 200, 100),
    (5, 64, 25, 5, 130, 120),           # three planes of 5-pixel rows back to back, 20 planes: the last band holds two
    (3, 48, 9, 4, 3, 250),              # four planes per band, 9 planes
    (7, 16, 6, 3, 250, 3),              # five planes per band and an unused lane
    (9, 32, 4, 2, 128, 7),              # eight planes per band
    (5, 16, 3, 1, 77, 200),             # sixteen one-pixel rows per band
    (770, 64, 25, 5, 130, 120),         # a full batch of them: 3080 planes, the last band holds two
]


@pytest.mark.parametrize("case", DW_LANES_U8_CASES)
def test_depthwise_lane_shift(case):
    """Quantized depthwise 3x3 with stride 1 and padding 1: the kernel that keeps rows in registers as exact floats
    and takes the horizontal neighbours from the next lanes; random filters, zero points away from 128 (the padding
    reads as zx, lanes at a unit's end shift in zero), a ReLU clamp in the middle of the codes."""
    N, C, H, W, zx, zw = case
    r = _rng(12)
    x, w = WL.u8_codes(r, (N, C, H, W)), WL.u8_codes(r, (C, 1, 3, 3))
    pad = (1, 1, 1, 1)
    q = _quant_for(Q.dwconv2d_acc(x, w, 1, pad, zx, zw), zx, zw, relu=True)
    ref = Q.dwconv2d(x, w, 1, pad, q)
    assert len(np.unique(ref)) > 8
    g = Guarded8(ref.size)
    S.small_dwconv2d_u8(dev8(Q.pack(x, 16)), dev8(Q.pack_dw_filter(w, 16)), g.t, N, C, H, W, 3, 3, 1, pad, 16, q)
    _same(Q.unpack(g.check(), ref.shape, 16), ref, f"dw u8 lanes {case}")


@pytest.mark.parametrize("mult,shift", [(1 << 20, 0), ((1 << 31) - 1, 0), (1, 31), (0, 5), ((1 << 31) - 1, 31), (3, 1)])
def test_depthwise_extreme_scales(mult, shift):
    """Scales from 'everything saturates' to 'everything rounds to the zero point': whichever requantization path the
    layer takes (the clamped one or the wide one), the codes are the oracle's."""
    r = _rng(13)
    x, w = WL.u8_codes(r, (3, 32, 9, 20)), WL.u8_codes(r, (32, 1, 3, 3))
    q = Q.Quant(zx=99, zw=140, zy=77, mult=mult, shift=shift, lo=3, hi=250)
    ref = Q.dwconv2d(x, w, 1, (1, 1, 1, 1), q)
    g = Guarded8(ref.size)
    S.small_dwconv2d_u8(dev8(Q.pack(x, 16)), dev8(Q.pack_dw_filter(w, 16)), g.t, 3, 32, 9, 20, 3, 3, 1, (1, 1, 1, 1), 16, q)
    _same(Q.unpack(g.check(), ref.shape, 16), ref, f"dw u8 scale {mult} / 2^{shift}")
