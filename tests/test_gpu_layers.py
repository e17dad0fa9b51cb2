"""GPU parity: every layer of the hot path, through the C ABI, against the CPU oracle.

Bit-exact for pack / unpack / max-pool / ReLU / add; |gpu - ref| <= 1e-4 (sqrt(K) max|ref| + 1)
for conv (K = Ci kh kw), depthwise and avg-pool (K = kh kw) and dense (K = Ci)."""
import numpy as np
import pytest
import torch

import paper_2303_04769_amd as S
from oracle import oracle as O
from gpu_util import DEV, Guarded, assert_bits, assert_close, dev

pytestmark = pytest.mark.gpu


def _blk(C):
    return min(16, C)


# ------------------------------------------------------------------ layouts

@pytest.mark.parametrize("N,C,H,W,Cb", [(2, 32, 5, 7, 16), (1, 3, 96, 96, 3), (3, 8, 9, 13, 8), (2, 1, 49, 10, 1),
                                         (1, 64, 1, 1, 16), (2, 10, 1, 1, 10), (1, 48, 17, 9, 16), (1, 12, 3, 70, 4),
                                         (2, 32, 20, 20, 16), (1, 16, 16, 16, 16), (3, 64, 56, 56, 16), (2, 16, 8, 8, 16),
                                         (5, 48, 14, 14, 16), (1, 16, 2, 2, 16), (3, 16, 2, 2, 16), (7, 32, 3, 4, 16), (2, 16, 50, 50, 16)])
def test_pack_unpack_bit_exact(N, C, H, W, Cb):
    rng = np.random.default_rng(N * 1000 + C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    g = Guarded(x.size)
    S.small_pack(dev(x), g.t, N, C, H, W, Cb)
    got = g.check()
    assert_bits(got, O.pack(x, Cb), "pack")
    g2 = Guarded(x.size)
    S.small_unpack(dev(got), g2.t, N, C, H, W, Cb)
    assert_bits(g2.check().reshape(x.shape), x, "unpack")


def test_pack_filters_bit_exact():
    rng = np.random.default_rng(3)
    for (Co, Ci, kh, kw, Cob, Cib) in [(32, 48, 3, 3, 16, 16), (16, 3, 3, 3, 16, 3), (64, 1, 10, 4, 16, 1),
                                       (10, 64, 1, 1, 10, 16), (16, 8, 1, 1, 16, 8)]:
        w = rng.standard_normal((Co, Ci, kh, kw)).astype(np.float32)
        g = Guarded(w.size)
        S.small_pack_filter(dev(w), g.t, Co, Ci, kh, kw, Cob, Cib)
        assert_bits(g.check(), O.pack_filter(w, Cob, Cib), "pack_filter")
    for (C, Cb) in [(32, 16), (8, 8), (3, 3)]:
        w = rng.standard_normal((C, 1, 3, 3)).astype(np.float32)
        g = Guarded(w.size)
        S.small_pack_dw_filter(dev(w), g.t, C, 3, 3, Cb)
        assert_bits(g.check(), O.pack_dw_filter(w, Cb), "pack_dw_filter")


# ------------------------------------------------------------------ single element

@pytest.mark.parametrize("n", [1, 3, 4, 1023, 4096, 16384, 100003])
def test_relu_add_bit_exact(n):
    rng = np.random.default_rng(n)
    a = rng.standard_normal(n).astype(np.float32)
    b = rng.standard_normal(n).astype(np.float32)
    special = np.array([-np.inf, -2.5, -0.0, 0.0, 1e-45, -1e-45, 3.0, np.inf, np.nan], np.float32)
    a[:min(n, special.size)] = special[:n]
    g = Guarded(n)
    S.small_relu(dev(a), g.t, n)
    assert_bits(g.check(), O.relu(a), "relu")
    g = Guarded(n)
    a2 = np.nan_to_num(a, nan=1.0, posinf=2.0, neginf=-2.0)
    S.small_add(dev(a2), dev(b), g.t, n)
    assert_bits(g.check(), O.add(a2, b), "add")
    # in place, and from an unaligned offset (scalar path)
    g = Guarded(n + 1)
    g.t[1:].copy_(dev(a))
    v = g.t[1:]
    S.small_relu(v, v, n)
    assert_bits(g.check()[1:], O.relu(a), "relu in place, unaligned")


# ------------------------------------------------------------------ convolution

def run_conv(x, w, stride, pad, Cib=None, Cob=None):
    N, Ci, H, W = x.shape
    Co, _, kh, kw = w.shape
    Cib, Cob = Cib or _blk(Ci), Cob or _blk(Co)
    xb, wb = dev(O.pack(x, Cib)), dev(O.pack_filter(w, Cob, Cib))
    Ho, Wo = O.out_dim(H, kh, stride, pad[0], pad[1]), O.out_dim(W, kw, stride, pad[2], pad[3])
    g = Guarded(N * Co * Ho * Wo)
    S.small_conv2d(xb, wb, g.t, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob)
    return O.unpack(g.check(), (N, Co, Ho, Wo), Cob)


CONV_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad
    (1, 16, 16, 32, 32, 3, 3, 1, (1, 1, 1, 1)),      # the single-layer workload
    (3, 32, 48, 13, 11, 3, 3, 1, (1, 1, 1, 1)),      # ragged pixel tail, Co not a power of two
    (2, 64, 64, 9, 9, 1, 1, 1, (0, 0, 0, 0)),
    (2, 16, 32, 16, 16, 1, 1, 2, (0, 0, 0, 0)),      # projection shortcut
    (2, 16, 32, 32, 32, 3, 3, 2, (0, 1, 0, 1)),      # 'same' stride 2
    (3, 32, 32, 31, 31, 3, 3, 2, (1, 1, 1, 1)),      # stride 2, odd image, left / top padding
    (5, 48, 64, 20, 12, 3, 3, 2, (0, 1, 0, 1)),      # stride 2, non-square, three input-channel blocks
    (2, 16, 32, 32, 32, 3, 3, 2, (1, 1, 1, 1)),      # stride 2 whose last tap stays inside the image: gather kernel
    (4, 64, 32, 15, 15, 1, 1, 2, (0, 0, 0, 0)),      # 1x1 stride 2, odd image, two planes per step
    (2, 16, 16, 9, 9, 1, 1, 3, (0, 0, 0, 0)),        # 1x1 stride 3
    (1, 32, 16, 7, 9, 5, 3, 2, (2, 2, 1, 1)),        # odd window
    (2, 16, 16, 6, 6, 3, 3, 1, (0, 0, 0, 0)),        # no padding
    (4, 256, 128, 7, 7, 3, 3, 1, (1, 1, 1, 1)),      # tiles straddle images, 128-wide channel tile
    (2, 1, 64, 49, 10, 10, 4, 2, (4, 5, 1, 1)),      # generic path: Ci = 1
    (2, 3, 16, 32, 32, 3, 3, 1, (1, 1, 1, 1)),       # generic path: Ci = 3
    (1, 3, 8, 96, 96, 3, 3, 2, (0, 1, 0, 1)),        # generic path: 8-channel output block
    (2, 8, 16, 24, 24, 1, 1, 1, (0, 0, 0, 0)),       # generic path: 8-channel input block
    (5, 64, 10, 1, 1, 1, 1, 1, (0, 0, 0, 0)),        # generic path: dense-like head
    (3, 16, 10, 4, 5, 4, 5, 1, (0, 0, 0, 0)),        # dense over a 4 x 5 image (window = image)
]


@pytest.mark.parametrize("case", CONV_CASES)
def test_conv2d(case):
    N, Ci, Co, H, W, kh, kw, s, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, Ci, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((Co, Ci, kh, kw), dtype=np.float32) * 2 - 1).astype(np.float32)
    got = run_conv(x, w, s, pad)
    assert_close(got, O.conv2d(x, w, s, pad), Ci * kh * kw, f"conv {case}")


def test_conv2d_large_tiles():
    """Enough pixels that the 128-pixel tiles are chosen (>= 256 workgroups) for every channel-tile width."""
    rng = np.random.default_rng(77)
    for Ci, Co, N, H in [(32, 128, 18, 45), (16, 64, 10, 58), (16, 32, 9, 61), (16, 16, 9, 61)]:
        x = (rng.random((N, Ci, H, H), dtype=np.float32) * 2 - 1).astype(np.float32)
        w = (rng.random((Co, Ci, 3, 3), dtype=np.float32) * 2 - 1).astype(np.float32)
        got = run_conv(x, w, 1, (1, 1, 1, 1))
        assert_close(got, O.conv2d(x, w, 1, (1, 1, 1, 1)), Ci * 9, f"conv large {Ci}->{Co}")


PERSISTENT_CASES = [  # N, Ci, Co, H, W, k: enough images that a workgroup walks several of them
    (131, 16, 16, 32, 32, 3),      # 16 tiles per image, last image group ragged
    (160, 16, 16, 30, 30, 3),      # image size not a multiple of the tile: masked lanes in each image's last tile
    (240, 16, 32, 24, 24, 3),      # 24 x 24 images: 9 full tiles, two output-channel blocks per wave
    (48, 32, 48, 40, 40, 3),       # three channel tiles per pixel tile
    (150, 16, 32, 48, 48, 3, 2),   # stride 2: two staged entries per output pixel
    (256, 16, 16, 32, 32, 3),      # the 128-pixel tile of the residual network's first stage at batch 256
]


@pytest.mark.parametrize("case", PERSISTENT_CASES)
def test_conv2d_persistent_variant(case):
    """Image-aligned persistent kernel: same results as the definition, and it really is the one that runs."""
    N, Ci, Co, H, W, k = case[:6]
    stride = case[6] if len(case) > 6 else 1
    pad = ((1, 1, 1, 1) if stride == 1 else (0, 1, 0, 1)) if k == 3 else (0, 0, 0, 0)
    assert S.small_conv2d_kernel(N, Ci, Co, H, W, k, k, stride, pad, 16, 16).startswith("conv16_img"), case
    rng = np.random.default_rng(1000 + N)
    x = (rng.random((N, Ci, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((Co, Ci, k, k), dtype=np.float32) * 2 - 1).astype(np.float32)
    got = run_conv(x, w, stride, pad)
    assert_close(got, O.conv2d(x, w, stride, pad), Ci * k * k, f"conv persistent {case}")


POINTWISE_STREAM_CASES = [  # N, C, H, W: 64 or 128 channels, at least 32768 pixels
    (3, 64, 105, 105),       # 33075 pixels: groups of 16 straddle images, the last group has 3 pixels
    (70, 64, 25, 19),        # 33250 pixels, many small images, ragged end (2 pixels)
    (11, 128, 55, 55),       # 128 channels: two waves share a pixel group; 33275 pixels (11 in the last group)
    (9, 128, 61, 60),        # 32940 pixels: a tail of units after the full rounds
    (16, 64, 64, 64),        # 65536 pixels: 4096 groups = 2 full rounds on 2048 waves, no tail, no ragged group
    (17, 64, 64, 64),        # ... and one image more: a short tail
    (40, 128, 30, 30),       # 36000 pixels = 2250 groups: fewer tasks than two rounds of 512 tasks
]


@pytest.mark.parametrize("case", POINTWISE_STREAM_CASES)
def test_conv2d_pointwise_stream(case):
    """1x1 convolutions on 64 / 128 channels with many pixels run in the persistent kernel with the filter resident
    (asserted by name): full rounds of tasks, the finer units of the tail, and the ragged last group."""
    N, C, H, W = case
    name = S.small_conv2d_kernel(N, C, C, H, W, 1, 1, 1, (0, 0, 0, 0), 16, 16)
    assert name.startswith("pw16_stream"), (case, name)
    rng = np.random.default_rng(6100 + N + C)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((C, C, 1, 1), dtype=np.float32) * 2 - 1).astype(np.float32)
    got = run_conv(x, w, 1, (0, 0, 0, 0))
    assert_close(got, O.conv2d(x, w, 1, (0, 0, 0, 0)), C, f"pointwise stream {case}")


FIRST_LAYER_CASES = [  # N, Ci, Co, H, W, kh, kw, stride, pad: at least 16384 output pixels, one short input block
    (17, 3, 16, 32, 32, 3, 3, 1, (1, 1, 1, 1)),      # K = 27: the residual network's first layer, ragged pixel tail
    (8, 3, 8, 96, 96, 3, 3, 2, (0, 1, 0, 1)),        # 8-channel output block, stride 2, bottom / right padding
    (140, 1, 64, 49, 10, 10, 4, 2, (4, 5, 1, 1)),    # K = 40: the audio network's first layer, four output blocks
    (20, 1, 16, 30, 31, 5, 5, 1, (2, 2, 2, 2)),      # K = 25 (padded to 28), wide padding on all sides
    (5, 2, 32, 60, 61, 2, 7, 1, (0, 1, 3, 3)),       # K = 28 exactly, two input channels
    (9, 5, 16, 44, 45, 2, 4, 1, (1, 0, 2, 1)),       # K = 40 with five input channels
    (3, 3, 16, 80, 81, 13, 1, 1, (6, 6, 0, 0)),      # K = 39: a tall window
    (40, 8, 16, 24, 24, 1, 1, 1, (0, 0, 0, 0)),      # K = 8: the pointwise layer after the 8-channel depthwise one
    (12, 2, 8, 40, 41, 2, 2, 1, (0, 1, 1, 0)),       # K = 8 from a 2 x 2 window of two channels
    (30, 5, 16, 30, 30, 1, 1, 1, (0, 0, 0, 0)),      # K = 5 (padded to 8)
]


@pytest.mark.parametrize("case", FIRST_LAYER_CASES)
def test_conv2d_first_layer_matrix_core(case):
    N, Ci, Co, H, W, kh, kw, s, pad = case
    name = S.small_conv2d_kernel(N, Ci, Co, H, W, kh, kw, s, pad, Ci, _blk(Co))
    assert name.startswith("conv_first_mfma"), (case, name)
    rng = np.random.default_rng(4000 + N)
    x = (rng.random((N, Ci, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((Co, Ci, kh, kw), dtype=np.float32) * 2 - 1).astype(np.float32)
    got = run_conv(x, w, s, pad)
    assert_close(got, O.conv2d(x, w, s, pad), Ci * kh * kw, f"first layer {case}, all {N} images")


def test_conv_identity_filter_is_exact():
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 32, 10, 12)).astype(np.float32)
    w = np.zeros((32, 32, 3, 3), np.float32)
    w[np.arange(32), np.arange(32), 1, 1] = 1
    assert_bits(run_conv(x, w, 1, (1, 1, 1, 1)), x, "delta filter")


def test_dense():
    rng = np.random.default_rng(6)
    for N, Ci, Co in [(7, 64, 10), (1, 256, 2), (33, 64, 12), (130, 128, 128), (3, 16, 16), (5, 6, 3), (1024, 64, 12)]:
        x = rng.standard_normal((N, Ci, 1, 1)).astype(np.float32)
        w = rng.standard_normal((Co, Ci, 1, 1)).astype(np.float32)
        Cib, Cob = _blk(Ci), _blk(Co)
        g = Guarded(N * Co)
        S.small_dense(dev(O.pack(x, Cib)), dev(O.pack_filter(w, Cob, Cib)), g.t, N, Ci, Co, Cib, Cob)
        got = O.unpack(g.check(), (N, Co, 1, 1), Cob)
        assert_close(got, O.dense(x, w), Ci, f"dense {N}x{Ci}->{Co}")


# ------------------------------------------------------------------ depthwise / pooling

DW_CASES = [  # N, C, H, W, k, stride, pad
    (2, 32, 13, 11, 3, 1, (1, 1, 1, 1)),
    (2, 64, 12, 12, 3, 2, (0, 1, 0, 1)),
    (1, 8, 48, 48, 3, 2, (0, 1, 0, 1)),        # 8-channel block
    (3, 128, 3, 3, 3, 2, (1, 1, 1, 1)),
    (2, 64, 25, 5, 3, 1, (1, 1, 1, 1)),
    (1, 16, 9, 9, 5, 1, (2, 2, 2, 2)),         # run-time window
    (2, 3, 10, 10, 3, 1, (1, 1, 1, 1)),        # scalar path
    (2, 256, 7, 7, 3, 1, (1, 1, 1, 1)),
]


@pytest.mark.parametrize("case", DW_CASES)
def test_dwconv2d(case):
    N, C, H, W, k, s, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((C, 1, k, k), dtype=np.float32) * 2 - 1).astype(np.float32)
    Cb = _blk(C)
    ref = O.dwconv2d(x, w, s, pad)
    g = Guarded(ref.size)
    S.small_dwconv2d(dev(O.pack(x, Cb)), dev(O.pack_dw_filter(w, Cb)), g.t, N, C, H, W, k, k, s, pad, Cb)
    assert_close(O.unpack(g.check(), ref.shape, Cb), ref, k * k, f"dw {case}")


DW_LARGE_CASES = [  # N, C, H, W, stride, pad: at least 40 MB of traffic, where the row-staged kernel takes over
    (8, 64, 161, 97, 1, (1, 1, 1, 1)),         # odd image: ragged row tiles, two row tiles of different height
    (6, 128, 120, 120, 2, (0, 1, 0, 1)),       # stride 2
    (700, 64, 25, 5, 1, (1, 1, 1, 1)),         # two whole small images per tile, last group shifted back (N odd / 2)
    (3501, 32, 7, 7, 1, (1, 1, 1, 1)),         # five images per tile, batch not a multiple of five
    (9, 16, 300, 140, 1, (0, 0, 0, 0)),        # rows wider than half a tile: one row per tile; no padding
    (8, 16, 150, 300, 1, (1, 1, 1, 1)),        # rows wider than a tile: too much to stage, the LDS-tiled kernel runs
]


@pytest.mark.parametrize("case", DW_LARGE_CASES)
def test_dwconv2d_large(case):
    N, C, H, W, s, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((C, 1, 3, 3), dtype=np.float32) * 2 - 1).astype(np.float32)
    ref = O.dwconv2d(x, w, s, pad)
    assert (x.size + ref.size) * 4 >= 40 << 20
    g = Guarded(ref.size)
    S.small_dwconv2d(dev(O.pack(x, 16)), dev(O.pack_dw_filter(w, 16)), g.t, N, C, H, W, 3, 3, s, pad, 16)
    assert_close(O.unpack(g.check(), ref.shape, 16), ref, 9, f"dw large {case}")


DW_LANES_CASES = [  # N, C, H, W: 3x3, stride 1, padding 1, 16-channel blocks
    (6, 64, 56, 56),           # four bands of 14 columns; the planes cut into row strips
    (20, 128, 28, 28),         # two bands
    (70, 256, 14, 14),         # one band: lanes 0 and 15 of a row of lanes stay zero
    (300, 512, 7, 7),          # two planes side by side in the 16 lanes
    (3, 16, 5, 5),             # ... an odd number of planes: the last pair has one
    (5, 48, 7, 3),             # ... narrow
    (1, 16, 1, 1),             # one pixel
    (2, 32, 1, 40),            # one row: every output touches the top and the bottom edge; three bands (14, 14, 12)
    (9, 48, 61, 63),           # three channel blocks, five bands (the last of 7 columns), strips of unequal height
    (70, 32, 33, 17),          # two bands, three columns in the second
    (12, 32, 52, 15),          # 15 columns: one more than a band
    (5, 32, 70, 100),          # eight bands, the last of two columns
    (600, 16, 2, 64),          # two rows
    (400, 16, 33, 8),          # eight columns: one plane per row of lanes again
    (64, 64, 56, 56),          # the benchmark row
]


@pytest.mark.parametrize("case", DW_LANES_CASES)
def test_dwconv2d_lane_shift(case):
    """Depthwise 3x3 layers with stride 1 and padding 1 run with the rows in registers and the horizontal neighbours
    taken from the next lanes: bands and their halo lanes, plane pairs, row strips, both image edges, ragged rows.
    The filters are random, so a shift in the wrong direction or a swapped row shows."""
    N, C, H, W = case
    rng = np.random.default_rng(7300 + N + C)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((C, 1, 3, 3), dtype=np.float32) * 2 - 1).astype(np.float32)
    ref = O.dwconv2d(x, w, 1, (1, 1, 1, 1))
    g = Guarded(ref.size)
    S.small_dwconv2d(dev(O.pack(x, 16)), dev(O.pack_dw_filter(w, 16)), g.t, N, C, H, W, 3, 3, 1, (1, 1, 1, 1), 16)
    assert_close(O.unpack(g.check(), ref.shape, 16), ref, 9, f"dw lanes {case}")


POOL_CASES = [  # N, C, H, W, kh, kw, stride, pad
    (2, 32, 13, 11, 3, 3, 2, (0, 0, 0, 0)),
    (1, 16, 56, 56, 3, 3, 2, (0, 0, 0, 0)),
    (2, 48, 9, 9, 3, 3, 1, (1, 1, 1, 1)),
    (2, 16, 8, 8, 2, 2, 2, (0, 0, 0, 0)),
    (3, 64, 8, 8, 8, 8, 1, (0, 0, 0, 0)),      # global
    (3, 256, 2, 2, 2, 2, 1, (0, 0, 0, 0)),     # global
    (5, 64, 25, 5, 25, 5, 1, (0, 0, 0, 0)),    # global
    (2, 8, 6, 6, 6, 6, 1, (0, 0, 0, 0)),       # global, 8-channel block
    (2, 3, 7, 7, 3, 3, 2, (1, 1, 1, 1)),       # scalar path
]


@pytest.mark.parametrize("case", POOL_CASES)
@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool2d(case, mode):
    N, C, H, W, kh, kw, s, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    Cb = _blk(C)
    ref = O.pool2d(x, (kh, kw), s, pad, mode)
    g = Guarded(ref.size)
    S.small_pool2d(dev(O.pack(x, Cb)), g.t, N, C, H, W, kh, kw, s, pad, Cb, S.POOL_MAX if mode == "max" else S.POOL_AVG)
    got = O.unpack(g.check(), ref.shape, Cb)
    if mode == "max":
        assert_bits(got, ref, f"maxpool {case}")
    else:
        assert_close(got, ref, kh * kw, f"avgpool {case}")


POOL_LARGE_CASES = [  # N, C, H, W, stride, pad: tens of MB, many workgroups per plane
    (16, 64, 112, 112, 2, (0, 0, 0, 0)),       # the sweep's pooling geometry, smaller batch
    (8, 64, 161, 97, 1, (1, 1, 1, 1)),         # padded: taps outside the image
    (4201, 32, 8, 8, 2, (0, 1, 0, 1)),         # many tiny images
]


@pytest.mark.parametrize("case", POOL_LARGE_CASES)
@pytest.mark.parametrize("mode", ["max", "avg"])
def test_pool2d_large(case, mode):
    N, C, H, W, s, pad = case
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    if mode == "max":      # ties between +0 and -0, NaNs, whole windows of NaN
        flat = x.reshape(-1)
        idx = rng.integers(0, flat.size, flat.size // 7)
        flat[idx[0::3]] = 0.0
        flat[idx[1::3]] = -0.0
        flat[idx[2::3]] = np.nan
        x[0, :, :6, :6] = np.nan
        x[-1, :, -5:, :] = -0.0
    ref = O.pool2d(x, (3, 3), s, pad, mode)
    g = Guarded(ref.size)
    S.small_pool2d(dev(O.pack(x, 16)), g.t, N, C, H, W, 3, 3, s, pad, 16, S.POOL_MAX if mode == "max" else S.POOL_AVG)
    got = O.unpack(g.check(), ref.shape, 16)
    if mode == "max":
        assert_bits(got, ref, f"maxpool large {case}")
    else:
        assert_close(got, ref, 9, f"avgpool large {case}")


@pytest.mark.parametrize("shape", [(2, 16, 3, 3), (2, 32, 16, 16), (1, 16, 20, 31), (3, 48, 33, 30), (2, 16, 4, 5), (1, 16, 57, 125),
                                   (2, 16, 31, 15), (1, 32, 16, 17), (7, 80, 14, 14), (4, 256, 56, 56)])
def test_maxpool_3x3_stride_2_by_lane_shifts(shape):
    """The 3x3 / stride 2 / unpadded window on 16-channel blocks: bands of 16 pixels (7 outputs) and strips of 7 output rows, at
    widths of one band, a band and one pixel, many bands, and heights that split into ragged strips; +0 / -0 ties, NaNs and
    whole windows of NaN as the reference scan resolves them."""
    N, C, H, W = shape
    rng = np.random.default_rng(N * 1000 + H * 10 + W)
    x = (rng.random((N, C, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    flat = x.reshape(-1)
    idx = rng.integers(0, flat.size, flat.size // 5)
    flat[idx[0::4]] = 0.0
    flat[idx[1::4]] = -0.0
    flat[idx[2::4]] = np.nan
    flat[idx[3::4]] = -np.inf
    x[0, :, :3, :3] = np.nan
    ref = O.pool2d(x, (3, 3), 2, (0, 0, 0, 0), "max")
    g = Guarded(ref.size)
    S.small_pool2d(dev(O.pack(x, 16)), g.t, N, C, H, W, 3, 3, 2, (0, 0, 0, 0), 16, S.POOL_MAX)
    assert_bits(O.unpack(g.check(), ref.shape, 16), ref, f"maxpool 3x3 s2 {shape}")


def test_maxpool_ties_and_nan_bit_exact():
    x = np.zeros((1, 16, 4, 4), np.float32)
    x[0, :, 0, 0], x[0, :, 0, 1] = -0.0, 0.0          # first seen is -0
    x[0, :, 2, 2], x[0, :, 2, 3], x[0, :, 3, 2], x[0, :, 3, 3] = np.nan, -3.0, np.nan, -5.0
    x[0, :, 0, 2], x[0, :, 0, 3], x[0, :, 1, 2], x[0, :, 1, 3] = 0.0, -0.0, -1.0, -2.0
    x[0, :, 1, 0], x[0, :, 1, 1] = -0.0, -0.0
    ref = O.pool2d(x, (2, 2), 2)
    g = Guarded(ref.size)
    S.small_pool2d(dev(O.pack(x, 16)), g.t, 1, 16, 4, 4, 2, 2, 2, (0, 0, 0, 0), 16, S.POOL_MAX)
    assert_bits(O.unpack(g.check(), ref.shape, 16), ref, "maxpool specials")


def test_errors_leave_output_untouched():
    x = dev(np.ones(16 * 64, np.float32))
    g = Guarded(16 * 64)
    with pytest.raises(S.binding.SmallError):
        S.small_conv2d(x, x, g.t, 1, 16, 24, 8, 8, 3, 3, 1, (1, 1, 1, 1), 16, 16)
    with pytest.raises(S.binding.SmallError):
        S.small_pool2d(x, x, 1, 16, 8, 8, 3, 3, 1, (1, 1, 1, 1), 16, S.POOL_MAX)
    assert (g.check() == np.float32(-7.25e37)).all()


def test_matrix_rate_probe_computes_what_it_says():
    """small_probe_mfma: eight accumulators, each `iters` times A x B with A[i][k] = 0.25 + (i & 7) / 1000 and
    B = 0.75, so D[i][j] = iters * 4 * 0.75 * A[i]; a lane holds rows 4q .. 4q+3 and stores the sum over its 32 values."""
    wgs, iters = 3, 5
    g = Guarded(wgs * 256)
    S.small_probe_mfma(g.t, wgs, iters)
    got = g.check().reshape(wgs, 4, 64)
    lane = np.arange(64)
    q = lane // 16
    rows = np.stack([4 * q + r for r in range(4)])                   # rows held by a lane
    ref = (8 * iters * 4 * 0.75 * (0.25 + (rows & 7) / 1000.0).sum(axis=0)).astype(np.float32)
    assert np.allclose(got, ref[None, None, :], rtol=1e-5, atol=0)


def test_matrix_and_vector_probe_computes_what_it_says():
    """small_probe_mfma_valu: four accumulators, each 4 * iters times A x B as above, and valu * iters multiply-adds
    a * b spread over eight registers, with a = 0.25 + (lane & 7) / 1000 and b = 0.75."""
    wgs, iters = 2, 3
    lane = np.arange(64)
    q = lane // 16
    rows = np.stack([4 * q + r for r in range(4)])
    for valu in (0, 32, 64, 96):
        g = Guarded(wgs * 256)
        S.small_probe_mfma_valu(g.t, wgs, iters, valu)
        got = g.check().reshape(wgs, 4, 64)
        ref = 4 * 4 * iters * 4 * 0.75 * (0.25 + (rows & 7) / 1000.0).sum(axis=0) + valu * iters * (0.25 + (lane & 7) / 1000.0) * 0.75
        assert np.allclose(got, ref.astype(np.float32)[None, None, :], rtol=1e-5, atol=0), valu
    with pytest.raises(RuntimeError):
        S.small_probe_mfma_valu(g.t, wgs, iters, 7)


# ------------------------------------------------------------------ seeded random geometries

def _random_geometry(rng, max_hw=34):
    kh, kw = int(rng.choice([1, 1, 3, 3, 3, 2, 5])), int(rng.choice([1, 1, 3, 3, 3, 2, 4]))
    if rng.random() < 0.6:
        kw = kh
    stride = int(rng.choice([1, 1, 1, 2, 2, 3]))
    H, W = int(rng.integers(kh, max_hw)), int(rng.integers(kw, max_hw))
    pad = (int(rng.integers(0, kh)), int(rng.integers(0, kh)), int(rng.integers(0, kw)), int(rng.integers(0, kw)))
    return H, W, kh, kw, stride, pad


@pytest.mark.parametrize("seed", range(48))
def test_conv2d_random_geometries(seed):
    """Channel counts, image sizes, windows, strides and paddings drawn from a seeded generator: whatever kernel the
    dispatcher picks for the geometry has to agree with the definition."""
    rng = np.random.default_rng(9000 + seed)
    Ci = int(rng.choice([1, 3, 8, 16, 16, 32, 48, 64, 128]))
    Co = int(rng.choice([8, 10, 16, 16, 32, 48, 64, 128]))
    H, W, kh, kw, stride, pad = _random_geometry(rng)
    N = int(rng.integers(1, 6)) if seed % 4 else int(rng.integers(20, 70))
    x = (rng.random((N, Ci, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((Co, Ci, kh, kw), dtype=np.float32) * 2 - 1).astype(np.float32)
    got = run_conv(x, w, stride, pad)
    assert_close(got, O.conv2d(x, w, stride, pad), Ci * kh * kw,
                 f"conv N={N} {Ci}->{Co} {H}x{W} k={kh}x{kw} s={stride} pad={pad}")


@pytest.mark.parametrize("seed", range(32))
def test_window_layers_random_geometries(seed):
    rng = np.random.default_rng(9500 + seed)
    C = int(rng.choice([3, 8, 16, 16, 32, 64, 80]))
    Cb = _blk(C)
    H, W, kh, kw, stride, pad = _random_geometry(rng, 40)
    N = int(rng.integers(1, 5)) if seed % 3 else int(rng.integers(30, 90))
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    w = rng.standard_normal((C, 1, kh, kw)).astype(np.float32)
    Ho, Wo = O.out_dim(H, kh, stride, pad[0], pad[1]), O.out_dim(W, kw, stride, pad[2], pad[3])
    xb = dev(O.pack(x, Cb))
    what = f"N={N} C={C} {H}x{W} k={kh}x{kw} s={stride} pad={pad}"
    g = Guarded(N * C * Ho * Wo)
    S.small_dwconv2d(xb, dev(O.pack_dw_filter(w, Cb)), g.t, N, C, H, W, kh, kw, stride, pad, Cb)
    assert_close(O.unpack(g.check(), (N, C, Ho, Wo), Cb), O.dwconv2d(x, w, stride, pad), kh * kw, "dw " + what)
    g = Guarded(N * C * Ho * Wo)
    S.small_pool2d(xb, g.t, N, C, H, W, kh, kw, stride, pad, Cb, S.POOL_MAX)
    assert_bits(O.unpack(g.check(), (N, C, Ho, Wo), Cb), O.pool2d(x, (kh, kw), stride, pad, "max"), "max pool " + what)
    g = Guarded(N * C * Ho * Wo)
    S.small_pool2d(xb, g.t, N, C, H, W, kh, kw, stride, pad, Cb, S.POOL_AVG)
    assert_close(O.unpack(g.check(), (N, C, Ho, Wo), Cb), O.pool2d(x, (kh, kw), stride, pad, "avg"), kh * kw, "avg pool " + what)
