"""GPU parity of the remaining Table 2 layers (batch normalization, nearest-neighbour upsampling, group
convolution) against the oracle, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2303_04769_amd as S
from oracle import oracle as O
from gpu_util import DEV, Guarded, assert_bits, assert_close, dev

pytestmark = pytest.mark.gpu


def _blk(c):
    return 16 if c % 16 == 0 else c


@pytest.mark.parametrize("N,C,H,W", [(2, 32, 13, 11), (1, 16, 56, 56), (3, 8, 5, 7), (2, 3, 9, 9), (5, 64, 1, 1),
                                     (64, 256, 14, 14)])
def test_batchnorm(N, C, H, W):
    rng = np.random.default_rng(41 + C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    scale = (rng.random(C) * 2 + 0.1).astype(np.float32)
    shift = rng.standard_normal(C).astype(np.float32)
    Cb = _blk(C)
    ref = O.batchnorm(x, scale, shift)
    g = Guarded(x.size)
    S.small_batchnorm(dev(O.pack(x, Cb)), dev(scale), dev(shift), g.t, N, C, H, W, Cb)
    assert_close(O.unpack(g.check(), x.shape, Cb), ref, 1, f"batchnorm {N}x{C}x{H}x{W}")
    # in place, and the identity parameters copy bit for bit
    t = dev(O.pack(x, Cb))
    S.small_batchnorm(t, dev(scale), dev(shift), t, N, C, H, W, Cb)
    assert_close(O.unpack(t.cpu().numpy(), x.shape, Cb), ref, 1, "batchnorm in place")
    g = Guarded(x.size)
    S.small_batchnorm(dev(O.pack(x, Cb)), dev(np.ones(C, np.float32)), dev(np.zeros(C, np.float32)), g.t, N, C, H, W, Cb)
    assert_bits(O.unpack(g.check(), x.shape, Cb), x, "batchnorm identity")


@pytest.mark.parametrize("N,C,H,W,fh,fw", [(2, 32, 7, 5, 2, 2), (1, 16, 20, 20, 3, 1), (3, 8, 4, 6, 2, 5), (2, 3, 5, 5, 2, 2),
                                           (1, 48, 9, 9, 1, 1), (32, 64, 28, 28, 2, 2)])
def test_upsample_bit_exact(N, C, H, W, fh, fw):
    rng = np.random.default_rng(43 + C)
    x = rng.standard_normal((N, C, H, W)).astype(np.float32)
    x.reshape(-1)[::97] = np.nan          # a copy: special values pass through
    x.reshape(-1)[1::89] = -0.0
    Cb = _blk(C)
    ref = O.upsample(x, fh, fw)
    g = Guarded(ref.size)
    S.small_upsample(dev(O.pack(x, Cb)), g.t, N, C, H, W, fh, fw, Cb)
    assert_bits(O.unpack(g.check(), ref.shape, Cb), ref, f"upsample {N}x{C}x{H}x{W} by {fh}x{fw}")


GROUP_CASES = [  # N, Ci, F_C, S_C, K, H, W, k, stride, pad, Cib, F_Cb, Cob
    (2, 32, 8, 8, 4, 9, 7, 3, 1, (1, 1, 1, 1), 16, 8, 16),       # 4 disjoint groups of 8 channels, 4 filters each
    (3, 64, 16, 16, 16, 6, 6, 3, 2, (0, 1, 0, 1), 16, 16, 16),   # one output block per group
    (2, 16, 4, 2, 3, 8, 8, 3, 1, (1, 1, 1, 1), 16, 4, 7),        # overlapping groups (S_C < F_C), 21 outputs in blocks of 7
    (2, 48, 1, 1, 1, 10, 10, 3, 1, (1, 1, 1, 1), 16, 1, 16),     # depthwise as a partial-channel reduction
    (2, 32, 32, 32, 24, 5, 5, 1, 1, (0, 0, 0, 0), 16, 16, 8),    # one group: a 1x1 convolution
    (1, 12, 6, 6, 5, 7, 9, 5, 2, (2, 2, 1, 1), 4, 3, 10),        # small blocks, odd window
    # whole 16-channel blocks per group: the matrix-core convolution kernels, every tile inside one group
    (2, 64, 32, 32, 32, 14, 13, 3, 1, (1, 1, 1, 1), 16, 16, 16),   # two groups of two blocks (64 x 32 tiles)
    (3, 48, 32, 16, 16, 9, 9, 3, 1, (1, 1, 1, 1), 16, 16, 16),     # overlapping groups: input blocks {0,1} and {1,2}
    (2, 128, 64, 64, 64, 7, 7, 1, 1, (0, 0, 0, 0), 16, 16, 16),    # 1x1, two input blocks per step (32 x 64 tiles)
    (2, 96, 32, 32, 16, 12, 12, 1, 1, (0, 0, 0, 0), 16, 16, 16),   # 1x1, three groups of one output block
    (40, 64, 32, 32, 32, 16, 16, 3, 1, (1, 1, 1, 1), 16, 16, 16),  # many images: the image-aligned persistent variant
    (5, 128, 32, 32, 48, 10, 10, 3, 2, (0, 1, 0, 1), 16, 16, 16),  # stride 2, four groups of three output blocks
    (8, 256, 32, 32, 32, 28, 28, 3, 1, (1, 1, 1, 1), 16, 16, 16),  # the sweep's group convolution on eight images
]


@pytest.mark.parametrize("case", GROUP_CASES)
def test_group_conv2d(case):
    N, Ci, F_C, S_C, K, H, W, k, s, pad, Cib, F_Cb, Cob = case
    G = (Ci - F_C) // S_C + 1
    rng = np.random.default_rng(abs(hash(case)) % 2**31)
    x = (rng.random((N, Ci, H, W), dtype=np.float32) * 2 - 1).astype(np.float32)
    w = (rng.random((G * K, F_C, k, k), dtype=np.float32) * 2 - 1).astype(np.float32)
    ref = O.group_conv2d(x, w, F_C, S_C, K, s, pad)
    g = Guarded(ref.size)
    S.small_group_conv2d(dev(O.pack(x, Cib)), dev(O.pack_filter(w, Cob, F_Cb)), g.t, N, Ci, F_C, S_C, K, H, W, k, k, s, pad,
                         Cib, F_Cb, Cob)
    assert_close(O.unpack(g.check(), ref.shape, Cob), ref, F_C * k * k, f"group conv {case}")


def test_group_conv_filters_packed_on_the_gpu():
    """small_pack_filter with Ci = F_C produces the layout small_group_conv2d reads."""
    N, Ci, F_C, S_C, K = 2, 32, 8, 8, 8
    rng = np.random.default_rng(45)
    x = rng.standard_normal((N, Ci, 6, 6)).astype(np.float32)
    w = rng.standard_normal((32, F_C, 3, 3)).astype(np.float32)
    wb = torch.empty(w.size, dtype=torch.float32, device=DEV)
    S.small_pack_filter(dev(w), wb, 32, F_C, 3, 3, 16, 8)
    ref = O.group_conv2d(x, w, F_C, S_C, K, 1, (1, 1, 1, 1))
    g = Guarded(ref.size)
    S.small_group_conv2d(dev(O.pack(x, 16)), wb, g.t, N, Ci, F_C, S_C, K, 6, 6, 3, 3, 1, (1, 1, 1, 1), 16, 8, 16)
    assert_close(O.unpack(g.check(), ref.shape, 16), ref, F_C * 9, "group conv, GPU-packed filter")


def test_table2_errors():
    t = torch.zeros(1024, dtype=torch.float32, device=DEV)
    for call in (lambda: S.small_group_conv2d(t, t, t, 1, 16, 6, 4, 2, 4, 4, 3, 3, 1, (1, 1, 1, 1), 16, 6, 4),   # (16 - 6) % 4 != 0
                 lambda: S.small_upsample(t, t, 1, 16, 4, 4, 0, 2, 16),
                 lambda: S.small_batchnorm(t, None, t, t, 1, 16, 4, 4, 16)):
        with pytest.raises(S.SmallError):
            call()


# ------------------------------------------------------------------ the same layers as ops of a layer table

def _run_table(net, x, ws, flags=0):
    N = x.shape[0]
    pn = S.PackedNetwork(net, ws, DEV)
    g = Guarded(pn.out_elems(N))
    pn.run_opt(pn.pack_input(dev(x)), g.t, N, flags)
    L = net.layers[-1]
    return O.unpack(g.check(), (N, L.Co, L.Ho, L.Wo), L.Cob), pn


def _bn_params(rng, C):
    return np.stack([(rng.random(C) * 1.5 + 0.25), rng.standard_normal(C) * 0.3]).astype(np.float32)


def _tensors(net, N, seed, bn_layers):
    """Seeded input and weights; the batch-normalization parameter sets ([2][C]: scale, shift) replace the drawn ones."""
    import workloads as WL
    x, ws = WL.network_tensors(net, N, seed)
    rng = np.random.default_rng(seed + 1)
    for w_index, C in bn_layers:
        ws[w_index] = _bn_params(rng, C)
    return x, ws


@pytest.mark.parametrize("N,C,H,W", [(3, 32, 12, 12), (2, 64, 9, 7), (20, 16, 32, 32)])
def test_residual_block_with_batch_normalization(N, C, H, W):
    """conv, norm, ReLU, conv, norm, add, ReLU on 16-channel blocks: both normalizations run in the store phase of
    the convolution before them (one launch each, asserted), the second together with the residual add and the ReLU."""
    from workloads.nets import Layer, Network, IN, OUT
    net = Network("bn_block", C, H, W)
    p1, z = (1, 1, 1, 1), (0, 0, 0, 0)
    net.wshapes = [((C, C, 3, 3), C * 9), ((2, C), 1), ((C, C, 3, 3), C * 9), ((2, C), 1)]
    net.layers = [
        Layer("conv", C, C, H, W, 3, 3, 1, p1, src=IN, dst=0, w=0),
        Layer("bn", C, C, H, W, src=0, dst=0, w=1),
        Layer("relu", C, C, H, W, src=0, dst=0),
        Layer("conv", C, C, H, W, 3, 3, 1, p1, src=0, dst=1, w=2),
        Layer("bn", C, C, H, W, src=1, dst=1, w=3),
        Layer("add", C, C, H, W, src=1, src2=IN, dst=1),
        Layer("relu", C, C, H, W, src=1, dst=1),
        Layer("maxpool", C, C, H, W, 1, 1, 1, z, src=1, dst=OUT),
    ]
    x, ws = _tensors(net, N, 7100 + C, [(1, C), (3, C)])
    got, pn = _run_table(net, x, ws, S.SMALL_RUN_RESIDENT_OFF)
    assert pn.launches_at(N, S.SMALL_RUN_RESIDENT_OFF) == [0, 3, 7]
    assert_close(got, O.run_network(net, x, ws), C * 9, f"residual block with batch normalization {N}x{C}x{H}x{W}")
    # image-resident runs do not take normalized layers: the same launches with them forced on
    got, _ = _run_table(net, x, ws, S.SMALL_RUN_RESIDENT_ON)
    assert_close(got, O.run_network(net, x, ws), C * 9, "the same with image-resident runs forced on")


def test_batch_normalization_after_kernels_without_that_epilogue():
    """A first layer on 3 channels (its kernel has no normalization epilogue) and a 5 x 5 convolution (the generic
    matrix-core kernel): the runner takes the fusion back and launches conv, norm (+ ReLU) as the table lists them;
    then nearest-neighbour upsampling, a group convolution and a normalization that stands alone."""
    from workloads.nets import Layer, Network, IN, OUT
    H = W = 40
    net = Network("bn_unfolded", 3, H, W)
    p1, p2, z = (1, 1, 1, 1), (2, 2, 2, 2), (0, 0, 0, 0)
    net.wshapes = [((16, 3, 3, 3), 27), ((2, 16), 1), ((32, 16, 5, 5), 400), ((2, 32), 1), ((32, 16, 3, 3), 144), ((2, 32), 1)]
    net.layers = [
        Layer("conv", 3, 16, H, W, 3, 3, 1, p1, src=IN, dst=0, w=0),
        Layer("bn", 16, 16, H, W, src=0, dst=0, w=1),
        Layer("relu", 16, 16, H, W, src=0, dst=0),
        Layer("maxpool", 16, 16, H, W, 2, 2, 2, z, src=0, dst=1),                     # 20 x 20
        Layer("conv", 16, 32, 20, 20, 5, 5, 1, p2, src=1, dst=0, w=2),
        Layer("bn", 32, 32, 20, 20, src=0, dst=0, w=3),
        Layer("upsample", 32, 32, 20, 20, 2, 3, src=0, dst=1),                       # 40 x 60
        Layer("gconv", 32, 32, 40, 60, 3, 3, 2, (0, 1, 0, 1), src=1, dst=0, w=4, F_C=16, S_C=16),   # two groups, 20 x 30
        Layer("bn", 32, 32, 20, 30, src=0, dst=2, w=5),                               # not in place
        Layer("relu", 32, 32, 20, 30, src=2, dst=2),
        Layer("add", 32, 32, 20, 30, src=2, src2=0, dst=OUT),
    ]
    N = 12
    x, ws = _tensors(net, N, 7200, [(1, 16), (3, 32), (5, 32)])
    got, pn = _run_table(net, x, ws)
    # conv | norm + ReLU | pool | conv | norm | upsample | group conv | norm + ReLU | add
    assert pn.launches_at(N) == [0, 1, 3, 4, 5, 6, 7, 8, 10], pn.launches_at(N)
    assert_close(got, O.run_network(net, x, ws), 400, "table with unfolded normalizations, upsampling and a group convolution")


def test_table2_ops_on_small_blocks():
    """8-channel tensors (one block of 8): normalization, upsampling and a group convolution with 4-channel groups run
    in the generic kernels."""
    from workloads.nets import Layer, Network, IN, OUT
    net = Network("table2_small_blocks", 8, 9, 7)
    net.wshapes = [((2, 8), 1), ((12, 4, 3, 3), 36)]
    net.layers = [
        Layer("bn", 8, 8, 9, 7, src=IN, dst=0, w=0),
        Layer("relu", 8, 8, 9, 7, src=0, dst=0),
        Layer("upsample", 8, 8, 9, 7, 2, 2, src=0, dst=1),
        Layer("gconv", 8, 12, 18, 14, 3, 3, 1, (1, 1, 1, 1), src=1, dst=OUT, w=1, F_C=4, S_C=2, Cob=12),   # 3 overlapping groups x 4 filters
    ]
    x, ws = _tensors(net, 3, 7300, [(0, 8)])
    got, pn = _run_table(net, x, ws)
    assert pn.launches_at(3) == [0, 2, 3]
    assert_close(got, O.run_network(net, x, ws), 36, "table 2 ops on 8-channel blocks")
