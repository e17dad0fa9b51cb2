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
