"""Pins for the oracle's remaining Table 2 layers: group convolution (partial-channel reduction),
batch normalization (single-element FMA) and nearest-neighbour upsampling (CPU only)."""
import numpy as np
import pytest
import torch

from oracle import oracle as O


# ---------------------------------------------------------------- group convolution

@pytest.mark.parametrize("Ci,F_C,S_C,K,s,pad", [(8, 2, 2, 3, 1, (1, 1, 1, 1)), (12, 4, 4, 2, 2, (0, 1, 0, 1)),
                                                 (6, 6, 6, 5, 1, (0, 0, 0, 0)), (6, 1, 1, 1, 1, (1, 1, 1, 1))])
def test_group_conv_disjoint_groups_equal_library_grouped_conv(Ci, F_C, S_C, K, s, pad):
    """S_C = F_C: the usual grouped convolution (Section 3.2, partial channel reductions)."""
    rng = np.random.default_rng(31)
    G = (Ci - F_C) // S_C + 1
    x = rng.standard_normal((2, Ci, 9, 7)).astype(np.float32)
    w = rng.standard_normal((G * K, F_C, 3, 3)).astype(np.float32)
    xp = torch.nn.functional.pad(torch.from_numpy(x).double(), (pad[2], pad[3], pad[0], pad[1]))
    ref = torch.nn.functional.conv2d(xp, torch.from_numpy(w).double(), stride=s, groups=G).float().numpy()
    got = O.group_conv2d(x, w, F_C, S_C, K, s, pad)
    assert got.shape == ref.shape
    np.testing.assert_allclose(got, ref, rtol=0, atol=2e-6)


def test_group_conv_overlapping_groups_are_per_group_full_convolutions():
    """S_C < F_C: group g is a full-channel convolution over channels g*S_C .. g*S_C + F_C - 1 (already pinned),
    and its K outputs land at channels g*K .. g*K + K - 1."""
    rng = np.random.default_rng(32)
    Ci, F_C, S_C, K = 10, 4, 2, 3
    G = (Ci - F_C) // S_C + 1
    assert G == 4
    x = rng.integers(-5, 6, (2, Ci, 6, 8)).astype(np.float32)
    w = rng.integers(-3, 4, (G * K, F_C, 3, 3)).astype(np.float32)
    got = O.group_conv2d(x, w, F_C, S_C, K, 1, (1, 1, 1, 1))
    for g in range(G):
        ref = O.conv2d(x[:, g * S_C:g * S_C + F_C], w[g * K:(g + 1) * K], 1, (1, 1, 1, 1))
        assert np.array_equal(got[:, g * K:(g + 1) * K], ref)


def test_group_conv_special_cases():
    rng = np.random.default_rng(33)
    x = rng.integers(-4, 5, (1, 6, 5, 5)).astype(np.float32)
    # one group over all channels == convolution; one channel per group and one filter == depthwise
    w = rng.integers(-2, 3, (7, 6, 3, 3)).astype(np.float32)
    assert np.array_equal(O.group_conv2d(x, w, 6, 6, 7, 1, (1, 1, 1, 1)), O.conv2d(x, w, 1, (1, 1, 1, 1)))
    wd = rng.integers(-2, 3, (6, 1, 3, 3)).astype(np.float32)
    assert np.array_equal(O.group_conv2d(x, wd, 1, 1, 1, 2, (0, 1, 0, 1)), O.dwconv2d(x, wd, 2, (0, 1, 0, 1)))


def test_group_conv_matches_algorithm_1_on_blocked_layouts():
    """O2 (the literal loop nest on the blocked layouts) == O1 for a partial-channel reduction."""
    rng = np.random.default_rng(34)
    Ci, F_C, S_C, K = 8, 4, 4, 4
    G = 2
    x = rng.integers(-4, 5, (2, Ci, 6, 7)).astype(np.float32)
    w = rng.integers(-3, 4, (G * K, F_C, 3, 3)).astype(np.float32)
    ref = O.group_conv2d(x, w, F_C, S_C, K, 1, (1, 1, 1, 1))
    wb = O.pack_filter(w, 4, 2)          # [Co/4][F_C/2][3][3][2][4]: G_b = 1, K_b = 4, F_Cb = 2
    yb, (oc, oh, ow) = O.abstract_layer_blocked("fma", O.pack(x, 4), wb, 2, Ci, 6, 7, 3, 3, F_C, 1, 1, S_C, K,
                                                (1, 1, 1, 1), Icb=4, G_b=1, K_b=4, F_Cb=2, O_wb=3)
    assert (oc, oh, ow) == (8, 6, 7)
    assert np.array_equal(O.unpack(yb, ref.shape, 4), ref)


# ---------------------------------------------------------------- batch normalization

def test_batchnorm_equals_library_inference_batchnorm_with_folded_statistics():
    rng = np.random.default_rng(35)
    x = rng.standard_normal((3, 5, 4, 6)).astype(np.float32)
    gamma, beta = rng.standard_normal(5), rng.standard_normal(5)
    mean, var, eps = rng.standard_normal(5), rng.random(5) + 0.5, 1e-5
    ref = torch.nn.functional.batch_norm(torch.from_numpy(x).double(), torch.from_numpy(mean), torch.from_numpy(var),
                                         torch.from_numpy(gamma), torch.from_numpy(beta), False, 0.0, eps).numpy()
    scale = gamma / np.sqrt(var + eps)
    shift = beta - mean * scale
    got = O.batchnorm(x, scale.astype(np.float32), shift.astype(np.float32))
    np.testing.assert_allclose(got, ref, rtol=0, atol=1e-6)


def test_batchnorm_closed_forms():
    rng = np.random.default_rng(36)
    x = rng.integers(-8, 9, (2, 3, 4, 5)).astype(np.float32)
    one, zero = np.ones(3, np.float32), np.zeros(3, np.float32)
    assert np.array_equal(O.batchnorm(x, one, zero), x)
    assert np.array_equal(O.batchnorm(x, zero, np.array([1, 2, 3], np.float32)),
                          np.broadcast_to(np.array([1, 2, 3], np.float32)[None, :, None, None], x.shape))
    # exact in fp32 for small integers: per-channel scale and shift
    sc, sh = np.array([2, -1, 0.5], np.float32), np.array([1, 0, -3], np.float32)
    assert np.array_equal(O.batchnorm(x, sc, sh), x * sc[None, :, None, None] + sh[None, :, None, None])
    # one rounding: x * s + t with an inexact product
    xs = np.full((1, 1, 1, 1), 1 + 2**-12, np.float32)
    s1, t1 = np.array([1 + 2**-12], np.float32), np.array([-1.0], np.float32)
    exact = float(np.float64(xs[0, 0, 0, 0]) * np.float64(s1[0]) + np.float64(t1[0]))
    assert O.batchnorm(xs, s1, t1)[0, 0, 0, 0] == np.float32(exact)


# ---------------------------------------------------------------- upsampling

@pytest.mark.parametrize("fh,fw", [(1, 1), (2, 2), (3, 1), (2, 5)])
def test_upsample_is_element_repetition(fh, fw):
    rng = np.random.default_rng(37)
    x = rng.standard_normal((2, 3, 4, 5)).astype(np.float32)
    got = O.upsample(x, fh, fw)
    assert np.array_equal(got, np.repeat(np.repeat(x, fh, axis=2), fw, axis=3))
    ref = torch.nn.functional.interpolate(torch.from_numpy(x), scale_factor=(fh, fw), mode="nearest").numpy()
    assert np.array_equal(got, ref)
    # every fh x fw block of the output is constant and strided sampling gives the input back
    assert np.array_equal(got[:, :, ::fh, ::fw], x)


def test_run_network_with_table2_ops_matches_a_library_composition():
    """The oracle's network runner on a table with batch normalization, upsampling and a group convolution against
    the same composition of a library's CPU ops in fp64."""
    import torch
    import torch.nn.functional as F
    from workloads.nets import Layer, Network, IN, OUT
    from oracle import oracle as O
    net = Network("table2_probe", 8, 6, 5)
    net.layers = [
        Layer("bn", 8, 8, 6, 5, src=IN, dst=0, w=0),
        Layer("relu", 8, 8, 6, 5, src=0, dst=0),
        Layer("upsample", 8, 8, 6, 5, 2, 3, src=0, dst=1),
        Layer("gconv", 8, 6, 12, 15, 3, 3, 2, (1, 0, 1, 1), src=1, dst=OUT, w=1, F_C=4, S_C=4, Cob=6),
    ]
    rng = np.random.default_rng(5)
    x = rng.standard_normal((2, 8, 6, 5)).astype(np.float32)
    bn = np.stack([rng.random(8) + 0.5, rng.standard_normal(8)]).astype(np.float32)
    w = rng.standard_normal((6, 4, 3, 3)).astype(np.float32)
    got = O.run_network(net, x, [bn, w])
    t = torch.from_numpy(x).double() * torch.from_numpy(bn[0]).double().view(1, 8, 1, 1) + torch.from_numpy(bn[1]).double().view(1, 8, 1, 1)
    t = t.float().double().clamp_min(0)                       # every layer's result is rounded to fp32
    t = F.interpolate(t, scale_factor=(2, 3), mode="nearest")
    t = F.conv2d(F.pad(t, (1, 1, 1, 0)), torch.from_numpy(w).double(), stride=2, groups=2)
    assert got.shape == tuple(t.shape) == (2, 6, 6, 8)
    assert np.allclose(got, t.numpy(), rtol=0, atol=1e-5)
