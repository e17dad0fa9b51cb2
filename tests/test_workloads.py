"""The synthetic stand-in networks: shapes, weight counts, buffer plan (CPU only)."""
import numpy as np

import workloads as WL
from oracle import oracle as O


def test_weight_and_mac_counts():
    r, d, a = WL.residual_cnn(), WL.dsep_cnn(), WL.audio_cnn()
    assert (r.n_weights, d.n_weights, a.n_weights) == (77360, 208112, 22016)
    assert r.macs_per_image() == 12_501_632 and sum(L.op == "conv" for L in r.layers) == 9
    assert d.macs_per_image() == 2_424_128
    assert WL.dsep_cnn(1).macs_per_image() > 7_000_000
    assert WL.single_conv_relu().macs_per_image() * 2 == 4_718_592
    # Table "tinyml_models": the autoencoder row prints 133120 parameters and a (1, 1, 128) input
    e = WL.dense_autoencoder()
    assert e.n_weights == 133120 == e.macs_per_image() and (e.C0, e.H0, e.W0) == (128, 1, 1)
    assert [L.Co for L in e.layers if L.op == "dense"] == [128] * 4 + [8] + [128] * 5


def test_spatial_sequences_and_paddings():
    d = WL.dsep_cnn()
    hs = [L.Ho for L in d.layers if L.op == "dw"]
    assert hs == [24, 12, 12, 6, 6, 3, 3, 3, 3, 3, 3, 2, 2]
    assert d.layers[0].pad == (0, 1, 0, 1) and d.layers[0].Ho == 48
    a = WL.audio_cnn()
    assert a.layers[0].pad == (4, 5, 1, 1) and (a.layers[0].Ho, a.layers[0].Wo) == (25, 5)
    r = WL.residual_cnn()
    s2 = [L for L in r.layers if L.op == "conv" and L.stride == 2 and L.kh == 3]
    assert [L.pad for L in s2] == [(0, 1, 0, 1)] * 2
    assert [L.pad for L in r.layers if L.op == "conv" and L.kh == 1] == [(0, 0, 0, 0)] * 2
    # on 3x3 inputs a stride-2 'same' 3x3 window pads 1 on each side -> 2x2
    dw12 = [L for L in d.layers if L.op == "dw"][11]
    assert dw12.H == 3 and dw12.pad == (1, 1, 1, 1) and dw12.Ho == 2


def test_no_reformat_invariant_and_buffer_plan():
    for net in (WL.residual_cnn(), WL.dsep_cnn(), WL.audio_cnn(), WL.dense_autoencoder(), WL.single_conv_relu()):
        block = {WL.nets.IN: WL.block_of(net.C0)}
        live = {}
        for L in net.layers:
            assert block[L.src] == L.Cib, (net.name, L)
            if L.op == "add":
                assert block[L.src2] == L.Cib
            if L.op in ("conv", "dw", "dense", "avgpool", "maxpool"):
                assert L.dst != L.src and L.dst != WL.nets.IN
            block[L.dst] = L.Cob
        assert net.layers[-1].dst == WL.nets.OUT


def test_network_oracle_runs_and_is_seeded():
    net = WL.audio_cnn()
    x, ws = WL.network_tensors(net, 2, WL.BASE_SEED + 4)
    x2, ws2 = WL.network_tensors(net, 2, WL.BASE_SEED + 4)
    assert np.array_equal(x, x2) and all(np.array_equal(a, b) for a, b in zip(ws, ws2))
    y = O.run_network(net, x, ws)
    assert y.shape == (2, 12) and np.isfinite(y).all() and np.abs(y).max() > 0
    # images are independent: batch of 2 == two batches of 1
    y0 = O.run_network(net, x[:1], ws)
    assert np.array_equal(y[:1], y0)


def test_residual_network_matches_torch_composition():
    """Third opinion on the network walk (buffer ids, skip branch): rebuild the residual CNN
    from torch CPU ops in fp64 and compare logits."""
    import torch
    import torch.nn.functional as F
    net = WL.residual_cnn()
    x, ws = WL.network_tensors(net, 2, 5)
    y = O.run_network(net, x, ws)
    t = [torch.from_numpy(w).double() for w in ws]
    h = F.relu(F.conv2d(torch.from_numpy(x).double(), t[0], padding=1))
    i = 1
    for s, proj in ((1, False), (2, True), (2, True)):
        hp = F.pad(h, (0, 1, 0, 1)) if s == 2 else F.pad(h, (1, 1, 1, 1))
        a = F.relu(F.conv2d(hp, t[i], stride=s))
        b = F.conv2d(a, t[i + 1], padding=1)
        sc = F.conv2d(h, t[i + 2], stride=s) if proj else h
        i += 3 if proj else 2
        h = F.relu(b + sc)
    logits = h.mean(dim=(2, 3)) @ t[i].reshape(10, 64).T
    np.testing.assert_allclose(y, logits.float().numpy(), rtol=0, atol=1e-4)


def test_autoencoder_matches_matrix_products():
    """The dense-only network is a chain of matrix products: rebuild it from numpy matmuls in fp64
    (a fully connected layer on a 1x1 image is y = W x) and compare."""
    net = WL.dense_autoencoder()
    x, ws = WL.network_tensors(net, 5, 11)
    y = O.run_network(net, x, ws)
    h = x.reshape(5, 128).astype(np.float64)
    for i, w in enumerate(ws):
        h = h @ w.reshape(w.shape[0], w.shape[1]).astype(np.float64).T
        if i + 1 < len(ws):
            h = np.maximum(h, 0.0)
    assert y.shape == (5, 128) and np.abs(y).max() > 0.01
    np.testing.assert_allclose(y, h.astype(np.float32), rtol=0, atol=1e-5)
    # the 8-wide code in the middle: the tensor after the fifth dense layer (+ ReLU) has 8 channels
    _, trace = O.run_network(net, x, ws, return_all=True)
    assert trace[9].shape[1] == 8 and (trace[9] >= 0).all() and trace[9].max() > 0
