"""The C-ABI library loads and exports every symbol include/small.h declares (no GPU needed:
only host-side entry points are called here)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    from paper_2303_04769_amd import binding
    return binding.load()


def _declared(header="small.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(small_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    from paper_2303_04769_amd import binding
    names = _declared()
    assert len(names) == 36 and set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None
    # the benchmark's probe is a library and a header of its own, outside the layer ABI
    assert _declared("small_probe.h") == ["small_probe_mfma", "small_probe_mfma_valu"] and not hasattr(lib, "small_probe_mfma")
    assert binding.load_probe().small_probe_mfma is not None and binding.load_probe().small_probe_mfma_valu is not None
    assert sorted(os.listdir(os.path.join(ROOT, "include"))) == ["small.h", "small_probe.h"]


def test_out_dim_and_strerror(lib):
    assert lib.small_out_dim(32, 3, 1, 1, 1) == 32
    assert lib.small_out_dim(56, 3, 2, 0, 0) == 27
    assert lib.small_out_dim(49, 10, 2, 4, 5) == 25
    assert lib.small_out_dim(2, 3, 1, 0, 0) == 0
    assert lib.small_strerror(0) == b"ok"
    assert b"overlap" in lib.small_strerror(4)


def test_argument_errors_are_reported_before_any_launch(lib):
    from paper_2303_04769_amd.binding import small_pad
    pad = small_pad(1, 1, 1, 1)
    fake = C.c_void_p(0x1000)     # never dereferenced: every call below fails validation first
    assert lib.small_relu(None, fake, 16, None) == 1
    assert lib.small_conv2d(fake, fake, fake, 1, 16, 16, 8, 8, 3, 3, 1, pad, 16, 16, None) == 4      # alias
    assert lib.small_conv2d(fake, fake, C.c_void_p(0x10000000), 1, 16, 24, 8, 8, 3, 3, 1, pad, 16, 16, None) == 2
    assert lib.small_conv2d(fake, fake, C.c_void_p(0x10000000), 1, 128, 128, 8, 8, 3, 3, 1, pad, 128, 16, None) == 3
    assert lib.small_conv2d(fake, fake, C.c_void_p(0x10000000), 0, 16, 16, 8, 8, 3, 3, 1, pad, 16, 16, None) == 2
    assert lib.small_pool2d(fake, C.c_void_p(0x10000000), 1, 16, 2, 2, 3, 3, 1, small_pad(0, 0, 0, 0), 16, 0, None) == 2
    assert lib.small_pool2d(fake, C.c_void_p(0x10000000), 1, 16, 8, 8, 3, 3, 1, pad, 16, 7, None) == 2
    assert lib.small_pack(fake, fake, 1, 16, 4, 4, 16, None) == 4
    # a padding as large as the window on its axis is refused (a window entirely in the padding has no maximum / mean)
    far0 = C.c_void_p(0x10000000)
    for bad in (small_pad(3, 0, 0, 0), small_pad(0, 3, 0, 0), small_pad(0, 0, 3, 0), small_pad(1, 1, 1, 5)):
        assert lib.small_conv2d(fake, fake, far0, 1, 16, 16, 8, 8, 3, 3, 1, bad, 16, 16, None) == 2
        assert lib.small_dwconv2d(fake, fake, far0, 1, 16, 8, 8, 3, 3, 1, bad, 16, None) == 2
        assert lib.small_pool2d(fake, far0, 1, 16, 8, 8, 3, 3, 1, bad, 16, 0, None) == 2
    # quantized layers: parameter ranges and the int32 bound on the reduction length
    from paper_2303_04769_amd.binding import small_quant
    far = C.c_void_p(0x10000000)
    ok = small_quant(128, 128, 128, 1 << 20, 30, 0, 255)
    q = lambda **k: C.byref(small_quant(*[k.get(f, getattr(ok, f)) for f, _ in small_quant._fields_]))
    conv = lambda qq, Ci=16, k=3: lib.small_conv2d_u8(fake, fake, far, 1, Ci, 16, 8, 8, k, k, 1, pad, 16, 16, qq, None, None)
    assert conv(None) == 1
    assert conv(q(zx=256)) == 8 and conv(q(zw=-1)) == 8 and conv(q(shift=32)) == 8 and conv(q(mult=-1)) == 8
    assert conv(q(lo=200, hi=100)) == 8 and conv(q(hi=256)) == 8
    assert conv(C.byref(ok), Ci=3680) == 8            # K = 33120: K * 255^2 >= 2^31
    assert lib.small_conv2d_u8(fake, fake, fake, 1, 16, 16, 8, 8, 3, 3, 1, pad, 16, 16, C.byref(ok), None, None) == 4
    assert lib.small_conv2d_u8(fake, fake, far, 1, 16, 16, 8, 8, 3, 3, 1, pad, 16, 16, C.byref(ok), C.c_void_p(0x2004), None) == 2
    assert lib.small_relu_u8(fake, far, 16, 256, None) == 2
    assert lib.small_pool2d_u8(fake, far, 1, 16, 8, 8, 3, 3, 1, pad, 16, 5, None) == 2


def test_workspace_follows_the_buffer_sharing_rule(lib, golden):
    """Section 'Memory Usage Comparison': only the largest buffers that are live together are
    allocated. The printed autoencoder row pins the formula bytes = 4 * (params + largest in+out):
    4 * (133120 + 2*128) B = 0.5088 MiB, printed as 0.509."""
    import workloads as WL
    from paper_2303_04769_amd import binding as B
    g = golden("paper_constants.txt")
    assert round(4 * (g["params"][3] + 2 * 128) / 2**20, 3) == g["memory_small_fp32_mib"][0]

    def ws(net, N):
        table = B.make_layer_table(net.layers, [None] * len(net.wshapes))
        for k, L in enumerate(net.layers):      # validation wants non-NULL filters; never dereferenced
            if L.w is not None:
                table[k].filt = 0x1000
        return B.small_network_workspace(table, N, net.C0, net.H0, net.W0)

    a = WL.audio_cnn()
    # chain network: two ping-pong slots, each as large as the largest tensor written to it
    assert ws(a, 1) == 2 * 64 * 25 * 5 * 4
    assert ws(a, 7) == 2 * 7 * 64 * 25 * 5 * 4
    r = WL.residual_cnn()
    # residual block: x, a, b live together (+ the projected shortcut from stage 2 on)
    sizes = {}
    for L in r.layers:
        if L.dst >= 0:
            sizes[L.dst] = max(sizes.get(L.dst, 0), L.Co * L.Ho * L.Wo * 4)
    assert ws(r, 1) == sum((v + 255) // 256 * 256 for v in sizes.values())
    assert ws(r, 1) <= 4 * 16 * 32 * 32 * 4
    # launches after cross-layer fusion: residual CNN = 9 convs (ReLU / add+ReLU folded) + the head (avgpool + dense)
    table = B.make_layer_table(r.layers, [None] * len(r.wshapes))
    heads = B.small_network_launches(table)
    assert len(r.layers) == 21 and len(heads) == 10
    assert [r.layers[h].op for h in heads] == ["conv"] * 9 + ["avgpool"]
    # image-resident runs: at batches that fill the chip in whole rounds the whole network (first layer, eight
    # convolutions with their ReLU / residual add, 72 KB + 72 KB of padded tensors at the widest point, and the pooling
    # + fully connected head) is ONE launch; never with the OFF flag,
    # always with the ON flag; the batch-independent list above stays as it is
    tr = B.make_layer_table(r.layers, [None] * len(r.wshapes))
    for k, L in enumerate(r.layers):
        if L.w is not None:
            tr[k].filt = 0x1000
    at = lambda N, flags=0: B.small_network_launches_at(tr, N, r.C0, r.H0, r.W0, flags)
    assert at(256) == [0] == at(144) == at(200) == at(448) == at(512) == at(1, B.SMALL_RUN_RESIDENT_ON) == at(1000, B.SMALL_RUN_RESIDENT_ON)
    assert at(1) == at(143) == at(257) == at(447) == at(513) == at(1024) == at(256, B.SMALL_RUN_RESIDENT_OFF) == B.small_network_launches(tr)
    # too little arithmetic per layer for a workgroup-per-image run: the depthwise-separable networks stay layer by
    # layer unless forced
    for other in (WL.dsep_cnn(), a):
        to = B.make_layer_table(other.layers, [None] * len(other.wshapes))
        for k, L in enumerate(other.layers):
            if L.w is not None:
                to[k].filt = 0x1000
        plan = lambda N, flags=0: B.small_network_launches_at(to, N, other.C0, other.H0, other.W0, flags)
        # layer by layer, except that consecutive depthwise + pointwise blocks on small images (known only with the
        # geometry) are one launch: the nine blocks from the 6x6 images on with the head (the audio CNN's 25x5 images are too large)
        # (from the 12x12 images on when a workgroup per image is one round of workgroups, else from the 3x3 images on,
        # several images per workgroup)
        expect = B.small_network_launches(to) if other is a else [0, 2, 6, 10, 14, 18, 22, 26]
        assert plan(512) == expect and set(expect) <= set(B.small_network_launches(to))
        if other is not a:
            assert plan(1, B.SMALL_RUN_RESIDENT_OFF) == [0, 2, 6, 10] == plan(256, B.SMALL_RUN_RESIDENT_OFF) and plan(257) == expect == plan(4096)
        assert len(plan(256, B.SMALL_RUN_RESIDENT_ON)) < len(plan(512))
        # the audio CNN (0.27 M multiply-adds per layer) is taken in one round, where it measures a few percent faster
        assert (plan(256) == [0]) == (other is a) and (plan(256) == [0, 2, 6, 10]) == (other is not a)
    assert at(256, B.SMALL_RUN_PLAIN_INPUT) == [0] == at(2, B.SMALL_RUN_PLAIN_INPUT | B.SMALL_RUN_RESIDENT_ON)
    n = C.c_int(0)
    assert lib.small_network_launches_at(tr, len(tr), 256, r.C0, r.H0, r.W0, 16, None, C.byref(n)) == 2    # unknown flag
    # plain output: only where the blocked result is the plain one (the classifiers' logits), not for a feature map
    assert at(256, B.SMALL_RUN_PLAIN_OUTPUT | B.SMALL_RUN_PLAIN_INPUT) == [0]
    s1 = WL.single_conv_relu()
    ts = B.make_layer_table(s1.layers, [None] * len(s1.wshapes))
    ts[0].filt = 0x1000
    assert lib.small_network_launches_at(ts, len(ts), 4, s1.C0, s1.H0, s1.W0, B.SMALL_RUN_PLAIN_OUTPUT, None, C.byref(n)) == 7
    assert lib.small_network_launches_at(tr, len(tr), 256, r.C0, r.H0, r.W0, 0, None, None) == 1
    # planning looks ahead over layers that have not been validated yet: a bad buffer id further down is an error
    # code, whatever the flags
    bad = B.make_layer_table(r.layers, [None] * len(r.wshapes))
    for k, L in enumerate(r.layers):
        if L.w is not None:
            bad[k].filt = 0x1000
    bad[5].src2 = 1000          # the first residual add
    for flags in (0, B.SMALL_RUN_RESIDENT_ON, B.SMALL_RUN_RESIDENT_OFF):
        assert lib.small_network_launches_at(bad, len(bad), 256, r.C0, r.H0, r.W0, flags, None, C.byref(n)) == 7
        assert lib.small_network_workspace(bad, len(bad), 256, r.C0, r.H0, r.W0, C.byref(C.c_size_t())) == 7
    bad[5].src2 = r.layers[5].src2
    bad[11].dst = -7
    assert lib.small_network_launches_at(bad, len(bad), 256, r.C0, r.H0, r.W0, 0, None, C.byref(n)) == 7
    ta = B.make_layer_table(a.layers, [None] * len(a.wshapes))
    # depthwise + ReLU + pointwise + ReLU blocks are one launch each
    assert [a.layers[h].op for h in B.small_network_launches(ta)] == ["conv"] + ["dw"] * 4 + ["avgpool"]
    d = WL.dsep_cnn()
    td = B.make_layer_table(d.layers, [None] * len(d.wshapes))
    # all 13 blocks are fused (the first, 8 -> 16 channels, on the vector units)
    assert [d.layers[h].op for h in B.small_network_launches(td)] == ["conv"] + ["dw"] * 13 + ["avgpool"]
    # the dense-only autoencoder is one run of pointwise layers: a single launch; workspace = two ping-pong rows
    e = WL.dense_autoencoder()
    te = B.make_layer_table(e.layers, [None] * len(e.wshapes))
    assert len(e.layers) == 19 and B.small_network_launches(te) == [0]
    assert ws(e, 3) == 2 * 3 * 128 * 4
    # malformed tables
    t = B.make_layer_table(a.layers, [None] * len(a.wshapes))
    assert lib.small_network_workspace(t, len(t), 1, a.C0, a.H0, a.W0, C.byref(C.c_size_t())) == 1   # NULL filter
    for k, L in enumerate(a.layers):
        if L.w is not None:
            t[k].filt = 0x1000
    t[3].Cib = 8
    assert lib.small_network_workspace(t, len(t), 1, a.C0, a.H0, a.W0, C.byref(C.c_size_t())) == 7


def _table(layers, n_w):
    from paper_2303_04769_amd import binding as B
    t = B.make_layer_table(layers, [None] * n_w)
    for k, L in enumerate(layers):
        if L.w is not None:
            t[k].filt = 0x1000          # validation wants non-NULL filters; never dereferenced
    return t


def test_a_folded_add_never_leaves_the_output_buffer_unwritten(lib):
    """conv -> OUT; add(OUT, slot) -> slot: folding the add into the convolution's store phase would write the sum into
    the slot and leave the caller's output buffer, which receives every write to SMALL_BUF_OUT, unwritten. The planner
    keeps the two apart, with and without image-resident runs; when OUT is rewritten later the fold is allowed."""
    from paper_2303_04769_amd import binding as B
    from workloads.nets import Layer, IN, OUT
    p1 = (1, 1, 1, 1)
    layers = [
        Layer("conv", 16, 16, 8, 8, 3, 3, 1, p1, src=IN, dst=0, w=0),
        Layer("conv", 16, 16, 8, 8, 1, 1, 1, (0, 0, 0, 0), src=IN, dst=1, w=1),
        Layer("conv", 16, 16, 8, 8, 3, 3, 1, p1, src=1, dst=OUT, w=0),
        Layer("add", 16, 16, 8, 8, src=OUT, src2=0, dst=0),
    ]
    t = _table(layers, 2)
    assert B.small_network_launches(t) == [0, 1, 2, 3]
    for flags in (B.SMALL_RUN_RESIDENT_OFF, B.SMALL_RUN_RESIDENT_ON):
        at = B.small_network_launches_at(t, 3, 16, 8, 8, flags)
        assert at[-1] == 3, (flags, at)          # the add is a launch of its own (the convolution before it may be
                                                 # the end of an image-resident run, whose last result is written)
    # OUT rewritten afterwards (and not read in between): the convolution's own result is dead, the fold is fine
    layers2 = layers + [Layer("conv", 16, 16, 8, 8, 1, 1, 1, (0, 0, 0, 0), src=0, dst=OUT, w=1)]
    assert B.small_network_launches(_table(layers2, 2)) == [0, 1, 2, 4]


def test_launch_list_applies_the_geometry_fallbacks_of_the_run(lib):
    """small_network_launches_at lists what a run with this input shape launches: an average pooling that does not
    cover the whole image is not fused with the fully connected layer after it, although the table alone (the
    batch-independent list) cannot tell."""
    from paper_2303_04769_amd import binding as B
    from workloads.nets import Layer, IN, OUT
    layers = [
        Layer("conv", 16, 16, 8, 8, 3, 3, 1, (1, 1, 1, 1), src=IN, dst=0, w=0),
        Layer("avgpool", 16, 16, 8, 8, 4, 4, 8, src=0, dst=1),
        Layer("dense", 16, 16, 1, 1, 1, 1, 1, src=1, dst=OUT, w=1, Ho=1, Wo=1),
    ]
    assert (layers[1].Ho, layers[1].Wo) == (1, 1)
    t = _table(layers, 2)
    assert B.small_network_launches(t) == [0, 1]
    assert B.small_network_launches_at(t, 2, 16, 8, 8, B.SMALL_RUN_RESIDENT_OFF) == [0, 1, 2]
    # the whole-image window is fused
    layers[1] = Layer("avgpool", 16, 16, 8, 8, 8, 8, 1, src=0, dst=1)
    assert B.small_network_launches_at(_table(layers, 2), 2, 16, 8, 8, B.SMALL_RUN_RESIDENT_OFF) == [0, 1]
    # a garbage buffer id is an error code, not a shift by it
    t = _table(layers, 2)
    t[0].src = 77
    n = C.c_int(0)
    assert lib.small_network_launches_at(t, len(t), 2, 16, 8, 8, 0, None, C.byref(n)) == 7


def test_batch_normalization_folds_into_the_convolution_before_it(lib):
    """conv, norm, [add], [ReLU]: one launch by the table; a run whose convolution kernel has no such epilogue (here: a
    window of 5 x 5) lists the layers one by one. A normalization that stands alone takes the ReLU after it."""
    from paper_2303_04769_amd import binding as B
    from workloads.nets import Layer, IN, OUT
    p1 = (1, 1, 1, 1)

    def block(k, pad):
        return [
            Layer("conv", 32, 32, 10, 10, k, k, 1, pad, src=IN, dst=0, w=0),
            Layer("bn", 32, 32, 10, 10, src=0, dst=0, w=1),
            Layer("add", 32, 32, 10, 10, src=0, src2=IN, dst=0),
            Layer("relu", 32, 32, 10, 10, src=0, dst=0),
            Layer("bn", 32, 32, 10, 10, src=0, dst=1, w=1),
            Layer("relu", 32, 32, 10, 10, src=1, dst=1),
            Layer("upsample", 32, 32, 10, 10, 2, 2, src=1, dst=OUT),
        ]
    t3 = _table(block(3, p1), 2)
    assert B.small_network_launches(t3) == [0, 4, 6]
    assert B.small_network_launches_at(t3, 2, 32, 10, 10, B.SMALL_RUN_RESIDENT_OFF) == [0, 4, 6]
    t5 = _table(block(5, (2, 2, 2, 2)), 2)
    assert B.small_network_launches(t5) == [0, 4, 6]                      # the table alone cannot tell
    assert B.small_network_launches_at(t5, 2, 32, 10, 10, 0) == [0, 1, 2, 3, 4, 6]
    # workspace: the upsampled tensor goes to OUT, slots 0 and 1 hold 32 x 10 x 10
    assert B.small_network_workspace(t3, 2, 32, 10, 10) == 2 * 2 * 32 * 100 * 4
    # malformed: a group convolution whose groups do not tile the channels, an upsampling factor of zero
    bad = _table([Layer("gconv", 32, 32, 10, 10, 3, 3, 1, p1, src=IN, dst=OUT, w=0, F_C=12, S_C=16)], 1)
    assert lib.small_network_workspace(bad, 1, 1, 32, 10, 10, C.byref(C.c_size_t())) == 7
    bad = _table([Layer("upsample", 32, 32, 10, 10, 2, 2, src=IN, dst=OUT)], 0)
    bad[0].kw = 0
    assert lib.small_network_workspace(bad, 1, 1, 32, 10, 10, C.byref(C.c_size_t())) == 7
