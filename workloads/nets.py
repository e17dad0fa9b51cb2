"""Layer tables for the synthetic stand-in networks (data only, no layer arithmetic).

A network is a list of `Layer` records that read and write logical buffers:
IN (-1) is the caller's blocked input (read-only), OUT (-2) the caller's blocked
output, 0..3 are workspace slots shared across layers (the paper's buffer-sharing
rule, Section "Memory Usage Comparison"). Paddings are explicit (t, b, l, r);
"same" paddings follow the Keras rule out = ceil(in/s), total = max((out-1)s+k-in, 0),
lo = total//2, hi = total-lo, because the stand-ins are Keras-style models.

Channel blocking: a tensor with C channels is stored with block min(16, C)
(every C used here is < 16 or a multiple of 16), so layer n's Cob equals layer
n+1's Cib and nothing is reformatted between layers (Section "Common Data Format").
"""
from dataclasses import dataclass, field
from typing import List, Optional, Tuple

IN, OUT = -1, -2
CB = 16  # machine block size C_b chosen for gfx950 (one 64-byte pixel row per block)


def block_of(C: int, cb: int = CB) -> int:
    """Stored channel-block size for a tensor with C channels."""
    b = min(cb, C)
    if C % b:
        raise ValueError(f"C={C} is not a multiple of its block {b}")
    return b


def same_pad(i: int, k: int, s: int) -> Tuple[int, int]:
    o = -(-i // s)
    total = max((o - 1) * s + k - i, 0)
    return total // 2, total - total // 2


@dataclass
class Layer:
    op: str                      # conv | dw | maxpool | avgpool | relu | add | dense | bn | upsample | gconv
    Ci: int
    Co: int
    H: int                       # input height / width seen by this layer
    W: int
    kh: int = 1
    kw: int = 1
    stride: int = 1
    pad: Tuple[int, int, int, int] = (0, 0, 0, 0)   # t, b, l, r
    Cib: int = 0
    Cob: int = 0
    src: int = IN
    src2: int = IN               # second operand of add; unused otherwise
    dst: int = OUT
    w: Optional[int] = None      # index into the network's weight list
    Ho: int = 0
    Wo: int = 0
    F_C: int = 0                 # gconv: channels of a group's window and its stride over the channels
    S_C: int = 0                 # (upsample: kh, kw are the factors; bn: w -> [2][C] scale, shift)

    def __post_init__(self):
        self.Cib = self.Cib or block_of(self.Ci)
        self.Cob = self.Cob or block_of(self.Co)
        if self.op == "upsample" and not self.Ho:
            self.Ho, self.Wo = self.H * self.kh, self.W * self.kw
        if not self.Ho:
            t, b, l, r = self.pad
            self.Ho = (self.H + t + b - self.kh) // self.stride + 1
            self.Wo = (self.W + l + r - self.kw) // self.stride + 1


@dataclass
class Network:
    name: str
    C0: int
    H0: int
    W0: int
    layers: List[Layer] = field(default_factory=list)
    # plain (unblocked) weight shapes, in layer order, with He fan-in
    wshapes: List[Tuple[Tuple[int, ...], int]] = field(default_factory=list)
    input_dist: str = "normal"       # "normal" = N(0,1), "uniform" = U[-1,1)
    weight_dist: str = "he_normal"   # "he_normal" = N(0, 2/fan_in), "uniform" = U[-1,1)

    @property
    def n_out(self) -> int:
        return self.layers[-1].Co

    @property
    def n_weights(self) -> int:
        n = 0
        for shp, _ in self.wshapes:
            m = 1
            for d in shp:
                m *= d
            n += m
        return n

    def macs_per_image(self) -> int:
        m = 0
        for L in self.layers:
            if L.op == "conv":
                m += L.Co * L.Ho * L.Wo * L.Ci * L.kh * L.kw
            elif L.op == "dw":
                m += L.Co * L.Ho * L.Wo * L.kh * L.kw
            elif L.op == "dense":
                m += L.Co * L.Ci * L.H * L.W
        return m


class _Builder:
    """Tracks the running (C, H, W) and the buffer that holds it."""

    def __init__(self, name, C0, H0, W0, input_dist="normal", weight_dist="he_normal"):
        self.net = Network(name, C0, H0, W0, input_dist=input_dist, weight_dist=weight_dist)
        self.C, self.H, self.W, self.buf = C0, H0, W0, IN

    def _free(self, *busy):
        for s in range(4):
            if s not in busy:
                return s
        raise RuntimeError("out of workspace slots")

    def _weight(self, shape, fan_in):
        self.net.wshapes.append((tuple(shape), fan_in))
        return len(self.net.wshapes) - 1

    def conv(self, Co, k, stride, pad, src=None, keep=()):
        kh, kw = k
        src = self.buf if src is None else src
        C, H, W = self._shape_of(src)
        if pad == "same":
            (t, b), (l, r) = same_pad(H, kh, stride), same_pad(W, kw, stride)
            pad = (t, b, l, r)
        dst = self._free(src, *keep)
        w = self._weight((Co, C, kh, kw), C * kh * kw)
        L = Layer("conv", C, Co, H, W, kh, kw, stride, pad, src=src, dst=dst, w=w)
        self.net.layers.append(L)
        self._set(dst, Co, L.Ho, L.Wo)
        return dst

    def dw(self, k, stride, pad):
        kh, kw = k
        if pad == "same":
            (t, b), (l, r) = same_pad(self.H, kh, stride), same_pad(self.W, kw, stride)
            pad = (t, b, l, r)
        dst = self._free(self.buf)
        w = self._weight((self.C, 1, kh, kw), kh * kw)
        L = Layer("dw", self.C, self.C, self.H, self.W, kh, kw, stride, pad,
                  src=self.buf, dst=dst, w=w)
        self.net.layers.append(L)
        self._set(dst, self.C, L.Ho, L.Wo)

    def relu(self):
        if self.buf == IN:
            raise RuntimeError("relu directly on the network input is not used here")
        self.net.layers.append(Layer("relu", self.C, self.C, self.H, self.W,
                                     src=self.buf, dst=self.buf))

    def add(self, other):
        self.net.layers.append(Layer("add", self.C, self.C, self.H, self.W,
                                     src=self.buf, src2=other, dst=self.buf))

    def global_avgpool(self):
        dst = self._free(self.buf)
        L = Layer("avgpool", self.C, self.C, self.H, self.W, self.H, self.W, 1,
                  src=self.buf, dst=dst)
        self.net.layers.append(L)
        self._set(dst, self.C, 1, 1)

    def dense(self, Co, last=True):
        dst = OUT if last else self._free(self.buf)
        w = self._weight((Co, self.C, self.H, self.W), self.C * self.H * self.W)
        L = Layer("dense", self.C, Co, self.H, self.W, self.H, self.W, 1,
                  src=self.buf, dst=dst, w=w, Ho=1, Wo=1)
        self.net.layers.append(L)
        self._set(dst, Co, 1, 1)

    # shapes per buffer so a skip branch can read an older buffer
    def _set(self, buf, C, H, W):
        self.C, self.H, self.W, self.buf = C, H, W, buf
        self._shapes[buf] = (C, H, W)

    def _shape_of(self, buf):
        return self._shapes[buf]

    _shapes = None

    def start(self):
        self._shapes = {IN: (self.C, self.H, self.W)}
        return self


def residual_cnn() -> Network:
    """32x32x3 residual CNN: stem 3x3 conv to 16 ch + ReLU; three stages of one
    residual block each (16, 32, 64 ch; stride 2 entering stages 2 and 3) where
    a = ReLU(conv3x3(x, s)), b = conv3x3(a), shortcut = x or conv1x1(x, s),
    x = ReLU(b + shortcut); 8x8 global average pool; dense 64 -> 10.
    The block structure follows the paper's description of ResNet (Section
    "MLPerf:Tiny Inference Models")."""
    B = _Builder("residual_cnn", 3, 32, 32).start()
    B.conv(16, (3, 3), 1, (1, 1, 1, 1))
    B.relu()
    for C, s in ((16, 1), (32, 2), (64, 2)):
        x, Cin = B.buf, B.C
        B.conv(C, (3, 3), s, "same")
        B.relu()
        B.conv(C, (3, 3), 1, (1, 1, 1, 1), keep=(x,))
        b = B.buf
        if s == 1 and Cin == C:
            sc = x
        else:
            sc = B.conv(C, (1, 1), s, (0, 0, 0, 0), src=x, keep=(b,))
            B._set(b, C, B.H, B.W)
        B.add(sc)
        B.relu()
    B.global_avgpool()
    B.dense(10)
    return B.net


_DSEP_WIDTHS = (16, 32, 32, 64, 64, 128, 128, 128, 128, 128, 128, 256, 256)


def dsep_cnn(first_block_stride: int = 2) -> Network:
    """96x96x3 depthwise-separable CNN: 3x3 stride-2 conv to 8 ch + ReLU, 13
    blocks of [3x3 depthwise + ReLU + 1x1 pointwise + ReLU], stride 2 on the
    depthwise conv of every block that widens (8->16 included when
    first_block_stride=2, the literal reading of the workload statement;
    first_block_stride=1 is the usual MobileNet-0.25 variant), global average
    pool, dense 256 -> 2."""
    B = _Builder("dsep_cnn" if first_block_stride == 2 else "dsep_cnn_b1s1", 3, 96, 96).start()
    B.conv(8, (3, 3), 2, "same")
    B.relu()
    for i, C in enumerate(_DSEP_WIDTHS):
        s = 2 if C != B.C else 1
        if i == 0:
            s = first_block_stride
        B.dw((3, 3), s, "same")
        B.relu()
        B.conv(C, (1, 1), 1, (0, 0, 0, 0))
        B.relu()
    B.global_avgpool()
    B.dense(2)
    return B.net


def audio_cnn() -> Network:
    """49x10x1 audio-feature CNN: 10x4 stride-2 'same' conv to 64 ch + ReLU, 4
    blocks of [3x3 depthwise + ReLU + 1x1 pointwise 64->64 + ReLU], global
    average pool (25x5), dense 64 -> 12."""
    B = _Builder("audio_cnn", 1, 49, 10).start()
    B.conv(64, (10, 4), 2, "same")
    B.relu()
    for _ in range(4):
        B.dw((3, 3), 1, (1, 1, 1, 1))
        B.relu()
        B.conv(64, (1, 1), 1, (0, 0, 0, 0))
        B.relu()
    B.global_avgpool()
    B.dense(12)
    return B.net


_AUTOENCODER_WIDTHS = (128, 128, 128, 128, 8, 128, 128, 128, 128, 128)


def dense_autoencoder() -> Network:
    """(1, 1, 128) dense-only autoencoder: ten fully connected layers, 128 wide except
    the 8-wide code in the middle, ReLU after every layer but the last. The widths
    are the ones that reproduce the weight count the paper lists for this model
    (Table "tinyml_models": 133120 = 8 * 128 * 128 + 2 * 128 * 8, no biases)."""
    B = _Builder("dense_autoencoder", 128, 1, 1).start()
    for i, C in enumerate(_AUTOENCODER_WIDTHS):
        last = i == len(_AUTOENCODER_WIDTHS) - 1
        B.dense(C, last=last)
        if not last:
            B.relu()
    return B.net


def single_conv_relu() -> Network:
    """1x16x32x32 input, 16x16x3x3 filters, stride 1, pad 1, then ReLU."""
    B = _Builder("single_conv_relu", 16, 32, 32, input_dist="uniform",
                 weight_dist="uniform").start()
    B.conv(16, (3, 3), 1, (1, 1, 1, 1))
    L = B.net.layers[-1]
    L.dst = OUT
    B.net.layers.append(Layer("relu", 16, 16, 32, 32, src=OUT, dst=OUT))
    return B.net
