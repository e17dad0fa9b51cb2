"""Seeded synthetic tensors (plain NCHW / OIHW float32), shared by oracle and HIP tests.

Everything is drawn from numpy's default_rng(seed) in a fixed order: the input
first, then each layer's weights in layer order. No layer arithmetic lives here.
"""
import numpy as np

BASE_SEED = 230304769   # seed of workload k is BASE_SEED + k


def uniform_pm1(rng, shape):
    """U[-1, 1) float32."""
    return (rng.random(shape, dtype=np.float32) * np.float32(2.0) - np.float32(1.0)).astype(np.float32)


def normal(rng, shape):
    """N(0, 1) float32."""
    return rng.standard_normal(shape, dtype=np.float32)


def he_normal(rng, shape, fan_in):
    """N(0, 2/fan_in) float32."""
    return (rng.standard_normal(shape, dtype=np.float32) * np.float32(np.sqrt(2.0 / fan_in))).astype(np.float32)


def network_tensors(net, N, seed):
    """Input batch [N, C0, H0, W0] and the list of plain weights of `net`."""
    rng = np.random.default_rng(seed)
    shape = (N, net.C0, net.H0, net.W0)
    x = uniform_pm1(rng, shape) if net.input_dist == "uniform" else normal(rng, shape)
    ws = []
    for shp, fan_in in net.wshapes:
        ws.append(uniform_pm1(rng, shp) if net.weight_dist == "uniform" else he_normal(rng, shp, fan_in))
    return x, ws


# Roofline layer sweep: fp32, batch 64, Cb = 16, everything U[-1, 1).
SWEEP_N = 64


def sweep_shapes():
    """(C, H) pairs of the conv / depthwise sweep, plus the pool / ReLU shape."""
    return {"conv": [(64, 56), (128, 28), (256, 14), (512, 7)],
            "pool_relu": (256, 56),
            # the two input sizes of the paper's own layer study (Section "Choice of layer types and sizes"):
            # 48 x 48 x 16 and 6 x 6 x 512 (height x width x channels), here at the sweep's batch of 64
            "paper_layer_study": [(16, 48), (512, 6)]}


# Quantized (uint8) layers: codes are uniform over 0..255; zero points and the fixed-point multiplier are
# parameters of the layer, chosen here so that the outputs spread over the whole code range.
def u8_codes(rng, shape):
    return rng.integers(0, 256, size=shape, dtype=np.uint8)


def u8_multiplier(K, spread=40.0, shift=31, x_rms=74.0):
    """(mult, shift) with mult / 2**shift = spread / (sqrt(K) * x_rms * 74): a sum of K products of a code minus its
    zero point with that root mean square (74 for uniform codes) and a uniform filter code minus its zero point has
    a standard deviation of about sqrt(K) * x_rms * 74."""
    m = spread / (np.sqrt(float(K)) * x_rms * 74.0)
    mult = int(round(m * (1 << shift)))
    return min(max(mult, 1), (1 << 31) - 1), shift


def quantized_network_tensors(net, N, seed):
    """A quantized stand-in of a float layer table: input codes [N, C0, H0, W0] and OIHW filter codes, uniform over
    0..255, and one parameter record per layer (plain dicts, no arithmetic): every tensor has zero point 128;
    conv / dw / dense: {"zx", "zw", "zy", "mult", "shift", "lo", "hi"} with the multiplier of u8_multiplier for
    the layer's reduction length; add: {"za", "zb", "zy", "mult_a", "mult_b", "shift", "lo", "hi"} with the two
    inputs weighted 3/4 and 1/2 (two different input scales); relu: {"z": 128}; pools: None."""
    rng = np.random.default_rng(seed)
    x = u8_codes(rng, (N, net.C0, net.H0, net.W0))
    ws = [u8_codes(rng, shp) for shp, _ in net.wshapes]
    # Multipliers are chosen so that the codes keep spreading through the network: a rough root mean square of
    # (code - 128) is carried per buffer (uniform input: 74; after a weighted layer: the spread asked for, 40; after
    # a ReLU: / sqrt 2; after an average over many values of a rectified tensor: about their mean, 0.56 of it).
    rms = {-1: 74.0}
    qs = []
    for l in net.layers:
        r = rms[l.src]
        if l.op in ("conv", "dw", "dense"):
            K = l.kh * l.kw * (1 if l.op == "dw" else l.Ci)
            mult, shift = u8_multiplier(K, x_rms=r)
            qs.append({"zx": 128, "zw": 128, "zy": 128, "mult": mult, "shift": shift, "lo": 0, "hi": 255})
            r = 40.0
        elif l.op == "add":
            qs.append({"za": 128, "zb": 128, "zy": 128, "mult_a": 3 << 28, "mult_b": 1 << 29, "shift": 30, "lo": 0, "hi": 255})
            r = float(np.hypot(0.75 * r, 0.5 * rms[l.src2]))
        elif l.op == "relu":
            qs.append({"z": 128})
            r = r / np.sqrt(2.0)
        elif l.op == "avgpool":
            qs.append(None)
            r = 0.56 * r if l.kh * l.kw >= 9 else r
        elif l.op == "maxpool":
            qs.append(None)
        else:
            raise ValueError("no quantized stand-in for op " + l.op)
        rms[l.dst] = r
    return x, ws, qs
