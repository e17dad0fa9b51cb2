"""ctypes front end of the CPU oracle (oracle/small_oracle.c). TEST INFRASTRUCTURE ONLY.

Only tests/, the smoke check and the benchmark's CPU-baseline leg may import this
module; the product package never does. Arrays are numpy float32, C-contiguous:
plain NCHW activations and OIHW filters for the definitional layers, flat blocked
buffers for the Algorithm-1 nest.
"""
import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "small_oracle.c")
_LIB = os.path.join(_HERE, "libsmall_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle with gcc (fp64 accumulation, OpenMP over (image, channel))."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-fno-fast-math",
                               "-ffp-contract=off", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.so_act_offset.restype = C.c_size_t
        _lib.so_filter_offset.restype = C.c_size_t
    return _lib


def _p(a):
    assert a.dtype == np.float32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_float))


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def set_threads(n):
    return lib().so_set_threads(int(n))


def out_dim(i, f, s, lo, hi):
    return lib().so_out_dim(i, f, s, lo, hi)


def conv2d(x, w, stride=1, pad=(0, 0, 0, 0)):
    x, w = _f32(x), _f32(w)
    N, Ci, H, W = x.shape
    Co, Ci2, kh, kw = w.shape
    assert Ci == Ci2
    t, b, l, r = pad
    y = np.empty((N, Co, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.float32)
    lib().so_conv2d(_p(x), _p(w), _p(y), N, Ci, Co, H, W, kh, kw, stride, t, b, l, r)
    return y


def dwconv2d(x, w, stride=1, pad=(0, 0, 0, 0)):
    x, w = _f32(x), _f32(w)
    N, Cc, H, W = x.shape
    assert w.shape[0] == Cc and w.shape[1] == 1
    kh, kw = w.shape[2:]
    t, b, l, r = pad
    y = np.empty((N, Cc, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.float32)
    lib().so_dwconv2d(_p(x), _p(w), _p(y), N, Cc, H, W, kh, kw, stride, t, b, l, r)
    return y


def pool2d(x, k, stride, pad=(0, 0, 0, 0), mode="max"):
    x = _f32(x)
    N, Cc, H, W = x.shape
    kh, kw = k
    t, b, l, r = pad
    y = np.empty((N, Cc, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.float32)
    lib().so_pool2d(_p(x), _p(y), N, Cc, H, W, kh, kw, stride, t, b, l, r, 0 if mode == "max" else 1)
    return y


def relu(x):
    x = _f32(x)
    y = np.empty_like(x)
    lib().so_relu(_p(x), _p(y), C.c_size_t(x.size))
    return y


def add(a, b):
    a, b = _f32(a), _f32(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().so_add(_p(a), _p(b), _p(y), C.c_size_t(a.size))
    return y


def batchnorm(x, scale, shift):
    """y = x * scale[c] + shift[c] on [N, C, H, W]."""
    x, scale, shift = _f32(x), _f32(scale), _f32(shift)
    N, Cc, H, W = x.shape
    assert scale.shape == (Cc,) and shift.shape == (Cc,)
    y = np.empty_like(x)
    lib().so_batchnorm(_p(x), _p(scale), _p(shift), _p(y), N, Cc, H, W)
    return y


def upsample(x, fh, fw):
    """Nearest-neighbour upsampling by integer factors."""
    x = _f32(x)
    N, Cc, H, W = x.shape
    y = np.empty((N, Cc, H * fh, W * fw), np.float32)
    lib().so_upsample(_p(x), _p(y), N, Cc, H, W, fh, fw)
    return y


def group_conv2d(x, w, F_C, S_C, K, stride=1, pad=(0, 0, 0, 0)):
    """x [N, Ci, H, W], w [G * K, F_C, kh, kw] with G = (Ci - F_C) / S_C + 1 -> [N, G * K, Ho, Wo]."""
    x, w = _f32(x), _f32(w)
    N, Ci, H, W = x.shape
    assert (Ci - F_C) % S_C == 0
    G = (Ci - F_C) // S_C + 1
    assert w.shape[0] == G * K and w.shape[1] == F_C
    kh, kw = w.shape[2:]
    t, b, l, r = pad
    y = np.empty((N, G * K, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.float32)
    lib().so_group_conv2d(_p(x), _p(w), _p(y), N, Ci, F_C, S_C, K, H, W, kh, kw, stride, t, b, l, r)
    return y


def dense(x, w):
    """x [N, Ci, H, W], w [Co, Ci, H, W] -> [N, Co, 1, 1]."""
    x, w = _f32(x), _f32(w)
    N, Ci, H, W = x.shape
    Co = w.shape[0]
    assert w.shape[1:] == (Ci, H, W)
    y = np.empty((N, Co, 1, 1), np.float32)
    lib().so_dense(_p(x), _p(w), _p(y), N, Ci, Co, H, W)
    return y


# ------------------------------------------------------------------ layouts

def pack(x, Cb):
    x = _f32(x)
    N, Cc, H, W = x.shape
    assert Cc % Cb == 0
    out = np.empty(x.size, np.float32)
    lib().so_pack(_p(x), _p(out), N, Cc, H, W, Cb)
    return out


def unpack(blk, shape, Cb):
    blk = _f32(blk)
    N, Cc, H, W = shape
    assert blk.size == N * Cc * H * W and Cc % Cb == 0
    out = np.empty(shape, np.float32)
    lib().so_unpack(_p(blk), _p(out), N, Cc, H, W, Cb)
    return out


def pack_filter(w, Cob, Cib):
    w = _f32(w)
    Co, Ci, kh, kw = w.shape
    assert Co % Cob == 0 and Ci % Cib == 0
    out = np.empty(w.size, np.float32)
    lib().so_pack_filter(_p(w), _p(out), Co, Ci, kh, kw, Cob, Cib)
    return out


def pack_dw_filter(w, Cb):
    w = _f32(w)
    Cc, one, kh, kw = w.shape
    assert one == 1 and Cc % Cb == 0
    out = np.empty(w.size, np.float32)
    lib().so_pack_dw_filter(_p(w), _p(out), Cc, kh, kw, Cb)
    return out


# ------------------------------------------------------------------ Algorithm 1 on blocked layouts

def abstract_layer_blocked(op, I, Wt, N, I_C, I_H, I_W, F_H, F_W, F_C, S_H, S_W, S_C, K, pad,
                           Icb, G_b, K_b, F_Cb, O_wb):
    """Runs the Algorithm-1 nest; returns the flat blocked output and (O_C, O_H, O_W)."""
    I = _f32(I)
    t, b, l, r = pad
    G = (I_C - F_C) // S_C + 1
    O_C = K * G
    O_H, O_W = out_dim(I_H, F_H, S_H, t, b), out_dim(I_W, F_W, S_W, l, r)
    O = np.empty(N * O_C * O_H * O_W, np.float32)
    wp = _p(_f32(Wt)) if Wt is not None else None
    rc = lib().so_abstract_layer_blocked({"fma": 0, "max": 1, "avg": 2}[op], _p(I), wp, _p(O), N, I_C, I_H, I_W,
                                         F_H, F_W, F_C, S_H, S_W, S_C, K, t, b, l, r, Icb, G_b, K_b, F_Cb, O_wb)
    if rc:
        raise ValueError(f"abstract layer tiling rejected (code {rc})")
    return O, (O_C, O_H, O_W)


def conv2d_blocked(xb, wb, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, O_wb=6):
    """Convolution = abstract layer with F_C = Ci, K = Co, G = 1 (Table 1 row 4)."""
    return abstract_layer_blocked("fma", xb, wb, N, Ci, H, W, kh, kw, Ci, stride, stride, 1, Co, pad,
                                  Cib, 1, Cob, Cib, O_wb)


def dwconv2d_blocked(xb, wb, N, Cc, H, W, kh, kw, stride, pad, Cb, O_wb=6):
    """Depthwise = abstract layer with F_C = 1, K = 1, G = C, G_b = O_cb (Table 1 row 2)."""
    return abstract_layer_blocked("fma", xb, wb, N, Cc, H, W, kh, kw, 1, stride, stride, 1, 1, pad,
                                  Cb, Cb, 1, 1, O_wb)


def pool2d_blocked(xb, N, Cc, H, W, kh, kw, stride, pad, Cb, mode="max", O_wb=6):
    return abstract_layer_blocked("max" if mode == "max" else "avg", xb, None, N, Cc, H, W, kh, kw, 1,
                                  stride, stride, 1, 1, pad, Cb, Cb, 1, 1, O_wb)


# ------------------------------------------------------------------ networks

def run_network(net, x, ws, return_all=False):
    """Chains the definitional layers over a workloads.Network table. Every layer's
    output is rounded to fp32 before the next one reads it. Returns logits [N, Co]."""
    bufs = {-1: _f32(x)}
    trace = []
    for L in net.layers:
        a = bufs[L.src]
        if L.op == "conv":
            y = conv2d(a, ws[L.w], L.stride, L.pad)
        elif L.op == "dw":
            y = dwconv2d(a, ws[L.w], L.stride, L.pad)
        elif L.op in ("maxpool", "avgpool"):
            y = pool2d(a, (L.kh, L.kw), L.stride, L.pad, "max" if L.op == "maxpool" else "avg")
        elif L.op == "relu":
            y = relu(a)
        elif L.op == "add":
            y = add(a, bufs[L.src2])
        elif L.op == "dense":
            y = dense(a, ws[L.w])
        elif L.op == "bn":
            y = batchnorm(a, ws[L.w][0], ws[L.w][1])
        elif L.op == "upsample":
            y = upsample(a, L.kh, L.kw)
        elif L.op == "gconv":
            G = (L.Ci - L.F_C) // L.S_C + 1
            y = group_conv2d(a, ws[L.w], L.F_C, L.S_C, L.Co // G, L.stride, L.pad)
        else:
            raise ValueError(L.op)
        bufs[L.dst] = y
        if return_all:
            trace.append(y)
    out = bufs[net.layers[-1].dst]
    out = out.reshape(out.shape[0], -1) if out.shape[2:] == (1, 1) else out
    return (out, trace) if return_all else out
