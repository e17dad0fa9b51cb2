"""ctypes front end of the quantized (uint8) CPU oracle (oracle/small_oracle_u8.c). TEST INFRASTRUCTURE ONLY.

Plain NCHW uint8 activations, OIHW uint8 filters; the requantization rule is stated in the C file's header.
Nothing under paper_2303_04769_amd/ imports this module.
"""
import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "small_oracle_u8.c")
_LIB = os.path.join(_HERE, "libsmall_oracle_u8.so")
_lib = None


@dataclass
class Quant:
    """y = clamp(zy + round_half_up(acc * mult / 2**shift), lo, hi); acc = sum (x - zx) * (w - zw)."""
    zx: int = 128
    zw: int = 128
    zy: int = 128
    mult: int = 1 << 20
    shift: int = 30
    lo: int = 0
    hi: int = 255


@dataclass
class QuantAdd:
    """y = clamp(zy + round_half_up(((a - za) * mult_a + (b - zb) * mult_b) / 2**shift), lo, hi)."""
    za: int = 128
    zb: int = 128
    zy: int = 128
    mult_a: int = 1 << 30
    mult_b: int = 1 << 30
    shift: int = 30
    lo: int = 0
    hi: int = 255


def build(force=False):
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-o", _LIB, _SRC])
    return _LIB


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.sq_act_offset.restype = C.c_size_t
        _lib.sq_filter_offset.restype = C.c_size_t
        _lib.sq_requant_one.restype = C.c_uint8
    return _lib


def _u8(a):
    return np.ascontiguousarray(a, dtype=np.uint8)


def _pu8(a):
    assert a.dtype == np.uint8 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_uint8))


def _pi32(a):
    assert a.dtype == np.int32 and a.flags["C_CONTIGUOUS"]
    return a.ctypes.data_as(C.POINTER(C.c_int32))


def out_dim(i, f, s, lo, hi):
    t = i + lo + hi - f
    return t // s + 1 if t >= 0 else 0


def requant(acc, q):
    acc = np.ascontiguousarray(acc, dtype=np.int32)
    y = np.empty(acc.shape, np.uint8)
    lib().sq_requant(_pi32(acc), _pu8(y), C.c_size_t(acc.size), q.zy, q.mult, q.shift, q.lo, q.hi)
    return y


def conv2d_acc(x, w, stride, pad, zx, zw):
    x, w = _u8(x), _u8(w)
    N, Ci, H, W = x.shape
    Co, Ci2, kh, kw = w.shape
    assert Ci == Ci2
    t, b, l, r = pad
    acc = np.empty((N, Co, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.int32)
    lib().sq_conv2d_acc(_pu8(x), _pu8(w), _pi32(acc), N, Ci, Co, H, W, kh, kw, stride, t, b, l, r, zx, zw)
    return acc


def conv2d(x, w, stride, pad, q):
    return requant(conv2d_acc(x, w, stride, pad, q.zx, q.zw), q)


def dwconv2d_acc(x, w, stride, pad, zx, zw):
    x, w = _u8(x), _u8(w)
    N, Cc, H, W = x.shape
    assert w.shape[0] == Cc and w.shape[1] == 1
    kh, kw = w.shape[2:]
    t, b, l, r = pad
    acc = np.empty((N, Cc, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.int32)
    lib().sq_dwconv2d_acc(_pu8(x), _pu8(w), _pi32(acc), N, Cc, H, W, kh, kw, stride, t, b, l, r, zx, zw)
    return acc


def dwconv2d(x, w, stride, pad, q):
    return requant(dwconv2d_acc(x, w, stride, pad, q.zx, q.zw), q)


def dense(x, w, q):
    """Window = whole image: conv with kh = H, kw = W, no padding."""
    return conv2d(x, w, 1, (0, 0, 0, 0), q)


def pool2d(x, k, stride, pad=(0, 0, 0, 0), mode="max"):
    x = _u8(x)
    N, Cc, H, W = x.shape
    kh, kw = k
    t, b, l, r = pad
    y = np.empty((N, Cc, out_dim(H, kh, stride, t, b), out_dim(W, kw, stride, l, r)), np.uint8)
    lib().sq_pool2d(_pu8(x), _pu8(y), N, Cc, H, W, kh, kw, stride, t, b, l, r, 0 if mode == "max" else 1)
    return y


def relu(x, z):
    x = _u8(x)
    y = np.empty_like(x)
    lib().sq_relu(_pu8(x), _pu8(y), C.c_size_t(x.size), int(z))
    return y


def add(a, b, q):
    a, b = _u8(a), _u8(b)
    assert a.shape == b.shape
    y = np.empty_like(a)
    lib().sq_add(_pu8(a), _pu8(b), _pu8(y), C.c_size_t(a.size), q.za, q.zb, q.zy, q.mult_a, q.mult_b, q.shift, q.lo, q.hi)
    return y


def run_network(net, x, ws, qs, upto=None, taps=None):
    """The layers of a table (workloads.nets.Network) on codes, one after the other on plain NCHW uint8 tensors.
    ws: OIHW uint8 filters by weight index; qs: one entry per layer -- Quant for conv / dw / dense, QuantAdd for add,
    the zero point (int) for relu, None for the pools (or the parameter dicts of workloads.quantized_network_tensors). Buffers are named by the table's ids; returns the tensor
    written to OUT (or by layer `upto`); taps, if a dict, receives every layer's result by layer index."""
    from workloads.nets import IN, OUT
    buf = {IN: _u8(x)}
    last = None
    for i, (l, q) in enumerate(zip(net.layers, qs)):
        if isinstance(q, dict):
            q = q["z"] if "z" in q else (QuantAdd(**q) if "za" in q else Quant(**q))
        src = buf[l.src]
        if l.op == "conv":
            y = conv2d(src, ws[l.w], l.stride, l.pad, q)
        elif l.op == "dw":
            y = dwconv2d(src, ws[l.w], l.stride, l.pad, q)
        elif l.op == "dense":
            y = dense(src, ws[l.w], q)
        elif l.op in ("maxpool", "avgpool"):
            y = pool2d(src, (l.kh, l.kw), l.stride, l.pad, "max" if l.op == "maxpool" else "avg")
        elif l.op == "relu":
            y = relu(src, q)
        elif l.op == "add":
            y = add(src, buf[l.src2], q)
        else:
            raise ValueError("no quantized layer for op " + l.op)
        buf[l.dst] = y
        last = y
        if taps is not None:
            taps[i] = y
        if upto is not None and i == upto:
            return y
    return buf.get(OUT, last)


def pack(x, Cb):
    x = _u8(x)
    N, Cc, H, W = x.shape
    blk = np.empty(x.size, np.uint8)
    lib().sq_pack(_pu8(x), _pu8(blk), N, Cc, H, W, Cb, 0)
    return blk


def unpack(blk, shape, Cb):
    blk = _u8(blk)
    N, Cc, H, W = shape
    x = np.empty(shape, np.uint8)
    lib().sq_pack(_pu8(x), _pu8(blk), N, Cc, H, W, Cb, 1)
    return x


def pack_filter(w, Cob, Cib):
    w = _u8(w)
    Co, Ci, kh, kw = w.shape
    blk = np.empty(w.size, np.uint8)
    lib().sq_pack_filter(_pu8(w), _pu8(blk), Co, Ci, kh, kw, Cob, Cib)
    return blk


def pack_dw_filter(w, Cb):
    """[C][1][kh][kw] -> [C/Cb][kh][kw][Cb] (the general layout with F_Cb = 1, G_b = Cb)."""
    w = _u8(w)
    Cc, one, kh, kw = w.shape
    assert one == 1
    return np.ascontiguousarray(w.reshape(Cc // Cb, Cb, kh, kw).transpose(0, 2, 3, 1)).reshape(-1)
