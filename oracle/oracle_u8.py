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
