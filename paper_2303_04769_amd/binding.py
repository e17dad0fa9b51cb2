"""ctypes binding of libsmall_hip.so: same names and arguments as include/small.h.

Tensor arguments are torch CUDA tensors (float32, contiguous); only their device
pointers cross the boundary. The stream is torch's current stream unless given.
Every wrapper raises SmallError on a non-zero status. No arithmetic happens here.
"""
import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsmall_hip.so")

OK = 0
POOL_MAX, POOL_AVG = 0, 1
OP_CONV, OP_DWCONV, OP_MAXPOOL, OP_AVGPOOL, OP_RELU, OP_ADD, OP_DENSE, OP_BATCHNORM, OP_UPSAMPLE, OP_GROUPCONV = range(10)
BUF_IN, BUF_OUT, MAX_SLOTS = -1, -2, 8
_OPS = {"conv": OP_CONV, "dw": OP_DWCONV, "maxpool": OP_MAXPOOL, "avgpool": OP_AVGPOOL, "relu": OP_RELU,
        "add": OP_ADD, "dense": OP_DENSE, "bn": OP_BATCHNORM, "upsample": OP_UPSAMPLE, "gconv": OP_GROUPCONV}

EXPORTS = ["small_out_dim", "small_strerror", "small_pack", "small_unpack", "small_pack_filter",
           "small_pack_dw_filter", "small_conv2d", "small_conv2d_kernel", "small_dwconv2d", "small_pool2d", "small_relu", "small_add",
           "small_dense", "small_batchnorm", "small_upsample", "small_group_conv2d", "small_pack_u8", "small_unpack_u8",
           "small_pack_filter_u8", "small_filter_sums_u8", "small_conv2d_u8", "small_dwconv2d_u8", "small_dense_u8", "small_pool2d_u8", "small_relu_u8",
           "small_add_u8", "small_network_workspace_u8", "small_network_run_u8",
           "small_network_workspace", "small_network_run", "small_network_run_plain", "small_network_run_opt", "small_network_launches", "small_network_launches_at",
           "small_network_run_range", "small_network_run_static"]


class SmallError(RuntimeError):
    def __init__(self, code, what):
        self.code = code
        super().__init__(f"{what}: error {code} ({strerror(code)})")


class small_pad(C.Structure):
    _fields_ = [("t", C.c_int), ("b", C.c_int), ("l", C.c_int), ("r", C.c_int)]


class small_quant(C.Structure):
    """y = clamp(zy + round_half_up(acc * mult / 2**shift), lo, hi), acc = sum (x - zx) * (w - zw)."""
    _fields_ = [("zx", C.c_int), ("zw", C.c_int), ("zy", C.c_int), ("mult", C.c_int), ("shift", C.c_int),
                ("lo", C.c_int), ("hi", C.c_int)]


class small_quant_add(C.Structure):
    """y = clamp(zy + round_half_up(((a - za) * mult_a + (b - zb) * mult_b) / 2**shift), lo, hi)."""
    _fields_ = [("za", C.c_int), ("zb", C.c_int), ("zy", C.c_int), ("mult_a", C.c_int), ("mult_b", C.c_int),
                ("shift", C.c_int), ("lo", C.c_int), ("hi", C.c_int)]


class small_layer_u8(C.Structure):
    _fields_ = [("op", C.c_int), ("Ci", C.c_int), ("Co", C.c_int), ("kh", C.c_int), ("kw", C.c_int),
                ("stride", C.c_int), ("pad", small_pad), ("Cib", C.c_int), ("Cob", C.c_int),
                ("src", C.c_int), ("src2", C.c_int), ("dst", C.c_int), ("filt", C.c_void_p), ("filt_sums", C.c_void_p),
                ("q", small_quant), ("qa", small_quant_add)]


class small_layer(C.Structure):
    _fields_ = [("op", C.c_int), ("Ci", C.c_int), ("Co", C.c_int), ("kh", C.c_int), ("kw", C.c_int),
                ("stride", C.c_int), ("pad", small_pad), ("Cib", C.c_int), ("Cob", C.c_int),
                ("src", C.c_int), ("src2", C.c_int), ("dst", C.c_int), ("filt", C.c_void_p),
                ("F_C", C.c_int), ("S_C", C.c_int)]


_lib = None


def load():
    """Loads the in-tree library; builds it first only when no built library exists."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        from .build import build_lib
        build_lib()
    lib = C.CDLL(LIB_PATH)
    i, p, sz = C.c_int, C.c_void_p, C.c_size_t
    sig = {
        "small_out_dim": (i, [i, i, i, i, i]),
        "small_strerror": (C.c_char_p, [i]),
        "small_pack": (i, [p, p, i, i, i, i, i, p]),
        "small_unpack": (i, [p, p, i, i, i, i, i, p]),
        "small_pack_filter": (i, [p, p, i, i, i, i, i, i, p]),
        "small_pack_dw_filter": (i, [p, p, i, i, i, i, p]),
        "small_conv2d": (i, [p, p, p, i, i, i, i, i, i, i, i, small_pad, i, i, p]),
        "small_conv2d_kernel": (C.c_char_p, [i, i, i, i, i, i, i, i, small_pad, i, i]),
        "small_dwconv2d": (i, [p, p, p, i, i, i, i, i, i, i, small_pad, i, p]),
        "small_pool2d": (i, [p, p, i, i, i, i, i, i, i, small_pad, i, i, p]),
        "small_relu": (i, [p, p, sz, p]),
        "small_add": (i, [p, p, p, sz, p]),
        "small_dense": (i, [p, p, p, i, i, i, i, i, p]),
        "small_batchnorm": (i, [p, p, p, p, i, i, i, i, i, p]),
        "small_upsample": (i, [p, p, i, i, i, i, i, i, i, p]),
        "small_group_conv2d": (i, [p, p, p, i, i, i, i, i, i, i, i, i, i, small_pad, i, i, i, p]),
        "small_pack_u8": (i, [p, p, i, i, i, i, i, p]),
        "small_unpack_u8": (i, [p, p, i, i, i, i, i, p]),
        "small_pack_filter_u8": (i, [p, p, i, i, i, i, i, i, p]),
        "small_filter_sums_u8": (i, [p, p, i, i, i, i, i, i, p]),
        "small_conv2d_u8": (i, [p, p, p, i, i, i, i, i, i, i, i, small_pad, i, i, C.POINTER(small_quant), p, p]),
        "small_dwconv2d_u8": (i, [p, p, p, i, i, i, i, i, i, i, small_pad, i, C.POINTER(small_quant), p]),
        "small_dense_u8": (i, [p, p, p, i, i, i, i, i, C.POINTER(small_quant), p, p]),
        "small_pool2d_u8": (i, [p, p, i, i, i, i, i, i, i, small_pad, i, i, p]),
        "small_relu_u8": (i, [p, p, sz, i, p]),
        "small_add_u8": (i, [p, p, p, sz, C.POINTER(small_quant_add), p]),
        "small_network_workspace_u8": (i, [C.POINTER(small_layer_u8), i, i, i, i, i, C.POINTER(sz)]),
        "small_network_run_u8": (i, [C.POINTER(small_layer_u8), i, p, p, p, sz, i, i, i, i, p]),
        "small_network_workspace": (i, [C.POINTER(small_layer), i, i, i, i, i, C.POINTER(sz)]),
        "small_network_run": (i, [C.POINTER(small_layer), i, p, p, p, sz, i, i, i, i, p]),
        "small_network_run_plain": (i, [C.POINTER(small_layer), i, p, p, p, sz, i, i, i, i, p]),
        "small_network_run_opt": (i, [C.POINTER(small_layer), i, p, p, p, sz, i, i, i, i, C.c_uint, p]),
        "small_network_launches_at": (i, [C.POINTER(small_layer), i, i, i, i, i, C.c_uint, C.POINTER(C.c_int),
                                          C.POINTER(C.c_int)]),
        "small_network_launches": (i, [C.POINTER(small_layer), i, C.POINTER(i), C.POINTER(i)]),
        "small_network_run_range": (i, [C.POINTER(small_layer), i, p, p, p, sz, i, i, i, i, i, i, p]),
        "small_network_run_static": (i, [C.POINTER(small_layer), i, p, p, i, i, i, i, C.c_uint, p]),
    }
    for name, (res, args) in sig.items():
        f = getattr(lib, name)     # AttributeError if the library does not export it
        f.restype, f.argtypes = res, args
    _lib = lib
    return lib


def strerror(code):
    return load().small_strerror(int(code)).decode()


def _check(rc, what):
    if rc != OK:
        raise SmallError(rc, what)


def _ptr(t):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.float32 and t.is_contiguous()):
        raise TypeError("expected a contiguous float32 CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


def _pad(pad):
    return small_pad(*[int(v) for v in pad])


def small_out_dim(i, k, stride, lo, hi):
    return load().small_out_dim(i, k, stride, lo, hi)


def small_pack(nchw, blocked, N, Cc, H, W, Cb, stream=None):
    _check(load().small_pack(_ptr(nchw), _ptr(blocked), N, Cc, H, W, Cb, _stream(stream)), "small_pack")


def small_unpack(blocked, nchw, N, Cc, H, W, Cb, stream=None):
    _check(load().small_unpack(_ptr(blocked), _ptr(nchw), N, Cc, H, W, Cb, _stream(stream)), "small_unpack")


def small_pack_filter(oihw, blocked, Co, Ci, kh, kw, Cob, Cib, stream=None):
    _check(load().small_pack_filter(_ptr(oihw), _ptr(blocked), Co, Ci, kh, kw, Cob, Cib, _stream(stream)),
           "small_pack_filter")


def small_pack_dw_filter(c1hw, blocked, Cc, kh, kw, Cb, stream=None):
    _check(load().small_pack_dw_filter(_ptr(c1hw), _ptr(blocked), Cc, kh, kw, Cb, _stream(stream)),
           "small_pack_dw_filter")


def small_conv2d(inp, filt, out, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, stream=None):
    _check(load().small_conv2d(_ptr(inp), _ptr(filt), _ptr(out), N, Ci, Co, H, W, kh, kw, stride, _pad(pad), Cib, Cob,
                               _stream(stream)), "small_conv2d")


def small_conv2d_kernel(N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob):
    name = load().small_conv2d_kernel(N, Ci, Co, H, W, kh, kw, stride, _pad(pad), Cib, Cob)
    return name.decode() if name else None


def small_dwconv2d(inp, filt, out, N, Cc, H, W, kh, kw, stride, pad, Cb, stream=None):
    _check(load().small_dwconv2d(_ptr(inp), _ptr(filt), _ptr(out), N, Cc, H, W, kh, kw, stride, _pad(pad), Cb,
                                 _stream(stream)), "small_dwconv2d")


def small_pool2d(inp, out, N, Cc, H, W, kh, kw, stride, pad, Cb, mode, stream=None):
    _check(load().small_pool2d(_ptr(inp), _ptr(out), N, Cc, H, W, kh, kw, stride, _pad(pad), Cb, mode,
                               _stream(stream)), "small_pool2d")


def small_relu(inp, out, n_elems, stream=None):
    _check(load().small_relu(_ptr(inp), _ptr(out), n_elems, _stream(stream)), "small_relu")


def small_add(a, b, out, n_elems, stream=None):
    _check(load().small_add(_ptr(a), _ptr(b), _ptr(out), n_elems, _stream(stream)), "small_add")


def small_dense(inp, filt, out, N, Ci, Co, Cib, Cob, stream=None):
    _check(load().small_dense(_ptr(inp), _ptr(filt), _ptr(out), N, Ci, Co, Cib, Cob, _stream(stream)), "small_dense")


def small_batchnorm(inp, scale, shift, out, N, Cc, H, W, Cb, stream=None):
    _check(load().small_batchnorm(_ptr(inp), _ptr(scale), _ptr(shift), _ptr(out), N, Cc, H, W, Cb, _stream(stream)),
           "small_batchnorm")


def small_upsample(inp, out, N, Cc, H, W, fh, fw, Cb, stream=None):
    _check(load().small_upsample(_ptr(inp), _ptr(out), N, Cc, H, W, fh, fw, Cb, _stream(stream)), "small_upsample")


def small_group_conv2d(inp, filt, out, N, Ci, F_C, S_C, K, H, W, kh, kw, stride, pad, Cib, F_Cb, Cob, stream=None):
    _check(load().small_group_conv2d(_ptr(inp), _ptr(filt), _ptr(out), N, Ci, F_C, S_C, K, H, W, kh, kw, stride, _pad(pad),
                                     Cib, F_Cb, Cob, _stream(stream)), "small_group_conv2d")


PROBE_LIB_PATH = os.path.join(_HERE, "libsmall_probe.so")
_probe = None


def load_probe():
    """The benchmark's matrix-rate probe (include/small_probe.h), a library of its own."""
    global _probe
    if _probe is None:
        if not os.path.exists(PROBE_LIB_PATH):
            from .build import build_lib
            build_lib()
        lib = C.CDLL(PROBE_LIB_PATH)
        lib.small_probe_mfma.restype, lib.small_probe_mfma.argtypes = C.c_int, [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
        lib.small_probe_mfma_valu.restype = C.c_int
        lib.small_probe_mfma_valu.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_int, C.c_void_p]
        _probe = lib
    return _probe


def small_probe_mfma(out, workgroups, iters, stream=None):
    rc = load_probe().small_probe_mfma(_ptr(out), workgroups, iters, _stream(stream))
    if rc:
        raise RuntimeError(f"small_probe_mfma: error {rc}")


def small_probe_mfma_valu(out, workgroups, iters, valu, stream=None):
    rc = load_probe().small_probe_mfma_valu(_ptr(out), workgroups, iters, valu, _stream(stream))
    if rc:
        raise RuntimeError(f"small_probe_mfma_valu: error {rc}")


def _ptr8(t):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.uint8 and t.is_contiguous()):
        raise TypeError("expected a contiguous uint8 CUDA tensor")
    return C.c_void_p(t.data_ptr())


def _quant(q):
    """q: small_quant, or any record with fields zx, zw, zy, mult, shift, lo, hi."""
    if isinstance(q, small_quant):
        return C.byref(q)
    return C.byref(small_quant(int(q.zx), int(q.zw), int(q.zy), int(q.mult), int(q.shift), int(q.lo), int(q.hi)))


def small_pack_u8(nchw, blocked, N, Cc, H, W, Cb, stream=None):
    _check(load().small_pack_u8(_ptr8(nchw), _ptr8(blocked), N, Cc, H, W, Cb, _stream(stream)), "small_pack_u8")


def small_unpack_u8(blocked, nchw, N, Cc, H, W, Cb, stream=None):
    _check(load().small_unpack_u8(_ptr8(blocked), _ptr8(nchw), N, Cc, H, W, Cb, _stream(stream)), "small_unpack_u8")


def small_pack_filter_u8(oihw, blocked, Co, Ci, kh, kw, Cob, Cib, stream=None):
    _check(load().small_pack_filter_u8(_ptr8(oihw), _ptr8(blocked), Co, Ci, kh, kw, Cob, Cib, _stream(stream)),
           "small_pack_filter_u8")


def _ptr32i(t):
    if t is None:
        return None
    if not (t.is_cuda and t.dtype == torch.int32 and t.is_contiguous()):
        raise TypeError("expected a contiguous int32 CUDA tensor")
    return C.c_void_p(t.data_ptr())


def small_filter_sums_u8(filt, sums, Co, Ci, kh, kw, Cob, Cib, stream=None):
    _check(load().small_filter_sums_u8(_ptr8(filt), _ptr32i(sums), Co, Ci, kh, kw, Cob, Cib, _stream(stream)),
           "small_filter_sums_u8")


def small_conv2d_u8(inp, filt, out, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, q, filt_sums=None, stream=None):
    _check(load().small_conv2d_u8(_ptr8(inp), _ptr8(filt), _ptr8(out), N, Ci, Co, H, W, kh, kw, stride, _pad(pad), Cib, Cob,
                                  _quant(q), _ptr32i(filt_sums), _stream(stream)), "small_conv2d_u8")


def small_dwconv2d_u8(inp, filt, out, N, Cc, H, W, kh, kw, stride, pad, Cb, q, stream=None):
    _check(load().small_dwconv2d_u8(_ptr8(inp), _ptr8(filt), _ptr8(out), N, Cc, H, W, kh, kw, stride, _pad(pad), Cb,
                                    _quant(q), _stream(stream)), "small_dwconv2d_u8")


def small_dense_u8(inp, filt, out, N, Ci, Co, Cib, Cob, q, filt_sums=None, stream=None):
    _check(load().small_dense_u8(_ptr8(inp), _ptr8(filt), _ptr8(out), N, Ci, Co, Cib, Cob, _quant(q), _ptr32i(filt_sums),
                                 _stream(stream)), "small_dense_u8")


def small_pool2d_u8(inp, out, N, Cc, H, W, kh, kw, stride, pad, Cb, mode, stream=None):
    _check(load().small_pool2d_u8(_ptr8(inp), _ptr8(out), N, Cc, H, W, kh, kw, stride, _pad(pad), Cb, mode,
                                  _stream(stream)), "small_pool2d_u8")


def small_relu_u8(inp, out, n, z, stream=None):
    _check(load().small_relu_u8(_ptr8(inp), _ptr8(out), n, z, _stream(stream)), "small_relu_u8")


def make_layer_table(layers, filters):
    """ctypes array of small_layer from records with fields op, Ci, Co, kh, kw, stride, pad,
    Cib, Cob, src, src2, dst, w (index into `filters`, the blocked device filters, or None), and for
    group convolutions F_C, S_C."""
    arr = (small_layer * len(layers))()
    for k, L in enumerate(layers):
        f = filters[L.w] if L.w is not None else None
        arr[k] = small_layer(_OPS[L.op], L.Ci, L.Co, L.kh, L.kw, L.stride, _pad(L.pad), L.Cib, L.Cob,
                             L.src, L.src2, L.dst, f.data_ptr() if f is not None else None,
                             getattr(L, "F_C", 0), getattr(L, "S_C", 0))
    return arr


def small_network_workspace(table, N, C0, H0, W0):
    n = C.c_size_t(0)
    _check(load().small_network_workspace(table, len(table), N, C0, H0, W0, C.byref(n)), "small_network_workspace")
    return n.value


def small_network_run(table, in_blocked, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, stream=None):
    _check(load().small_network_run(table, len(table), _ptr(in_blocked), _ptr(out_blocked),
                                    C.c_void_p(workspace.data_ptr()) if workspace is not None else None,
                                    workspace_bytes, N, C0, H0, W0, _stream(stream)), "small_network_run")


def small_network_run_plain(table, in_nchw, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, stream=None):
    _check(load().small_network_run_plain(table, len(table), _ptr(in_nchw), _ptr(out_blocked),
                                          C.c_void_p(workspace.data_ptr()) if workspace is not None else None,
                                          workspace_bytes, N, C0, H0, W0, _stream(stream)), "small_network_run_plain")


SMALL_RUN_PLAIN_INPUT, SMALL_RUN_RESIDENT_OFF, SMALL_RUN_RESIDENT_ON, SMALL_RUN_PLAIN_OUTPUT = 1, 2, 4, 8


def small_network_run_opt(table, in_tensor, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, flags, stream=None):
    _check(load().small_network_run_opt(table, len(table), _ptr(in_tensor), _ptr(out_blocked),
                                        C.c_void_p(workspace.data_ptr()) if workspace is not None else None,
                                        workspace_bytes, N, C0, H0, W0, flags, _stream(stream)), "small_network_run_opt")


def small_network_launches_at(table, N, C0, H0, W0, flags=0):
    """List of first-layer indices, one per kernel launch of a run with this batch size and these flags."""
    first = (C.c_int * len(table))()
    n = C.c_int(0)
    _check(load().small_network_launches_at(table, len(table), N, C0, H0, W0, flags, first, C.byref(n)),
           "small_network_launches_at")
    return list(first[:n.value])


def small_network_launches(table):
    """List of first-layer indices, one per kernel launch of small_network_run."""
    first = (C.c_int * len(table))()
    n = C.c_int(0)
    _check(load().small_network_launches(table, len(table), first, C.byref(n)), "small_network_launches")
    return [first[k] for k in range(n.value)]


def small_network_run_range(table, in_blocked, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, first, count,
                            stream=None):
    _check(load().small_network_run_range(table, len(table), _ptr(in_blocked), _ptr(out_blocked),
                                          C.c_void_p(workspace.data_ptr()) if workspace is not None else None,
                                          workspace_bytes, N, C0, H0, W0, first, count, _stream(stream)),
           "small_network_run_range")


STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024


def small_network_run_static(table, in_tensor, out_blocked, N, C0, H0, W0, flags=0, stream=None):
    _check(load().small_network_run_static(table, len(table), _ptr(in_tensor), _ptr(out_blocked), N, C0, H0, W0, flags,
                                           _stream(stream)), "small_network_run_static")


def small_add_u8(a, b, out, n, q, stream=None):
    """q: small_quant_add, or anything with its eight fields (a dict, oracle-side records)."""
    _check(load().small_add_u8(_ptr8(a), _ptr8(b), _ptr8(out), n, C.byref(_quant_add(q)), _stream(stream)), "small_add_u8")


def _quant_add(q):
    if isinstance(q, small_quant_add):
        return q
    get = (lambda k: q[k]) if isinstance(q, dict) else (lambda k: getattr(q, k))
    return small_quant_add(*[int(get(k)) for k in ("za", "zb", "zy", "mult_a", "mult_b", "shift", "lo", "hi")])


def _quant_of(q):
    if isinstance(q, small_quant):
        return q
    get = (lambda k: q[k]) if isinstance(q, dict) else (lambda k: getattr(q, k))
    return small_quant(*[int(get(k)) for k in ("zx", "zw", "zy", "mult", "shift", "lo", "hi")])


class PackedNetworkU8:
    """Device-resident form of a quantized layer table: uint8 filters packed once (small_pack_filter_u8; depthwise
    filters [C/Cb][kh][kw][Cb]), their per-channel sums taken once (small_filter_sums_u8), the table of small_layer_u8
    records built from a workloads layer table and its per-layer parameter records."""

    def __init__(self, net, weights, params, device="cuda:0"):
        self.net, self.device = net, torch.device(device)
        self.filters, self.sums = {}, {}
        for L in net.layers:
            if L.w is None:
                continue
            src = torch.from_numpy(weights[L.w]).to(self.device).contiguous()
            if L.op == "dw":
                dst = src.reshape(L.Ci // L.Cib, L.Cib, L.kh, L.kw).permute(0, 2, 3, 1).contiguous().reshape(-1)
            else:
                dst = torch.empty(src.numel(), dtype=torch.uint8, device=self.device)
                small_pack_filter_u8(src, dst, L.Co, L.Ci, L.kh, L.kw, L.Cob, L.Cib)
                sums = torch.empty(L.Co, dtype=torch.int32, device=self.device)
                small_filter_sums_u8(dst, sums, L.Co, L.Ci, L.kh, L.kw, L.Cob, L.Cib)
                self.sums[L.w] = sums
            self.filters[L.w] = dst
        arr = (small_layer_u8 * len(net.layers))()
        for k, (L, q) in enumerate(zip(net.layers, params)):
            arr[k].op = _OPS[L.op]
            arr[k].Ci, arr[k].Co, arr[k].kh, arr[k].kw, arr[k].stride = L.Ci, L.Co, L.kh, L.kw, L.stride
            arr[k].pad = small_pad(*L.pad)
            arr[k].Cib, arr[k].Cob = L.Cib, L.Cob
            arr[k].src, arr[k].src2, arr[k].dst = L.src, L.src2, L.dst
            arr[k].filt = self.filters[L.w].data_ptr() if L.w is not None else None
            arr[k].filt_sums = self.sums[L.w].data_ptr() if L.w in self.sums else None
            if L.op in ("conv", "dw", "dense"):
                arr[k].q = _quant_of(q)
            elif L.op == "add":
                arr[k].qa = _quant_add(q)
            elif L.op == "relu":
                arr[k].q = small_quant(0, 0, int(q["z"] if isinstance(q, dict) else q), 0, 0, 0, 255)
        self.table = arr
        self._ws = {}

    def workspace(self, N):
        if N not in self._ws:
            nbytes = C.c_size_t(0)
            _check(load().small_network_workspace_u8(self.table, len(self.table), N, self.net.C0, self.net.H0, self.net.W0,
                                                     C.byref(nbytes)), "small_network_workspace_u8")
            self._ws[N] = (torch.empty(max(nbytes.value, 256), dtype=torch.uint8, device=self.device), nbytes.value)
        return self._ws[N]

    def pack_input(self, x_nchw):
        N = x_nchw.shape[0]
        xb = torch.empty(x_nchw.numel(), dtype=torch.uint8, device=self.device)
        small_pack_u8(x_nchw, xb, N, self.net.C0, self.net.H0, self.net.W0, self.net.layers[0].Cib)
        return xb

    def out_elems(self, N):
        L = self.net.layers[-1]
        return N * L.Co * L.Ho * L.Wo

    def run(self, in_blocked, out_blocked, N, stream=None):
        ws, nbytes = self.workspace(N)
        _check(load().small_network_run_u8(self.table, len(self.table), _ptr8(in_blocked), _ptr8(out_blocked), _ptr8(ws), nbytes,
                                           N, self.net.C0, self.net.H0, self.net.W0, _stream(stream)), "small_network_run_u8")


class PackedNetwork:
    """Device-resident form of a layer table: filters packed once into the blocked layout
    (by small_pack_filter / small_pack_dw_filter), workspace allocated once per batch size."""

    def __init__(self, net, weights, device="cuda:0"):
        self.net, self.device = net, torch.device(device)
        self.filters = []
        by_w = {L.w: L for L in net.layers if L.w is not None}
        for k, w in enumerate(weights):
            L = by_w[k]
            src = torch.from_numpy(w).to(self.device).contiguous()
            dst = torch.empty(src.numel(), dtype=torch.float32, device=self.device)
            if L.op == "dw":
                small_pack_dw_filter(src, dst, L.Ci, L.kh, L.kw, L.Cib)
            elif L.op == "bn":                   # [2][C]: scale, then shift, as they are
                dst.copy_(src.reshape(-1))
            elif L.op == "gconv":                # [Co][F_C][kh][kw] in the general layout with Ci = F_C
                small_pack_filter(src, dst, L.Co, L.F_C, L.kh, L.kw, L.Cob, min(16, L.F_C))
            else:
                small_pack_filter(src, dst, L.Co, L.Ci, L.kh, L.kw, L.Cob, L.Cib)
            self.filters.append(dst)
        self.table = make_layer_table(net.layers, self.filters)
        self._ws = {}

    def workspace(self, N):
        if N not in self._ws:
            nbytes = small_network_workspace(self.table, N, self.net.C0, self.net.H0, self.net.W0)
            self._ws[N] = (torch.empty(max(nbytes, 256) // 4, dtype=torch.float32, device=self.device), nbytes)
        return self._ws[N]

    def pack_input(self, x_nchw):
        N = x_nchw.shape[0]
        xb = torch.empty(x_nchw.numel(), dtype=torch.float32, device=self.device)
        small_pack(x_nchw, xb, N, self.net.C0, self.net.H0, self.net.W0, self.net.layers[0].Cib)
        return xb

    def out_elems(self, N):
        L = self.net.layers[-1]
        return N * L.Co * L.Ho * L.Wo

    def run(self, in_blocked, out_blocked, N, stream=None):
        ws, nbytes = self.workspace(N)
        small_network_run(self.table, in_blocked, out_blocked, ws, nbytes, N, self.net.C0, self.net.H0, self.net.W0,
                          stream)

    def run_opt(self, in_tensor, out_blocked, N, flags, stream=None):
        ws, nbytes = self.workspace(N)
        small_network_run_opt(self.table, in_tensor, out_blocked, ws, nbytes, N, self.net.C0, self.net.H0, self.net.W0,
                              flags, stream)

    def launches_at(self, N, flags=0):
        return small_network_launches_at(self.table, N, self.net.C0, self.net.H0, self.net.W0, flags)

    def run_plain(self, in_nchw, out_blocked, N, stream=None):
        """The run from a plain [N][C0][H0][W0] input (no small_pack launch); raises SmallError with
        SMALL_ERR_LAYER when the first layer cannot take a plain tensor."""
        ws, nbytes = self.workspace(N)
        small_network_run_plain(self.table, in_nchw, out_blocked, ws, nbytes, N, self.net.C0, self.net.H0,
                                self.net.W0, stream)

    def capture(self, in_blocked, out_blocked, N):
        """Records one run on these buffers into a HIP graph (torch.cuda.CUDAGraph). graph.replay() enqueues the
        same launches again without the per-launch host cost, which bounds small batches (about 4 us of host
        time per launch against kernels of a few microseconds). The library allocates nothing and never
        synchronises, so a run is capturable once every kernel has been launched once (first launches may
        set kernel attributes)."""
        self.run(in_blocked, out_blocked, N)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            self.run(in_blocked, out_blocked, N)
        return graph

    def run_range(self, in_blocked, out_blocked, N, first, count, stream=None):
        ws, nbytes = self.workspace(N)
        small_network_run_range(self.table, in_blocked, out_blocked, ws, nbytes, N, self.net.C0, self.net.H0,
                                self.net.W0, first, count, stream)
