// C-ABI layer of libsmall_hip (see include/small.h for the contract of every entry point).
// Everything here is host code: argument validation, shape arithmetic, the layer-table walk.
#include "../../include/small.h"
#include "small_internal.h"

#include <algorithm>
#include <utility>

#include <limits.h>
#include <string.h>

using namespace small;

namespace {

constexpr int kMaxBlock = 64;
constexpr size_t kMaxElems = (size_t)INT_MAX;   // kernels index a tensor with 32-bit element offsets
constexpr size_t kSlotAlign = 256;

inline hipStream_t as_stream(void *s) { return reinterpret_cast<hipStream_t>(s); }

inline int from_hip(hipError_t e) { return e == hipSuccess ? SMALL_OK : SMALL_ERR_LAUNCH; }

inline bool overlap(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb * sizeof(float) && b0 < a0 + na * sizeof(float);
}

// elems = product of the dims, or 0 when any dim is non-positive or the product exceeds kMaxElems
size_t elems(int a, int b, int c, int d)
{
    if (a <= 0 || b <= 0 || c <= 0 || d <= 0) return 0;
    size_t p = (size_t)a;
    const int rest[3] = {b, c, d};
    for (int v : rest) {
        if (p > kMaxElems / (size_t)v) return 0;
        p *= (size_t)v;
    }
    return p;
}

int check_block(int C, int Cb)
{
    if (C <= 0 || Cb <= 0) return SMALL_ERR_SHAPE;
    if (Cb > kMaxBlock) return SMALL_ERR_BLOCK;
    if (C % Cb) return SMALL_ERR_SHAPE;
    return SMALL_OK;
}

// Fills the geometry of a windowed layer and validates it. Cob/Co may equal Cib/Ci (pool, depthwise).
int window_geom(LayerGeom &g, int N, int Ci, int Co, int H, int W, int kh, int kw, int stride, small_pad pad, int Cib,
                int Cob, size_t *in_elems, size_t *out_elems)
{
    if (N <= 0 || H <= 0 || W <= 0 || kh <= 0 || kw <= 0 || stride <= 0) return SMALL_ERR_SHAPE;
    if (pad.t < 0 || pad.b < 0 || pad.l < 0 || pad.r < 0) return SMALL_ERR_SHAPE;
    int rc = check_block(Ci, Cib);
    if (rc) return rc;
    rc = check_block(Co, Cob);
    if (rc) return rc;
    // a window row/column that lies entirely in the padding would make empty reductions possible
    if (pad.t >= kh || pad.b >= kh || pad.l >= kw || pad.r >= kw) return SMALL_ERR_SHAPE;
    const int Ho = small_out_dim(H, kh, stride, pad.t, pad.b), Wo = small_out_dim(W, kw, stride, pad.l, pad.r);
    if (Ho <= 0 || Wo <= 0) return SMALL_ERR_SHAPE;
    *in_elems = elems(N, Ci, H, W);
    *out_elems = elems(N, Co, Ho, Wo);
    if (!*in_elems || !*out_elems) return SMALL_ERR_SHAPE;
    g.N = N; g.H = H; g.W = W; g.Ho = Ho; g.Wo = Wo; g.Ci = Ci; g.Co = Co; g.Cib = Cib; g.Cob = Cob;
    g.kh = kh; g.kw = kw; g.stride = stride; g.pt = pad.t; g.pl = pad.l;
    return SMALL_OK;
}

struct ConvPlan { LayerGeom g; size_t in_elems, out_elems, filt_elems; };

int plan_conv(ConvPlan &p, int N, int Ci, int Co, int H, int W, int kh, int kw, int stride, small_pad pad, int Cib,
              int Cob)
{
    int rc = window_geom(p.g, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, &p.in_elems, &p.out_elems);
    if (rc) return rc;
    p.filt_elems = elems(Co, Ci, kh, kw);
    return p.filt_elems ? SMALL_OK : SMALL_ERR_SHAPE;
}

// bn (EPI_BN): scale[0 .. Co) then shift[0 .. Co); the caller has made sure that the layer's kernel has that epilogue
// (conv_epilogue_takes_bn).
int run_conv(const float *in, const float *filt, float *out, const float *res, const ConvPlan &p, int epilogue,
             hipStream_t s, bool plain_input = false, const float *bn = nullptr)
{
    if (!in || !filt || !out) return SMALL_ERR_NULL;
    if ((epilogue & EPI_BN) && !bn) return SMALL_ERR_NULL;
    if (overlap(in, p.in_elems, out, p.out_elems) || overlap(filt, p.filt_elems, out, p.out_elems)) return SMALL_ERR_ALIAS;
    return from_hip(launch_conv(in, filt, out, res, p.g, epilogue, s, plain_input, bn));
}

}  // namespace

extern "C" {

int small_out_dim(int in, int k, int stride, int pad_lo, int pad_hi)
{
    if (in <= 0 || k <= 0 || stride <= 0 || pad_lo < 0 || pad_hi < 0) return 0;
    const long t = (long)in + pad_lo + pad_hi - k;
    if (t < 0) return 0;
    return (int)(t / stride) + 1;
}

const char *small_strerror(int code)
{
    switch (code) {
        case SMALL_OK: return "ok";
        case SMALL_ERR_NULL: return "null pointer";
        case SMALL_ERR_SHAPE: return "bad shape (non-positive dim, window does not fit, C % Cb != 0, or tensor too large)";
        case SMALL_ERR_BLOCK: return "channel block size has no kernel (Cb > 64)";
        case SMALL_ERR_ALIAS: return "input and output overlap";
        case SMALL_ERR_LAUNCH: return "HIP launch failed";
        case SMALL_ERR_WORKSPACE: return "workspace too small or misaligned";
        case SMALL_ERR_LAYER: return "malformed layer table";
        case SMALL_ERR_QUANT: return "quantization parameters out of range or reduction too long for int32";
        case SMALL_ERR_STATIC: return "table and batch need more workspace than the built-in array holds (SMALL_STATIC_WORKSPACE_BYTES)";
        default: return "unknown error";
    }
}

int small_pack(const float *nchw, float *blocked, int N, int C, int H, int W, int Cb, void *stream)
{
    if (!nchw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    const size_t n = elems(N, C, H, W);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap(nchw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack(nchw, blocked, N, C, H, W, Cb, false, as_stream(stream)));
}

int small_unpack(const float *blocked, float *nchw, int N, int C, int H, int W, int Cb, void *stream)
{
    if (!nchw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    const size_t n = elems(N, C, H, W);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap(nchw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack(blocked, nchw, N, C, H, W, Cb, true, as_stream(stream)));
}

int small_pack_filter(const float *oihw, float *blocked, int Co, int Ci, int kh, int kw, int Cob, int Cib, void *stream)
{
    if (!oihw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(Co, Cob)) return rc;
    if (int rc = check_block(Ci, Cib)) return rc;
    const size_t n = elems(Co, Ci, kh, kw);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap(oihw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack_filter(oihw, blocked, Co, Ci, kh, kw, Cob, Cib, as_stream(stream)));
}

int small_pack_dw_filter(const float *c1hw, float *blocked, int C, int kh, int kw, int Cb, void *stream)
{
    // [C][1][kh][kw] -> [C/Cb][kh][kw][Cb] is the general filter layout with one input channel per filter
    return small_pack_filter(c1hw, blocked, C, 1, kh, kw, Cb, 1, stream);
}

int small_conv2d(const float *in, const float *filt, float *out, int N, int Ci, int Co, int H, int W, int kh, int kw,
                 int stride, small_pad pad, int Cib, int Cob, void *stream)
{
    ConvPlan p;
    if (int rc = plan_conv(p, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob)) return rc;
    return run_conv(in, filt, out, nullptr, p, EPI_NONE, as_stream(stream));
}

const char *small_conv2d_kernel(int N, int Ci, int Co, int H, int W, int kh, int kw, int stride, small_pad pad,
                                int Cib, int Cob)
{
    ConvPlan p;
    if (plan_conv(p, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob)) return nullptr;
    return conv_kernel_name(p.g);
}

int small_dwconv2d(const float *in, const float *filt, float *out, int N, int C, int H, int W, int kh, int kw,
                   int stride, small_pad pad, int Cb, void *stream)
{
    LayerGeom g;
    size_t ni, no;
    if (int rc = window_geom(g, N, C, C, H, W, kh, kw, stride, pad, Cb, Cb, &ni, &no)) return rc;
    if (!in || !filt || !out) return SMALL_ERR_NULL;
    if (overlap(in, ni, out, no) || overlap(filt, (size_t)C * kh * kw, out, no)) return SMALL_ERR_ALIAS;
    return from_hip(launch_dwconv(in, filt, out, g, EPI_NONE, as_stream(stream)));
}

int small_pool2d(const float *in, float *out, int N, int C, int H, int W, int kh, int kw, int stride, small_pad pad,
                 int Cb, int mode, void *stream)
{
    LayerGeom g;
    size_t ni, no;
    if (mode != SMALL_POOL_MAX && mode != SMALL_POOL_AVG) return SMALL_ERR_SHAPE;
    if (int rc = window_geom(g, N, C, C, H, W, kh, kw, stride, pad, Cb, Cb, &ni, &no)) return rc;
    if (!in || !out) return SMALL_ERR_NULL;
    if (overlap(in, ni, out, no)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pool(in, out, g, mode, as_stream(stream)));
}

int small_relu(const float *in, float *out, size_t n_elems, void *stream)
{
    if (!in || !out) return SMALL_ERR_NULL;
    if (n_elems > (size_t)1 << 40) return SMALL_ERR_SHAPE;
    if (in != out && overlap(in, n_elems, out, n_elems)) return SMALL_ERR_ALIAS;
    return from_hip(launch_relu(in, out, n_elems, as_stream(stream)));
}

int small_add(const float *a, const float *b, float *out, size_t n_elems, void *stream)
{
    if (!a || !b || !out) return SMALL_ERR_NULL;
    if (n_elems > (size_t)1 << 40) return SMALL_ERR_SHAPE;
    if ((a != out && overlap(a, n_elems, out, n_elems)) || (b != out && overlap(b, n_elems, out, n_elems)))
        return SMALL_ERR_ALIAS;
    return from_hip(launch_add(a, b, out, n_elems, as_stream(stream)));
}

int small_dense(const float *in, const float *filt, float *out, int N, int Ci, int Co, int Cib, int Cob, void *stream)
{
    // Full reduction on a 1x1 image == 1x1 convolution over N "pixels" (one per image).
    ConvPlan p;
    const small_pad nopad = {0, 0, 0, 0};
    if (int rc = plan_conv(p, N, Ci, Co, 1, 1, 1, 1, 1, nopad, Cib, Cob)) return rc;
    return run_conv(in, filt, out, nullptr, p, EPI_NONE, as_stream(stream));
}

int small_batchnorm(const float *in, const float *scale, const float *shift, float *out, int N, int C, int H, int W, int Cb,
                    void *stream)
{
    if (!in || !scale || !shift || !out) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    const size_t n = elems(N, C, H, W);
    if (!n || (size_t)H * W * Cb > kMaxElems) return SMALL_ERR_SHAPE;
    if (in != out && overlap(in, n, out, n)) return SMALL_ERR_ALIAS;
    if (overlap(scale, (size_t)C, out, n) || overlap(shift, (size_t)C, out, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_batchnorm(in, scale, shift, out, N, C, H, W, Cb, as_stream(stream)));
}

int small_upsample(const float *in, float *out, int N, int C, int H, int W, int fh, int fw, int Cb, void *stream)
{
    if (!in || !out) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    if (fh <= 0 || fw <= 0 || H <= 0 || W <= 0 || (size_t)H * fh > kMaxElems || (size_t)W * fw > kMaxElems) return SMALL_ERR_SHAPE;
    const size_t ni = elems(N, C, H, W), no = elems(N, C, H * fh, W * fw);
    if (!ni || !no) return SMALL_ERR_SHAPE;
    if (overlap(in, ni, out, no)) return SMALL_ERR_ALIAS;
    return from_hip(launch_upsample(in, out, N, C, H, W, fh, fw, Cb, as_stream(stream)));
}

int small_group_conv2d(const float *in, const float *filt, float *out, int N, int Ci, int F_C, int S_C, int K, int H, int W,
                       int kh, int kw, int stride, small_pad pad, int Cib, int F_Cb, int Cob, void *stream)
{
    if (F_C <= 0 || S_C <= 0 || K <= 0 || F_C > Ci || (Ci - F_C) % S_C) return SMALL_ERR_SHAPE;
    const long groups = (Ci - F_C) / S_C + 1;
    if (groups * K > INT_MAX) return SMALL_ERR_SHAPE;
    const int Co = (int)(groups * K);
    if (int rc = check_block(F_C, F_Cb)) return rc;
    LayerGeom g;
    size_t ni, no;
    if (int rc = window_geom(g, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob, &ni, &no)) return rc;
    const size_t nf = elems(Co, F_C, kh, kw);
    if (!nf) return SMALL_ERR_SHAPE;
    if (!in || !filt || !out) return SMALL_ERR_NULL;
    if (overlap(in, ni, out, no) || overlap(filt, nf, out, no)) return SMALL_ERR_ALIAS;
    return from_hip(launch_group_conv(in, filt, out, g, F_C, S_C, K, F_Cb, as_stream(stream)));
}

// ---- quantized (uint8) layers

}  // extern "C"

namespace {

inline bool overlap_bytes(const void *a, size_t na, const void *b, size_t nb)
{
    const uintptr_t a0 = (uintptr_t)a, b0 = (uintptr_t)b;
    return a0 < b0 + nb && b0 < a0 + na;
}

// K: reduction length; |acc| <= K * 255 * 255 must stay below 2^31
int check_quant(const small_quant *q, long K, QuantParams &out)
{
    if (!q) return SMALL_ERR_NULL;
    if (q->zx < 0 || q->zx > 255 || q->zw < 0 || q->zw > 255 || q->zy < 0 || q->zy > 255) return SMALL_ERR_QUANT;
    if (q->mult < 0 || q->shift < 0 || q->shift > 31) return SMALL_ERR_QUANT;
    if (q->lo < 0 || q->hi > 255 || q->lo > q->hi) return SMALL_ERR_QUANT;
    if (K <= 0 || K * 255L * 255L >= (1L << 31)) return SMALL_ERR_QUANT;
    // Sums beyond +-amax saturate the output whatever they are (amax * mult / 2^shift >= 512 > 255 + 255), and
    // up to amax the scaled sum fits 32 bits: the kernels then clamp the sum first and work in 32 bits.
    int amax = 0;
    if (q->mult == 0) {
        amax = INT_MAX;
    } else {
        const __int128 num = (__int128)512 << q->shift;
        const __int128 need = (num + q->mult - 1) / q->mult;
        if (need > INT_MAX) amax = INT_MAX;
        else if (need * q->mult < ((__int128)((1LL << 31) - 1024) << q->shift)) amax = (int)need;
    }
    out = QuantParams{q->zx, q->zw, q->zy, q->mult, q->shift, q->lo, q->hi, amax};
    return SMALL_OK;
}

}  // namespace

extern "C" {

int small_pack_u8(const unsigned char *nchw, unsigned char *blocked, int N, int C, int H, int W, int Cb, void *stream)
{
    if (!nchw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    const size_t n = elems(N, C, H, W);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap_bytes(nchw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack_u8(nchw, blocked, N, C, H, W, Cb, false, as_stream(stream)));
}

int small_unpack_u8(const unsigned char *blocked, unsigned char *nchw, int N, int C, int H, int W, int Cb, void *stream)
{
    if (!nchw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(C, Cb)) return rc;
    const size_t n = elems(N, C, H, W);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap_bytes(nchw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack_u8(nchw, const_cast<unsigned char *>(blocked), N, C, H, W, Cb, true, as_stream(stream)));
}

int small_pack_filter_u8(const unsigned char *oihw, unsigned char *blocked, int Co, int Ci, int kh, int kw, int Cob,
                         int Cib, void *stream)
{
    if (!oihw || !blocked) return SMALL_ERR_NULL;
    if (int rc = check_block(Co, Cob)) return rc;
    if (int rc = check_block(Ci, Cib)) return rc;
    const size_t n = elems(Co, Ci, kh, kw);
    if (!n) return SMALL_ERR_SHAPE;
    if (overlap_bytes(oihw, n, blocked, n)) return SMALL_ERR_ALIAS;
    return from_hip(launch_pack_filter_u8(oihw, blocked, Co, Ci, kh, kw, Cob, Cib, as_stream(stream)));
}

int small_filter_sums_u8(const unsigned char *filt, int *sums, int Co, int Ci, int kh, int kw, int Cob, int Cib, void *stream)
{
    if (!filt || !sums) return SMALL_ERR_NULL;
    if (int rc = check_block(Co, Cob)) return rc;
    if (int rc = check_block(Ci, Cib)) return rc;
    const size_t n = elems(Co, Ci, kh, kw);
    if (!n) return SMALL_ERR_SHAPE;
    if ((long)Ci * kh * kw * 255L >= (1L << 31)) return SMALL_ERR_QUANT;
    if (overlap_bytes(filt, n, sums, (size_t)Co * sizeof(int))) return SMALL_ERR_ALIAS;
    return from_hip(launch_filter_sums_u8(filt, sums, Co, Ci, kh, kw, Cob, Cib, as_stream(stream)));
}

int small_conv2d_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int Ci, int Co, int H,
                    int W, int kh, int kw, int stride, small_pad pad, int Cib, int Cob, const small_quant *q,
                    const int *filt_sums, void *stream)
{
    ConvPlan p;
    if (int rc = plan_conv(p, N, Ci, Co, H, W, kh, kw, stride, pad, Cib, Cob)) return rc;
    QuantParams qp;
    if (int rc = check_quant(q, (long)Ci * kh * kw, qp)) return rc;
    if (!in || !filt || !out) return SMALL_ERR_NULL;
    if (overlap_bytes(in, p.in_elems, out, p.out_elems) || overlap_bytes(filt, p.filt_elems, out, p.out_elems))
        return SMALL_ERR_ALIAS;
    if (filt_sums) {
        if ((uintptr_t)filt_sums & 15u) return SMALL_ERR_SHAPE;
        if (overlap_bytes(filt_sums, (size_t)Co * sizeof(int), out, p.out_elems)) return SMALL_ERR_ALIAS;
    }
    return from_hip(launch_conv_u8(in, filt, out, p.g, qp, filt_sums, as_stream(stream)));
}

int small_dense_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int Ci, int Co, int Cib,
                   int Cob, const small_quant *q, const int *filt_sums, void *stream)
{
    const small_pad nopad = {0, 0, 0, 0};
    return small_conv2d_u8(in, filt, out, N, Ci, Co, 1, 1, 1, 1, 1, nopad, Cib, Cob, q, filt_sums, stream);
}

int small_dwconv2d_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int C, int H, int W,
                      int kh, int kw, int stride, small_pad pad, int Cb, const small_quant *q, void *stream)
{
    LayerGeom g;
    size_t ni, no;
    if (int rc = window_geom(g, N, C, C, H, W, kh, kw, stride, pad, Cb, Cb, &ni, &no)) return rc;
    QuantParams qp;
    if (int rc = check_quant(q, (long)kh * kw, qp)) return rc;
    const size_t nf = elems(C, 1, kh, kw);
    if (!nf) return SMALL_ERR_SHAPE;
    if (!in || !filt || !out) return SMALL_ERR_NULL;
    if (overlap_bytes(in, ni, out, no) || overlap_bytes(filt, nf, out, no)) return SMALL_ERR_ALIAS;
    return from_hip(launch_window_u8(in, filt, out, g, 0, qp, as_stream(stream)));
}

int small_pool2d_u8(const unsigned char *in, unsigned char *out, int N, int C, int H, int W, int kh, int kw, int stride,
                    small_pad pad, int Cb, int mode, void *stream)
{
    LayerGeom g;
    size_t ni, no;
    if (mode != SMALL_POOL_MAX && mode != SMALL_POOL_AVG) return SMALL_ERR_SHAPE;
    if (int rc = window_geom(g, N, C, C, H, W, kh, kw, stride, pad, Cb, Cb, &ni, &no)) return rc;
    if ((long)kh * kw * 255L >= (1L << 31)) return SMALL_ERR_SHAPE;
    if (!in || !out) return SMALL_ERR_NULL;
    if (overlap_bytes(in, ni, out, no)) return SMALL_ERR_ALIAS;
    const QuantParams none = {0, 0, 0, 0, 0, 0, 255, 0};
    return from_hip(launch_window_u8(in, nullptr, out, g, mode == SMALL_POOL_MAX ? 1 : 2, none, as_stream(stream)));
}

int small_relu_u8(const unsigned char *in, unsigned char *out, size_t n_elems, int z, void *stream)
{
    if (!in || !out) return SMALL_ERR_NULL;
    if (!n_elems || z < 0 || z > 255) return SMALL_ERR_SHAPE;
    if (in != out && overlap_bytes(in, n_elems, out, n_elems)) return SMALL_ERR_ALIAS;
    return from_hip(launch_relu_u8(in, out, n_elems, z, as_stream(stream)));
}


}  // extern "C"

namespace {

int check_quant_add(const small_quant_add *q, AddQuantParams &out)
{
    if (!q) return SMALL_ERR_NULL;
    if (q->za < 0 || q->za > 255 || q->zb < 0 || q->zb > 255 || q->zy < 0 || q->zy > 255) return SMALL_ERR_QUANT;
    if (q->mult_a < 0 || q->mult_b < 0 || q->shift < 0 || q->shift > 31) return SMALL_ERR_QUANT;
    if (q->lo < 0 || q->hi > 255 || q->lo > q->hi) return SMALL_ERR_QUANT;
    out = AddQuantParams{q->za, q->zb, q->zy, q->mult_a, q->mult_b, q->shift, q->lo, q->hi};
    return SMALL_OK;
}

// ---- a table of quantized layers over shared buffers: the walk of small_network_run on bytes, layer by layer.
struct ShapeU8 { int C, H, W, Cb; bool set; };

struct NetPlanU8 {
    size_t slot_bytes[SMALL_MAX_SLOTS];
    size_t slot_off[SMALL_MAX_SLOTS];
    size_t bytes;
};

inline bool valid_buf(int id) { return id >= SMALL_BUF_OUT && id < SMALL_MAX_SLOTS; }

// An in-place ReLU (zero point z) directly after layer i, whose lower clamp can take it: clamp(v, max(lo, z), hi)
// is relu(clamp(v, lo, hi)) for z <= hi, the same codes.
bool relu_follows_u8(const small_layer_u8 *L, int nL, int i)
{
    if (i + 1 >= nL) return false;
    const small_layer_u8 &l = L[i], &r = L[i + 1];
    if (r.op != SMALL_OP_RELU || r.src != l.dst || r.dst != l.dst) return false;
    const int hi = l.op == SMALL_OP_ADD ? l.qa.hi : l.q.hi;
    return r.q.zy >= 0 && r.q.zy <= hi;
}

// run = false: shapes, parameters and workspace sizes only. Every layer is checked before the first one runs
// (the caller walks twice).
int walk_u8(const small_layer_u8 *L, int nL, int N, int C0, int H0, int W0, NetPlanU8 &plan, bool run, const unsigned char *in,
            unsigned char *out, unsigned char *ws, hipStream_t s)
{
    if (!L || nL <= 0 || N <= 0 || C0 <= 0 || H0 <= 0 || W0 <= 0) return SMALL_ERR_SHAPE;
    ShapeU8 shp_store[SMALL_MAX_SLOTS + 2] = {};
    ShapeU8 *shp = shp_store + 2;                              // ids -2 .. SMALL_MAX_SLOTS - 1
    shp[SMALL_BUF_IN] = ShapeU8{C0, H0, W0, L[0].Cib, true};
    if (!run) {
        for (int k = 0; k < SMALL_MAX_SLOTS; ++k) plan.slot_bytes[k] = 0;
    }
    auto ptr = [&](int id) -> unsigned char * {
        if (id == SMALL_BUF_IN) return const_cast<unsigned char *>(in);
        if (id == SMALL_BUF_OUT) return out;
        return ws + plan.slot_off[id];
    };
    for (int i = 0; i < nL; ++i) {
        small_layer_u8 l = L[i];
        if (!valid_buf(l.src) || !valid_buf(l.dst) || l.dst == SMALL_BUF_IN || !shp[l.src].set) return SMALL_ERR_LAYER;
        const ShapeU8 si = shp[l.src];
        if (l.Ci != si.C || l.Cib != si.Cb) return SMALL_ERR_LAYER;
        const bool fold = (l.op == SMALL_OP_CONV || l.op == SMALL_OP_DWCONV || l.op == SMALL_OP_DENSE || l.op == SMALL_OP_ADD) &&
                          relu_follows_u8(L, nL, i);
        if (fold) {
            if (l.op == SMALL_OP_ADD) l.qa.lo = l.qa.lo > L[i + 1].q.zy ? l.qa.lo : L[i + 1].q.zy;
            else l.q.lo = l.q.lo > L[i + 1].q.zy ? l.q.lo : L[i + 1].q.zy;
        }
        ShapeU8 so = ShapeU8{l.Co, si.H, si.W, l.Cob, true};
        int rc = SMALL_OK;
        LayerGeom g;
        size_t ni = 0, no = 0;
        QuantParams qp;
        switch (l.op) {
        case SMALL_OP_CONV:
        case SMALL_OP_DENSE: {
            if (l.op == SMALL_OP_DENSE && (l.kh != si.H || l.kw != si.W)) return SMALL_ERR_LAYER;
            const small_pad pad = l.op == SMALL_OP_DENSE ? small_pad{0, 0, 0, 0} : l.pad;
            const int stride = l.op == SMALL_OP_DENSE ? 1 : l.stride;
            if ((rc = window_geom(g, N, l.Ci, l.Co, si.H, si.W, l.kh, l.kw, stride, pad, l.Cib, l.Cob, &ni, &no))) return rc;
            if ((rc = check_quant(&l.q, (long)l.Ci * l.kh * l.kw, qp))) return rc;
            if (!l.filt) return SMALL_ERR_NULL;
            so.H = g.Ho; so.W = g.Wo;
            if (run) rc = small_conv2d_u8(ptr(l.src), l.filt, ptr(l.dst), N, l.Ci, l.Co, si.H, si.W, l.kh, l.kw, stride, pad, l.Cib,
                                          l.Cob, &l.q, l.filt_sums, s);
            break;
        }
        case SMALL_OP_DWCONV:
            if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
            if ((rc = window_geom(g, N, l.Ci, l.Co, si.H, si.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cob, &ni, &no))) return rc;
            if ((rc = check_quant(&l.q, (long)l.kh * l.kw, qp))) return rc;
            if (!l.filt) return SMALL_ERR_NULL;
            so.H = g.Ho; so.W = g.Wo;
            if (run) rc = small_dwconv2d_u8(ptr(l.src), l.filt, ptr(l.dst), N, l.Ci, si.H, si.W, l.kh, l.kw, l.stride, l.pad, l.Cib,
                                            &l.q, s);
            break;
        case SMALL_OP_MAXPOOL:
        case SMALL_OP_AVGPOOL:
            if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
            if ((rc = window_geom(g, N, l.Ci, l.Co, si.H, si.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cob, &ni, &no))) return rc;
            so.H = g.Ho; so.W = g.Wo;
            if (run) rc = small_pool2d_u8(ptr(l.src), ptr(l.dst), N, l.Ci, si.H, si.W, l.kh, l.kw, l.stride, l.pad, l.Cib,
                                          l.op == SMALL_OP_MAXPOOL ? SMALL_POOL_MAX : SMALL_POOL_AVG, s);
            break;
        case SMALL_OP_RELU:
            if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
            if (l.q.zy < 0 || l.q.zy > 255) return SMALL_ERR_QUANT;
            if (run) rc = small_relu_u8(ptr(l.src), ptr(l.dst), (size_t)N * si.C * si.H * si.W, l.q.zy, s);
            break;
        case SMALL_OP_ADD: {
            if (l.Co != l.Ci || l.Cob != l.Cib || !valid_buf(l.src2) || !shp[l.src2].set) return SMALL_ERR_LAYER;
            const ShapeU8 s2 = shp[l.src2];
            if (s2.C != si.C || s2.H != si.H || s2.W != si.W || s2.Cb != si.Cb) return SMALL_ERR_LAYER;
            AddQuantParams ap;
            if ((rc = check_quant_add(&l.qa, ap))) return rc;
            if (run) rc = small_add_u8(ptr(l.src), ptr(l.src2), ptr(l.dst), (size_t)N * si.C * si.H * si.W, &l.qa, s);
            break;
        }
        default:
            return SMALL_ERR_LAYER;
        }
        if (rc) return rc;
        shp[l.dst] = so;
        if (!run && l.dst >= 0) {
            const size_t b = (size_t)N * so.C * so.H * so.W;
            if (b > plan.slot_bytes[l.dst]) plan.slot_bytes[l.dst] = b;
        }
        if (fold) ++i;                                         // the ReLU went into the layer's lower clamp
    }
    if (!run) {
        size_t off = 0;
        for (int k = 0; k < SMALL_MAX_SLOTS; ++k) {
            plan.slot_off[k] = off;
            off += (plan.slot_bytes[k] + 255) / 256 * 256;
        }
        plan.bytes = off;
    }
    return SMALL_OK;
}

}  // namespace

extern "C" {

int small_add_u8(const unsigned char *a, const unsigned char *b, unsigned char *out, size_t n_elems, const small_quant_add *q,
                 void *stream)
{
    AddQuantParams ap;
    if (int rc = check_quant_add(q, ap)) return rc;
    if (!a || !b || !out) return SMALL_ERR_NULL;
    if (!n_elems) return SMALL_ERR_SHAPE;
    if ((a != out && overlap_bytes(a, n_elems, out, n_elems)) || (b != out && overlap_bytes(b, n_elems, out, n_elems)))
        return SMALL_ERR_ALIAS;
    return from_hip(launch_add_u8(a, b, out, n_elems, ap, as_stream(stream)));
}

int small_network_workspace_u8(const small_layer_u8 *layers, int n_layers, int N, int C0, int H0, int W0, size_t *bytes)
{
    if (!bytes) return SMALL_ERR_NULL;
    NetPlanU8 plan;
    if (int rc = walk_u8(layers, n_layers, N, C0, H0, W0, plan, false, nullptr, nullptr, nullptr, nullptr)) return rc;
    *bytes = plan.bytes;
    return SMALL_OK;
}

int small_network_run_u8(const small_layer_u8 *layers, int n_layers, const unsigned char *in_blocked, unsigned char *out_blocked,
                         void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, void *stream)
{
    NetPlanU8 plan;
    if (int rc = walk_u8(layers, n_layers, N, C0, H0, W0, plan, false, nullptr, nullptr, nullptr, nullptr)) return rc;
    if (!in_blocked || !out_blocked) return SMALL_ERR_NULL;
    if (plan.bytes && (!workspace || workspace_bytes < plan.bytes || ((uintptr_t)workspace & 255u))) return SMALL_ERR_WORKSPACE;
    return walk_u8(layers, n_layers, N, C0, H0, W0, plan, true, in_blocked, out_blocked, static_cast<unsigned char *>(workspace),
                   as_stream(stream));
}

}  // extern "C"

// ------------------------------------------------------------------------------------------------
// Layer tables
namespace {

struct Shape { int C, H, W, Cb; bool set; };

struct NetPlan {
    size_t slot_elems[SMALL_MAX_SLOTS];
    size_t slot_off[SMALL_MAX_SLOTS];
    size_t bytes;
    size_t out_elems;   // largest tensor written to SMALL_BUF_OUT
};

inline size_t align_up(size_t v, size_t a) { return (v + a - 1) / a * a; }

inline bool reads(const small_layer &l, int id) { return l.src == id || (l.op == SMALL_OP_ADD && l.src2 == id); }

// Cross-layer fusion on the common layout (the paper's "abstract fused layer" direction): layers
// that follow a convolution and only touch its output element by element are folded into the
// convolution's STORE phase. The table keeps its meaning: every buffer that is read later holds
// exactly what the unfused sequence would have left there.
// pw > 0: layer i is a depthwise 3x3 and layer i + pw the 1x1 convolution that alone consumes its output; both
// run in one kernel (the depthwise buffer is never written), pw_relu: an in-place ReLU after that convolution.
// rename: the convolution's destination is the depthwise layer's source (two buffers used in turn); one kernel
// cannot overwrite the tensor its other workgroups still read, so it writes into the (dead) depthwise buffer
// instead and the runner swaps the memory behind the two logical buffers from then on.
// chain >= 2: layer i starts a run of `chain` pointwise layers (dense on 1x1 images, 1x1 stride-1 unpadded
// convolution), each consumed only by the next, that one kernel takes from the first layer's source to the last
// layer's destination; chain_idx / chain_relu: their table indices and whether an in-place ReLU follows each.
// The tensors between them are never written.
// head: layer i is an average pooling whose output only the fully connected layer i + 1 reads; when the pooling
// window turns out to be the whole image, both run in one kernel and the pooled tensor is never written.
// bn > 0: layer i + bn is an in-place batch normalization of layer i's result, folded into its store phase (EPI_BN).
struct Fusion {
    int epilogue; int out_id; int res_id; int skip; int pw; int pw_relu; int rename;
    int chain; int chain_idx[kChainMaxLayers]; int chain_relu[kChainMaxLayers];
    int head; int bn;
};

bool pointwise(const small_layer &l)
{
    if (l.op == SMALL_OP_CONV) {
        if (l.stride != 1 || l.pad.t || l.pad.b || l.pad.l || l.pad.r) return false;
    } else if (l.op != SMALL_OP_DENSE) {
        return false;
    }
    return l.kh == 1 && l.kw == 1 && l.dst != l.src && l.dst != SMALL_BUF_IN && chain_layer_eligible(l.Ci, l.Co, l.Cib, l.Cob);
}

// True when nothing from layer `from` on needs the tensor that buffer D holds at that point.
bool dead_from(const small_layer *L, int nL, int from, int D)
{
    for (int k = from; k < nL; ++k) {
        if (reads(L[k], D)) return false;
        if (L[k].dst == D) return true;
    }
    return D != SMALL_BUF_OUT;
}

// Fills f.chain* for the longest run of pointwise layers that starts at layer i; f.skip covers the run.
void plan_chain(const small_layer *L, int nL, int i, Fusion &f)
{
    int n = 0, end[kChainMaxLayers];
    int k = i;
    while (k < nL && n < kChainMaxLayers && pointwise(L[k])) {
        if (n > 0) {
            const small_layer &prev = L[f.chain_idx[n - 1]];
            // the previous result is this layer's input, and nothing else ever looks at it
            if (L[k].src != prev.dst || L[k].Ci != prev.Co || L[k].Cib != prev.Cob || !dead_from(L, nL, k + 1, prev.dst)) break;
        }
        f.chain_idx[n] = k;
        f.chain_relu[n] = 0;
        int next = k + 1;
        if (next < nL && L[next].op == SMALL_OP_RELU && L[next].src == L[k].dst && L[next].dst == L[k].dst) {
            f.chain_relu[n] = 1;
            ++next;
        }
        end[n++] = next;
        k = next;
    }
    if (n && L[i].Cib != 16) n = 0;
    // the run's output is a 16-blocked tensor in a buffer other than the run's input
    while (n && (L[f.chain_idx[n - 1]].Cob != 16 || L[f.chain_idx[n - 1]].dst == L[i].src)) --n;
    if (n < 2) return;
    f.chain = n;
    f.skip = end[n - 1] - i - 1;
    f.out_id = f.res_id = L[f.chain_idx[n - 1]].dst;
}

// What plan_fusion yields when the depthwise + pointwise kernel cannot take the layer (image geometry, alignment).
Fusion without_pointwise(Fusion f)
{
    if (f.pw) {
        f.skip = f.pw - 1;
        f.pw = 0;
        f.pw_relu = 0;
        f.rename = 0;
    }
    return f;
}

Fusion plan_fusion(const small_layer *L, int nL, int i, bool allow_chain = true)
{
    const small_layer &c = L[i];
    Fusion f = {EPI_NONE, c.dst, c.dst, 0, 0, 0, 0};
    const bool conv = c.op == SMALL_OP_CONV || c.op == SMALL_OP_DENSE;
    if (c.op == SMALL_OP_AVGPOOL && allow_chain && i + 1 < nL) {
        const small_layer &d = L[i + 1];
        if (d.op == SMALL_OP_DENSE && d.src == c.dst && d.kh == 1 && d.kw == 1 && d.Ci == c.Ci && d.Cib == c.Cib &&
            d.dst != c.src && d.dst != SMALL_BUF_IN && c.pad.t == 0 && c.pad.b == 0 && c.pad.l == 0 && c.pad.r == 0 &&
            avgpool_dense_eligible(c.Ci, c.Cib, d.Co, d.Cob) && dead_from(L, nL, i + 2, c.dst)) {
            f.head = 1;
            f.skip = 1;
            f.out_id = f.res_id = d.dst;
        }
        return f;
    }
    if (c.op == SMALL_OP_BATCHNORM) {
        // a ReLU in place on the normalized tensor runs in the normalization's kernel
        if (i + 1 < nL && L[i + 1].op == SMALL_OP_RELU && L[i + 1].src == c.dst && L[i + 1].dst == c.dst) {
            f.epilogue |= EPI_RELU;
            f.skip = 1;
        }
        return f;
    }
    if (!conv && c.op != SMALL_OP_DWCONV) return f;
    if (conv && allow_chain) {
        plan_chain(L, nL, i, f);
        if (f.chain) return f;
    }
    int j = i + 1;
    const int D = c.dst;
    // conv, norm (in place), [add], [ReLU]: the normalization becomes the first step of the store phase (where the
    // layer's kernel turns out to have no such epilogue, the runner takes this fusion back and runs the layers as the
    // table lists them)
    if (conv && j < nL && L[j].op == SMALL_OP_BATCHNORM && L[j].src == D && L[j].dst == D && L[j].Ci == c.Co &&
        L[j].Cib == c.Cob) {
        f.epilogue |= EPI_BN;
        f.bn = j - i;
        f.skip = 1;
        ++j;
    }
    if (conv && j < nL && L[j].op == SMALL_OP_ADD && L[j].src != L[j].src2 && (L[j].src == D || L[j].src2 == D)) {
        const int E = L[j].src == D ? L[j].src2 : L[j].src, T = L[j].dst;
        bool ok = (T == D || T == E) && T != c.src;
        if (ok && T == E) {
            if (E == SMALL_BUF_IN) ok = false;
            // the convolution's own buffer D is then never written: nobody may read it before it is rewritten, and
            // the caller's output buffer receives every write the table makes to it
            if (!dead_from(L, nL, j + 1, D)) ok = false;
        }
        if (ok) {
            f.epilogue |= EPI_ADD;
            f.out_id = T;
            f.res_id = E;
            ++f.skip;
            ++j;
        }
    }
    if (j < nL && L[j].op == SMALL_OP_RELU && L[j].src == f.out_id && L[j].dst == f.out_id) {
        f.epilogue |= EPI_RELU;
        ++f.skip;
        ++j;
    }
    if (c.op == SMALL_OP_DWCONV && j < nL && L[j].op == SMALL_OP_CONV && L[j].src == D && L[j].dst != SMALL_BUF_IN &&
        (L[j].dst != c.src || (c.src >= 0 && D >= 0)) && L[j].Cib == c.Cib && L[j].Ci == c.Ci &&
        L[j].pad.t == 0 && L[j].pad.b == 0 && L[j].pad.l == 0 && L[j].pad.r == 0 &&
        dwpw_eligible(c.Ci, L[j].Co, c.Cib, L[j].Cob, c.kh, c.kw, c.stride, L[j].kh, L[j].kw, L[j].stride)) {
        // the depthwise buffer D is never written: nobody may read it before it is rewritten
        if (L[j].dst == D || dead_from(L, nL, j + 1, D)) {
            f.pw = j - i;
            f.skip = j - i;
            f.rename = L[j].dst == c.src;
            const int T = L[j].dst;
            if (j + 1 < nL && L[j + 1].op == SMALL_OP_RELU && L[j + 1].src == T && L[j + 1].dst == T) {
                f.pw_relu = 1;
                ++f.skip;
            }
        }
    }
    return f;
}

// A run of depthwise + pointwise blocks that one launch of dwpw_run.hip takes: every block is a pair plan_fusion already
// joins (depthwise 3x3 -> 1x1 convolution, in-place ReLUs folded) on images of at most 64 pixels, each block reading what
// the one before wrote; strides, paddings and channel counts may change from block to block. The launch writes the last
// block's result only, so every other buffer the table writes inside the run must be dead afterwards.
struct DwpwRun {
    int n;                                  // blocks (0: no run)
    int dw_idx[kDwpwChainMaxBlocks], pw_idx[kDwpwChainMaxBlocks];
    DwpwRunBlock block[kDwpwChainMaxBlocks];
    int covered;                            // layers behind layer i that the launch covers
    int rename;                             // the result goes to the memory of the last depthwise layer's destination,
                                            // which then changes places with the memory of the last convolution's
    int head;                               // table index of a fully connected layer that closes the run (behind an
                                            // average over the whole image), or 0: the launch then writes that layer's
                                            // destination and never the run's last tensor
};

// The run of depthwise + pointwise blocks from layer i on (a depthwise layer whose input is an H x W image) that one
// launch of dwpw_run.hip takes at batch N. Pointer-free: the same answer whether the table is being planned or run.
DwpwRun plan_dwpw_run(const small_layer *L, int nL, int i, int H, int W, int N)
{
    DwpwRun r;
    memset(&r, 0, sizeof(r));
    int n = 0, k = i, C = L[i].Ci;
    while (k < nL && n < kDwpwChainMaxBlocks) {
        const small_layer &d = L[k];
        if (d.op != SMALL_OP_DWCONV || d.Ci != C || d.Cib != 16 || d.kh != 3 || d.kw != 3 || d.stride < 1) break;
        if (d.pad.t < 0 || d.pad.b < 0 || d.pad.l < 0 || d.pad.r < 0 || d.pad.t > 2 || d.pad.b > 2 || d.pad.l > 2 || d.pad.r > 2) break;
        const Fusion f = plan_fusion(L, nL, k);
        if (!f.pw) break;
        const small_layer &pw = L[k + f.pw];
        if (pw.Cob != 16 || pw.Co % 16) break;
        if (n > 0 && d.src != L[r.pw_idx[n - 1]].dst) break;
        const int Ho = small_out_dim(H, 3, d.stride, d.pad.t, d.pad.b), Wo = small_out_dim(W, 3, d.stride, d.pad.l, d.pad.r);
        if (Ho < 1 || Wo < 1 || (long)H * W > kDwpwRunMaxPixels || (long)Ho * Wo > kDwpwRunMaxPixels) break;
        r.dw_idx[n] = k;
        r.pw_idx[n] = k + f.pw;
        r.block[n] = DwpwRunBlock{d.filt, pw.filt, (f.epilogue & EPI_RELU) != 0, f.pw_relu, C, pw.Co, H, W, Ho, Wo, d.stride,
                                  d.pad.t, d.pad.l};
        ++n;
        C = pw.Co; H = Ho; W = Wo;
        k = k + f.skip + 1;
    }
    // shorten the run until its shapes fit, everything it does not write is dead behind it, and its result has a
    // place that is not its input
    for (; n >= 2; --n) {
        if (!dwpw_run_eligible(r.block, n)) continue;
        // a workgroup that holds one image takes it through the whole run: beyond one round of such workgroups a launch per
        // block is faster, and so is a later, shorter run on smaller images, several per workgroup (depthwise-separable
        // CNN at 384 / 512 / 1024 images: one run from the 12 x 12 images on 152 / 162 / 302 us, blocks up to the 3 x 3
        // images layer by layer and a run from there 133 / 147 / 216 us, all layer by layer 165 / 181 / 271 us)
        if (dwpw_run_images(r.block, n, N) == 1 && N > device_cus()) continue;
        const int last = r.pw_idx[n - 1], T = L[last].dst, S = L[i].src;
        const int after = last + 1 + r.block[n - 1].pw_relu;
        bool ok = T != SMALL_BUF_IN;
        for (int b = 0; b < n && ok; ++b) {
            const int ids[2] = {L[r.dw_idx[b]].dst, L[r.pw_idx[b]].dst};
            for (int id : ids)
                if (id != T && !dead_from(L, nL, after, id)) ok = false;
        }
        if (!ok) continue;
        bool same_shape = true;
        for (int b = 0; b < n; ++b)
            if (r.block[b].Cin != r.block[b].Cout || r.block[b].Hi != r.block[b].Ho || r.block[b].Wi != r.block[b].Wo) same_shape = false;
        int rename = 0;
        if (T == S && !same_shape) {
            // in place with changing shapes: workgroups would write over images others have not read yet
            const int B = L[r.dw_idx[n - 1]].dst;
            if (S < 0 || B < 0 || B == S) continue;
            rename = 1;
        }
        r.n = n;
        r.covered = after - 1 - i;
        r.rename = rename;
        // the network's head behind the run: average over the whole (last) image + fully connected layer
        if (after + 1 < nL && L[after].op == SMALL_OP_AVGPOOL && L[after].src == T && T >= 0) {
            const small_layer &pl = L[after], &d = L[after + 1];
            const DwpwRunBlock &lb = r.block[n - 1];
            const Fusion hf = plan_fusion(L, nL, after);
            if (hf.head && pl.kh == lb.Ho && pl.kw == lb.Wo && pl.Ci == lb.Cout && pl.Cib == 16 && d.dst != S &&
                dead_from(L, nL, after + 2, T)) {
                r.head = after + 1;
                r.covered += 2;
                r.rename = 0;
            }
        }
        return r;
    }
    r.n = 0;
    return r;
}

// The convolution groups from layer i on that may run as one image-resident launch (resident.hip): fills rg
// and the table index of every group's last layer, returns how many groups the launch takes (0: none).
// shp: the shapes the logical buffers hold before layer i (indexed by id + 2).
int plan_resident_run(const small_layer *L, int nL, int i, const Shape *shp_now, ResGroup *rg, int *last_layer,
                      bool in_plain, bool forced, int N)
{
    Shape shp[SMALL_MAX_SLOTS + 2];
    memcpy(shp, shp_now, sizeof(shp));
    bool closed[kResMaxLayers];
    unsigned long long produced = 0;      // buffers written inside the run so far
    int n = 0, k = i;
    while (k < nL && n < kResMaxLayers) {
        const small_layer &l = L[k];
        if (l.op == SMALL_OP_AVGPOOL && n > 0 && k + 1 < nL) {
            // a head: pooling over the whole image of the run's last result + fully connected layer
            const small_layer &d = L[k + 1];
            const Fusion fu = plan_fusion(L, nL, k);
            const Shape a = l.src >= SMALL_BUF_OUT && l.src < SMALL_MAX_SLOTS ? shp[l.src + 2] : Shape{};
            if (fu.head && d.filt && a.set && a.C == l.Ci && a.Cb == 16 && l.Cib == 16 && l.kh == a.H && l.kw == a.W &&
                l.src == rg[n - 1].dst && d.dst >= SMALL_BUF_OUT && d.dst < SMALL_MAX_SLOTS) {
                rg[n] = ResGroup{d.filt, l.src, d.dst, d.dst, l.Ci, d.Co, 16, d.Cob, a.H, a.W, 1, 1, l.kh, l.kw, 1, 0, 0,
                                 EPI_NONE, RESIDENT_HEAD, 0};
                last_layer[n] = k + 1;
                bool c = true;
                for (int id = SMALL_BUF_OUT; id < SMALL_MAX_SLOTS; ++id)
                    if (((produced >> (id + 2)) & 1ull) && id != d.dst && !dead_from(L, nL, k + 2, id)) c = false;
                closed[n] = c;
                ++n;
            }
            break;
        }
        if (l.op == SMALL_OP_DWCONV) {
            // depthwise convolution (+ ReLU in place)
            if (l.dst == l.src || l.dst == SMALL_BUF_IN || !l.filt || l.Co != l.Ci || l.Cib != 16 || l.Cob != 16) break;
            if (l.src < SMALL_BUF_OUT || l.src >= SMALL_MAX_SLOTS || l.dst < SMALL_BUF_OUT || l.dst >= SMALL_MAX_SLOTS) break;
            const Shape a = shp[l.src + 2];
            if (!a.set || a.C != l.Ci || a.Cb != l.Cib) break;
            ConvPlan p;
            if (plan_conv(p, 1, l.Ci, l.Ci, a.H, a.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cib)) break;
            const bool relu = k + 1 < nL && L[k + 1].op == SMALL_OP_RELU && L[k + 1].src == l.dst && L[k + 1].dst == l.dst;
            rg[n] = ResGroup{l.filt, l.src, l.dst, l.dst, l.Ci, l.Ci, 16, 16, a.H, a.W, p.g.Ho, p.g.Wo, l.kh, l.kw, l.stride,
                             l.pad.t, l.pad.l, relu ? EPI_RELU : EPI_NONE, RESIDENT_DW, 0};
            shp[l.dst + 2] = Shape{l.Ci, p.g.Ho, p.g.Wo, 16, true};
            const int next = k + 1 + (relu ? 1 : 0);
            last_layer[n] = next - 1;
            bool c = true;
            for (int id = SMALL_BUF_OUT; id < SMALL_MAX_SLOTS; ++id)
                if (((produced >> (id + 2)) & 1ull) && id != l.dst && !dead_from(L, nL, next, id)) c = false;
            closed[n] = c;
            produced |= 1ull << (l.dst + 2);
            ++n;
            k = next;
            continue;
        }
        if (l.op != SMALL_OP_CONV || l.dst == l.src || l.dst == SMALL_BUF_IN || !l.filt) break;
        if (l.src < SMALL_BUF_OUT || l.src >= SMALL_MAX_SLOTS || l.dst < SMALL_BUF_OUT || l.dst >= SMALL_MAX_SLOTS) break;
        const Shape a = shp[l.src + 2];
        if (!a.set || a.C != l.Ci || a.Cb != l.Cib) break;
        ConvPlan p;
        if (plan_conv(p, 1, l.Ci, l.Co, a.H, a.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cob)) break;
        const Fusion fu = plan_fusion(L, nL, k, false);
        if (fu.pw || fu.head || fu.chain || (fu.epilogue & EPI_BN)) break;
        // (the layers ahead have not been validated yet: ids taken from them are checked here)
        if (fu.out_id < SMALL_BUF_OUT || fu.out_id >= SMALL_MAX_SLOTS || fu.out_id == SMALL_BUF_IN ||
            fu.res_id < SMALL_BUF_OUT || fu.res_id >= SMALL_MAX_SLOTS)
            break;
        const Shape o = Shape{l.Co, p.g.Ho, p.g.Wo, l.Cob, true};
        if (fu.epilogue & EPI_ADD) {
            const Shape r = shp[fu.res_id + 2];
            if (!r.set || r.C != o.C || r.H != o.H || r.W != o.W || r.Cb != o.Cb) break;
        }
        // a first layer on fewer than 16 channels can only open a run, reading the network input
        const bool stem = l.Cib < 16;
        if (stem && !(k == 0 && n == 0 && l.src == SMALL_BUF_IN)) break;
        rg[n] = ResGroup{l.filt, l.src, fu.res_id, fu.out_id, l.Ci, l.Co, l.Cib, l.Cob, a.H, a.W, p.g.Ho, p.g.Wo,
                         l.kh, l.kw, l.stride, l.pad.t, l.pad.l, fu.epilogue, stem ? RESIDENT_STEM : RESIDENT_CONV,
                         stem && in_plain ? 1 : 0};
        shp[l.dst + 2] = o;
        shp[fu.out_id + 2] = o;
        const int next = k + 1 + fu.skip;
        last_layer[n] = next - 1;
        // closed: nothing the run has produced, other than this group's result, is read from here on
        bool c = true;
        for (int id = SMALL_BUF_OUT; id < SMALL_MAX_SLOTS; ++id)
            if (((produced >> (id + 2)) & 1ull) && id != fu.out_id && !dead_from(L, nL, next, id)) c = false;
        closed[n] = c;
        produced |= 1ull << (fu.out_id + 2);
        ++n;
        k = next;
    }
    if (n < 2) return 0;
    const int taken = resident_groups(rg, n, closed);
    if (!taken || forced) return taken;
    // Every layer of a run costs a workgroup a few microseconds of set-up, barrier and store whatever its size: with
    // little arithmetic per layer (depthwise-separable blocks on small images) the layer-by-layer kernels win.
    double macs = 0;
    for (int k = 0; k < taken; ++k) {
        const ResGroup &g = rg[k];
        const double per_out = g.kind == RESIDENT_DW ? (double)g.kh * g.kw
                             : (g.kind == RESIDENT_HEAD ? (double)g.Ci : (double)g.Ci * g.kh * g.kw);
        macs += per_out * g.Co * g.Ho * g.Wo;
    }
    // (measured break-even: the audio CNN, 0.27 M multiply-adds per layer, gains 2..10 % in one round and loses 10 %
    // in two; the depthwise-separable CNN, 0.09 M, always loses)
    const double least = N <= device_cus() ? 2.5e5 : 5e5;
    return macs >= least * taken ? taken : 0;
}

// Image-resident runs pay off when the batch is about one or two images per compute unit. A run costs rounds x
// (one image in one workgroup); layer-by-layer launches cost a fixed part plus a part per image, so with few images
// they win because most of the chip would idle for the time one image takes, and from three rounds on because
// their fixed part is spread over more images. Measured on the residual CNN (us, layer by layer / resident):
// 81 / 82 at 128 images, 96 / 82 at 160, 109 / 82 at 256, 141 / 156 at 384, 164 / 156 at 448, 169 / 156 at 512,
// 231 / 230 at 768, 289 / 305 at 1024.
bool resident_batch(int N, unsigned flags)
{
    if (flags & SMALL_RUN_RESIDENT_OFF) return false;
    if (flags & SMALL_RUN_RESIDENT_ON) return true;
    const int cus = device_cus();
    const int rounds = (N + cus - 1) / cus;
    if (rounds == 1) return 16 * N >= 9 * cus;        // at least 9/16 of a round: 144 images on 256 compute units
    if (rounds == 2) return 8 * N >= 14 * cus;        // at least 1 3/4 rounds: 448
    return false;
}

// Walks the table once: validates every layer, tracks the shape held by every logical buffer and
// the largest tensor written to every workspace slot. With `run` set, launches as it goes (the
// caller has already walked the table once without `run`, so no error can occur midway).
// in_plain: the network input is a plain [N][C0][H0][W0] tensor; only layer 0 may read it, and only as a
// convolution that launch_conv can feed from a plain tensor (the layout change then happens inside that kernel).
// flags: SMALL_RUN_*; heads / n_heads (optional, without `run`): the first layer of every launch a run would make.
int walk(const small_layer *L, int nL, int N, int C0, int H0, int W0, NetPlan &plan, bool run, const float *in_blocked,
         float *out_blocked, char *ws, hipStream_t s, int first = 0, int count = INT_MAX, unsigned flags = 0,
         int *heads = nullptr, int *n_heads = nullptr)
{
    const bool in_plain = (flags & SMALL_RUN_PLAIN_INPUT) != 0;
    const bool track = true;                           // follow which layers start a launch
    const bool resident = resident_batch(N, flags);
    if (n_heads) *n_heads = 0;
    if (!L) return SMALL_ERR_NULL;
    if (nL <= 0 || N <= 0 || C0 <= 0 || H0 <= 0 || W0 <= 0) return SMALL_ERR_SHAPE;
    Shape shp[SMALL_MAX_SLOTS + 2];
    memset(shp, 0, sizeof(shp));
    auto idx = [](int id) { return id + 2; };   // OUT(-2) -> 0, IN(-1) -> 1, slot k -> k + 2
    auto valid_id = [](int id) { return id >= SMALL_BUF_OUT && id < SMALL_MAX_SLOTS; };
    int phys[SMALL_MAX_SLOTS];                     // memory slot behind every logical slot id (see Fusion::rename)
    for (int k = 0; k < SMALL_MAX_SLOTS; ++k) phys[k] = k;
    unsigned may_swap = 0;
    auto ptr = [&](int id) -> float * {
        if (id == SMALL_BUF_IN) return const_cast<float *>(in_blocked);
        if (id == SMALL_BUF_OUT) return out_blocked;
        return reinterpret_cast<float *>(ws + plan.slot_off[phys[id]]);
    };
    if (!run) memset(&plan, 0, sizeof(plan));
    shp[idx(SMALL_BUF_IN)] = Shape{C0, H0, W0, L[0].Cib, true};
    if (check_block(C0, L[0].Cib)) return SMALL_ERR_SHAPE;

    int fused_away = 0;      // layers after the current one that its launch already covers
    for (int i = 0; i < nL; ++i) {
        const small_layer &l = L[i];
        const bool head = fused_away == 0;             // this layer starts a launch (it is not folded into an earlier one)
        if (fused_away > 0) --fused_away;
        if (!valid_id(l.src) || !valid_id(l.dst) || l.dst == SMALL_BUF_IN) return SMALL_ERR_LAYER;
        Fusion fu = {EPI_NONE, l.dst, l.dst, 0, 0, 0, 0};
        if (track && head) {
            fu = plan_fusion(L, nL, i);
            fused_away = fu.skip;
            if (n_heads) {
                if (heads) heads[*n_heads] = i;
                ++*n_heads;
            }
        }
        if (!run && l.op == SMALL_OP_DWCONV) {
            // a run may swap the memory behind these two slots: both must then hold either one's tensors
            const Fusion f = plan_fusion(L, nL, i);
            if (f.rename && l.src >= 0 && l.dst >= 0) may_swap |= (1u << l.src) | (1u << l.dst);
        }
        // a run of convolutions with every tensor between them in LDS, one image per workgroup
        int res_n = 0;
        ResGroup res_g[kResMaxLayers];
        if (track && head && resident && (l.op == SMALL_OP_CONV || l.op == SMALL_OP_DWCONV) && !fu.chain && valid_id(l.src) &&
            valid_id(l.dst) && (l.Cib == 16 || (i == 0 && l.op == SMALL_OP_CONV))) {
            int last_layer[kResMaxLayers];
            res_n = plan_resident_run(L, nL, i, shp, res_g, last_layer, in_plain, (flags & SMALL_RUN_RESIDENT_ON) != 0, N);
            if (in_plain && i == 0 && res_n && res_g[0].kind != RESIDENT_STEM) res_n = 0;
            if (res_n && run &&
                ((((uintptr_t)ptr(l.src) | (uintptr_t)ptr(res_g[res_n - 1].dst)) & 15u) ||
                 overlap(ptr(l.src), elems(N, l.Ci, shp[idx(l.src)].H, shp[idx(l.src)].W), ptr(res_g[res_n - 1].dst),
                         elems(N, res_g[res_n - 1].Co, res_g[res_n - 1].Ho, res_g[res_n - 1].Wo))))
                res_n = 0;
            if (res_n) {
                fused_away = last_layer[res_n - 1] - i;
                fu.pw = fu.pw_relu = fu.rename = fu.head = 0;      // the run covers what these would have fused
            }
        }
        const bool launch = run && head && i >= first && (long)i < (long)first + count;
        if (in_plain && reads(l, SMALL_BUF_IN) && !(i == 0 && l.op == SMALL_OP_CONV)) return SMALL_ERR_LAYER;
        const Shape a = shp[idx(l.src)];
        if (!a.set || a.C != l.Ci || a.Cb != l.Cib) return SMALL_ERR_LAYER;
        Shape o = a;
        const size_t in_elems = elems(N, a.C, a.H, a.W);
        int rc = SMALL_OK;
        switch (l.op) {
            case SMALL_OP_CONV:
            case SMALL_OP_DENSE: {
                ConvPlan p;
                const bool dense = l.op == SMALL_OP_DENSE;
                if (dense && (l.kh != a.H || l.kw != a.W)) return SMALL_ERR_LAYER;
                const small_pad nopad = {0, 0, 0, 0};
                rc = plan_conv(p, N, l.Ci, l.Co, a.H, a.W, l.kh, l.kw, dense ? 1 : l.stride, dense ? nopad : l.pad,
                               l.Cib, l.Cob);
                if (rc) return rc;
                if (l.dst == l.src) return SMALL_ERR_ALIAS;
                if (!l.filt) return SMALL_ERR_NULL;
                o = Shape{l.Co, p.g.Ho, p.g.Wo, l.Cob, true};
                if (head && (fu.epilogue & EPI_BN)) {
                    // the normalization is folded only into kernels that have the epilogue (geometry; when running
                    // also the pointers): otherwise this layer and the ones after it run as the table lists them
                    const small_layer &b = L[i + fu.bn];
                    bool ok = !fu.chain && !res_n && p.g.Cib == 16 && p.g.Cob == 16 && (conv_pw_eligible(p.g) || conv_same_eligible(p.g));
                    if (ok && run)
                        ok = b.filt && conv_epilogue_takes_bn(p.g, ptr(l.src), l.filt, ptr(fu.out_id),
                                                              (fu.epilogue & EPI_ADD) ? ptr(fu.res_id) : ptr(fu.out_id), b.filt);
                    if (!ok) {
                        fu = Fusion{EPI_NONE, l.dst, l.dst, 0, 0, 0, 0};
                        fused_away = 0;
                    }
                }
                const bool plain = in_plain && i == 0 && !res_n;
                if (plain) {
                    if (fu.chain) return SMALL_ERR_LAYER;        // a pointwise run does not start from a plain tensor
                    const bool with_ptrs = run && head;
                    if (!conv_takes_plain_input(p.g, with_ptrs ? ptr(l.src) : nullptr, with_ptrs ? l.filt : nullptr,
                                                with_ptrs ? ptr(fu.out_id) : nullptr, with_ptrs ? ptr(fu.res_id) : nullptr))
                        return SMALL_ERR_LAYER;
                }
                if (head && fu.chain) {
                    // the one-kernel run of pointwise layers needs 32-bit input offsets and, known only when running,
                    // aligned pointers; otherwise every layer of the run is planned on its own
                    bool ok = in_elems * sizeof(float) < (1ull << 32) && (size_t)N * a.H * a.W <= (size_t)INT_MAX - 64;
                    if (ok && run) {
                        uintptr_t bits = (uintptr_t)ptr(l.src) | (uintptr_t)ptr(fu.out_id);
                        for (int k = 0; k < fu.chain; ++k) bits |= (uintptr_t)L[fu.chain_idx[k]].filt;
                        const size_t n_out = elems(N, L[fu.chain_idx[fu.chain - 1]].Co, a.H, a.W);
                        ok = !(bits & 15u) && !overlap(ptr(l.src), in_elems, ptr(fu.out_id), n_out);
                    }
                    if (!ok) {
                        fu = plan_fusion(L, nL, i, false);
                        fused_away = fu.skip;
                    }
                }
                if (launch && fu.chain) {
                    ChainLayer cl[kChainMaxLayers];
                    for (int k = 0; k < fu.chain; ++k) {
                        const small_layer &t = L[fu.chain_idx[k]];
                        if (!t.filt) return SMALL_ERR_NULL;
                        cl[k] = ChainLayer{t.filt, t.Ci, t.Co, fu.chain_relu[k]};
                    }
                    rc = from_hip(launch_dense_chain(ptr(l.src), ptr(fu.out_id), cl, fu.chain, (long)N * a.H * a.W, a.H * a.W, s));
                } else if (launch && res_n) {
                    rc = from_hip(launch_resident(res_g, res_n, ptr(l.src), ptr(res_g[res_n - 1].dst), N, s));
                } else if (launch) {
                    rc = run_conv(ptr(l.src), l.filt, ptr(fu.out_id), ptr(fu.res_id), p, fu.epilogue, s, plain,
                                  (fu.epilogue & EPI_BN) ? L[i + fu.bn].filt : nullptr);
                }
                break;
            }
            case SMALL_OP_DWCONV:
            case SMALL_OP_MAXPOOL:
            case SMALL_OP_AVGPOOL: {
                LayerGeom g;
                size_t ni, no;
                if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
                rc = window_geom(g, N, l.Ci, l.Ci, a.H, a.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cib, &ni, &no);
                if (rc) return rc;
                if (l.dst == l.src) return SMALL_ERR_ALIAS;
                if (l.op == SMALL_OP_DWCONV && !l.filt) return SMALL_ERR_NULL;
                o = Shape{l.Ci, g.Ho, g.Wo, l.Cib, true};
                // several such blocks in a row on small images: one launch for the whole run
                DwpwRun dr;
                dr.n = 0;
                if (head && fu.pw && !res_n && l.op == SMALL_OP_DWCONV && l.Cib == 16 && (long)a.H * a.W <= kDwpwRunMaxPixels &&
                    in_elems * sizeof(float) < ((size_t)1 << 32)) {
                    dr = plan_dwpw_run(L, nL, i, a.H, a.W, N);
                    if (dr.n && run) {
                        const small_layer &ldw = L[dr.dw_idx[dr.n - 1]], &lpw = L[dr.pw_idx[dr.n - 1]];
                        const DwpwRunBlock &lb = dr.block[dr.n - 1];
                        const float *rin = ptr(l.src);
                        float *rout = ptr(dr.head ? L[dr.head].dst : (dr.rename ? ldw.dst : lpw.dst));
                        const size_t out_elems = dr.head ? (size_t)N * L[dr.head].Co : (size_t)N * lb.Cout * lb.Ho * lb.Wo;
                        uintptr_t bits = (uintptr_t)rin | (uintptr_t)(dr.head ? nullptr : rout);
                        for (int b = 0; b < dr.n; ++b) bits |= (uintptr_t)dr.block[b].dw | (uintptr_t)dr.block[b].pw;
                        if (dr.head && !L[dr.head].filt) bits |= 1u;
                        if ((bits & 15u) || (rin != rout && overlap(rin, in_elems, rout, out_elems)) || (dr.head && rin == rout))
                            dr.n = 0;
                    }
                }
                if (!dr.n && head && fu.pw && !res_n) {
                    // the one-kernel depthwise + pointwise path also needs a geometry and (known only when running)
                    // pointers it can take; otherwise the pointwise convolution becomes a launch of its own
                    const small_layer &pw = L[i + fu.pw];
                    bool ok = dwpw_geom_ok(g, pw.Co);
                    if (ok && run)
                        ok = !(((uintptr_t)ptr(l.src) | (uintptr_t)ptr(fu.rename ? l.dst : pw.dst) | (uintptr_t)l.filt |
                                (uintptr_t)pw.filt) & 15u);
                    if (!ok) {
                        fu = without_pointwise(fu);
                        fused_away = fu.skip;
                    }
                }
                if (dr.n) {
                    const small_layer &ldw = L[dr.dw_idx[dr.n - 1]], &lpw = L[dr.pw_idx[dr.n - 1]];
                    fused_away = dr.covered;
                    const DwpwRunHead hd = dr.head ? DwpwRunHead{L[dr.head].filt, L[dr.head].Co, L[dr.head].Cob} : DwpwRunHead{nullptr, 0, 0};
                    if (launch)
                        rc = from_hip(launch_dwpw_run(ptr(l.src), ptr(dr.head ? L[dr.head].dst : (dr.rename ? ldw.dst : lpw.dst)),
                                                      dr.block, dr.n, N, hd, s));
                    if (dr.rename) std::swap(phys[ldw.dst], phys[lpw.dst]);
                } else if (l.op == SMALL_OP_DWCONV && res_n) {
                    if (launch) rc = from_hip(launch_resident(res_g, res_n, ptr(l.src), ptr(res_g[res_n - 1].dst), N, s));
                } else if (l.op == SMALL_OP_DWCONV && fu.pw) {
                    const small_layer &pw = L[i + fu.pw];
                    float *dst = ptr(fu.rename ? l.dst : pw.dst);
                    if (launch)
                        rc = from_hip(launch_dwpw(ptr(l.src), l.filt, pw.filt, dst, g, pw.Co,
                                                  (fu.epilogue & EPI_RELU) != 0, fu.pw_relu, s));
                    if (fu.rename) std::swap(phys[l.dst], phys[pw.dst]);
                } else if (head && fu.head) {
                    // pooling over the whole image + the fully connected layer in one kernel, if that is what it is
                    // (and, known only when running, if the pointers are aligned)
                    const small_layer &d = L[i + 1];
                    const bool global = g.Ho == 1 && g.Wo == 1 && l.kh == a.H && l.kw == a.W;
                    if (!global || (run && (!d.filt || (((uintptr_t)ptr(l.src) | (uintptr_t)d.filt) & 15u)))) {
                        fu.head = 0;
                        fused_away = 0;
                        if (launch) rc = from_hip(launch_pool(ptr(l.src), ptr(l.dst), g, SMALL_POOL_AVG, s));
                    } else if (launch) {
                        rc = from_hip(launch_avgpool_dense(ptr(l.src), d.filt, ptr(d.dst), N, l.Ci, a.H * a.W, d.Co, d.Cob, s));
                    }
                } else if (launch) {
                    if (l.op == SMALL_OP_DWCONV)
                        rc = from_hip(launch_dwconv(ptr(l.src), l.filt, ptr(l.dst), g, fu.epilogue, s));
                    else rc = from_hip(launch_pool(ptr(l.src), ptr(l.dst), g,
                                                   l.op == SMALL_OP_MAXPOOL ? SMALL_POOL_MAX : SMALL_POOL_AVG, s));
                }
                break;
            }
            case SMALL_OP_RELU:
                if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
                if (launch) rc = from_hip(launch_relu(ptr(l.src), ptr(l.dst), in_elems, s));
                break;
            case SMALL_OP_BATCHNORM:
                if (l.Co != l.Ci || l.Cob != l.Cib) return SMALL_ERR_LAYER;
                if (!l.filt) return SMALL_ERR_NULL;
                if ((size_t)a.H * a.W * a.Cb > kMaxElems) return SMALL_ERR_SHAPE;
                if (launch)
                    rc = from_hip(launch_batchnorm(ptr(l.src), l.filt, l.filt + l.Ci, ptr(l.dst), N, l.Ci, a.H, a.W, l.Cib, s,
                                                   (fu.epilogue & EPI_RELU) != 0));
                break;
            case SMALL_OP_UPSAMPLE: {
                if (l.Co != l.Ci || l.Cob != l.Cib || l.kh <= 0 || l.kw <= 0) return SMALL_ERR_LAYER;
                if (l.dst == l.src) return SMALL_ERR_ALIAS;
                if ((size_t)a.H * l.kh > kMaxElems || (size_t)a.W * l.kw > kMaxElems) return SMALL_ERR_SHAPE;
                o = Shape{l.Ci, a.H * l.kh, a.W * l.kw, l.Cib, true};
                if (!elems(N, o.C, o.H, o.W)) return SMALL_ERR_SHAPE;
                if (launch) rc = from_hip(launch_upsample(ptr(l.src), ptr(l.dst), N, l.Ci, a.H, a.W, l.kh, l.kw, l.Cib, s));
                break;
            }
            case SMALL_OP_GROUPCONV: {
                if (l.F_C <= 0 || l.S_C <= 0 || l.F_C > l.Ci || (l.Ci - l.F_C) % l.S_C) return SMALL_ERR_LAYER;
                const int groups = (l.Ci - l.F_C) / l.S_C + 1;
                if (l.Co <= 0 || l.Co % groups) return SMALL_ERR_LAYER;
                const int F_Cb = l.F_C < 16 ? l.F_C : 16;
                if (l.F_C % F_Cb) return SMALL_ERR_LAYER;
                LayerGeom g;
                size_t ni, no;
                rc = window_geom(g, N, l.Ci, l.Co, a.H, a.W, l.kh, l.kw, l.stride, l.pad, l.Cib, l.Cob, &ni, &no);
                if (rc) return rc;
                if (l.dst == l.src) return SMALL_ERR_ALIAS;
                if (!l.filt) return SMALL_ERR_NULL;
                if (!elems(l.Co, l.F_C, l.kh, l.kw)) return SMALL_ERR_SHAPE;
                o = Shape{l.Co, g.Ho, g.Wo, l.Cob, true};
                if (launch)
                    rc = from_hip(launch_group_conv(ptr(l.src), l.filt, ptr(l.dst), g, l.F_C, l.S_C, l.Co / groups, F_Cb, s));
                break;
            }
            case SMALL_OP_ADD: {
                if (l.Co != l.Ci || l.Cob != l.Cib || !valid_id(l.src2)) return SMALL_ERR_LAYER;
                const Shape b = shp[idx(l.src2)];
                if (!b.set || b.C != a.C || b.H != a.H || b.W != a.W || b.Cb != a.Cb) return SMALL_ERR_LAYER;
                if (launch) rc = from_hip(launch_add(ptr(l.src), ptr(l.src2), ptr(l.dst), in_elems, s));
                break;
            }
            default:
                return SMALL_ERR_LAYER;
        }
        if (rc) return rc;
        const size_t out_elems = elems(N, o.C, o.H, o.W);
        if (!out_elems) return SMALL_ERR_SHAPE;
        shp[idx(l.dst)] = o;
        if (!run && l.dst >= 0 && out_elems > plan.slot_elems[l.dst]) plan.slot_elems[l.dst] = out_elems;
        if (!run && l.dst == SMALL_BUF_OUT && out_elems > plan.out_elems) plan.out_elems = out_elems;
    }
    if (flags & SMALL_RUN_PLAIN_OUTPUT) {
        // The caller takes the result as a plain [N][C][H][W] tensor. That is what the last layer writes anyway when
        // the two layouts coincide: one pixel per image and one channel block (the logits of a classifier head).
        const Shape &r = shp[idx(SMALL_BUF_OUT)];
        if (!r.set || r.H != 1 || r.W != 1 || r.C != r.Cb) return SMALL_ERR_LAYER;
    }
    if (!run) {
        size_t m = 0;
        for (int k = 0; k < SMALL_MAX_SLOTS; ++k)
            if ((may_swap >> k) & 1u) m = std::max(m, plan.slot_elems[k]);
        for (int k = 0; k < SMALL_MAX_SLOTS; ++k)
            if ((may_swap >> k) & 1u) plan.slot_elems[k] = m;
        size_t off = 0;
        for (int k = 0; k < SMALL_MAX_SLOTS; ++k) {
            plan.slot_off[k] = off;
            off += align_up(plan.slot_elems[k] * sizeof(float), kSlotAlign);
        }
        plan.bytes = off;
    }
    return SMALL_OK;
}

}  // namespace

extern "C" {

int small_network_workspace(const small_layer *layers, int n_layers, int N, int C0, int H0, int W0, size_t *bytes)
{
    if (!bytes) return SMALL_ERR_NULL;
    NetPlan plan;
    const int rc = walk(layers, n_layers, N, C0, H0, W0, plan, false, nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
    *bytes = plan.bytes;
    return SMALL_OK;
}

int small_network_launches(const small_layer *layers, int n_layers, int *first_layer, int *n_launches)
{
    if (!layers || !n_launches) return SMALL_ERR_NULL;
    if (n_layers <= 0) return SMALL_ERR_SHAPE;
    int n = 0;
    for (int i = 0; i < n_layers; ++i) {
        if (first_layer) first_layer[n] = i;
        ++n;
        i += plan_fusion(layers, n_layers, i).skip;
    }
    *n_launches = n;
    return SMALL_OK;
}

static int network_run_impl(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, int first, int count,
                            void *stream, unsigned flags = 0);

int small_network_run_opt(const small_layer *layers, int n_layers, const float *in, float *out_blocked, void *workspace,
                          size_t workspace_bytes, int N, int C0, int H0, int W0, unsigned flags, void *stream)
{
    if (flags & ~(unsigned)(SMALL_RUN_PLAIN_INPUT | SMALL_RUN_RESIDENT_OFF | SMALL_RUN_RESIDENT_ON | SMALL_RUN_PLAIN_OUTPUT)) return SMALL_ERR_SHAPE;
    return network_run_impl(layers, n_layers, in, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, 0, INT_MAX,
                            stream, flags);
}

int small_network_launches_at(const small_layer *layers, int n_layers, int N, int C0, int H0, int W0, unsigned flags,
                              int *first_layer, int *n_launches)
{
    if (!layers || !n_launches) return SMALL_ERR_NULL;
    if (flags & ~(unsigned)(SMALL_RUN_PLAIN_INPUT | SMALL_RUN_RESIDENT_OFF | SMALL_RUN_RESIDENT_ON | SMALL_RUN_PLAIN_OUTPUT)) return SMALL_ERR_SHAPE;
    NetPlan plan;
    return walk(layers, n_layers, N, C0, H0, W0, plan, false, nullptr, nullptr, nullptr, nullptr, 0, INT_MAX, flags,
                first_layer, n_launches);
}

int small_network_run_plain(const small_layer *layers, int n_layers, const float *in_nchw, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, void *stream)
{
    return network_run_impl(layers, n_layers, in_nchw, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, 0,
                            INT_MAX, stream, SMALL_RUN_PLAIN_INPUT);
}

// The layer workspace of small_network_run_static: one array per GPU, part of the library's device image, held from
// the moment the library is loaded on that GPU until the process ends.
static __device__ __align__(256) unsigned char scratch[SMALL_STATIC_WORKSPACE_BYTES];

namespace {
constexpr int kMaxDevices = 64;
void *g_scratch_ptr[kMaxDevices];      // the array's address on every device that has asked for it

// The device address of `scratch` on the current device (in host code the array's name is not an address).
int scratch_address(void **ptr)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return SMALL_ERR_LAUNCH;
    void *q = __atomic_load_n(&g_scratch_ptr[dev], __ATOMIC_ACQUIRE);
    if (!q) {
        if (hipGetSymbolAddress(&q, HIP_SYMBOL(scratch)) != hipSuccess || !q) return SMALL_ERR_LAUNCH;
        __atomic_store_n(&g_scratch_ptr[dev], q, __ATOMIC_RELEASE);     // every thread obtains the same address
    }
    *ptr = q;
    return SMALL_OK;
}
}  // namespace

int small_network_run_static(const small_layer *layers, int n_layers, const float *in, float *out_blocked, int N, int C0,
                             int H0, int W0, unsigned flags, void *stream)
{
    if (flags & ~(unsigned)(SMALL_RUN_PLAIN_INPUT | SMALL_RUN_RESIDENT_OFF | SMALL_RUN_RESIDENT_ON | SMALL_RUN_PLAIN_OUTPUT)) return SMALL_ERR_SHAPE;
    size_t need = 0;
    if (int rc = small_network_workspace(layers, n_layers, N, C0, H0, W0, &need)) return rc;
    if (need > (size_t)SMALL_STATIC_WORKSPACE_BYTES) return SMALL_ERR_STATIC;
    void *ws = nullptr;
    if (int rc = scratch_address(&ws)) return rc;
    return network_run_impl(layers, n_layers, in, out_blocked, ws, (size_t)SMALL_STATIC_WORKSPACE_BYTES, N, C0, H0, W0, 0,
                            INT_MAX, stream, flags);
}

int small_network_run_range(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, int first, int count,
                            void *stream)
{
    if (first < 0 || count < 0) return SMALL_ERR_SHAPE;
    return network_run_impl(layers, n_layers, in_blocked, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, first,
                            count, stream);
}

int small_network_run(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                      void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, void *stream)
{
    return network_run_impl(layers, n_layers, in_blocked, out_blocked, workspace, workspace_bytes, N, C0, H0, W0, 0,
                            INT_MAX, stream);
}

static int network_run_impl(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, int first, int count,
                            void *stream, unsigned flags)
{
    NetPlan plan;
    int rc = walk(layers, n_layers, N, C0, H0, W0, plan, false, nullptr, nullptr, nullptr, nullptr, 0, INT_MAX, flags);
    if (rc) return rc;
    if (!in_blocked || !out_blocked) return SMALL_ERR_NULL;
    if (plan.bytes && !workspace) return SMALL_ERR_NULL;
    if (workspace_bytes < plan.bytes || ((uintptr_t)workspace % kSlotAlign)) return SMALL_ERR_WORKSPACE;
    const size_t in_elems = elems(N, C0, H0, W0), ws_elems = plan.bytes / sizeof(float);
    if (overlap(in_blocked, in_elems, out_blocked, plan.out_elems) ||
        (plan.bytes && (overlap(in_blocked, in_elems, workspace, ws_elems) ||
                        overlap(out_blocked, plan.out_elems, workspace, ws_elems))))
        return SMALL_ERR_ALIAS;
    return walk(layers, n_layers, N, C0, H0, W0, plan, true, in_blocked, out_blocked, static_cast<char *>(workspace),
                as_stream(stream), first, count, flags);
}

}  // extern "C"
