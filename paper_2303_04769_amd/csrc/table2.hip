// The remaining layers of the paper's Table 2 on the shared blocked layout (gfx950): batch normalization
// (single-element reduction, FMA), nearest-neighbour upsampling (single element, strided mapping) and group
// convolution (partial-channel reduction, Table 1 row 3). None of them is on the networks' hot path: plain
// one-lane-per-output kernels, memory-bound, coalesced along the channel block.
#include "small_internal.h"

namespace small {

namespace {

constexpr int kBlock = 256;

// y = x * scale[c] + shift[c]; element e of [N][C/Cb][HW][Cb] belongs to channel ((e / (HW * Cb)) % nCb) * Cb + e % Cb.
// VEC = 4: Cb % 4 == 0 and 16-byte aligned tensors, the four lanes' channels are consecutive.
template <int VEC>
__global__ void __launch_bounds__(kBlock) batchnorm_kernel(const float *__restrict__ in, const float *__restrict__ scale,
                                                           const float *__restrict__ shift, float *__restrict__ out,
                                                           unsigned n_vec, int Cb, int nCb, FastDiv by_plane, FastDiv by_nCb,
                                                           FastDiv by_Cb, int relu)
{
    const unsigned v = blockIdx.x * kBlock + threadIdx.x;
    if (v >= n_vec) return;
    const int e = (int)v * VEC;                                  // element index (< 2^31, checked by the caller)
    // plane index and position inside the plane (planes hold HW * Cb elements): 32-bit divisions by launch constants
    const int plane = by_plane.div(e), within = e - plane * (int)by_plane.d;
    const int c = (plane - by_nCb.div(plane) * nCb) * Cb + (within - by_Cb.div(within) * Cb);
    if (VEC == 4) {
        const floatx4 x = __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(in + e));
        const floatx4 sc = *reinterpret_cast<const floatx4 *>(scale + c), sh = *reinterpret_cast<const floatx4 *>(shift + c);
        floatx4 y;
        y.x = fmaf(x.x, sc.x, sh.x); y.y = fmaf(x.y, sc.y, sh.y);
        y.z = fmaf(x.z, sc.z, sh.z); y.w = fmaf(x.w, sc.w, sh.w);
        if (relu) {
            y.x = y.x > 0.f ? y.x : 0.f; y.y = y.y > 0.f ? y.y : 0.f;
            y.z = y.z > 0.f ? y.z : 0.f; y.w = y.w > 0.f ? y.w : 0.f;
        }
        __builtin_nontemporal_store(y, reinterpret_cast<floatx4 *>(out + e));
    } else {
        const float y = fmaf(in[e], scale[c], shift[c]);
        out[e] = relu ? (y > 0.f ? y : 0.f) : y;
    }
}

// out[n][cb][oh][ow][:] = in[n][cb][oh / fh][ow / fw][:]. One lane per VEC output floats, so a wave's stores are one
// contiguous run of the output (streaming); the copies of an input pixel along a row are neighbouring lanes (one
// request to the cache), the copies along a column come from L2. Index arithmetic in 32 bits by launch constants.
struct UpsampleDivs { FastDiv per_px, Wo, Ho, fw, fh; };

template <int VEC>
__global__ void __launch_bounds__(kBlock) upsample_kernel(const float *__restrict__ in, float *__restrict__ out, unsigned n_vec,
                                                          int H, int W, int Cb, UpsampleDivs d)
{
    const unsigned v = blockIdx.x * kBlock + threadIdx.x;
    if (v >= n_vec) return;
    const int per_px = Cb / VEC, Wo = (int)d.Wo.d, Ho = (int)d.Ho.d;
    const int opx = d.per_px.div((int)v), q = (int)v - opx * per_px;        // output pixel over (plane, row, column)
    const int orow = d.Wo.div(opx), ow = opx - orow * Wo;                    // output row over (plane, row)
    const int plane = d.Ho.div(orow), oh = orow - plane * Ho;
    const size_t src = (((size_t)plane * H + d.fh.div(oh)) * W + d.fw.div(ow)) * Cb + q * VEC;
    if (VEC == 4)
        __builtin_nontemporal_store(*reinterpret_cast<const floatx4 *>(in + src), reinterpret_cast<floatx4 *>(out) + v);
    else
        out[v] = in[src];
}

struct GroupArgs {
    const float *in;
    const float *filt;
    float *out;
    int N, H, W, Ho, Wo;
    int Ci, F_C, S_C, K, Co;
    int Cib, F_Cb, Cob;
    int kh, kw, stride, pt, pl;
};

// One lane per output element, output channel fastest inside a block (filter reads coalesced, input reads
// broadcast within a group). Output channel oc = g * K + k reduces input channels g * S_C .. g * S_C + F_C - 1.
__global__ void __launch_bounds__(kBlock) group_conv_direct(GroupArgs a, size_t total)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= total) return;
    const size_t dst = e;
    const int co_in = (int)(e % a.Cob); e /= a.Cob;
    const int ow = (int)(e % a.Wo); e /= a.Wo;
    const int oh = (int)(e % a.Ho); e /= a.Ho;
    const int nCob = a.Co / a.Cob, nCib = a.Ci / a.Cib, nFb = a.F_C / a.F_Cb;
    const int cob = (int)(e % nCob);
    const int n = (int)(e / nCob);
    const int oc = cob * a.Cob + co_in;
    const int c0 = (oc / a.K) * a.S_C;               // first input channel of the group
    float acc = 0.f;
    for (int fc = 0; fc < a.F_C; ++fc) {
        const int ic = c0 + fc;
        const float *plane = a.in + (size_t)(n * nCib + ic / a.Cib) * a.H * a.W * a.Cib + ic % a.Cib;
        const float *wp = a.filt + ((size_t)(cob * nFb + fc / a.F_Cb) * a.kh * a.kw * a.F_Cb + fc % a.F_Cb) * a.Cob + co_in;
        for (int y = 0; y < a.kh; ++y) {
            const int ih = oh * a.stride - a.pt + y;
            if (ih < 0 || ih >= a.H) continue;
            for (int x = 0; x < a.kw; ++x) {
                const int iw = ow * a.stride - a.pl + x;
                if (iw < 0 || iw >= a.W) continue;
                acc = fmaf(plane[(size_t)(ih * a.W + iw) * a.Cib], wp[(size_t)(y * a.kw + x) * a.F_Cb * a.Cob], acc);
            }
        }
    }
    a.out[dst] = acc;
}

}  // namespace

hipError_t launch_batchnorm(const float *in, const float *scale, const float *shift, float *out, int N, int C, int H, int W,
                            int Cb, hipStream_t s, bool relu)
{
    const size_t total = (size_t)N * C * H * W;
    const FastDiv plane = make_fastdiv(H * W * Cb), by_nCb = make_fastdiv(C / Cb), by_Cb = make_fastdiv(Cb);
    // float4 accesses: blocks of a multiple of four channels, and scale / shift 16-byte aligned as well
    const bool vec = Cb % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)scale | (uintptr_t)shift) & 15u) == 0);
    const unsigned n = (unsigned)(vec ? total / 4 : total);
    if (vec)
        hipLaunchKernelGGL((batchnorm_kernel<4>), dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, in, scale, shift, out, n, Cb,
                           C / Cb, plane, by_nCb, by_Cb, relu ? 1 : 0);
    else
        hipLaunchKernelGGL((batchnorm_kernel<1>), dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, in, scale, shift, out, n, Cb,
                           C / Cb, plane, by_nCb, by_Cb, relu ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_upsample(const float *in, float *out, int N, int C, int H, int W, int fh, int fw, int Cb, hipStream_t s)
{
    const size_t total = (size_t)N * C * H * fh * W * fw;         // output elements (< 2^31: checked by the caller)
    const bool vec = Cb % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out) & 15u) == 0);
    const unsigned n = (unsigned)(vec ? total / 4 : total);
    const UpsampleDivs d = {make_fastdiv(vec ? Cb / 4 : Cb), make_fastdiv(W * fw), make_fastdiv(H * fh), make_fastdiv(fw),
                            make_fastdiv(fh)};
    if (vec) hipLaunchKernelGGL((upsample_kernel<4>), dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, in, out, n, H, W, Cb, d);
    else hipLaunchKernelGGL((upsample_kernel<1>), dim3((n + kBlock - 1) / kBlock), dim3(kBlock), 0, s, in, out, n, H, W, Cb, d);
    return hipGetLastError();
}

hipError_t launch_group_conv(const float *in, const float *filt, float *out, const LayerGeom &g, int F_C, int S_C, int K,
                             int F_Cb, hipStream_t s)
{
    // channel counts in whole 16-blocks and a geometry the matrix-core convolution takes: the same kernels, every
    // tile inside one group (Table 1 row "Partial Channel Reduction" on the full-reduction kernels)
    const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt) & 15u) == 0);
    const int tile = aligned && F_Cb == 16 ? group_conv_same_tile(g, F_C, S_C, K) : -1;
    if (tile >= 0) return launch_conv_same(in, filt, out, out, g, tile, EPI_NONE, s, F_C, S_C, K);
    GroupArgs a;
    a.in = in; a.filt = filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo;
    a.Ci = g.Ci; a.F_C = F_C; a.S_C = S_C; a.K = K; a.Co = g.Co;
    a.Cib = g.Cib; a.F_Cb = F_Cb; a.Cob = g.Cob;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    const size_t total = (size_t)g.N * g.Co * g.Ho * g.Wo;
    hipLaunchKernelGGL(group_conv_direct, dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, a, total);
    return hipGetLastError();
}

}  // namespace small
