// Single-channel reductions (paper Table 1 row 2; Section 3.2 item 2): depthwise
// convolution (FMA with one filter per channel, G_b = Cb, K_b = 1), max pooling and
// average pooling. HBM-bound: no matrix cores. One lane owns four adjacent channels of one
// output pixel (a 16-byte slice of the Cb-contiguous axis), so a wavefront covers 16
// consecutive pixels = 1 KiB of contiguous output, and window taps that overlap between
// neighbouring pixels are served by the vector L1 / L2 rather than by HBM.
#include "small_internal.h"

namespace small {

namespace {

constexpr int kBlock = 256;
enum : int { OP_DW = 0, OP_MAX = 1, OP_AVG = 2 };

__device__ __forceinline__ floatx4 ld4(const float *p) { return *reinterpret_cast<const floatx4 *>(p); }
__device__ __forceinline__ void st4(float *p, floatx4 v) { *reinterpret_cast<floatx4 *>(p) = v; }

__device__ __forceinline__ float max_first(float m, float v) { return (v > m) ? v : m; }   // first value seen wins ties

// grid.x = (image, channel block) plane, grid.y = chunks of kBlock lanes over Ho*Wo*(Cb/4).
// KS > 0: square KS x KS window fully unrolled; KS == 0: run-time kh x kw.
// CQ > 0: Cb/4 known at compile time; CQ == 0: run-time.
template <int OP, int KS, int CQ>
__global__ void __launch_bounds__(kBlock) window_vec4(const float *__restrict__ in, const float *__restrict__ filt,
                                                       float *__restrict__ out, LayerGeom g)
{
    const int Cb = g.Cib;
    const int cq = CQ > 0 ? CQ : Cb / 4;
    const int kh = KS > 0 ? KS : g.kh, kw = KS > 0 ? KS : g.kw;
    const int plane = blockIdx.x;
    const int e = blockIdx.y * kBlock + threadIdx.x;
    if (e >= g.Ho * g.Wo * cq) return;
    const int p = e / cq, c4 = (e - p * cq) * 4;
    const int oh = p / g.Wo, ow = p - oh * g.Wo;
    const int ih0 = oh * g.stride - g.pt, iw0 = ow * g.stride - g.pl;
    const float *src = in + (size_t)plane * g.H * g.W * Cb + c4;
    const int cb = plane % (g.Ci / Cb);
    const float *wsrc = (OP == OP_DW) ? filt + (size_t)cb * kh * kw * Cb + c4 : nullptr;

    floatx4 acc;
    if (OP == OP_MAX) acc = floatx4{-INFINITY, -INFINITY, -INFINITY, -INFINITY};
    else acc = floatx4{0.f, 0.f, 0.f, 0.f};
    int cnt = 0;
#pragma unroll
    for (int y = 0; y < kh; ++y) {
        const int ih = ih0 + y;
        if (ih < 0 || ih >= g.H) continue;
#pragma unroll
        for (int x = 0; x < kw; ++x) {
            const int iw = iw0 + x;
            if (iw < 0 || iw >= g.W) continue;
            const floatx4 v = ld4(src + (size_t)(ih * g.W + iw) * Cb);
            if (OP == OP_DW) {
                const floatx4 w = ld4(wsrc + (y * kw + x) * Cb);
                acc.x = fmaf(v.x, w.x, acc.x); acc.y = fmaf(v.y, w.y, acc.y);
                acc.z = fmaf(v.z, w.z, acc.z); acc.w = fmaf(v.w, w.w, acc.w);
            } else if (OP == OP_MAX) {
                acc.x = max_first(acc.x, v.x); acc.y = max_first(acc.y, v.y);
                acc.z = max_first(acc.z, v.z); acc.w = max_first(acc.w, v.w);
            } else {
                acc += v;
                ++cnt;
            }
        }
    }
    if (OP == OP_AVG) {
        const float d = (float)(cnt > 0 ? cnt : 1);
        acc.x /= d; acc.y /= d; acc.z /= d; acc.w /= d;
    }
    st4(out + ((size_t)plane * g.Ho * g.Wo + p) * Cb + c4, acc);
}

// Any block size: one lane per output element (used when Cb is not a multiple of 4).
template <int OP>
__global__ void __launch_bounds__(kBlock) window_scalar(const float *__restrict__ in, const float *__restrict__ filt,
                                                         float *__restrict__ out, LayerGeom g, size_t total)
{
    size_t e = (size_t)blockIdx.x * kBlock + threadIdx.x;
    if (e >= total) return;
    const size_t dst = e;
    const int Cb = g.Cib;
    const int c = (int)(e % Cb); e /= Cb;
    const int ow = (int)(e % g.Wo); e /= g.Wo;
    const int oh = (int)(e % g.Ho); e /= g.Ho;
    const size_t plane = e;
    const int cb = (int)(plane % (g.Ci / Cb));
    const float *src = in + plane * g.H * g.W * Cb + c;
    float acc = OP == OP_MAX ? -INFINITY : 0.f;
    int cnt = 0;
    for (int y = 0; y < g.kh; ++y) {
        const int ih = oh * g.stride - g.pt + y;
        if (ih < 0 || ih >= g.H) continue;
        for (int x = 0; x < g.kw; ++x) {
            const int iw = ow * g.stride - g.pl + x;
            if (iw < 0 || iw >= g.W) continue;
            const float v = src[(size_t)(ih * g.W + iw) * Cb];
            if (OP == OP_DW) acc = fmaf(v, filt[((size_t)(cb * g.kh + y) * g.kw + x) * Cb + c], acc);
            else if (OP == OP_MAX) acc = max_first(acc, v);
            else { acc += v; ++cnt; }
        }
    }
    if (OP == OP_AVG) acc /= (float)(cnt > 0 ? cnt : 1);
    out[dst] = acc;
}

// Global average pooling (window = whole image, no padding): one wavefront per (image,
// channel block) plane. Lane = (pixel slot, channel quad); every load instruction reads
// 1 KiB of contiguous input; the pixel slots are then folded with wavefront shuffles.
template <int CQ>
__global__ void __launch_bounds__(kBlock) global_avgpool(const float *__restrict__ in, float *__restrict__ out,
                                                          int planes, int HW)
{
    constexpr int Cb = CQ * 4, kSlots = 64 / CQ;
    const int plane = (blockIdx.x * kBlock + threadIdx.x) >> 6;
    if (plane >= planes) return;                      // uniform per wavefront
    const int lane = threadIdx.x & 63;
    const int slot = lane / CQ, c4 = (lane % CQ) * 4;
    const float *src = in + (size_t)plane * HW * Cb + c4;
    floatx4 acc{0.f, 0.f, 0.f, 0.f};
    for (int p = slot; p < HW; p += kSlots) acc += ld4(src + (size_t)p * Cb);
#pragma unroll
    for (int off = CQ; off < 64; off <<= 1) {
        acc.x += __shfl_xor(acc.x, off); acc.y += __shfl_xor(acc.y, off);
        acc.z += __shfl_xor(acc.z, off); acc.w += __shfl_xor(acc.w, off);
    }
    if (slot == 0) {
        const float d = (float)HW;
        st4(out + (size_t)plane * Cb + c4, floatx4{acc.x / d, acc.y / d, acc.z / d, acc.w / d});
    }
}

template <int OP>
hipError_t launch_window(const float *in, const float *filt, float *out, const LayerGeom &g, hipStream_t s)
{
    const int Cb = g.Cib;
    const int planes = g.N * (g.Ci / Cb);
    const bool vec = (Cb % 4 == 0) && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt) & 15u) == 0);
    if (vec) {
        const int cq = Cb / 4;
        const int per_plane = g.Ho * g.Wo * cq;
        const dim3 grid((unsigned)planes, (unsigned)((per_plane + kBlock - 1) / kBlock));
        const bool k3 = g.kh == 3 && g.kw == 3;
        if (k3 && cq == 4)
            hipLaunchKernelGGL((window_vec4<OP, 3, 4>), grid, dim3(kBlock), 0, s, in, filt, out, g);
        else if (cq == 4)
            hipLaunchKernelGGL((window_vec4<OP, 0, 4>), grid, dim3(kBlock), 0, s, in, filt, out, g);
        else
            hipLaunchKernelGGL((window_vec4<OP, 0, 0>), grid, dim3(kBlock), 0, s, in, filt, out, g);
    } else {
        const size_t total = (size_t)planes * g.Ho * g.Wo * Cb;
        hipLaunchKernelGGL((window_scalar<OP>), dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, in,
                           filt, out, g, total);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_dwconv(const float *in, const float *filt, float *out, const LayerGeom &g, hipStream_t s)
{
    return launch_window<OP_DW>(in, filt, out, g, s);
}

hipError_t launch_pool(const float *in, float *out, const LayerGeom &g, int mode, hipStream_t s)
{
    if (mode == 0) return launch_window<OP_MAX>(in, nullptr, out, g, s);
    const bool global = g.Ho == 1 && g.Wo == 1 && g.kh == g.H && g.kw == g.W && g.pt == 0 && g.pl == 0;
    const bool aligned = ((((uintptr_t)in | (uintptr_t)out) & 15u) == 0);
    if (global && aligned && (g.Cib == 16 || g.Cib == 8 || g.Cib == 4)) {
        const int planes = g.N * (g.Ci / g.Cib), HW = g.H * g.W;
        const dim3 grid((unsigned)((planes + 3) / 4));
        if (g.Cib == 16) hipLaunchKernelGGL((global_avgpool<4>), grid, dim3(kBlock), 0, s, in, out, planes, HW);
        else if (g.Cib == 8) hipLaunchKernelGGL((global_avgpool<2>), grid, dim3(kBlock), 0, s, in, out, planes, HW);
        else hipLaunchKernelGGL((global_avgpool<1>), grid, dim3(kBlock), 0, s, in, out, planes, HW);
        return hipGetLastError();
    }
    return launch_window<OP_AVG>(in, nullptr, out, g, s);
}

}  // namespace small
