// Single-channel reductions (paper Table 1 row 2; Section 3.2 item 2): depthwise
// convolution (FMA with one filter per channel, G_b = Cb, K_b = 1), max pooling and
// average pooling. HBM-bound: no matrix cores. One lane owns four adjacent channels of one
// output pixel (a 16-byte slice of the Cb-contiguous axis), so a wavefront covers 16
// consecutive pixels = 1 KiB of contiguous output, and window taps that overlap between
// neighbouring pixels are served from an LDS tile (Cb = 16) or the vector L1 / L2 (other blocks).
#include "small_internal.h"

#include <algorithm>

namespace small {

namespace {

constexpr int kBlock = 256;
enum : int { OP_DW = 0, OP_MAX = 1, OP_AVG = 2 };

__device__ __forceinline__ floatx4 ld4(const float *p) { return *reinterpret_cast<const floatx4 *>(p); }
__device__ __forceinline__ void st4(float *p, floatx4 v) { *reinterpret_cast<floatx4 *>(p) = v; }
// streaming variants: data that is touched once should not displace reusable lines
__device__ __forceinline__ floatx4 ld4_stream(const float *p) { return __builtin_nontemporal_load(reinterpret_cast<const floatx4 *>(p)); }
__device__ __forceinline__ void st4_stream(float *p, floatx4 v) { __builtin_nontemporal_store(v, reinterpret_cast<floatx4 *>(p)); }

__device__ __forceinline__ float max_first(float m, float v) { return (v > m) ? v : m; }   // first value seen wins ties
__device__ __forceinline__ floatx4 relu4(floatx4 v)
{
    return floatx4{v.x > 0.f ? v.x : 0.f, v.y > 0.f ? v.y : 0.f, v.z > 0.f ? v.z : 0.f, v.w > 0.f ? v.w : 0.f};
}

// 1-D grid over (plane, chunk): plane = (image, channel block), chunk = kBlock lanes of the plane's
// Ho*Wo*(Cb/4) float4 outputs; chunks of one plane are consecutive logical workgroups on one XCD.
// KS > 0: square KS x KS window fully unrolled; KS == 0: run-time kh x kw.
// CQ > 0: Cb/4 known at compile time; CQ == 0: run-time.
template <int OP, int KS, int CQ>
__global__ void __launch_bounds__(kBlock) window_vec4(const float *__restrict__ in, const float *__restrict__ filt,
                                                       float *__restrict__ out, LayerGeom g, int chunks, int epilogue)
{
    const int Cb = g.Cib;
    const int cq = CQ > 0 ? CQ : Cb / 4;
    const int kh = KS > 0 ? KS : g.kh, kw = KS > 0 ? KS : g.kw;
    const unsigned wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int plane = wg / chunks;
    const int e = (wg - plane * chunks) * kBlock + threadIdx.x;
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
    // Branch-free taps: an out-of-range tap reads a clamped (valid) address and is then replaced by
    // the reduction's neutral value (0 for FMA / Add, -inf for Max, which "v > m" never selects), so
    // all loads of a window can be in flight together.
    const float neutral = OP == OP_MAX ? -INFINITY : 0.f;
#pragma unroll
    for (int y = 0; y < kh; ++y) {
        const int ih = ih0 + y;
        const bool oky = ih >= 0 && ih < g.H;
        const int ihc = min(max(ih, 0), g.H - 1);
#pragma unroll
        for (int x = 0; x < kw; ++x) {
            const int iw = iw0 + x;
            const bool ok = oky && iw >= 0 && iw < g.W;
            const int iwc = min(max(iw, 0), g.W - 1);
            floatx4 v = ld4(src + (size_t)(ihc * g.W + iwc) * Cb);
            if (!ok) v = floatx4{neutral, neutral, neutral, neutral};
            if (OP == OP_DW) {
                const floatx4 w = ld4(wsrc + (y * kw + x) * Cb);
                acc.x = fmaf(v.x, w.x, acc.x); acc.y = fmaf(v.y, w.y, acc.y);
                acc.z = fmaf(v.z, w.z, acc.z); acc.w = fmaf(v.w, w.w, acc.w);
            } else if (OP == OP_MAX) {
                acc.x = max_first(acc.x, v.x); acc.y = max_first(acc.y, v.y);
                acc.z = max_first(acc.z, v.z); acc.w = max_first(acc.w, v.w);
            } else {
                acc += v;
                cnt += ok ? 1 : 0;
            }
        }
    }
    if (OP == OP_AVG) {
        const float d = (float)(cnt > 0 ? cnt : 1);
        acc.x /= d; acc.y /= d; acc.z /= d; acc.w /= d;
    }
    if (epilogue & EPI_RELU) acc = relu4(acc);
    st4(out + ((size_t)plane * g.Ho * g.Wo + p) * Cb + c4, acc);
}

// LDS-tiled single-channel reduction, Cb = 16: one workgroup owns TR output rows (full width) of one
// (image, channel block) plane. Phase 1 copies the input rows the tile needs into LDS with
// consecutive lanes on consecutive 16-byte pieces, so every global line is requested exactly once
// per workgroup (repeated requests to a line that is still in flight stall the vector L1);
// padding cells are written with the reduction's neutral value, so phase 2 has no bounds checks.
// Phase 2: one lane = 4 channels of one output pixel, taps read from LDS (ds_read_b128, lanes on
// consecutive addresses), depthwise filter taps held in registers.
// LDS tile: IR rows x IW padded columns x 16 floats, IR = (TR-1)*stride + kh, IW = max(W + pl, (Wo-1)*stride + kw).
template <int OP, int KS, int kCopyBatch>
__global__ void __launch_bounds__(kBlock) window_lds16(const float *__restrict__ in, const float *__restrict__ filt,
                                                        float *__restrict__ out, LayerGeom g, int TR, int tiles, int IW, int epilogue)
{
    extern __shared__ floatx4 tile[];                 // [IR][IW][4 quads]
    const int kh = KS > 0 ? KS : g.kh, kw = KS > 0 ? KS : g.kw;
    const unsigned wg = xcd_contiguous(blockIdx.x, gridDim.x);
    const int plane = wg / tiles;
    const int oy0 = (wg - plane * tiles) * TR;
    const int trc = min(TR, g.Ho - oy0);              // output rows of this tile
    const int IR = (trc - 1) * g.stride + kh;
    const int iy0 = oy0 * g.stride - g.pt;
    const int tid = threadIdx.x;
    const float neutral = OP == OP_MAX ? -INFINITY : 0.f;
    const floatx4 nv{neutral, neutral, neutral, neutral};

    // output decomposition of phase 2, computed early so the filter taps are requested before the tile
    const int ow4 = g.Wo * 4;
    const int rows_per_iter = ow4 >= kBlock ? 1 : kBlock / ow4;
    const int ry = ow4 >= kBlock ? 0 : tid / ow4;
    const int oc = ow4 >= kBlock ? tid : tid - ry * ow4;
    const int cb = plane % (g.Ci / 16);
    floatx4 w[KS > 0 ? KS * KS : 1];
    if (OP == OP_DW && KS > 0) {
        // a lane's channel quad is the same for all of its outputs (columns advance by 256 lanes = 64 pixels)
#pragma unroll
        for (int k = 0; k < KS * KS; ++k) w[k] = ld4(filt + ((size_t)cb * KS * KS + k) * 16 + (oc & 3) * 4);
    }

    // ---- phase 1: global -> LDS. Lane t copies float4 items t, t + 256, ... of the IR x IW x 4 tile;
    // kCopyBatch loads are issued back to back (clamped addresses, so no branches) before the first
    // LDS write, which keeps that many 16-byte requests per lane in flight.
    {
        const int iw4 = IW * 4, items = IR * iw4;
        const int step_r = kBlock / iw4, step_c = kBlock - step_r * iw4;
        int r = tid / iw4, c = tid - r * iw4;
        const float *src = in + (size_t)plane * g.H * g.W * 16;
        for (int base = 0; base < items; base += kCopyBatch * kBlock) {
            floatx4 v[kCopyBatch];
            bool ok[kCopyBatch];
#pragma unroll
            for (int k = 0; k < kCopyBatch; ++k) {
                const int iy = iy0 + r, ix = (c >> 2) - g.pl;
                ok[k] = iy >= 0 && iy < g.H && ix >= 0 && ix < g.W;
                const int iyc = min(max(iy, 0), g.H - 1), ixc = min(max(ix, 0), g.W - 1);
                v[k] = ld4_stream(src + ((size_t)iyc * g.W + ixc) * 16 + (c & 3) * 4);
                c += step_c; r += step_r;
                if (c >= iw4) { c -= iw4; ++r; }
            }
#pragma unroll
            for (int k = 0; k < kCopyBatch; ++k) {
                const int f = base + k * kBlock + tid;
                if (f < items) tile[f] = ok[k] ? v[k] : nv;
            }
        }
    }
    __syncthreads();

    // ---- phase 2: LDS -> registers -> global
    if (ry >= rows_per_iter) return;
    float *dst = out + (size_t)plane * g.Ho * g.Wo * 16;
    for (int c = oc; c < ow4; c += kBlock) {
        const int ox = c >> 2, q = c & 3;
        for (int r = ry; r < trc; r += rows_per_iter) {
            const floatx4 *t0 = tile + ((r * g.stride) * IW + ox * g.stride) * 4 + q;
            floatx4 acc = (OP == OP_MAX) ? nv : floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int y = 0; y < kh; ++y) {
#pragma unroll
                for (int x = 0; x < kw; ++x) {
                    const floatx4 v = t0[(y * IW + x) * 4];
                    if (OP == OP_DW) {
                        const floatx4 wv = KS > 0 ? w[y * kw + x] : ld4(filt + ((size_t)(cb * kh + y) * kw + x) * 16 + q * 4);
                        acc.x = fmaf(v.x, wv.x, acc.x); acc.y = fmaf(v.y, wv.y, acc.y);
                        acc.z = fmaf(v.z, wv.z, acc.z); acc.w = fmaf(v.w, wv.w, acc.w);
                    } else if (OP == OP_MAX) {
                        acc.x = max_first(acc.x, v.x); acc.y = max_first(acc.y, v.y);
                        acc.z = max_first(acc.z, v.z); acc.w = max_first(acc.w, v.w);
                    } else {
                        acc += v;
                    }
                }
            }
            if (OP == OP_AVG) {
                // divisor = taps inside the image (padding cells hold 0 and are not counted)
                const int y0 = (oy0 + r) * g.stride - g.pt, x0 = ox * g.stride - g.pl;
                const int ny = min(y0 + kh, g.H) - max(y0, 0), nx = min(x0 + kw, g.W) - max(x0, 0);
                const float d = (float)(ny * nx);
                acc.x /= d; acc.y /= d; acc.z /= d; acc.w /= d;
            }
            if (epilogue & EPI_RELU) acc = relu4(acc);
            st4_stream(dst + ((size_t)(oy0 + r) * g.Wo + ox) * 16 + q * 4, acc);
        }
    }
}

// Any block size: one lane per output element (used when Cb is not a multiple of 4).
template <int OP>
__global__ void __launch_bounds__(kBlock) window_scalar(const float *__restrict__ in, const float *__restrict__ filt,
                                                         float *__restrict__ out, LayerGeom g, size_t total, int epilogue)
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
    if (epilogue & EPI_RELU) acc = acc > 0.f ? acc : 0.f;
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
hipError_t launch_window(const float *in, const float *filt, float *out, const LayerGeom &g, int epilogue, hipStream_t s)
{
    const int Cb = g.Cib;
    const int planes = g.N * (g.Ci / Cb);
    const bool vec = (Cb % 4 == 0) && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt) & 15u) == 0);
    if (vec && Cb == 16) {
        // LDS-tiled path when at least one output row's input rows fit the LDS budget
        const int IW = std::max(g.W + g.pl, (g.Wo - 1) * g.stride + g.kw);
        constexpr int kLdsBudget = 40 * 1024;   // measured best: 4 workgroups per compute unit
        const int max_ir = kLdsBudget / (IW * 64);
        if (max_ir >= g.kh) {
            int TR = std::min(g.Ho, (max_ir - g.kh) / g.stride + 1);
            // keep at least ~4 workgroups per compute unit when the layer is large enough
            while (TR > 1 && (long)planes * ((g.Ho + TR - 1) / TR) < 1024) TR = (TR + 1) / 2;
            const int tiles = (g.Ho + TR - 1) / TR;
            const size_t lds = (size_t)((TR - 1) * g.stride + g.kh) * IW * 64;
            const dim3 grid((unsigned)planes * (unsigned)tiles);
            const int items = (int)(lds / 16);
            const bool k3 = g.kh == 3 && g.kw == 3;
#define SMALL_LAUNCH_LDS(KS, CB) \
    hipLaunchKernelGGL((window_lds16<OP, KS, CB>), grid, dim3(kBlock), lds, s, in, filt, out, g, TR, tiles, IW, epilogue)
            if (items <= 2 * kBlock) { if (k3) SMALL_LAUNCH_LDS(3, 2); else SMALL_LAUNCH_LDS(0, 2); }
            else if (items <= 4 * kBlock) { if (k3) SMALL_LAUNCH_LDS(3, 4); else SMALL_LAUNCH_LDS(0, 4); }
            else { if (k3) SMALL_LAUNCH_LDS(3, 10); else SMALL_LAUNCH_LDS(0, 10); }
#undef SMALL_LAUNCH_LDS
            return hipGetLastError();
        }
    }
    if (vec) {
        const int cq = Cb / 4;
        const int per_plane = g.Ho * g.Wo * cq;
        const int chunks = (per_plane + kBlock - 1) / kBlock;
        const dim3 grid((unsigned)planes * (unsigned)chunks);
        const bool k3 = g.kh == 3 && g.kw == 3;
        if (k3 && cq == 4)
            hipLaunchKernelGGL((window_vec4<OP, 3, 4>), grid, dim3(kBlock), 0, s, in, filt, out, g, chunks, epilogue);
        else if (cq == 4)
            hipLaunchKernelGGL((window_vec4<OP, 0, 4>), grid, dim3(kBlock), 0, s, in, filt, out, g, chunks, epilogue);
        else
            hipLaunchKernelGGL((window_vec4<OP, 0, 0>), grid, dim3(kBlock), 0, s, in, filt, out, g, chunks, epilogue);
    } else {
        const size_t total = (size_t)planes * g.Ho * g.Wo * Cb;
        hipLaunchKernelGGL((window_scalar<OP>), dim3((unsigned)((total + kBlock - 1) / kBlock)), dim3(kBlock), 0, s, in,
                           filt, out, g, total, epilogue);
    }
    return hipGetLastError();
}

}  // namespace

hipError_t launch_dwconv(const float *in, const float *filt, float *out, const LayerGeom &g, int epilogue, hipStream_t s)
{
    const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt) & 15u) == 0);
    if (aligned && (epilogue & ~EPI_RELU) == 0 && dw_dpp_eligible(g))
        return launch_dw_dpp(in, filt, out, g, (epilogue & EPI_RELU) != 0, s);
    if (aligned && (epilogue & ~EPI_RELU) == 0 && dw_rows_eligible(g))
        return launch_dw_rows(in, filt, out, g, (epilogue & EPI_RELU) != 0, s);
    return launch_window<OP_DW>(in, filt, out, g, epilogue, s);
}

namespace {

// Network head in one launch: global average pooling followed by a fully connected layer, one workgroup per image.
// in [N][C/16][HW][16], filt [Co/Cob][C/16][1][1][16][Cob], out [N][Co]. Phase 1: 64 lanes per 16-channel block
// (a float4 of channels each, 16 pixels in flight) sum the block's pixels; phase 2: lane (o, part) adds up a
// sixteenth of the channels for output o. C <= 256, Co <= 16 (LDS: 256 means and 256 partial sums).
__global__ void __launch_bounds__(256) avgpool_dense_head(const float *__restrict__ in, const float *__restrict__ filt,
                                                          float *__restrict__ out, int C, int HW, int Co, int Cob)
{
    __shared__ float part4[16][16][4][4];    // [pixel lane][block][quad][channel in quad]
    __shared__ float mean[256];
    __shared__ float partial[16][16];
    const int t = threadIdx.x, n = blockIdx.x;
    const int nCb = C >> 4;
    const int quad = t & 3, plane_lane = (t >> 2) & 15, cbl = t >> 6;          // 4 blocks in flight, 16 pixels x 4 quads each
    for (int cb0 = 0; cb0 < nCb; cb0 += 4) {
        const int cb = cb0 + cbl;
        floatx4 sum = {0.f, 0.f, 0.f, 0.f};
        if (cb < nCb) {
            const floatx4 *src = reinterpret_cast<const floatx4 *>(in + ((size_t)n * nCb + cb) * HW * 16) + quad;
            for (int px = plane_lane; px < HW; px += 16) sum += src[px * 4];
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) part4[plane_lane][cbl][quad][k] = sum[k];
        __syncthreads();
        if (t < 64 && cb0 + (t >> 4) < nCb) {                                    // 4 blocks x 16 channels
            float v = 0.f;
#pragma unroll
            for (int l = 0; l < 16; ++l) v += part4[l][t >> 4][(t >> 2) & 3][t & 3];
            mean[(cb0 + (t >> 4)) * 16 + (t & 15)] = v / (float)HW;
        }
        __syncthreads();
    }
    const int o = t & 15, part = t >> 4;
    float acc = 0.f;
    if (o < Co) {
        const int cob = o / Cob, co_in = o - cob * Cob;
        for (int c = part; c < C; c += 16)
            acc += mean[c] * filt[(((size_t)cob * nCb + (c >> 4)) * 16 + (c & 15)) * Cob + co_in];
    }
    partial[part][o] = acc;
    __syncthreads();
    if (t < Co) {
        float v = 0.f;
#pragma unroll
        for (int l = 0; l < 16; ++l) v += partial[l][t];
        out[(size_t)n * Co + t] = v;
    }
}

}  // namespace

bool avgpool_dense_eligible(int C, int Cb, int Co, int Cob)
{
    return Cb == 16 && C % 16 == 0 && C <= 256 && Co >= 1 && Co <= 16 && Cob >= 1 && Co % Cob == 0;
}

hipError_t launch_avgpool_dense(const float *in, const float *filt, float *out, int N, int C, int HW, int Co, int Cob,
                                hipStream_t s)
{
    hipLaunchKernelGGL(avgpool_dense_head, dim3((unsigned)N), dim3(256), 0, s, in, filt, out, C, HW, Co, Cob);
    return hipGetLastError();
}

hipError_t launch_pool(const float *in, float *out, const LayerGeom &g, int mode, hipStream_t s)
{
    if (mode == 0 && pool_dpp_eligible(g, in, out)) return launch_pool_dpp(in, out, g, s);
    if (mode == 0) return launch_window<OP_MAX>(in, nullptr, out, g, EPI_NONE, s);
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
    return launch_window<OP_AVG>(in, nullptr, out, g, EPI_NONE, s);
}

}  // namespace small
