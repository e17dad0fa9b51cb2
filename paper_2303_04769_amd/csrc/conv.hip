// Full-channel reduction: direct convolution on the blocked layout (paper Table 1 row 4,
// Algorithm 1 with G = 1, K = Co, F_C = Ci; kernel phases of Algorithm 2).
//
// Mapping of Algorithm 1 onto gfx950:
//   loops g, k (output-channel blocks, "in parallel")  -> blockIdx.y / wave column
//   loops j, l (output pixels, tile O_wb)              -> blockIdx.x / wave row; pixels of all
//                                                         images are one flattened axis
//   loop  i    (input-channel blocks)                  -> moved INSIDE the tile: the output tile
//                                                         stays in accumulator registers for the
//                                                         whole reduction, LOAD/STORE happen once
//   kernel loops x, y, ii over a O_wb x K_b tile       -> v_mfma_f32_16x16x4_f32 on LDS-staged
//                                                         [pixel][Cib] and [Cib][Cob] slabs
// The blocked layouts are already matrix-core operands: for a fixed (Ci block, tap) a run of
// pixels is a row-major [pixels][16] matrix and the filter slab is a row-major [16][16] matrix.
#include "small_internal.h"

#include <cstdio>

namespace small {

namespace {

struct ConvArgs {
    const float *in;
    const float *filt;
    float *out;
    const float *res;
    int N, H, W, Ho, Wo;
    int nCib, nCob;
    int kh, kw, stride, pt, pl;
    int M;        // N * Ho * Wo flattened output pixels
    int HoWo;
    int epilogue;
};

__device__ __forceinline__ floatx4 epilogue4(floatx4 v, int epi, const float *res)
{
    if (epi & EPI_ADD) v += *reinterpret_cast<const floatx4 *>(res);
    if (epi & EPI_RELU) {
        v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
        v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
    }
    return v;
}

// ---------------------------------------------------------------------------------------------
// Matrix-core path, Cib = Cob = 16, any window / stride / padding.
//
// Workgroup tile: TM = WAVES_M*WM*16 flattened output pixels x TN = WAVES_N*WN*16 output channels.
// Reduction step ("k-step") = one (Ci block, tap y, tap x): 16 input channels.
//   A-stage: for every tile pixel the 16 input channels of the tap's input pixel (zeros when the
//            tap falls outside the image or the pixel is beyond M), gathered into LDS as
//            sA[quad q][pixel] float4 (q = which 4 of the 16 channels).
//   B-stage: the [16 ci][TN co] filter slab, re-tiled in LDS per 16-co subtile as
//            float4 groups (q, co) -> W[4q..4q+3][co], so that one ds_read_b128 per lane yields
//            the operand registers of four MFMAs.
// MFMA operand roles: "A" (16x4, row i) = filter with i = co; "B" (4x16, col j) = input with
// j = pixel; D[i = co][j = pixel]: lane l holds co = 4*(l/16) + v (v = 0..3), pixel = l%16, i.e. a
// float4 of four adjacent output channels of one pixel, and the 16 lanes x 4 lane-groups of a
// wave store one contiguous 1 KiB run of the [pixel][Cob] output.
// The reduction index inside a k-step is permuted (MFMA r takes ci = 4*(l/16) + r); both
// operands use the same permutation, and a sum does not depend on it.
// Global -> LDS copies are software-pipelined one k-step ahead through registers (double-buffered
// LDS, one barrier per k-step).
template <int WAVES_M, int WAVES_N, int WM, int WN>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) conv16_mfma(ConvArgs a)
{
    constexpr int NT = 64 * WAVES_M * WAVES_N;
    constexpr int TM = WAVES_M * WM * 16;
    constexpr int TN = WAVES_N * WN * 16;
    constexpr int NSUB = TN / 16;
    constexpr int A_ITEMS = TM * 4, B_ITEMS = TN * 4;           // float4 items per stage
    constexpr int A_IT = (A_ITEMS + NT - 1) / NT, B_IT = (B_ITEMS + NT - 1) / NT;
    constexpr int A_LD = TM + 2;                                 // skewed quad stride (float4 units)

    __shared__ floatx4 sA[2][4 * A_LD];
    __shared__ float sB[2][TN * 16];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int m0 = blockIdx.x * TM;
    const int cob0 = blockIdx.y * NSUB;
    const int HW = a.H * a.W;

    // ---- per-thread staging descriptors (fixed over the reduction)
    int a_off[A_IT], a_ih0[A_IT], a_iw0[A_IT];
    bool a_ok[A_IT];
#pragma unroll
    for (int i = 0; i < A_IT; ++i) {
        const int item = tid + i * NT;
        const int px = item >> 2, quad = item & 3;
        const int m = m0 + px;
        a_ok[i] = (item < A_ITEMS) && (m < a.M);
        const int mm = a_ok[i] ? m : 0;
        const int n = mm / a.HoWo, rem = mm - n * a.HoWo;
        const int oh = rem / a.Wo, ow = rem - oh * a.Wo;
        a_ih0[i] = oh * a.stride - a.pt;
        a_iw0[i] = ow * a.stride - a.pl;
        a_off[i] = n * a.nCib * HW * 16 + quad * 4;
    }
    int b_src[B_IT], b_dst[B_IT];
    bool b_ok[B_IT];
#pragma unroll
    for (int i = 0; i < B_IT; ++i) {
        const int item = tid + i * NT;
        const int sub = item >> 6, w = item & 63;
        const int ci = w >> 2, cq = w & 3;
        b_ok[i] = (item < B_ITEMS) && (cob0 + sub < a.nCob);
        // element offset inside the filter of (cob0+sub, cib = 0, tap 0), row ci, channels 4cq..4cq+3
        b_src[i] = (cob0 + sub) * a.nCib * a.kh * a.kw * 256 + ci * 16 + cq * 4;
        // LDS float index of group (q = ci/4, co = 4cq + j), component r = ci%4; j is added at store time
        b_dst[i] = sub * 256 + (ci >> 2) * 64 + (ci & 3);
    }

    floatx4 ra[A_IT], rb[B_IT];
    auto load_stage = [&](int cib, int y, int x) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int ih = a_ih0[i] + y, iw = a_iw0[i] + x;
            const bool ok = a_ok[i] && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            ra[i] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (ok) ra[i] = *reinterpret_cast<const floatx4 *>(a.in + a_off[i] + (cib * HW + ih * a.W + iw) * 16);
        }
        const int tap = ((cib * a.kh + y) * a.kw + x) * 256;
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            rb[i] = floatx4{0.f, 0.f, 0.f, 0.f};
            if (b_ok[i]) rb[i] = *reinterpret_cast<const floatx4 *>(a.filt + b_src[i] + tap);
        }
    };
    auto store_stage = [&](int buf) {
#pragma unroll
        for (int i = 0; i < A_IT; ++i) {
            const int item = tid + i * NT;
            if (item < A_ITEMS) sA[buf][(item & 3) * A_LD + (item >> 2)] = ra[i];
        }
#pragma unroll
        for (int i = 0; i < B_IT; ++i) {
            const int item = tid + i * NT;
            if (item < B_ITEMS) {
                const int w = item & 63, q = w >> 4, cq = w & 3;
                float *d = &sB[buf][b_dst[i]];
                // group index inside the quarter is swizzled with q to spread LDS banks
                d[((4 * cq + 0) ^ q) * 4] = rb[i].x;
                d[((4 * cq + 1) ^ q) * 4] = rb[i].y;
                d[((4 * cq + 2) ^ q) * 4] = rb[i].z;
                d[((4 * cq + 3) ^ q) * 4] = rb[i].w;
            }
        }
    };

    floatx4 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    const int lp = lane & 15, lq = lane >> 4;
    const int ksteps = a.nCib * a.kh * a.kw;
    int cib = 0, y = 0, x = 0;

    load_stage(0, 0, 0);
    store_stage(0);
    __syncthreads();

    for (int ks = 0; ks < ksteps; ++ks) {
        const int buf = ks & 1;
        // advance (cib, y, x) to k-step ks + 1
        if (++x == a.kw) { x = 0; if (++y == a.kh) { y = 0; ++cib; } }
        const bool more = ks + 1 < ksteps;
        if (more) load_stage(cib, y, x);

        floatx4 fa[WM], fb[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j)
            fb[j] = *reinterpret_cast<const floatx4 *>(&sB[buf][(wave_n * WN + j) * 256 + (lq * 16 + (lp ^ lq)) * 4]);
#pragma unroll
        for (int i = 0; i < WM; ++i) fa[i] = sA[buf][lq * A_LD + (wave_m * WM + i) * 16 + lp];
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int i = 0; i < WM; ++i)
#pragma unroll
                for (int j = 0; j < WN; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fb[j][r], fa[i][r], acc[i][j], 0, 0, 0);

        if (more) store_stage(buf ^ 1);
        __syncthreads();
    }

    // ---- STORE phase: each lane owns 4 adjacent output channels of one pixel
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = m0 + (wave_m * WM + i) * 16 + lp;
        if (m >= a.M) continue;
        const int n = m / a.HoWo, rem = m - n * a.HoWo;
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cob = cob0 + wave_n * WN + j;
            if (cob >= a.nCob) continue;
            const size_t o = ((size_t)(n * a.nCob + cob) * a.HoWo + rem) * 16 + lq * 4;
            *reinterpret_cast<floatx4 *>(a.out + o) = epilogue4(acc[i][j], a.epilogue, a.res + o);
        }
    }
}

// ---------------------------------------------------------------------------------------------
// Generic path, any block sizes (first layers with Ci = 1 or 3, 8-channel blocks, dense heads
// with Co = 2, 10, 12): one lane per output element, output channel fastest, so the filter
// reads of a wavefront are contiguous and its input reads are broadcasts.
__global__ void __launch_bounds__(256) conv_direct(ConvArgs a, int Cib, int Cob, size_t total)
{
    size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const size_t dst = e;
    const int co = (int)(e % Cob); e /= Cob;
    const int ow = (int)(e % a.Wo); e /= a.Wo;
    const int oh = (int)(e % a.Ho); e /= a.Ho;
    const int cob = (int)(e % a.nCob);
    const int n = (int)(e / a.nCob);
    float acc = 0.f;
    for (int cib = 0; cib < a.nCib; ++cib)
        for (int y = 0; y < a.kh; ++y) {
            const int ih = oh * a.stride - a.pt + y;
            if (ih < 0 || ih >= a.H) continue;
            for (int x = 0; x < a.kw; ++x) {
                const int iw = ow * a.stride - a.pl + x;
                if (iw < 0 || iw >= a.W) continue;
                const float *ip = a.in + (((size_t)(n * a.nCib + cib) * a.H + ih) * a.W + iw) * Cib;
                const float *wp = a.filt + ((((size_t)cob * a.nCib + cib) * a.kh + y) * a.kw + x) * Cib * Cob + co;
                for (int ci = 0; ci < Cib; ++ci) acc = fmaf(ip[ci], wp[(size_t)ci * Cob], acc);
            }
        }
    if (a.epilogue & EPI_ADD) acc += a.res[dst];
    if (a.epilogue & EPI_RELU) acc = acc > 0.f ? acc : 0.f;
    a.out[dst] = acc;
}

// ---------------------------------------------------------------------------------------------
// Dense head (window = whole unpadded image, one output pixel): the blocked input of an image is one
// contiguous vector in exactly the filter's reduction order, so every output is a plain dot product.
// One lane per output, output channel fastest (filter reads coalesced, input reads broadcast), four
// independent partial sums and vector loads so that the short loop is not one long latency chain.
__global__ void __launch_bounds__(256) dense_rows(ConvArgs a, int Cob, int K, size_t total, int vec)
{
    const size_t e = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (e >= total) return;
    const int co = (int)(e % Cob);
    const size_t t = e / Cob;
    const int cob = (int)(t % a.nCob);
    const size_t n = t / a.nCob;
    const float *x = a.in + n * K;
    const float *w = a.filt + (size_t)cob * K * Cob + co;
    float s0 = 0.f, s1 = 0.f, s2 = 0.f, s3 = 0.f;
    int k = 0;
    if (vec) {
#pragma unroll 4
        for (; k + 4 <= K; k += 4) {
            const floatx4 v = *reinterpret_cast<const floatx4 *>(x + k);
            s0 = fmaf(v.x, w[(size_t)(k + 0) * Cob], s0);
            s1 = fmaf(v.y, w[(size_t)(k + 1) * Cob], s1);
            s2 = fmaf(v.z, w[(size_t)(k + 2) * Cob], s2);
            s3 = fmaf(v.w, w[(size_t)(k + 3) * Cob], s3);
        }
    }
    for (; k < K; ++k) s0 = fmaf(x[k], w[(size_t)k * Cob], s0);
    float acc = (s0 + s1) + (s2 + s3);
    if (a.epilogue & EPI_ADD) acc += a.res[e];
    if (a.epilogue & EPI_RELU) acc = acc > 0.f ? acc : 0.f;
    a.out[e] = acc;
}

// ---------------------------------------------------------------------------------------------
// Small-channel path (first layers with Ci = 1 or 3, 8-channel blocks, dense heads with few
// outputs): one lane computes one output pixel for a whole output-channel block (up to 16
// accumulators = the G_b x K_b tile of Algorithm 1 with O_wb = 1 per lane, 256 pixels per
// workgroup). The block's filters sit in LDS, zero-padded to 16 output channels, and are read as
// broadcast float4; input values are read once per lane. HBM-bound in practice (K is tiny).
constexpr int kSmallMaxFilterFloats = 12 * 1024;     // 48 KiB of LDS

// CIB, KH, KW: compile-time input block and window of the common first layers (0: taken from the arguments).
// Taps are branch-free (address clamped into the image, value replaced by zero outside), so with
// compile-time bounds all input loads of a pixel are in flight together instead of one round trip per tap.
template <int CIB, int KH, int KW>
__global__ void __launch_bounds__(256) conv_small(ConvArgs a, int Cib_rt, int Cob, int kfloats)
{
    const int Cib = CIB ? CIB : Cib_rt, kh = KH ? KH : a.kh, kw = KW ? KW : a.kw;
    extern __shared__ floatx4 wl[];                   // [nCib][kh][kw][Cib] rows of 16 output channels
    const int cob = blockIdx.y;
    const int K = a.nCib * kh * kw * Cib;             // reduction length
    // filter of this block: [cib][y][x][ci][Cob] with cib stride kh*kw*Cib*Cob, block stride nCib * that
    const float *wsrc = a.filt + (size_t)cob * K * Cob;
    for (int e = threadIdx.x; e < K * 16; e += 256) {
        const int k = e >> 4, co = e & 15;
        reinterpret_cast<float *>(wl)[e] = co < Cob ? wsrc[(size_t)k * Cob + co] : 0.f;
    }
    __syncthreads();
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= a.M) return;
    const int n = m / a.HoWo, rem = m - n * a.HoWo;
    const int oh = rem / a.Wo, ow = rem - oh * a.Wo;
    floatx4 acc[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) acc[q] = floatx4{0.f, 0.f, 0.f, 0.f};
    int k = 0;
    for (int cib = 0; cib < a.nCib; ++cib) {
        const float *plane = a.in + (size_t)(n * a.nCib + cib) * a.H * a.W * Cib;
        if constexpr (CIB * KH * KW != 0) {
            // all input values of the window first (one batch of loads), then the multiply-adds tap by tap
            float v[KH * KW * CIB];
#pragma unroll
            for (int y = 0; y < KH; ++y) {
                const int ih = oh * a.stride - a.pt + y;
                const int ihc = min(max(ih, 0), a.H - 1);
#pragma unroll
                for (int x = 0; x < KW; ++x) {
                    const int iw = ow * a.stride - a.pl + x;
                    const int iwc = min(max(iw, 0), a.W - 1);
                    const bool ok = ih == ihc && iw == iwc;
                    const float *ip = plane + (size_t)(ihc * a.W + iwc) * CIB;
#pragma unroll
                    for (int ci = 0; ci < CIB; ++ci) v[(y * KW + x) * CIB + ci] = ok ? ip[ci] : 0.f;
                }
            }
#pragma unroll
            for (int t = 0; t < KH * KW * CIB; ++t) {
                const floatx4 *w = wl + (size_t)(k + t) * 4;
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const floatx4 wq = w[q];
                    acc[q].x = fmaf(v[t], wq.x, acc[q].x); acc[q].y = fmaf(v[t], wq.y, acc[q].y);
                    acc[q].z = fmaf(v[t], wq.z, acc[q].z); acc[q].w = fmaf(v[t], wq.w, acc[q].w);
                }
                if (t % 2 == 1) __builtin_amdgcn_sched_barrier(0);    // keeps the filter reads from being hoisted wholesale
            }
            k += KH * KW * CIB;
        } else {
            for (int y = 0; y < kh; ++y) {
                const int ih = oh * a.stride - a.pt + y;
                const int ihc = min(max(ih, 0), a.H - 1);
                for (int x = 0; x < kw; ++x, k += Cib) {
                    const int iw = ow * a.stride - a.pl + x;
                    const int iwc = min(max(iw, 0), a.W - 1);
                    const bool ok = ih == ihc && iw == iwc;
                    const float *ip = plane + (size_t)(ihc * a.W + iwc) * Cib;
                    for (int ci = 0; ci < Cib; ++ci) {
                        const float v = ok ? ip[ci] : 0.f;
                        const floatx4 *w = wl + (size_t)(k + ci) * 4;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            const floatx4 wq = w[q];
                            acc[q].x = fmaf(v, wq.x, acc[q].x); acc[q].y = fmaf(v, wq.y, acc[q].y);
                            acc[q].z = fmaf(v, wq.z, acc[q].z); acc[q].w = fmaf(v, wq.w, acc[q].w);
                        }
                    }
                }
            }
        }
    }
    const size_t o = ((size_t)(n * a.nCob + cob) * a.HoWo + rem) * Cob;
    float *dst = a.out + o;
    if (Cob == 16 && (((uintptr_t)a.out | (uintptr_t)a.res) & 15u) == 0) {
#pragma unroll
        for (int q = 0; q < 4; ++q) reinterpret_cast<floatx4 *>(dst)[q] = epilogue4(acc[q], a.epilogue, a.res + o + 4 * q);
    } else {
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            floatx4 r = acc[q];
            if (a.epilogue & EPI_ADD) {
                if (4 * q + 0 < Cob) r.x += a.res[o + 4 * q + 0];
                if (4 * q + 1 < Cob) r.y += a.res[o + 4 * q + 1];
                if (4 * q + 2 < Cob) r.z += a.res[o + 4 * q + 2];
                if (4 * q + 3 < Cob) r.w += a.res[o + 4 * q + 3];
            }
            r = epilogue4(r, a.epilogue & ~EPI_ADD, nullptr);
            if (4 * q + 0 < Cob) dst[4 * q + 0] = r.x;
            if (4 * q + 1 < Cob) dst[4 * q + 1] = r.y;
            if (4 * q + 2 < Cob) dst[4 * q + 2] = r.z;
            if (4 * q + 3 < Cob) dst[4 * q + 3] = r.w;
        }
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN>
void launch_mfma(const ConvArgs &a, hipStream_t s)
{
    constexpr int TM = WAVES_M * WM * 16, TN = WAVES_N * WN * 16;
    const dim3 grid((unsigned)((a.M + TM - 1) / TM), (unsigned)((a.nCob * 16 + TN - 1) / TN));
    hipLaunchKernelGGL((conv16_mfma<WAVES_M, WAVES_N, WM, WN>), grid, dim3(64 * WAVES_M * WAVES_N), 0, s, a);
}

// Tile choice for the 16 x 16 blocked matrix-core kernels, from measurements on the layer sweep at
// steady clocks. Small tiles win: many short workgroups balance better over 256 compute units and
// leave 4 or more of them resident per compute unit, which hides each other's prologue, barrier and
// store phases. 1x1 (little work per pixel): 32 pixels x 64 channels, or 32 x 32 for narrow layers.
// 3x3: the candidate with the least work on the busiest compute unit (workgroups are spread evenly,
// so that is ceil(workgroups / compute units) x tile area), 64 x 32 preferred on near-ties for its operand reuse.
int pick_tile(const LayerGeom &g)
{
    const long M = (long)g.N * g.Ho * g.Wo;
    const bool pointwise = g.kh == 1 && g.kw == 1;
    if (pointwise) return g.Co >= 64 ? SAME_32x64 : g.Co >= 32 ? SAME_32x32 : SAME_64x16;
    struct Cand { int tile, tm, tn; double penalty; };
    static const Cand wide[] = {{SAME_64x32, 64, 32, 1.0}, {SAME_64x16, 64, 16, 1.07}, {SAME_32x32, 32, 32, 1.08}};
    static const Cand narrow[] = {{SAME_128x16, 128, 16, 1.0}, {SAME_64x16, 64, 16, 1.05}};
    const Cand *cands = g.Co >= 32 ? wide : narrow;
    const int n = g.Co >= 32 ? 3 : 2;
    const long cus = device_cus();
    int best = cands[0].tile;
    double best_cost = 0;
    for (int i = 0; i < n; ++i) {
        const long wgs = ((M + cands[i].tm - 1) / cands[i].tm) * ((g.Co + cands[i].tn - 1) / cands[i].tn);
        const double cost = (double)((wgs + cus - 1) / cus) * cands[i].tm * cands[i].tn * cands[i].penalty;
        if (i == 0 || cost < best_cost) { best = cands[i].tile; best_cost = cost; }
    }
    return best;
}

// ---------------------------------------------------------------------------------------------
// First layers on the matrix cores: one input block of fewer than 16 channels (Ci = 1, 3, ...) and a short
// reduction K = Ci * kh * kw (27 for the 3x3 RGB layers, 40 for the 10x4 single-channel one), 8 or 16 output
// channels per block. The reduction is padded to 4 * KT and runs as KT 16x16x4 matrix instructions per 16
// pixels: the filter operands (one float per lane and instruction) stay in registers for the whole kernel, the
// input operand of lane (pixel p, q) in instruction t is the single input value k = 4t + q = (tap, channel) of
// the pixel's window, gathered straight from global memory (neighbouring lanes read neighbouring pixels; the
// nine values of one filter row are contiguous). No LDS: conv_small spends its time re-reading broadcast filter
// values from LDS, 16 per tap and lane.
struct FirstArgs {
    ConvArgs c;
    int Cib, Cob, K;
    int plain_input;      // the input is a plain [N][C][H][W] tensor (the network's own input): the layout change
                          // of the network boundary then happens in this kernel's gathers
    FastDiv div_HoWo, div_Wo;
    unsigned in_bytes, filt_bytes, out_bytes;       // each below 2 GiB
};

// CIB, KW > 0: the layer's input block and window width as compile-time constants (the decoding of k into
// (tap, channel) is then free); 0, 0: read from the arguments.
// A wave gathers the input values of its WM groups of 16 pixels once and walks the output blocks with them in
// registers (a workgroup per output block would gather them once per block: 24.6 against 21 us on the audio
// CNN's first layer, 64 output channels, at batch 1024). Every access goes through a buffer descriptor over its
// whole tensor (tensors below 2 GiB): an offset of 32 bits per access instead of a 64-bit address, and masks (a
// tap outside the image, a pixel past the end, a channel the block does not have) are offsets beyond the
// descriptor, which read zero and drop stores, instead of selects on the values. The kernel's time is the
// output stream, address arithmetic and waiting, not matrix instructions: 1600 vector instructions per wave
// with 64-bit addresses and selects, 500 this way (21 -> 16 us on that layer).
template <int KT, int WM, int CIB, int KW>
__global__ void __launch_bounds__(256) conv_first_mfma(FirstArgs f)
{
    const ConvArgs &a = f.c;
    const int cib = CIB ? CIB : f.Cib, kw = KW ? KW : a.kw;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, q = lane >> 4;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.in), 0, f.in_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t flt = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.filt), 0, f.filt_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, f.out_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t res = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.res), 0, f.out_bytes, kRawBuffer);

    // this lane's reduction elements: k = 4t + q -> (dy, dx, ci), byte offset inside the window
    int koff[KT], kdy[KT], kdx[KT];
#pragma unroll
    for (int t = 0; t < KT; ++t) {
        const int k = 4 * t + q;
        const int tap = k / cib, ci = k - tap * cib;
        kdy[t] = tap / kw;
        kdx[t] = tap - kdy[t] * kw;
        koff[t] = 4 * (f.plain_input ? ci * a.H * a.W + kdy[t] * a.W + kdx[t] : (kdy[t] * a.W + kdx[t]) * cib + ci);
        if (k >= f.K) kdy[t] = 1 << 20;      // never inside the image: the operand reads as zero
    }
    // filter value (block cob, k = 4t + q, channel p) sits at ((cob K + k) Cob + p) floats
    const unsigned f_at = p < f.Cob ? (unsigned)(q * f.Cob + p) * 4u : kBeyond;
    const int f_step = 16 * f.Cob, f_block = 4 * f.K * f.Cob;
    auto filter_of = [&](int cob, float (&fa)[KT]) __attribute__((always_inline)) {
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const bool live = t + 1 < KT || 4 * t + q < f.K;
            fa[t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(flt, live ? f_at + (unsigned)(cob * f_block + t * f_step) : kBeyond, 0, 0));
        }
    };
    float fa[KT];
    filter_of(0, fa);

    // All input values of the wave's WM pixel groups are requested before the first matrix instruction: a wave
    // has only a few hundred cycles of arithmetic, so the loads of one group after the other would each expose
    // their full latency (and the grid is a single round of waves). They serve every output block: the wave walks
    // the blocks with the gathered values in registers (a workgroup per output block would gather them again).
    float fb[WM][KT];
    unsigned o_at[WM];
    const int image_bytes = 4 * a.H * a.W * cib, px_bytes = 4 * (f.plain_input ? 1 : cib);
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        const int m_own = tile0 + wm * 16 + p;
        const int m = m_own < a.M ? m_own : a.M - 1;
        const int n = f.div_HoWo.div(m), rem = m - n * a.HoWo;
        const int oy = f.div_Wo.div(rem), ox = rem - oy * a.Wo;
        const int iy0 = oy * a.stride - a.pt, ix0 = ox * a.stride - a.pl;
        const int org = n * image_bytes + (iy0 * a.W + ix0) * px_bytes;       // window origin, may lie before the image
#pragma unroll
        for (int t = 0; t < KT; ++t) {
            const bool inside = (unsigned)(iy0 + kdy[t]) < (unsigned)a.H && (unsigned)(ix0 + kdx[t]) < (unsigned)a.W;
            fb[wm][t] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(src, inside ? (unsigned)(org + koff[t]) : kBeyond, 0, 0));
        }
        // lane (p, q) holds output channels 4q .. 4q+3 of pixel p
        o_at[wm] = (m_own < a.M && 4 * q < f.Cob) ? (unsigned)(((n * a.nCob * a.HoWo + rem) * f.Cob + 4 * q) * 4) : kBeyond;
    }
    const int o_block = 4 * a.HoWo * f.Cob;
    for (int cob = 0; cob < a.nCob; ++cob) {
        float fn[KT];
        filter_of(cob + 1 < a.nCob ? cob + 1 : cob, fn);          // the next block's filter values, under way early
        floatx4 acc[WM];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            acc[wm] = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < KT; ++t) acc[wm] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[t], fb[wm][t], acc[wm], 0, 0, 0);
        }
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            const unsigned o = o_at[wm] + (unsigned)(cob * o_block);
            floatx4 v = acc[wm];
            if (a.epilogue & EPI_ADD) v += __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(res, o, 0, 0));
            if (a.epilogue & EPI_RELU) {
                v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
                v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
            }
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, v), dst, o, 0, 0);
        }
#pragma unroll
        for (int t = 0; t < KT; ++t) fa[t] = fn[t];
    }
}

// Which layers the kernel above takes: one input block of fewer than 16 channels, a reduction of 5..8 (the
// pointwise layer after an 8-channel depthwise one), 25..28 or 37..40 values, input and output tensors below 2 GiB
// each (32-bit buffer offsets).
int first_mfma_steps(const LayerGeom &g)
{
    if (g.Ci != g.Cib || g.Cib >= 16 || (g.Cob != 8 && g.Cob != 16)) return 0;
    if ((size_t)g.N * g.H * g.W * g.Ci * 4 >= kBeyond || (size_t)g.N * g.Ho * g.Wo * g.Co * 4 >= kBeyond) return 0;
    const int K = g.Cib * g.kh * g.kw, kt = (K + 3) / 4;
    return (kt == 2 || kt == 7 || kt == 10) ? kt : 0;
}

// One lane per pixel (conv_small) needs enough pixels to fill the chip; dense heads and other layers with
// few output pixels take one lane per output element instead.
bool use_small(const LayerGeom &g)
{
    const long M = (long)g.N * g.Ho * g.Wo;
    return g.Cob <= 16 && (g.Ci / g.Cib) * g.kh * g.kw * g.Cib * 16 <= kSmallMaxFilterFloats && M >= 16384;
}

bool is_dense(const LayerGeom &g)
{
    return g.Ho == 1 && g.Wo == 1 && g.kh == g.H && g.kw == g.W && g.pt == 0 && g.pl == 0;
}

const char *const kTileWaves[] = {"2,2,4,4", "1,4,4,2", "2,2,4,2", "2,2,2,2", "4,1,2,2", "4,1,1,2", "4,1,2,1", "4,1,1,1",
                                  "2,2,1,2", "2,2,1,1", "4,1,4,1"};

}  // namespace

int group_conv_same_tile(const LayerGeom &g, int F_C, int S_C, int K)
{
    if (g.Cib != 16 || g.Cob != 16 || F_C % 16 || S_C % 16 || K % 16 || F_C <= 0 || S_C <= 0 || K <= 0) return -1;
    LayerGeom one = g;                   // one group as a convolution of its own: what the kernels must be able to take
    one.Ci = F_C;
    one.Co = K;
    // (byte offsets are those of the whole tensors)
    if (!conv_same_eligible(one) || !((size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30)) ||
        !((size_t)g.N * g.Co * g.Ho * g.Wo < ((size_t)1 << 30)))
        return -1;
    // the tile's output channels must not straddle groups
    if (g.kh == 1) return K % 64 == 0 ? SAME_32x64 : K % 32 == 0 ? SAME_32x32 : SAME_64x16;
    return K % 32 == 0 ? SAME_64x32 : SAME_64x16;
}

const char *conv_kernel_name(const LayerGeom &g)
{
    static thread_local char name[64];
    if (g.Cib != 16 || g.Cob != 16)
    {
        if (!use_small(g)) return is_dense(g) ? "dense_rows" : "conv_direct";
        if (first_mfma_steps(g) == 2) return "conv_first_mfma<2,4>";
        if (first_mfma_steps(g)) return first_mfma_steps(g) == 7 ? "conv_first_mfma<7,4>" : "conv_first_mfma<10,4>";
        if (g.Cib == 3 && g.kh == 3 && g.kw == 3) return "conv_small<3,3,3>";
        if (g.Cib == 1 && g.kh == 10 && g.kw == 4) return "conv_small<1,10,4>";
        if (g.Cib == 8 && g.kh == 1 && g.kw == 1) return "conv_small<8,1,1>";
        return "conv_small<0,0,0>";
    }
    if (conv_pw_eligible(g)) return conv_pw_kernel_name(g);
    const int tile = pick_tile(g);
    if (conv_same_eligible(g))
        snprintf(name, sizeof(name), "%s<%s,%d,%d,%d>", conv_same_images_per_workgroup(g, tile) ? "conv16_img" : "conv16_same",
                 kTileWaves[tile], g.kw, conv_same_planes(g), (g.kw == 3 && g.stride == 2) ? 2 : 1);
    else
        snprintf(name, sizeof(name), "conv16_mfma<%s>", kTileWaves[tile]);
    return name;
}

bool conv_takes_plain_input(const LayerGeom &g, const void *in, const void *filt, const void *out, const void *res)
{
    const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt | (uintptr_t)res) & 15u) == 0);
    return aligned && first_mfma_steps(g) && use_small(g);
}

bool conv_epilogue_takes_bn(const LayerGeom &g, const void *in, const void *filt, const void *out, const void *res,
                            const void *bn)
{
    const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt | (uintptr_t)res | (uintptr_t)bn) & 15u) == 0);
    return aligned && g.Cib == 16 && g.Cob == 16 && (conv_pw_eligible(g) || conv_same_eligible(g));
}

hipError_t launch_conv(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g, int epilogue,
                       hipStream_t s, bool plain_input, const float *bn)
{
    if ((epilogue & EPI_BN) && !conv_epilogue_takes_bn(g, in, filt, out, (epilogue & EPI_ADD) ? res : out, bn))
        return hipErrorInvalidValue;        // (the runner launches the normalization on its own in that case)
    ConvArgs a;
    a.in = in; a.filt = filt; a.out = out; a.res = (epilogue & EPI_ADD) ? res : out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo;
    a.nCib = g.Ci / g.Cib; a.nCob = g.Co / g.Cob;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    a.HoWo = g.Ho * g.Wo;
    a.M = g.N * a.HoWo;
    a.epilogue = epilogue;

    const bool aligned = ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt | (uintptr_t)a.res) & 15u) == 0);
    if (plain_input && !conv_takes_plain_input(g, in, filt, out, a.res)) return hipErrorInvalidValue;
    if (aligned && first_mfma_steps(g) && use_small(g)) {
        FirstArgs f;
        f.c = a;
        f.Cib = g.Cib; f.Cob = g.Cob; f.K = g.Cib * g.kh * g.kw;
        f.plain_input = plain_input ? 1 : 0;
        f.div_HoWo = make_fastdiv(a.HoWo);
        f.div_Wo = make_fastdiv(g.Wo);
        const dim3 grid((unsigned)((a.M + 255) / 256));
        const int kt = first_mfma_steps(g);
        f.in_bytes = (unsigned)((size_t)g.N * g.H * g.W * g.Ci * 4);
        f.out_bytes = (unsigned)((size_t)a.M * g.Co * 4);
        f.filt_bytes = (unsigned)((size_t)g.Co * f.K * 4);
        if (g.Cib == 3 && g.kw == 3 && kt == 7) hipLaunchKernelGGL((conv_first_mfma<7, 4, 3, 3>), grid, dim3(256), 0, s, f);
        else if (g.Cib == 1 && g.kw == 4 && kt == 10) hipLaunchKernelGGL((conv_first_mfma<10, 4, 1, 4>), grid, dim3(256), 0, s, f);
        else if (g.Cib == 8 && g.kw == 1 && kt == 2) hipLaunchKernelGGL((conv_first_mfma<2, 4, 8, 1>), grid, dim3(256), 0, s, f);
        else if (kt == 2) hipLaunchKernelGGL((conv_first_mfma<2, 4, 0, 0>), grid, dim3(256), 0, s, f);
        else if (kt == 7) hipLaunchKernelGGL((conv_first_mfma<7, 4, 0, 0>), grid, dim3(256), 0, s, f);
        else hipLaunchKernelGGL((conv_first_mfma<10, 4, 0, 0>), grid, dim3(256), 0, s, f);
        return hipGetLastError();
    }
    if (!aligned || g.Cib != 16 || g.Cob != 16) {
        const int kfloats = a.nCib * g.kh * g.kw * g.Cib * 16;
        if (use_small(g)) {
            const dim3 grid((unsigned)((a.M + 255) / 256), (unsigned)a.nCob);
            const size_t lds = (size_t)kfloats * 4;
            if (g.Cib == 3 && g.kh == 3 && g.kw == 3)
                hipLaunchKernelGGL((conv_small<3, 3, 3>), grid, dim3(256), lds, s, a, g.Cib, g.Cob, kfloats);
            else if (g.Cib == 1 && g.kh == 10 && g.kw == 4)
                hipLaunchKernelGGL((conv_small<1, 10, 4>), grid, dim3(256), lds, s, a, g.Cib, g.Cob, kfloats);
            else if (g.Cib == 8 && g.kh == 1 && g.kw == 1)
                hipLaunchKernelGGL((conv_small<8, 1, 1>), grid, dim3(256), lds, s, a, g.Cib, g.Cob, kfloats);
            else
                hipLaunchKernelGGL((conv_small<0, 0, 0>), grid, dim3(256), lds, s, a, g.Cib, g.Cob, kfloats);
            return hipGetLastError();
        }
        const size_t total = (size_t)a.M * g.Co;
        if (is_dense(g)) {
            const int K = g.Ci * g.kh * g.kw;
            const int vec = K % 4 == 0 && ((uintptr_t)in & 15u) == 0;
            hipLaunchKernelGGL(dense_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a, g.Cob, K, total, vec);
            return hipGetLastError();
        }
        hipLaunchKernelGGL(conv_direct, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s, a, g.Cib, g.Cob, total);
        return hipGetLastError();
    }
    if (conv_pw_eligible(g)) return launch_conv_pw(in, filt, out, a.res, g, epilogue, s, bn);
    const int tile = pick_tile(g);
    if (conv_same_eligible(g)) return launch_conv_same(in, filt, out, a.res, g, tile, epilogue, s, 0, 0, 0, bn);
    switch (tile) {
        case SAME_128x128: launch_mfma<2, 2, 4, 4>(a, s); break;
        case SAME_64x128: launch_mfma<1, 4, 4, 2>(a, s); break;
        case SAME_128x64: launch_mfma<2, 2, 4, 2>(a, s); break;
        case SAME_64x64: launch_mfma<2, 2, 2, 2>(a, s); break;
        case SAME_128x32: launch_mfma<4, 1, 2, 2>(a, s); break;
        case SAME_64x32: launch_mfma<4, 1, 1, 2>(a, s); break;
        case SAME_128x16: launch_mfma<4, 1, 2, 1>(a, s); break;
        case SAME_32x64: launch_mfma<2, 2, 1, 2>(a, s); break;
        case SAME_32x32: launch_mfma<2, 2, 1, 1>(a, s); break;
        case SAME_256x16: launch_mfma<4, 1, 4, 1>(a, s); break;
        default: launch_mfma<4, 1, 1, 1>(a, s); break;
    }
    return hipGetLastError();
}

}  // namespace small
