// A run of depthwise-separable blocks in one kernel: [depthwise 3x3, stride 1, padding 1 (+ ReLU)] -> [pointwise 1x1
// (+ ReLU)], repeated, every block C -> C channels with C = 64 or 128, on images small enough that a workgroup holds
// whole images (at most 128 pixels each). This is the abstract fused layer of the paper's "Conclusion & Future
// Directions" across a single-channel reduction and a full-channel reduction (Table 1), several times over: the
// tail of the depthwise-separable CNN (five 128-channel blocks on 3x3 images) and the body of the audio CNN (four
// 64-channel blocks on 25x5 images) of Section "MLPerf:Tiny Inference Models" are such runs. Only the run's input,
// its last output and the filters touch memory; layer by layer every block costs a launch, a prologue and a round
// trip of its tensors.
//
// A workgroup (8 waves) takes G = floor(16 WM / HW) whole images, 16 WM pixel slots (WM groups of 16). Activations
// live in LDS in two buffers of [channel block][pixel group][lane (pixel p, quad q)] float4 -- the accumulator
// layout of v_mfma_f32_16x16x4_f32, which is also its B-operand layout (chain.hip). Wave w owns channel block
// w % nCb; with four channel blocks the two waves of a block split the pixel groups.
//   depthwise stage: buffer 0 -> buffer 1. A lane gathers the nine window entries of its pixel from LDS (a bit mask
//     per pixel says which lie in the image; the others contribute nothing), multiplies with the taps of its
//     channel quad and applies the ReLU. A wave touches its own channel block only.
//   pointwise stage: buffer 1 -> buffer 0 (or, in the last block, memory). One reduction step per input block: B is
//     a plain 16-byte LDS read, A the wave's 16 x 16 filter block.
//   Two workgroup barriers per block. Filters never wait for activations: every wave copies its blocks -- per
//     block of the run the 9 x 16 depthwise taps of its channel block, then its nCb pointwise blocks -- global ->
//     LDS with the load unit into a ring of its own, STAGES - 1 steps ahead and across stage and block boundaries;
//     one copy is issued per step consumed, so the wait before a step is a constant count.
#include "small_internal.h"

namespace small {
namespace {

constexpr int kDcWaves = 8;
constexpr int kDcThreads = kDcWaves * 64;
constexpr int kDcStages = 4;

struct DcBlock {
    const float *dw;       // [C/16][3][3][16]
    const float *pw;       // [C/16][C/16][1][1][16][16]
    int dw_relu, pw_relu;
};

struct DcArgs {
    const float *in;
    float *out;
    int N, H, W, HW, nCb;
    int G;                 // images per workgroup
    int n_blocks;
    DcBlock block[kDwpwChainMaxBlocks];
};

typedef const __attribute__((address_space(4))) DcArgs *DcKernArgs;

__device__ __forceinline__ const float *dc_uniform(const float *p)
{
    const uintptr_t v = (uintptr_t)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const float *)(((uintptr_t)hi << 32) | lo);
}

// The wave's flat sequence of filter copies: per block of the run the depthwise taps, then the pointwise blocks.
struct DcCursor { int block, step; };       // step 0: depthwise taps; 1 .. nCb: pointwise input block step - 1

// WM: groups of 16 pixel slots per workgroup; NG: groups per wave (WM with eight channel blocks, WM / 2 with four)
template <int WM, int NG>
__global__ void __launch_bounds__(kDcThreads) dwpw_chain(DcArgs args)
{
    (void)args;
    const DcKernArgs ka = (DcKernArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const int N = ka->N, W = ka->W, H = ka->H, HW = ka->HW, nCb = ka->nCb, G = ka->G, n_blocks = ka->n_blocks;

    extern __shared__ floatx4 lds[];
    char *lds_c = reinterpret_cast<char *>(lds);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = lane & 15, q = lane >> 4;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;

    // LDS: [ring: 8 waves x kDcStages KB][buffer 0: nCb x WM KB][buffer 1: nCb x WM KB]
    const int ring_off = w * kDcStages * 1024;
    const int act_bytes = nCb * WM * 1024;
    const int act0 = kDcWaves * kDcStages * 1024, act1 = act0 + act_bytes;

    // this wave's channel block and pixel groups
    const int cb = w % nCb, half = w / nCb;             // half: 0 with eight channel blocks, 0 or 1 with four
    constexpr int kMaxGroups = NG, n_groups = NG;
    const int g0 = half * NG;

    // per pixel slot of this lane: where the pixel lies, which window entries exist
    const int img0 = (int)blockIdx.x * G;
    unsigned in_off[kMaxGroups];                        // byte offset of (image, block cb, pixel, quad q) in the tensors
    unsigned tapmask[kMaxGroups];                       // bit t: window entry t lies inside the image; bit 9: a real pixel
#pragma unroll
    for (int k = 0; k < kMaxGroups; ++k) {
        in_off[k] = 0;
        tapmask[k] = 0;
        if (k < n_groups) {
            const int m = (g0 + k) * 16 + p;
            const int im = m / HW, pix = m - im * HW;
            const bool real = im < G && img0 + im < N;
            const int imc = real ? im : 0, pc = real ? pix : 0;
            const int y = pc / W, x = pc - y * W;
            unsigned mask = real ? 1u << 9 : 0u;
            if (real) {
#pragma unroll
                for (int t = 0; t < 9; ++t) {
                    const int yy = y + t / 3 - 1, xx = x + t % 3 - 1;
                    if (yy >= 0 && yy < H && xx >= 0 && xx < W) mask |= 1u << t;
                }
            }
            tapmask[k] = mask;
            in_off[k] = (unsigned)((((size_t)(img0 + imc) * nCb + cb) * HW + pc) * 64 + q * 16);
        }
    }

    // ---- the filter ring
    const unsigned off_pw = (unsigned)((4 * ((lane >> 2) & 3) + (lane >> 4)) * 64 + (lane & 3) * 16);   // rows permuted (chain.hip)
    const unsigned off_dw = (unsigned)(min(lane, 35) * 16);                                            // 576 bytes of taps
    DcCursor cur = {0, 0};
    auto issue = [&](int slot) __attribute__((always_inline)) {
        const int b = min(cur.block, n_blocks - 1);     // past the run's end: the last copy again (never read)
        const float *src = cur.step == 0 ? ka->block[b].dw + (size_t)cb * 144
                                         : ka->block[b].pw + ((size_t)cb * nCb + (cur.step - 1)) * 256;
        dma16(dc_uniform(src), cur.step == 0 ? off_dw : off_pw, lds0 + (unsigned)(ring_off + slot * 1024));
        if (cur.block < n_blocks && ++cur.step > nCb) {
            cur.step = 0;
            ++cur.block;
        }
    };

    // input tile -> buffer 0 (this wave's channel block, its pixel groups), then the ring's first copies
#pragma unroll
    for (int k = 0; k < kMaxGroups; ++k)
        if (k < n_groups) dma16(dc_uniform(ka->in), in_off[k], lds0 + (unsigned)(act0 + (cb * WM + g0 + k) * 1024));
#pragma unroll
    for (int s = 0; s < kDcStages - 1; ++s) issue(s);
    wait_vmcnt<kDcStages - 1>();                        // the input copies of this wave have landed
    __syncthreads();                                    // ... and those of the wave it shares the block with

    int s = 0;                                          // steps consumed: ring slot s % kDcStages
    for (int b = 0; b < n_blocks; ++b) {
        const int dw_relu = ka->block[b].dw_relu, pw_relu = ka->block[b].pw_relu;
        // ---------------- depthwise stage: buffer 0 -> buffer 1
        wait_vmcnt<kDcStages - 2>();
        issue((s + kDcStages - 1) % kDcStages);
        {
            const floatx4 *taps = reinterpret_cast<const floatx4 *>(lds_c + ring_off + (s % kDcStages) * 1024) + q;
            floatx4 wt[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) wt[t] = taps[t * 4];
            const floatx4 *src = reinterpret_cast<const floatx4 *>(lds_c + act0) + cb * WM * 64 + q * 16;
            floatx4 *dst = reinterpret_cast<floatx4 *>(lds_c + act1) + (cb * WM + g0) * 64 + lane;
#pragma unroll
            for (int k = 0; k < kMaxGroups; ++k) {
                if (k < n_groups) {
                    const int m = (g0 + k) * 16 + p;
                    floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
                    for (int t = 0; t < 9; ++t) {
                        const int mm = m + (t / 3 - 1) * W + (t % 3 - 1);
                        const bool on = (tapmask[k] >> t) & 1u;
                        const int at = on ? (mm >> 4) * 64 + (mm & 15) : 0;
                        const floatx4 v = src[at];
                        if (on) acc += v * wt[t];
                    }
                    if (dw_relu) {
                        acc.x = acc.x > 0.f ? acc.x : 0.f; acc.y = acc.y > 0.f ? acc.y : 0.f;
                        acc.z = acc.z > 0.f ? acc.z : 0.f; acc.w = acc.w > 0.f ? acc.w : 0.f;
                    }
                    dst[k * 64] = acc;
                }
            }
        }
        ++s;
        __syncthreads();                                // buffer 1 is complete
        // ---------------- pointwise stage: buffer 1 -> buffer 0 / memory
        floatx4 acc[kMaxGroups];
#pragma unroll
        for (int k = 0; k < kMaxGroups; ++k) acc[k] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int ci = 0; ci < nCb; ++ci, ++s) {
            wait_vmcnt<kDcStages - 2>();
            issue((s + kDcStages - 1) % kDcStages);
            const float *af = reinterpret_cast<const float *>(lds_c + ring_off + (s % kDcStages) * 1024) + lane;
            float a4[4];
#pragma unroll
            for (int r = 0; r < 4; ++r) a4[r] = af[r * 64];
            const floatx4 *bsrc = reinterpret_cast<const floatx4 *>(lds_c + act1) + (ci * WM + g0) * 64 + lane;
            floatx4 bv[kMaxGroups];
#pragma unroll
            for (int k = 0; k < kMaxGroups; ++k)
                if (k < n_groups) bv[k] = bsrc[k * 64];
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int k = 0; k < kMaxGroups; ++k)
                    if (k < n_groups) acc[k] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[r], bv[k][r], acc[k], 0, 0, 0);
        }
        const bool last = b + 1 == n_blocks;
#pragma unroll
        for (int k = 0; k < kMaxGroups; ++k) {
            if (k < n_groups) {
                floatx4 v = acc[k];
                if (pw_relu) {
                    v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
                    v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
                }
                if (last) {
                    if ((tapmask[k] >> 9) & 1u)
                        *reinterpret_cast<floatx4 *>(reinterpret_cast<char *>(ka->out) + in_off[k]) = v;
                } else {
                    reinterpret_cast<floatx4 *>(lds_c + act0)[(cb * WM + g0 + k) * 64 + lane] = v;
                }
            }
        }
        if (!last) __syncthreads();                     // buffer 0 is complete (and buffer 1 free again)
    }
    wait_vmcnt<0>();        // copies issued past the run's last step must land before the workgroup's LDS is released
}

template <int WM, int NG>
hipError_t launch_dc(const DcArgs &a, hipStream_t s)
{
    const size_t lds = (size_t)kDcWaves * kDcStages * 1024 + 2 * (size_t)a.nCb * WM * 1024;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(dwpw_chain<WM, NG>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    const unsigned wgs = (unsigned)((a.N + a.G - 1) / a.G);
    hipLaunchKernelGGL((dwpw_chain<WM, NG>), dim3(wgs), dim3(kDcThreads), lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool dwpw_chain_eligible(int C, int H, int W)
{
    // whole images in at most 64 pixel slots (measured on the audio network's 25 x 5 images with 128 slots and one
    // workgroup per compute unit: no faster than a launch per block)
    return (C == 64 || C == 128) && H >= 1 && W >= 1 && (long)H * W <= 64;
}

hipError_t launch_dwpw_chain(const float *in, float *out, const DwpwChainBlock *blocks, int n_blocks, int N, int C, int H, int W,
                             hipStream_t s)
{
    DcArgs a;
    a.in = in; a.out = out;
    a.N = N; a.H = H; a.W = W; a.HW = H * W; a.nCb = C / 16;
    a.n_blocks = n_blocks;
    for (int i = 0; i < kDwpwChainMaxBlocks; ++i) {
        const DwpwChainBlock &b = blocks[i < n_blocks ? i : n_blocks - 1];
        a.block[i] = DcBlock{b.dw, b.pw, b.dw_relu, b.pw_relu};
    }
    // Pixel slots per workgroup (16, 32 or 64; with four channel blocks at least 32, two waves sharing a block): the
    // largest tile that still gives every compute unit a workgroup, else the smallest that holds an image. Small tiles
    // waste matrix-instruction lanes (a 3 x 3 image fills 9 of 16) and stream the filters more often, but these runs
    // are bound by the chain of stages of one workgroup, not by arithmetic.
    const int wm_min = a.nCb == 4 ? 2 : 1;
    int wm = 4;
    while (wm > wm_min && wm * 8 >= a.HW && (N + (16 * wm / a.HW) - 1) / (16 * wm / a.HW) < device_cus()) wm /= 2;
    while (16 * wm < a.HW) wm *= 2;
    a.G = 16 * wm / a.HW;
    if (a.nCb == 8) return wm == 1 ? launch_dc<1, 1>(a, s) : (wm == 2 ? launch_dc<2, 2>(a, s) : launch_dc<4, 4>(a, s));
    return wm == 2 ? launch_dc<2, 1>(a, s) : launch_dc<4, 2>(a, s);
}

}  // namespace small
