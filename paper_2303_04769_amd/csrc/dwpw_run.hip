// A run of depthwise-separable blocks in one kernel, the blocks' shapes free to change inside the run:
// [depthwise 3x3, any stride and padding (+ ReLU)] -> [pointwise 1x1, Cin -> Cout (+ ReLU)], repeated, on images
// small enough that a workgroup holds whole images (at most 64 pixels where the run starts). This is the abstract
// fused layer of the paper's "Conclusion & Future Directions" across single-channel and full-channel reductions
// (Table 1), several times over: the second half of the depthwise-separable CNN of Section "MLPerf:Tiny Inference
// Models" -- nine blocks from 64 channels on 6x6 images to 256 channels on 2x2 -- is one such run. Only the run's
// input, its last output and the filters touch memory; layer by layer every block costs a launch, a prologue and a
// round trip of its tensors, which at these sizes is all of its time.
//
// A workgroup (8 waves) takes G whole images. Activations live in LDS in two buffers of
// [channel block][pixel group][lane (pixel p, quad q)] float4 -- the accumulator layout of v_mfma_f32_16x16x4_f32,
// which is also its B-operand layout; pixel slot m = image * (pixels per image) + pixel, so the slots move when a
// strided block shrinks the images.
//   depthwise stage: buffer 0 -> buffer 1. Work items (channel block, pixel group) go round the waves; a lane
//     finds its output pixel's window entries in buffer 0 (those outside the image contribute nothing), multiplies
//     with the taps of its channel quad and applies the ReLU.
//   pointwise stage: buffer 1 -> buffer 0 (or, in the last block, memory). Work items are output channel blocks
//     (with fewer than eight of them, halves or quarters of the pixel groups as well); one reduction step per
//     input block: B is a plain 16-byte LDS read, A the item's 16 x 16 filter block.
//   Two workgroup barriers per block. Filters never wait for activations: every wave copies the filter blocks of
//     its items -- in the order it will use them, through all stages and blocks of the run -- global -> LDS with
//     the load unit into a ring of its own, STAGES - 1 steps ahead; one copy is issued per step consumed, so the
//     wait before a step is a constant count.
#include "small_internal.h"

#include <algorithm>

namespace small {
namespace {

constexpr int kDrWaves = 8;
constexpr int kDrThreads = kDrWaves * 64;

struct DrBlock {
    const float *dw;       // [Cin/16][3][3][16]
    const float *pw;       // [Cout/16][Cin/16][1][1][16][16]
    int dw_relu, pw_relu;
    int nCbi, nCbo;
    int Hi, Wi, Ho, Wo, stride, pt, pl;
    FastDiv by_HWo, by_Wo, by_nCbi, by_nCbo;
};

struct DrArgs {
    const float *in;
    float *out;
    int N, G, n_blocks;
    int act_bytes;         // of one activation buffer
    FastDiv by_HWi0;       // pixels per image of the run's input
    const float *head;     // closing average over the last result's pixels + fully connected layer [Co/Cob][C/16][16][Cob],
    int head_Co, head_Cob; // or null: the last result goes to memory
    DrBlock block[kDwpwChainMaxBlocks];
};

typedef const __attribute__((address_space(4))) DrArgs *DrKernArgs;

__device__ __forceinline__ const float *dr_uniform(const float *p)
{
    const uintptr_t v = (uintptr_t)p;
    const unsigned lo = __builtin_amdgcn_readfirstlane((unsigned)v), hi = __builtin_amdgcn_readfirstlane((unsigned)(v >> 32));
    return (const float *)(((uintptr_t)hi << 32) | lo);
}

// A division constant read from the kernel arguments (scalar loads), in two registers instead of three: the kernel
// lives at the limit of the scalar registers (what does not fit is kept in lanes of a vector register and fetched from
// there, inside the loops too), and it holds six of these. A divisor of 1 is marked in the shift.
struct DrDiv {
    unsigned magic, shift;
    __device__ __forceinline__ int div(int n) const { return (shift & 0x80u) ? n : (int)(__umulhi((unsigned)n, magic) >> shift); }
};
__device__ __forceinline__ DrDiv dr_fd(const __attribute__((address_space(4))) FastDiv &x)
{
    DrDiv f;
    f.magic = x.magic;
    f.shift = x.d == 1 ? 0x80u : x.shift;
    return f;
}
// pixel groups of a tensor of G images
__device__ __forceinline__ int dr_groups(int G, int HW) { return (G * HW + 15) >> 4; }
// how the pointwise stage splits the pixel groups when there are fewer output blocks than waves
__device__ __forceinline__ int dr_parts(int nCbo, int ng) { return nCbo >= kDrWaves ? 1 : min(kDrWaves / nCbo, ng); }

// These kernels run two waves per SIMD and are bound by how many instructions a step costs, not by memory: everything
// a step needs is kept in registers, the copy cursor has a fast path of a handful of scalar instructions (the filter
// blocks of a pointwise item are consecutive in memory), and the reduction loop is compiled per number of pixel groups.

// The pointwise reduction of one item over NK pixel groups: one step per input block. (Two blocks per turn into two sets
// of accumulators, so that the matrix instructions of a step do not wait for each other, measured slower: 110 against
// 102 us for the depthwise-separable CNN at batch 256.)
template <int NK, int STAGES, typename Issue>
__device__ __forceinline__ void dr_reduce(floatx4 (&acc)[NK], int nCbi, const char *ring_lane, const floatx4 *bsrc, int b_stride,
                                          unsigned &rs, Issue &issue)
{
#pragma unroll
    for (int k = 0; k < NK; ++k) acc[k] = floatx4{0.f, 0.f, 0.f, 0.f};
    for (int ci = 0; ci < nCbi; ++ci) {
        wait_vmcnt<STAGES - 2>();
        issue();
        const float *af = reinterpret_cast<const float *>(ring_lane + rs * 1024);    // this lane's column of the filter block
        rs = (rs + 1) & (STAGES - 1);
        float a4[4];
#pragma unroll
        for (int r = 0; r < 4; ++r) a4[r] = af[r * 64];
        floatx4 bv[NK];
#pragma unroll
        for (int k = 0; k < NK; ++k) bv[k] = bsrc[k * 64];
        bsrc += b_stride;
#pragma unroll
        for (int r = 0; r < 4; ++r)
#pragma unroll
            for (int k = 0; k < NK; ++k) acc[k] = __builtin_amdgcn_mfma_f32_16x16x4f32(a4[r], bv[k][r], acc[k], 0, 0, 0);
    }
}

// STAGES: kilobytes of a wave's filter ring (a power of two)
template <int STAGES>
__global__ void __launch_bounds__(kDrThreads) dwpw_run(DrArgs args)
{
    (void)args;
    const DrKernArgs ka = (DrKernArgs)__builtin_amdgcn_kernarg_segment_ptr();
    const int N = ka->N, G = ka->G, n_blocks = ka->n_blocks;

    extern __shared__ floatx4 lds[];
    char *lds_c = reinterpret_cast<char *>(lds);
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int p = lane & 15, q = lane >> 4;
    const unsigned lds0 = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;

    // LDS: [ring: 8 waves x STAGES KB][buffer 0][buffer 1]
    const int ring_off = w * STAGES * 1024;
    const int act0 = kDrWaves * STAGES * 1024, act1 = act0 + ka->act_bytes;
    const int img0 = (int)blockIdx.x * G;

    // ---- the filter ring: this wave's copies in the order of use
    const unsigned off_pw = (unsigned)((4 * ((lane >> 2) & 3) + (lane >> 4)) * 64 + (lane & 3) * 16);   // rows permuted (chain.hip)
    const unsigned off_dw = (unsigned)(min(lane, 35) * 16);                                            // 576 bytes of taps
    // cursor: block, stage (0 depthwise, 1 pointwise), item; and, for the fast path, the item's next copy
    int c_b = 0, c_phase = 0, c_item = w;
    const float *c_dw, *c_pw;
    int c_nCbi, c_nCbo, c_lim_dw, c_lim_pw;
    DrDiv c_by_nCbi, c_by_nCbo;
    const float *c_src;
    int c_left = 0, c_stride = 0;
    unsigned c_off = off_dw, ws = 0;                    // ws: ring slot of the next copy
    auto enter_block = [&](int b) __attribute__((always_inline)) {
        const int ng = dr_groups(G, ka->block[b].Ho * ka->block[b].Wo);
        c_dw = ka->block[b].dw; c_pw = ka->block[b].pw;
        c_nCbi = ka->block[b].nCbi; c_nCbo = ka->block[b].nCbo;
        c_lim_dw = c_nCbi * ng; c_lim_pw = c_nCbo * dr_parts(c_nCbo, ng);
        c_by_nCbi = dr_fd(ka->block[b].by_nCbi); c_by_nCbo = dr_fd(ka->block[b].by_nCbo);
    };
    enter_block(0);
    c_src = c_dw;
    auto next_item = [&]() __attribute__((always_inline)) {
        while (c_b < n_blocks && c_item >= (c_phase == 0 ? c_lim_dw : c_lim_pw)) {      // stages without an item left
            c_item = w;
            if (c_phase == 0) c_phase = 1;
            else {
                c_phase = 0;
                if (++c_b < n_blocks) enter_block(c_b);
            }
        }
        if (c_b >= n_blocks) {                          // past the run's end: copies nobody reads
            c_src = c_dw; c_off = off_dw; c_stride = 0; c_left = 1 << 30;
        } else if (c_phase == 0) {
            const int grp = c_by_nCbi.div(c_item), cb = c_item - grp * c_nCbi;
            c_src = c_dw + (size_t)cb * 144; c_off = off_dw; c_stride = 0; c_left = 1;
        } else {
            const int part = c_by_nCbo.div(c_item), cob = c_item - part * c_nCbo;
            c_src = c_pw + (size_t)cob * c_nCbi * 256; c_off = off_pw; c_stride = 256; c_left = c_nCbi;
        }
        c_item += kDrWaves;
    };
    auto issue = [&]() __attribute__((always_inline)) {
        if (c_left == 0) next_item();
        dma16(dr_uniform(c_src), c_off, lds0 + (unsigned)ring_off + ws * 1024);
        ws = (ws + 1) & (STAGES - 1);
        c_src += c_stride;
        --c_left;
    };

    // ---- the run's input -> buffer 0, items (channel block, pixel group) round the waves; then the ring's first copies
    {
        const int nCb = ka->block[0].nCbi, HW = ka->block[0].Hi * ka->block[0].Wi;
        const int ng = dr_groups(G, HW);
        for (int item = w; item < nCb * ng; item += kDrWaves) {
            const int grp = c_by_nCbi.div(item), cb = item - grp * nCb;
            const int m = grp * 16 + p;
            const int im = dr_fd(ka->by_HWi0).div(m), pix = m - im * HW;
            const bool real = im < G && img0 + im < N;
            const unsigned off = (unsigned)((((size_t)(img0 + (real ? im : 0)) * nCb + cb) * HW + (real ? pix : 0)) * 64 + q * 16);
            dma16(dr_uniform(ka->in), off, lds0 + (unsigned)(act0 + (cb * ng + grp) * 1024));
        }
    }
#pragma unroll 1
    for (int s = 0; s < STAGES - 1; ++s) issue();
    wait_vmcnt<STAGES - 1>();                           // this wave's input copies have landed
    __syncthreads();                                    // ... and everybody else's

    const char *ring = lds_c + ring_off;
    unsigned rs = 0;                                    // ring slot of the next step consumed
    for (int b = 0; b < n_blocks; ++b) {
        const int nCbi = ka->block[b].nCbi, nCbo = ka->block[b].nCbo;
        const int Hi = ka->block[b].Hi, Wi = ka->block[b].Wi, Wo = ka->block[b].Wo;
        const int HWi = Hi * Wi, HWo = ka->block[b].Ho * Wo;
        const int stride = ka->block[b].stride, pt = ka->block[b].pt, pl = ka->block[b].pl;
        const int dw_relu = ka->block[b].dw_relu, pw_relu = ka->block[b].pw_relu;
        const DrDiv by_HWo = dr_fd(ka->block[b].by_HWo), by_Wo = dr_fd(ka->block[b].by_Wo);
        const DrDiv by_nCbi = dr_fd(ka->block[b].by_nCbi), by_nCbo = dr_fd(ka->block[b].by_nCbo);
        const int ngi = dr_groups(G, HWi), ng = dr_groups(G, HWo);
        const bool last = b + 1 == n_blocks;
        const bool to_memory = last && ka->head == nullptr;

        // ---------------- depthwise stage: buffer 0 [nCbi][ngi] -> buffer 1 [nCbi][ng]
        for (int item = w; item < nCbi * ng; item += kDrWaves) {
            const int grp = by_nCbi.div(item), cb = item - grp * nCbi;
            wait_vmcnt<STAGES - 2>();
            issue();
            const floatx4 *taps = reinterpret_cast<const floatx4 *>(ring + rs * 1024) + q;
            rs = (rs + 1) & (STAGES - 1);
            floatx4 wt[9];
#pragma unroll
            for (int t = 0; t < 9; ++t) wt[t] = taps[t * 4];
            const int m = grp * 16 + p;
            const int im = by_HWo.div(m), pix = m - im * HWo;
            const bool real = im < G && img0 + im < N;
            const int oy = by_Wo.div(pix), ox = pix - oy * Wo;
            const int iy0 = oy * stride - pt, ix0 = ox * stride - pl;
            const floatx4 *src = reinterpret_cast<const floatx4 *>(lds_c + act0) + cb * ngi * 64 + q * 16;
            const int m_in = im * HWi + iy0 * Wi + ix0;         // slot of the window's first entry (may lie outside)
            floatx4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < 9; ++t) {
                const int iy = iy0 + t / 3, ix = ix0 + t % 3;
                const bool on = real && (unsigned)iy < (unsigned)Hi && (unsigned)ix < (unsigned)Wi;
                const int mm = m_in + (t / 3) * Wi + t % 3;
                const int at = on ? (mm >> 4) * 64 + (mm & 15) : 0;
                const floatx4 v = src[at];
                acc.x = fmaf(on ? v.x : 0.f, wt[t].x, acc.x); acc.y = fmaf(on ? v.y : 0.f, wt[t].y, acc.y);
                acc.z = fmaf(on ? v.z : 0.f, wt[t].z, acc.z); acc.w = fmaf(on ? v.w : 0.f, wt[t].w, acc.w);
            }
            if (dw_relu) {
                acc.x = acc.x > 0.f ? acc.x : 0.f; acc.y = acc.y > 0.f ? acc.y : 0.f;
                acc.z = acc.z > 0.f ? acc.z : 0.f; acc.w = acc.w > 0.f ? acc.w : 0.f;
            }
            reinterpret_cast<floatx4 *>(lds_c + act1)[(cb * ng + grp) * 64 + lane] = acc;
        }
        __syncthreads();                                // buffer 1 is complete

        // ---------------- pointwise stage: buffer 1 [nCbi][ng] -> buffer 0 [nCbo][ng] / memory
        const int parts = dr_parts(nCbo, ng), per_part = (ng + parts - 1) / parts;
        for (int item = w; item < nCbo * parts; item += kDrWaves) {
            const int part = by_nCbo.div(item), cob = item - part * nCbo;
            const int g0 = part * per_part, nk = min(per_part, ng - g0);
            const floatx4 *bsrc = reinterpret_cast<const floatx4 *>(lds_c + act1) + g0 * 64 + lane;
            floatx4 acc[4];
            if (nk == 1) {
                floatx4 a1[1];
                dr_reduce<1, STAGES>(a1, nCbi, ring + lane * 4, bsrc, ng * 64, rs, issue);
                acc[0] = a1[0];
            } else if (nk == 2) {
                floatx4 a2[2];
                dr_reduce<2, STAGES>(a2, nCbi, ring + lane * 4, bsrc, ng * 64, rs, issue);
                acc[0] = a2[0]; acc[1] = a2[1];
            } else if (nk == 3) {
                floatx4 a3[3];
                dr_reduce<3, STAGES>(a3, nCbi, ring + lane * 4, bsrc, ng * 64, rs, issue);
                acc[0] = a3[0]; acc[1] = a3[1]; acc[2] = a3[2];
            } else {
                dr_reduce<4, STAGES>(acc, nCbi, ring + lane * 4, bsrc, ng * 64, rs, issue);
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                if (k < nk) {
                    floatx4 v = acc[k];
                    if (pw_relu) {
                        v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
                        v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
                    }
                    if (to_memory) {
                        const int m = (g0 + k) * 16 + p;
                        const int im = by_HWo.div(m), pix = m - im * HWo;
                        if (im < G && img0 + im < N)
                            *reinterpret_cast<floatx4 *>(reinterpret_cast<char *>(ka->out) +
                                                         ((((size_t)(img0 + im) * nCbo + cob) * HWo + pix) * 64 + q * 16)) = v;
                    } else {
                        reinterpret_cast<floatx4 *>(lds_c + act0)[(cob * ng + g0 + k) * 64 + lane] = v;
                    }
                }
            }
        }
        if (!to_memory) __syncthreads();                // buffer 0 is complete (and buffer 1 free again)
    }

    // ---------------- the network's head on the last result (buffer 0): mean over the pixels, fully connected layer
    if (ka->head != nullptr) {
        const int nCb = ka->block[n_blocks - 1].nCbo, C = nCb * 16;
        const int HW = ka->block[n_blocks - 1].Ho * ka->block[n_blocks - 1].Wo, ng = dr_groups(G, HW);
        const int Co = ka->head_Co, Cob = ka->head_Cob;
        const float *act = reinterpret_cast<const float *>(lds_c + act0);
        float *red = reinterpret_cast<float *>(lds_c + act1);          // [wave][16 outputs]
        const float scale = 1.f / (float)HW;
        const int tid = threadIdx.x;
        for (int im = 0; im < G && img0 + im < N; ++im) {
            float part[16];
#pragma unroll
            for (int o = 0; o < 16; ++o) part[o] = 0.f;
            for (int c = tid; c < C; c += kDrThreads) {
                float sum = 0.f;
                for (int pix = 0; pix < HW; ++pix) {
                    const int m = im * HW + pix;
                    sum += act[(((c >> 4) * ng + (m >> 4)) * 64 + ((c & 15) >> 2) * 16 + (m & 15)) * 4 + (c & 3)];
                }
#pragma unroll
                for (int o = 0; o < 16; ++o)
                    if (o < Co) part[o] = fmaf(sum, ka->head[((size_t)(o / Cob) * C + c) * Cob + o % Cob], part[o]);
            }
#pragma unroll
            for (int o = 0; o < 16; ++o) {
                if (o < Co) {
                    float v = part[o];
#pragma unroll
                    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, 64);
                    if (lane == 0) red[w * 16 + o] = v;
                }
            }
            __syncthreads();
            if (tid < Co) {
                float v = 0.f;
#pragma unroll
                for (int k = 0; k < kDrWaves; ++k) v += red[k * 16 + tid];
                ka->out[(size_t)(img0 + im) * Co + tid] = v * scale;
            }
            __syncthreads();
        }
    }
    wait_vmcnt<0>();        // copies issued past the run's last step must land before the workgroup's LDS is released
}

template <int STAGES>
hipError_t launch_dr(const DrArgs &a, hipStream_t s)
{
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(dwpw_run<STAGES>),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (attr != hipSuccess) return attr;
    const unsigned wgs = (unsigned)((a.N + a.G - 1) / a.G);
    const size_t lds = (size_t)kDrWaves * STAGES * 1024 + 2 * (size_t)a.act_bytes;
    hipLaunchKernelGGL((dwpw_run<STAGES>), dim3(wgs), dim3(kDrThreads), lds, s, a);
    return hipGetLastError();
}
// bytes of one activation buffer for G images per workgroup: the largest tensor of the run
size_t dr_act_bytes(const DwpwRunBlock *b, int n, int G)
{
    size_t most = 0;
    for (int i = 0; i < n; ++i) {
        const size_t gi = (size_t)(G * b[i].Hi * b[i].Wi + 15) / 16, go = (size_t)(G * b[i].Ho * b[i].Wo + 15) / 16;
        most = std::max({most, (size_t)(b[i].Cin / 16) * gi, (size_t)(b[i].Cin / 16) * go, (size_t)(b[i].Cout / 16) * go});
    }
    return most * 1024;
}

constexpr size_t kDrRingBytes = (size_t)kDrWaves * 4 * 1024;       // the shallowest ring
constexpr size_t kDrLdsMax = 160 * 1024;

}  // namespace

bool dwpw_run_eligible(const DwpwRunBlock *b, int n)
{
    if (n < 2 || n > kDwpwChainMaxBlocks) return false;
    for (int i = 0; i < n; ++i) {
        if (b[i].Cin % 16 || b[i].Cout % 16 || b[i].Cin < 16 || b[i].Cout < 16) return false;
        if (b[i].Hi < 1 || b[i].Wi < 1 || b[i].Ho < 1 || b[i].Wo < 1 || b[i].stride < 1) return false;
        if ((long)b[i].Hi * b[i].Wi > kDwpwRunMaxPixels || (long)b[i].Ho * b[i].Wo > kDwpwRunMaxPixels) return false;
        // one workgroup per image must beat a launch per block: images of 8000 values (the audio CNN's 64 x 25 x 5) lose,
        // 35 -> 53 us for the network at batch 1 and 116 -> 190 at 1024; images of 4608 (32 x 12 x 12) gain
        if ((long)b[i].Cin * b[i].Hi * b[i].Wi > kDwpwRunMaxValues || (long)b[i].Cout * b[i].Ho * b[i].Wo > kDwpwRunMaxValues) return false;
        // a pointwise item holds accumulators for at most four pixel groups (one image per workgroup; with more images
        // per workgroup the launch keeps within 64 pixel slots)
        const int ng = (b[i].Ho * b[i].Wo + 15) / 16, nCbo = b[i].Cout / 16;
        const int parts = nCbo >= kDrWaves ? 1 : std::min(kDrWaves / nCbo, ng);
        if ((ng + parts - 1) / parts > 4) return false;
        if (i > 0 && (b[i].Cin != b[i - 1].Cout || b[i].Hi != b[i - 1].Ho || b[i].Wi != b[i - 1].Wo)) return false;
    }
    return kDrRingBytes + 2 * dr_act_bytes(b, n, 1) <= kDrLdsMax;
}

int dwpw_run_images(const DwpwRunBlock *blocks, int n_blocks, int N)
{
    // As many images as 64 pixel slots (and LDS) hold, fewer where one round of workgroups does with fewer. Small tiles waste matrix-instruction lanes (a 3 x 3 image fills 9 of 16) and stream the filters more often,
    // but these runs are bound by the chain of stages of one workgroup, not by arithmetic.
    int most_px = 1;
    for (int i = 0; i < n_blocks; ++i) most_px = std::max({most_px, blocks[i].Hi * blocks[i].Wi, blocks[i].Ho * blocks[i].Wo});
    int G = std::max(1, 64 / most_px);
    while (G > 1 && kDrRingBytes + 2 * dr_act_bytes(blocks, n_blocks, G) > kDrLdsMax) --G;
    // no more than one round of workgroups needs (640 images on 256 compute units: three per workgroup, 214 workgroups,
    // not two and 320)
    const int one_round = (N + device_cus() - 1) / device_cus();
    return std::max(1, std::min(G, one_round));
}

hipError_t launch_dwpw_run(const float *in, float *out, const DwpwRunBlock *blocks, int n_blocks, int N, const DwpwRunHead &head,
                           hipStream_t s)
{
    DrArgs a;
    a.in = in; a.out = out;
    a.head = head.filt; a.head_Co = head.Co; a.head_Cob = head.Cob;
    a.N = N; a.n_blocks = n_blocks;
    for (int i = 0; i < kDwpwChainMaxBlocks; ++i) {
        const DwpwRunBlock &b = blocks[i < n_blocks ? i : n_blocks - 1];
        DrBlock &d = a.block[i];
        d.dw = b.dw; d.pw = b.pw; d.dw_relu = b.dw_relu; d.pw_relu = b.pw_relu;
        d.nCbi = b.Cin / 16; d.nCbo = b.Cout / 16;
        d.Hi = b.Hi; d.Wi = b.Wi; d.Ho = b.Ho; d.Wo = b.Wo; d.stride = b.stride; d.pt = b.pt; d.pl = b.pl;
        d.by_HWo = make_fastdiv(b.Ho * b.Wo); d.by_Wo = make_fastdiv(b.Wo);
        d.by_nCbi = make_fastdiv(d.nCbi); d.by_nCbo = make_fastdiv(d.nCbo);
    }
    a.by_HWi0 = make_fastdiv(blocks[0].Hi * blocks[0].Wi);
    const int G = dwpw_run_images(blocks, n_blocks, N);
    a.G = G;
    a.act_bytes = (int)dr_act_bytes(blocks, n_blocks, G);
    // the filter ring as deep as LDS allows: a run streams all its filters through every workgroup, and what bounds it is
    // how many kilobytes a wave has in flight (4 stages: 80 us for the nine blocks of the depthwise-separable CNN)
    const int stages = kDrWaves * 16 * 1024 + 2 * (size_t)a.act_bytes <= kDrLdsMax ? 16
                     : (kDrWaves * 8 * 1024 + 2 * (size_t)a.act_bytes <= kDrLdsMax ? 8 : 4);
    return stages == 16 ? launch_dr<16>(a, s) : (stages == 8 ? launch_dr<8>(a, s) : launch_dr<4>(a, s));
}

}  // namespace small
