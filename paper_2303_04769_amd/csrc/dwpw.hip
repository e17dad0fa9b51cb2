// Depthwise 3x3 -> (ReLU) -> pointwise 1x1 -> (ReLU) in one kernel (gfx950), the "abstract fused layer"
// direction the paper names as future work: the depthwise result of a pixel tile never leaves the
// compute unit, so one launch and one HBM round trip of the intermediate tensor disappear.
//
// Both layers are instances of the abstract layer on the shared blocked layout (Cb = 16):
// depthwise = single-channel reduction (Table 1), pointwise = full-channel reduction with a 1x1 window.
//
// A workgroup (4 waves) owns one tile of 64 output pixels and one tile of up to 64 output channels, and
// walks over images with all per-lane state fixed (see conv16_img in conv_same.hip). Images of at most 32
// output pixels are taken several at a time (a tile is then a group of whole consecutive images), so that
// the 3 x 3 and 2 x 2 layers at the end of a network still fill their lanes.
//   1. depthwise phase, one step per 16-channel block: all input rows the tile's windows touch are staged
//      global -> LDS as whole rows (ring of `stages` steps, loads run stages - 1 steps ahead; for short
//      channel counts that is the whole tile at once); lane (pixel p, quad q) reads its nine taps as float4
//      (channels 4q .. 4q + 3) from precomputed addresses and multiplies by the filter taps held in LDS;
//   2. pointwise part of the same step: that (ReLU'd) float4 is exactly this lane's pixel operand of the
//      16x16x4 fp32 MFMAs (B[k = 4q + r][pixel p]), so it goes from registers straight into the matrix
//      instructions against the filter slabs of this channel block, which stay resident in LDS for the
//      whole kernel (loaded once per workgroup). After the last block: accumulators -> (ReLU) -> global.
// Taps outside the image are redirected to an all-zero LDS entry, as in the convolution kernels.
#include "small_internal.h"

#include <algorithm>
#include <type_traits>

namespace small {

namespace {

constexpr int kTM = 64;              // output pixels per tile
constexpr int kMaxStages = 8;

struct DwPwArgs {
    const float *in;
    const float *dwf;    // [C/16][3][3][16]
    const float *pwf;    // [Co/16][C/16][16][16]
    float *out;
    int N, H, W, HW;
    int Ho, Wo, HWo, stride;
    int nCb, nCob;       // channel blocks of the depthwise layer / of the pointwise output
    int pt, pl;
    int ipt;             // images per tile group (1 unless an output image has at most 32 pixels)
    int GHW;             // output pixels of a tile group: ipt * Ho * Wo
    int n_igroups;       // tile groups in the batch: ceil(N / ipt); the last one is shifted back to end at image N - 1
    int n_mtiles, n_cotiles, n_groups;     // tiles per tile group, channel tiles, workgroups along the batch
    int stages;          // ring depth
    int stage_bytes;     // staged entries of a step (64 B each, a whole number of 16-entry chunks) + the zero entry
    FastDiv dW, dH, dWo, dHWo, dMt, dCt;
    int relu_mid, relu_out;
};

// Staged input rows of the tile that starts at output pixel m0 of a tile group: rows are numbered through the
// images of the group (image * H + row); the tile needs rows [lo, hi]. Same arithmetic on host and device (the
// device divides by multiplication: an integer division is some thirty vector instructions, four of them here).
struct PlainDiv {
    int d;
    __host__ __device__ int div(int n) const { return n / d; }
};
template <typename Div>
__host__ __device__ inline void tile_rows(int m0, int TM, int GHW, int HWo, int Wo, int H, int stride, int pt, const Div &by_HWo,
                                          const Div &by_Wo, int &lo, int &hi)
{
    const int f0 = m0, f1 = (m0 + TM - 1 < GHW - 1) ? m0 + TM - 1 : GHW - 1;
    const int img0 = by_HWo.div(f0), oh0 = by_Wo.div(f0 - img0 * HWo);
    const int img1 = by_HWo.div(f1), oh1 = by_Wo.div(f1 - img1 * HWo);
    int r0 = oh0 * stride - pt, r1 = oh1 * stride - pt + 2;
    r0 = r0 < 0 ? 0 : (r0 > H - 1 ? H - 1 : r0);
    r1 = r1 < 0 ? 0 : (r1 > H - 1 ? H - 1 : r1);
    lo = img0 * H + r0;
    hi = img1 * H + r1;
}

// max(x, 0) in one instruction per value (the compiler's form quiets the operand first: two)
__device__ __forceinline__ float relu1(float x)
{
    float r;
    asm("v_max_f32 %0, 0, %1" : "=v"(r) : "v"(x));
    return r;
}
__device__ __forceinline__ floatx4 relu4(floatx4 v) { return floatx4{relu1(v.x), relu1(v.y), relu1(v.z), relu1(v.w)}; }

// LPS: load instructions per wave and step (a stage holds up to 64 * LPS entries). WN: 16-channel output blocks.
// OWN: narrow images, whose 16-pixel tiles touch at most 16 * LPS input pixels. Every wave (eight per workgroup) then
// stages the rows of its own 16 pixels into a ring of its own (kOwnStages steps) and nothing in the step loop couples
// the waves: no barrier, and a wait on a fixed number of outstanding loads. With shared stages the four waves of a
// workgroup, each on another SIMD and held up there by other workgroups' matrix instructions, meet at a barrier every
// step, and the step takes as long as the slowest of them. The halo rows of neighbouring tiles are fetched by both
// waves (from L2).
constexpr int kOwnStages = 3;
template <int WN, int LPS, bool OWN>
__global__ void __launch_bounds__(OWN ? 512 : 256) dwpw16_img(DwPwArgs a)
{
    constexpr int NW = OWN ? 8 : 4, NT = 64 * NW, TM = OWN ? 16 : kTM;
    static_assert((kMaxStages - 1) * LPS < 64, "too many loads in flight for vmcnt");
    static_assert(kOwnStages == 3, "the step loop is unrolled over the ring");

    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    char *lds_c = reinterpret_cast<char *>(lds);
    const int zero_rel = a.stage_bytes - 16;
    const int stages = OWN ? kOwnStages : a.stages;
    const int pwf_off = ((OWN ? NW : 1) * stages * a.stage_bytes + 255) & ~255;
    const int dwf_off = pwf_off + a.nCb * (WN * 1024);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 15, lq = lane >> 4;
    const int ring = OWN ? wave * stages * a.stage_bytes : 0;       // this wave's stages start here

    // workgroup (OWN: wave) -> (image group, pixel tile of the group, channel tile), channel tile fastest
    int co_tile, grp, m_tile;
    if (OWN) {
        const int wv = (int)xcd_contiguous(blockIdx.x, gridDim.x) * NW + wave;
        co_tile = (int)blockIdx.y;
        grp = a.dMt.div(wv);
        m_tile = wv - grp * a.n_mtiles;
        if (grp >= a.n_groups) { grp = a.n_igroups; m_tile = 0; }    // a wave without work: it only helps fetch the filters
    } else {
        const int wg = (int)xcd_contiguous(blockIdx.x, gridDim.x);
        const int t = a.dCt.div(wg);
        co_tile = wg - t * a.n_cotiles;
        grp = a.dMt.div(t);
        m_tile = t - grp * a.n_mtiles;
    }
    const int m0 = m_tile * TM;            // first pixel of the tile inside its tile group
    const int cob0 = co_tile * WN;
    const size_t planeA = (size_t)a.HW * 64;
    const size_t imgA = (size_t)a.nCb * planeA;
    const size_t imgO = (size_t)a.nCob * a.HWo * 64;
    int row_lo, row_hi;
    tile_rows(m0, TM, a.GHW, a.HWo, a.Wo, a.H, a.stride, a.pt, a.dHWo, a.dWo, row_lo, row_hi);

    // ---- load descriptors of a step (one 16-channel block of the tile's input rows), relative to the first
    // image of the tile group and to the channel block. Chunks past the tile's rows repeat its last row.
    unsigned d_voff[LPS];
    unsigned d_lds[LPS];
    const int n_chunks = (a.stage_bytes - 16) / 1024;
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int chunk = min(OWN ? j : j * NW + wave, n_chunks - 1);
        const int e = chunk * 16 + (lane >> 2);
        const int quad = (lane & 3) ^ ((e >> 1) & 3);
        const int er = a.dW.div(e);
        const int R = min(row_lo + er, row_hi), col = e - er * a.W;
        const int img = a.dH.div(R), row = R - img * a.H;
        d_voff[j] = (unsigned)(img * imgA) + (unsigned)(((row * a.W + col) * 16 + quad * 4) * 4);
        d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)(chunk * 1024));
    }

    // ---- this lane's pixel: tap addresses in a stage, mid-tile address, output offset
    const int px = OWN ? lp : wave * 16 + lp;
    const bool o_ok = m0 + px < a.GHW;
    unsigned p_addr[9];
    unsigned o_off;
    {
        const int f = min(m0 + px, a.GHW - 1);
        const int img = a.dHWo.div(f), pix = f - img * a.HWo;
        const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
        o_off = (unsigned)(img * imgO) + (unsigned)((pix * 16 + lq * 4) * 4);
#pragma unroll
        for (int y = 0; y < 3; ++y)
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const int ir = oh * a.stride + y - a.pt, ic = ow * a.stride + x - a.pl;
                const bool ok = (unsigned)ir < (unsigned)a.H && (unsigned)ic < (unsigned)a.W;
                const int e = (img * a.H + ir - row_lo) * a.W + ic;
                p_addr[y * 3 + x] = (unsigned)ring + (ok ? (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16) : (unsigned)zero_rel);
            }
    }
    const unsigned b_addr = (unsigned)(pwf_off + lane * 4);
    const unsigned w_addr = (unsigned)(dwf_off + lq * 16);

    // ---- issue side of the input pipeline: (tile group, channel block) of the next step to load
    const char *in_c = reinterpret_cast<const char *>(a.in);
    char *out_c = reinterpret_cast<char *>(a.out);
    // tile group q covers images first_image(q) .. + ipt - 1
    auto first_image = [&](int q) __attribute__((always_inline)) { return min(q * a.ipt, a.N - a.ipt); };
    int i_n = grp, i_cb = 0, i_slot = 0, ahead = 0;        // i_n, n: tile groups
    // (OWN: a step is issued in every turn of the loop, so that the number of loads in flight is a constant; past the
    // wave's last step it fetches the batch's last tile group again, into a slot nobody reads any more)
    auto issue_step = [&]() __attribute__((always_inline)) {
        const char *base = in_c + (size_t)first_image(OWN ? min(i_n, a.n_igroups - 1) : i_n) * imgA + (size_t)i_cb * planeA;
        const unsigned stage_lds = lds_base + (unsigned)(ring + i_slot * a.stage_bytes);
#pragma unroll
        for (int j = 0; j < LPS; ++j) dma16(base, d_voff[j], stage_lds + d_lds[j]);
        ++ahead;
        if (++i_slot == stages) i_slot = 0;
        if (++i_cb == a.nCb) { i_cb = 0; i_n += a.n_groups; }
    };
    // the input pipeline starts before the resident operands are fetched, so that both latencies overlap
    for (int s = 0; s < stages - 1; ++s)
        if (OWN || i_n < a.n_igroups) issue_step();

    // ---- resident operands: pointwise filter slabs of this channel tile and all depthwise taps
    {
        const int row = lane >> 2, ci = 4 * (row & 3) + (row >> 2);      // LDS row 4r + q holds input channel 4q + r
        const int nslab = a.nCb * WN;
        for (int sidx = wave; sidx < nslab; sidx += NW) {
            const int cb = sidx / WN, j = sidx - cb * WN;
            const int cob = min(cob0 + j, a.nCob - 1);
            const unsigned off = (unsigned)(((cob * a.nCb + cb) * 256 + ci * 16 + (lane & 3) * 4) * 4);
            dma16(a.pwf, off, lds_base + (unsigned)(pwf_off + sidx * 1024));
        }
        const int ndw = a.nCb * 9 * 4;                                   // float4s
        for (int e = tid; e < ndw; e += NT)
            *reinterpret_cast<floatx4 *>(lds_c + dwf_off + e * 16) = reinterpret_cast<const floatx4 *>(a.dwf)[e];
        if (OWN ? lane < stages : tid < stages)
            *reinterpret_cast<floatx4 *>(lds_c + ring + (OWN ? lane : tid) * a.stage_bytes + zero_rel) = floatx4{0.f, 0.f, 0.f, 0.f};
        wait_vmcnt<0>();                                                 // also the first input steps: they are older
        __syncthreads();
    }

    int cb = 0, slot = 0, n = grp;                         // channel block being reduced, its ring slot, its tile group
    floatx4 acc[WN];
#pragma unroll
    for (int j = 0; j < WN; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
    // One step: a channel block of the tile. stage_off: where the step's stage starts in the ring (OWN: a constant, so
    // that it becomes the immediate offset of the window reads: a vector instruction costs its full issue time here,
    // the matrix pipe does not hide it).
    auto step = [&](auto stage_off) __attribute__((always_inline)) {
        // pointwise filter fragments of this channel block: independent of the staged input, requested first
        float fb[WN][4];
        {
            const char *bs = lds_c + b_addr + cb * (WN * 1024);
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) fb[j][r] = *reinterpret_cast<const float *>(bs + j * 1024 + r * 256);
        }
        // the step to compute has landed once at most the loads of the steps issued after it are outstanding
        if (OWN) {
            issue_step();                                  // into the slot that was computed one step ago
            wait_vmcnt<(kOwnStages - 1) * LPS>();
        } else {
            switch (ahead - 1) {
                case 0: wait_vmcnt<0>(); break;
                case 1: wait_vmcnt<LPS>(); break;
                case 2: wait_vmcnt<2 * LPS>(); break;
                case 3: wait_vmcnt<3 * LPS>(); break;
                case 4: wait_vmcnt<4 * LPS>(); break;
                case 5: wait_vmcnt<5 * LPS>(); break;
                case 6: wait_vmcnt<6 * LPS>(); break;
                default: wait_vmcnt<7 * LPS>(); break;
            }
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            --ahead;
            if (i_n < a.n_igroups) issue_step();           // into the slot that was computed one step ago
        }
        floatx4 dw = floatx4{0.f, 0.f, 0.f, 0.f};
        {
            const char *stage = lds_c + stage_off;
            const char *wrow = lds_c + w_addr + cb * (9 * 64);
            // the window in two batches of reads (five taps, then four): left to itself the compiler reads a tap and its
            // filter value and waits for them before it reads the next, nine LDS latencies in a row per step (all nine at
            // once measure the same and take 32 more registers)
            floatx4 v[5], w[5];
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                v[k] = *reinterpret_cast<const floatx4 *>(stage + p_addr[k]);
                w[k] = *reinterpret_cast<const floatx4 *>(wrow + k * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 5; ++k) {
                dw.x = fmaf(v[k].x, w[k].x, dw.x); dw.y = fmaf(v[k].y, w[k].y, dw.y);
                dw.z = fmaf(v[k].z, w[k].z, dw.z); dw.w = fmaf(v[k].w, w[k].w, dw.w);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                v[k] = *reinterpret_cast<const floatx4 *>(stage + p_addr[5 + k]);
                w[k] = *reinterpret_cast<const floatx4 *>(wrow + (5 + k) * 64);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                dw.x = fmaf(v[k].x, w[k].x, dw.x); dw.y = fmaf(v[k].y, w[k].y, dw.y);
                dw.z = fmaf(v[k].z, w[k].z, dw.z); dw.w = fmaf(v[k].w, w[k].w, dw.w);
            }
            if (a.relu_mid) dw = relu4(dw);
        }
        // (the accumulators named as tied operands: through the builtin the compiler renames them from step to step and
        // copies all sixteen registers twice per step to undo it; a tile's first matrix instructions start from zero
        // instead of sixteen cleared registers per tile)
        {
            const float d0 = dw.x, d1 = dw.y, d2 = dw.z, d3 = dw.w;
            if (cb == 0) {
#pragma unroll
                for (int j = 0; j < WN; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, 0" : "=&v"(acc[j]) : "v"(fb[j][0]), "v"(d0));
            } else {
#pragma unroll
                for (int j = 0; j < WN; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(fb[j][0]), "v"(d0));
            }
#pragma unroll
            for (int j = 0; j < WN; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(fb[j][1]), "v"(d1));
#pragma unroll
            for (int j = 0; j < WN; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(fb[j][2]), "v"(d2));
#pragma unroll
            for (int j = 0; j < WN; ++j) asm volatile("v_mfma_f32_16x16x4_f32 %0, %1, %2, %0" : "+v"(acc[j]) : "v"(fb[j][3]), "v"(d3));
        }
        if (++cb < a.nCb) return;
        cb = 0;

        // ---- STORE phase of this tile
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cob = cob0 + j;
            if (cob < a.nCob && o_ok)
                *reinterpret_cast<floatx4 *>(out_c + (size_t)first_image(n) * imgO + (size_t)cob * a.HWo * 64 + o_off) =
                    a.relu_out ? relu4(acc[j]) : acc[j];
        }
        n += a.n_groups;
    };
    if constexpr (OWN) {
        constexpr int SB = LPS * 1024 + 16;                // bytes of a stage, the host's figure
        if (n < a.n_igroups)
            for (;;) {
                step(std::integral_constant<int, 0>{});
                if (n >= a.n_igroups) break;
                step(std::integral_constant<int, SB>{});
                if (n >= a.n_igroups) break;
                step(std::integral_constant<int, 2 * SB>{});
                if (n >= a.n_igroups) break;
            }
    } else {
        while (n < a.n_igroups) {
            step(slot * a.stage_bytes);
            if (++slot == stages) slot = 0;
        }
    }
    if (OWN) wait_vmcnt<0>();          // (the extra steps still write to this workgroup's LDS)
}

// Host-side shape of a launch: images per tile, staged entries per step, ring depth, LDS bytes.
struct DwPwPlan {
    int ipt, GHW, n_mtiles, chunks, stage_bytes, stages, lps, wn;
    size_t lds;
    bool ok;
    bool own;       // every wave stages the rows of its own 16 pixels (n_mtiles then counts 16-pixel tiles)
};

DwPwPlan make_plan(const LayerGeom &g, int Co)
{
    DwPwPlan p = {};
    const int HWo = g.Ho * g.Wo, nCb = g.Ci / 16, nCob = Co / 16;
    p.ipt = HWo <= 32 ? std::max(1, std::min(g.N, kTM / HWo)) : 1;
    p.GHW = p.ipt * HWo;
    p.n_mtiles = (p.GHW + kTM - 1) / kTM;
    // output channel blocks per workgroup: up to 4 (the depthwise part is redone by every channel tile), fewer
    // when that leaves compute units without a workgroup
    int wn = std::min(4, nCob);
    const long tiles = (long)p.n_mtiles * ((g.N + p.ipt - 1) / p.ipt);
    while (wn > 1 && tiles * ((nCob + wn - 1) / wn) < device_cus()) wn = (wn + 1) / 2;
    p.wn = wn;
    int ent = 0;
    for (int m = 0; m < p.n_mtiles; ++m) {
        int lo, hi;
        tile_rows(m * kTM, kTM, p.GHW, HWo, g.Wo, g.H, g.stride, g.pt, PlainDiv{HWo}, PlainDiv{g.Wo}, lo, hi);
        ent = std::max(ent, (hi - lo + 1) * g.W);
    }
    p.chunks = (ent + 15) / 16;
    p.stage_bytes = p.chunks * 1024 + 16;
    p.lps = (p.chunks + 3) / 4;
    p.lps = p.lps <= 2 ? 2 : p.lps <= 4 ? 4 : p.lps <= 6 ? 6 : 8;
    const size_t fixed = (size_t)nCb * (wn * 1024 + 9 * 64);
    // ring: as deep as 8 steps and never more loads in flight than the 6-bit counter can track. With work for
    // four workgroups per compute unit, latencies are hidden by occupancy: the workgroup stays within 40 KiB of
    // LDS if three stages fit in that; otherwise by depth: up to 48 KiB of ring.
    const size_t room = kDwPwMaxLds > fixed + 256 ? kDwPwMaxLds - fixed - 256 : 0;
    size_t budget = std::min<size_t>(48 * 1024, room);
    if (tiles * ((nCob + wn - 1) / wn) >= 4 * device_cus() && fixed + 256 + 3 * (size_t)p.stage_bytes <= 40 * 1024)
        budget = 40 * 1024 - fixed - 256;
    p.stages = (int)std::min<size_t>({(size_t)kMaxStages, budget / (size_t)p.stage_bytes, (size_t)(63 / p.lps + 1)});
    p.lds = (size_t)((p.stages * p.stage_bytes + 255) & ~255) + fixed;
    p.ok = p.chunks <= 32 && p.stages >= 2 && p.lds <= kDwPwMaxLds;
    // narrow images: a ring per wave, when two workgroups of eight waves still fit a compute unit
    if (p.ok) {
        const int n16 = (p.GHW + 15) / 16;
        int ent16 = 0;
        for (int m = 0; m < n16; ++m) {
            int lo, hi;
            tile_rows(m * 16, 16, p.GHW, HWo, g.Wo, g.H, g.stride, g.pt, PlainDiv{HWo}, PlainDiv{g.Wo}, lo, hi);
            ent16 = std::max(ent16, (hi - lo + 1) * g.W);
        }
        const int stage16 = 2 * 1024 + 16;
        const size_t lds16 = (size_t)((8 * kOwnStages * stage16 + 255) & ~255) + fixed;
        // (eight waves to a workgroup: with fewer than a workgroup per compute unit the four-wave kernel covers more of them)
        const long waves16 = (long)n16 * ((g.N + p.ipt - 1) / p.ipt) * ((nCob + wn - 1) / wn);
        if (ent16 <= 32 && 2 * lds16 <= 160 * 1024 && waves16 >= 8L * device_cus()) {
            p.own = true;
            p.n_mtiles = n16;
            p.chunks = (ent16 + 15) / 16;
            p.stage_bytes = stage16;
            p.lps = 2;
            p.stages = kOwnStages;
            p.lds = lds16;
        }
    }
    return p;
}

template <int WN, int LPS, bool OWN = false>
hipError_t launch_cfg(DwPwArgs a, const DwPwPlan &p, hipStream_t s)
{
    auto kern = dwpw16_img<WN, LPS, OWN>;
    static size_t lds_allowed = 64 * 1024;
    if (p.lds > lds_allowed) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)kDwPwMaxLds);
        if (e != hipSuccess) return e;
        lds_allowed = kDwPwMaxLds;
    }
    a.ipt = p.ipt;
    a.GHW = p.GHW;
    a.n_igroups = (a.N + a.ipt - 1) / a.ipt;
    a.n_mtiles = p.n_mtiles;
    a.n_cotiles = (a.nCob + WN - 1) / WN;
    a.stages = p.stages;
    a.stage_bytes = p.stage_bytes;
    // tile groups per workgroup: enough workgroups to fill the chip (as many as LDS lets be resident, at most 4
    // per compute unit), the rest of the batch is walked by each workgroup with its set-up paid once
    // (with a ring per wave, positions are taken by waves, eight to a workgroup, two workgroups per compute unit)
    const long positions = (long)a.n_mtiles * a.n_cotiles;
    const long resident = OWN ? 256 * 8 * std::max<long>(1, std::min<long>(2, (long)(160 * 1024 / p.lds)))
                              : 256 * std::max<long>(1, std::min<long>(4, (long)(160 * 1024 / p.lds)));
    const long per_wg = std::max<long>(1, std::min<long>(a.n_igroups, (positions * a.n_igroups + resident - 1) / resident));
    a.n_groups = (int)((a.n_igroups + per_wg - 1) / per_wg);
    a.dW = make_fastdiv(a.W);
    a.dH = make_fastdiv(a.H);
    a.dWo = make_fastdiv(a.Wo);
    a.dHWo = make_fastdiv(a.HWo);
    a.dMt = make_fastdiv(a.n_mtiles);
    a.dCt = make_fastdiv(a.n_cotiles);
    if (OWN) {
        const dim3 grid((unsigned)(((long)a.n_mtiles * a.n_groups + 7) / 8), (unsigned)a.n_cotiles);
        hipLaunchKernelGGL(kern, grid, dim3(512), p.lds, s, a);
        return hipGetLastError();
    }
    const unsigned grid = (unsigned)(positions * a.n_groups);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(256), p.lds, s, a);
    return hipGetLastError();
}

template <int WN>
hipError_t launch_wn(const DwPwArgs &a, const DwPwPlan &p, hipStream_t s)
{
    if (p.own) return launch_cfg<WN, 2, true>(a, p, s);
    switch (p.lps) {
        case 2: return launch_cfg<WN, 2>(a, p, s);
        case 4: return launch_cfg<WN, 4>(a, p, s);
        case 6: return launch_cfg<WN, 6>(a, p, s);
        default: return launch_cfg<WN, 8>(a, p, s);
    }
}

// Eight input channels in one 8-channel block -> sixteen output channels: too little reduction for the matrix cores
// (K = 8), so the block runs on the vector units: a lane owns one output pixel, gathers its window (two float4 per
// tap, taps outside the image skipped), forms the eight depthwise sums, applies the ReLU and multiplies them with the
// 8 x 16 pointwise filter; both filters are broadcast from LDS. in [N][1][H][W][8], dw [1][3][3][8], pw
// [1][1][1][1][8][16], out [N][1][Ho][Wo][16].
struct DwPw8Args {
    const float *in, *dwf, *pwf;
    float *out;
    int H, W, Ho, Wo, stride, pt, pl;
    int total;            // output pixels over all images
    int relu_mid, relu_out;
    FastDiv by_Wo, by_Ho;
};

// What a lane does with its window (eighteen float4: two per tap) and the filters in LDS
__device__ __forceinline__ void dwpw8_finish(const floatx4 (&v)[18], const float (&on)[9], const floatx4 *w_dw, const floatx4 *w_pw,
                                             floatx4 *o, int relu_mid, int relu_out)
{
    floatx4 lo = {0.f, 0.f, 0.f, 0.f}, hi = {0.f, 0.f, 0.f, 0.f};       // depthwise sums of channels 0..3, 4..7
    // filter values in batches of reads (left to itself the compiler reads two, waits, uses them, reads the next two:
    // 25 LDS latencies in a row per pixel)
#pragma unroll
    for (int t0 = 0; t0 < 9; t0 += 3) {
        floatx4 f[6];
#pragma unroll
        for (int k = 0; k < 6; ++k) f[k] = w_dw[2 * t0 + k];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int t = 0; t < 3; ++t) {
            lo += v[2 * (t0 + t)] * (f[2 * t] * on[t0 + t]);
            hi += v[2 * (t0 + t) + 1] * (f[2 * t + 1] * on[t0 + t]);
        }
        __builtin_amdgcn_sched_barrier(0);
    }
    if (relu_mid) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            lo[c] = lo[c] > 0.f ? lo[c] : 0.f;
            hi[c] = hi[c] > 0.f ? hi[c] : 0.f;
        }
    }
    floatx4 acc[4] = {{0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}, {0.f, 0.f, 0.f, 0.f}};
#pragma unroll
    for (int c0 = 0; c0 < 8; c0 += 2) {
        floatx4 f[8];
#pragma unroll
        for (int k = 0; k < 8; ++k) f[k] = w_pw[c0 * 4 + k];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int c = 0; c < 2; ++c) {
            const int ci = c0 + c;
            const float x = ci < 4 ? lo[ci] : hi[ci - 4];
#pragma unroll
            for (int k = 0; k < 4; ++k) acc[k] += f[c * 4 + k] * x;
        }
        __builtin_amdgcn_sched_barrier(0);
    }
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        floatx4 y = acc[k];
        if (relu_out) {
            y.x = y.x > 0.f ? y.x : 0.f; y.y = y.y > 0.f ? y.y : 0.f;
            y.z = y.z > 0.f ? y.z : 0.f; y.w = y.w > 0.f ? y.w : 0.f;
        }
        __builtin_nontemporal_store(y, o + k);
    }
}

// A lane per output pixel, the window gathered from memory: all eighteen loads are issued unconditionally (a tap
// outside the image reads a valid pixel and is dropped by a zero factor: loads under a divergent branch would be
// waited for one by one).
__global__ void __launch_bounds__(256) dwpw8_16(DwPw8Args a)
{
    __shared__ floatx4 w_dw[18], w_pw[32];
    if (threadIdx.x < 18) w_dw[threadIdx.x] = reinterpret_cast<const floatx4 *>(a.dwf)[threadIdx.x];
    else if (threadIdx.x >= 64 && threadIdx.x < 96) w_pw[threadIdx.x - 64] = reinterpret_cast<const floatx4 *>(a.pwf)[threadIdx.x - 64];
    __syncthreads();
    const int m = (int)blockIdx.x * 256 + (int)threadIdx.x;
    if (m >= a.total) return;
    const int t = a.by_Wo.div(m), ow = m - t * a.Wo;
    const int n = a.by_Ho.div(t), oh = t - n * a.Ho;
    const floatx4 *img = reinterpret_cast<const floatx4 *>(a.in) + (size_t)n * a.H * a.W * 2;
    floatx4 v[18];
    float on[9];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const int ih = oh * a.stride + ky - a.pt;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int iw = ow * a.stride + kx - a.pl;
            const bool inside = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            const floatx4 *px = img + (inside ? (ih * a.W + iw) * 2 : 0);
            v[(ky * 3 + kx) * 2] = px[0];
            v[(ky * 3 + kx) * 2 + 1] = px[1];
            on[ky * 3 + kx] = inside ? 1.f : 0.f;
        }
    }
    dwpw8_finish(v, on, w_dw, w_pw, reinterpret_cast<floatx4 *>(a.out) + (size_t)m * 4, a.relu_mid, a.relu_out);
}

// The same with the input rows of a tile staged in LDS: a workgroup owns TR whole output rows of one image
// (TR * Wo <= 256 lanes); the input rows they touch are one contiguous piece of memory, copied with consecutive lanes
// on consecutive 16 bytes (a lane-per-pixel gather from memory touches every cache line of the piece in every load
// instruction: 15 us instead of 7 on the first block of the depthwise-separable CNN at batch 256).
struct DwPw8Tile { int TR, tiles_per_image, rows_max; };

__global__ void __launch_bounds__(256) dwpw8_16_rows(DwPw8Args a, DwPw8Tile tl)
{
    extern __shared__ floatx4 lds[];
    floatx4 *w_dw = lds, *w_pw = lds + 18, *rows = lds + 50;
    const int tid = (int)threadIdx.x;
    if (tid < 18) w_dw[tid] = reinterpret_cast<const floatx4 *>(a.dwf)[tid];
    else if (tid >= 64 && tid < 96) w_pw[tid - 64] = reinterpret_cast<const floatx4 *>(a.pwf)[tid - 64];
    const int n = (int)blockIdx.x / tl.tiles_per_image, tile = (int)blockIdx.x - n * tl.tiles_per_image;
    const int oh0 = tile * tl.TR, n_out_rows = min(tl.TR, a.Ho - oh0);
    // input rows ih0 .. ih1 - 1 (inside the image) serve the tile
    const int ih0 = max(oh0 * a.stride - a.pt, 0), ih1 = min((oh0 + n_out_rows - 1) * a.stride - a.pt + 3, a.H);
    const floatx4 *img = reinterpret_cast<const floatx4 *>(a.in) + (size_t)n * a.H * a.W * 2;
    const int n_vec = (ih1 - ih0) * a.W * 2;
    for (int c = tid; c < n_vec; c += 256) rows[c] = __builtin_nontemporal_load(img + ih0 * a.W * 2 + c);
    __syncthreads();
    const int r = a.by_Wo.div(tid), ow = tid - r * a.Wo;
    if (r >= n_out_rows) return;
    const int oh = oh0 + r;
    floatx4 v[18];
    float on[9];
#pragma unroll
    for (int ky = 0; ky < 3; ++ky) {
        const int ih = oh * a.stride + ky - a.pt;
#pragma unroll
        for (int kx = 0; kx < 3; ++kx) {
            const int iw = ow * a.stride + kx - a.pl;
            const bool inside = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            const floatx4 *px = rows + (inside ? ((ih - ih0) * a.W + iw) * 2 : 0);
            v[(ky * 3 + kx) * 2] = px[0];
            v[(ky * 3 + kx) * 2 + 1] = px[1];
            on[ky * 3 + kx] = inside ? 1.f : 0.f;
        }
    }
    const size_t m = ((size_t)n * a.Ho + oh) * a.Wo + ow;
    dwpw8_finish(v, on, w_dw, w_pw, reinterpret_cast<floatx4 *>(a.out) + m * 4, a.relu_mid, a.relu_out);
}

}  // namespace

bool dwpw_eligible(int C, int Co, int Cb, int Cob_pw, int kh, int kw, int stride, int pw_kh, int pw_kw, int pw_stride)
{
    if (kh != 3 || kw != 3 || stride < 1 || pw_kh != 1 || pw_kw != 1 || pw_stride != 1) return false;
    if (C == 8 && Cb == 8 && Co == 16 && Cob_pw == 16) return true;        // the vector-unit kernel
    if (Cb != 16 || Cob_pw != 16 || C % 16 || Co % 16) return false;
    // resident filters + the smallest ring must fit
    const size_t fixed = (size_t)(C / 16) * (std::min(4, Co / 16) * 1024 + 9 * 64);
    return fixed + 2 * (4 * 1024 + 16) + 256 <= kDwPwMaxLds;
}

bool dwpw_geom_ok(const LayerGeom &g, int Co)
{
    if (g.Cib == 8) return (size_t)g.N * g.Ho * g.Wo < ((size_t)1 << 31) && (size_t)g.N * g.H * g.W * 8 < ((size_t)1 << 31);
    // per-lane 32-bit byte offsets span the images of a tile group
    const bool small_enough = (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30) &&
                              (size_t)64 * g.Ci * g.H * g.W * 4 < ((size_t)1 << 31) &&
                              (size_t)64 * Co * g.Ho * g.Wo * 4 < ((size_t)1 << 31);
    return small_enough && g.pt < 3 && g.pl < 3 && make_plan(g, Co).ok;
}

hipError_t launch_dwpw(const float *in, const float *dw_filt, const float *pw_filt, float *out, const LayerGeom &g, int Co,
                       int relu_mid, int relu_out, hipStream_t s)
{
    if (g.Cib == 8) {
        DwPw8Args b;
        b.in = in; b.dwf = dw_filt; b.pwf = pw_filt; b.out = out;
        b.H = g.H; b.W = g.W; b.Ho = g.Ho; b.Wo = g.Wo; b.stride = g.stride; b.pt = g.pt; b.pl = g.pl;
        b.total = g.N * g.Ho * g.Wo;
        b.relu_mid = relu_mid; b.relu_out = relu_out;
        b.by_Wo = make_fastdiv(g.Wo); b.by_Ho = make_fastdiv(g.Ho);
        // whole output rows per workgroup with their input rows in LDS, where rows are short enough
        if (g.Wo <= 128) {
            DwPw8Tile tl;
            tl.TR = std::min(g.Ho, 256 / g.Wo);
            tl.rows_max = std::min(g.H, (tl.TR - 1) * g.stride + 3);
            const size_t lds = (size_t)(50 + tl.rows_max * g.W * 2) * 16;
            if (lds <= 64 * 1024) {
                tl.tiles_per_image = (g.Ho + tl.TR - 1) / tl.TR;
                hipLaunchKernelGGL(dwpw8_16_rows, dim3((unsigned)(g.N * tl.tiles_per_image)), dim3(256), lds, s, b, tl);
                return hipGetLastError();
            }
        }
        hipLaunchKernelGGL(dwpw8_16, dim3((unsigned)((b.total + 255) / 256)), dim3(256), 0, s, b);
        return hipGetLastError();
    }
    DwPwArgs a = {};
    a.in = in; a.dwf = dw_filt; a.pwf = pw_filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.HW = g.H * g.W;
    a.Ho = g.Ho; a.Wo = g.Wo; a.HWo = g.Ho * g.Wo; a.stride = g.stride;
    a.nCb = g.Ci / 16; a.nCob = Co / 16;
    a.pt = g.pt; a.pl = g.pl;
    a.relu_mid = relu_mid; a.relu_out = relu_out;
    const DwPwPlan p = make_plan(g, Co);
    if (!p.ok) return hipErrorInvalidValue;
    switch (p.wn) {
        case 1: return launch_wn<1>(a, p, s);
        case 2: return launch_wn<2>(a, p, s);
        case 3: return launch_wn<3>(a, p, s);
        default: return launch_wn<4>(a, p, s);
    }
}

}  // namespace small
