// Matrix-core convolution for "same" geometry: stride 1 and output size == input size
// (pad.t + pad.b = kh - 1, pad.l + pad.r = kw - 1), Cib = Cob = 16, kw in {1, 3}. This is the
// shape of every 3x3 / 1x1 layer of the roofline sweep and of most network layers.
//
// Geometry. With stride 1 and equal sizes, the flattened pixel index m = (n, oh, ow) of an output
// and the flattened index of the input pixel under tap (y, x) differ by the constant
// (y - pad.t) * W + (x - pad.l). A tile of TM consecutive output pixels therefore needs, for one
// filter row y, one run of TM + kw - 1 consecutive input pixels, and tap x is that run shifted by
// x entries. One reduction step = (Ci block(s), filter row y): the run is staged once and feeds
// all kw taps, so the input crosses the L2 -> LDS path kh times instead of kh * kw times. For 1x1
// filters a step stages NA consecutive Ci blocks ("planes") to get comparable work per step.
// Taps that fall outside the image would read a neighbouring row's (or image's) pixel from the
// run; each lane redirects those reads to an all-zero LDS entry (Algorithm 1's "edge cases are
// handled around the kernel"): one v_cndmask on an LDS address per 16x16 tile and tap. Every
// entry that is read without redirection is a pixel of the right image row, so entries whose
// source would be outside the tensor may hold anything.
//
// Data movement. Both operands go from global memory straight into LDS with the gfx950
// global_load_lds_dwordx4 instruction (no staging registers, no ds_write): one wave instruction
// moves 64 x 16 B and the LDS destination is linear in the lane id, so
//   - an input chunk of 16 pixels x 64 B lands as [entry][4 quads]; the lane chooses WHICH quad of
//     its pixel it fetches so that quad q of entry e sits at position q ^ ((e >> 1) & 3): the
//     ds_read_b128 of 8 consecutive entries then hits 8 distinct 16-byte bank groups;
//   - a 16 x 16 filter slab lands as 16 rows of 64 B; the lane chooses WHICH input-channel row it
//     fetches so that LDS row 4r + q holds channel 4q + r: MFMA number r of a slab then reads
//     LDS words 64 r + lane, conflict-free, and no transposition is ever materialised.
// LDS is a ring of STAGES steps; loads run STAGES - 1 steps ahead of the matrix instructions and
// are tracked by hand with s_waitcnt vmcnt(n) (they are issued from inline assembly so that the
// compiler does not serialise them against every LDS read). One s_barrier per step.
//
// MFMA operand roles, the reduction-index permutation and the output mapping are those of the
// gather kernel in conv.hip: v_mfma_f32_16x16x4_f32 with A = filter (row = output channel),
// B = input (column = pixel); lane l ends up with 4 adjacent output channels of pixel l % 16.
#include "small_internal.h"

namespace small {

namespace {

struct SameArgs {
    const float *in;
    const float *filt;
    float *out;
    const float *res;
    int N, H, W, HW;
    int nCib, nCob;
    int kh, pt, pl;
    int M;          // N * H * W
    int n_mtiles, n_cotiles;
    FastDiv dHW, dW, dMt, dCt;   // divisions by H*W, W, n_mtiles, n_cotiles
    int co_fast;    // workgroup order: channel tile fastest (input tile shared in L2) or pixel tile fastest (filter shared)
    int epilogue;
};

__device__ __forceinline__ floatx4 epi4(floatx4 v, int epi, const float *res)
{
    if (epi & EPI_ADD) v += *reinterpret_cast<const floatx4 *>(res);
    if (epi & EPI_RELU) {
        v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
        v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
    }
    return v;
}

// 64 lanes x 16 B: global (base + per-lane byte offset) -> LDS (wave-uniform byte address + 16 * lane).
__device__ __forceinline__ void dma16(const void *gbase, unsigned lane_off_bytes, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off_bytes), "s"(gbase), "s"(__builtin_amdgcn_readfirstlane(lds_addr_uniform))
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

constexpr int gcd_(int a, int b) { return b == 0 ? a : gcd_(b, a % b); }

// KS: square filter size (1 or 3). NA: Ci blocks staged per reduction step (1 for 3x3).
template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int STAGES>
struct SameCfg {
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int NT = 64 * NW;
    static constexpr int TM = WAVES_M * WM * 16;
    static constexpr int TN = WAVES_N * WN * 16;
    static constexpr int NSUB = TN / 16;
    static constexpr int ENT = TM + KS - 1;                  // staged input pixels per plane
    static constexpr int ENTP = (ENT + 15) / 16 * 16;        // rounded up to whole wave instructions
    static constexpr int NS = NA * KS;                       // filter slabs per step
    static constexpr int A_BYTES = NA * ENTP * 64;
    static constexpr int B_BYTES = NS * NSUB * 1024;
    static constexpr int ZERO_REL = A_BYTES + B_BYTES;       // one all-zero float4 at the end of every stage
    static constexpr int STAGE_BYTES = ZERO_REL + 16;
    static constexpr int NAI = NA * ENTP / 16, NBI = NS * NSUB;   // wave instructions per step
    static constexpr int LPS = (NAI + NBI + NW - 1) / NW;         // ... per wave
    static constexpr int UNROLL = STAGES * KS / gcd_(STAGES, KS); // steps after which (ring slot, filter row) repeat
    static constexpr size_t LDS_BYTES = (size_t)STAGES * STAGE_BYTES;
    static_assert((STAGES - 2) * LPS < 64, "too many loads in flight for vmcnt");
    static_assert(KS == 1 || NA == 1, "several planes per step only for 1x1 filters");
};

template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int STAGES>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) conv16_same(SameArgs a)
{
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, STAGES>;
    constexpr int NW = C::NW, TM = C::TM, NSUB = C::NSUB, ENT = C::ENT, ENTP = C::ENTP, LPS = C::LPS, NS = C::NS;

    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    const char *lds_c = reinterpret_cast<const char *>(lds);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const unsigned wg = xcd_contiguous(blockIdx.x, gridDim.x);
    int co_tile, m_tile;
    if (a.co_fast) { m_tile = a.dCt.div((int)wg); co_tile = (int)wg - m_tile * a.n_cotiles; }
    else { co_tile = a.dMt.div((int)wg); m_tile = (int)wg - co_tile * a.n_mtiles; }
    const int m0 = m_tile * TM;
    const int cob0 = co_tile * NSUB;
    const int lp = lane & 15, lq = lane >> 4;

    // Everything that depends on the lane is computed here, once: inside the reduction loop only
    // scalar instructions touch addresses (vector ALU instructions do not overlap with MFMA on
    // this hardware, each one in the loop costs matrix-pipe time).
    //
    // ---- load descriptors: slot j of this wave is wave instruction k = j * NW + wave of a step
    // (k < NAI: input chunk, else filter slab; k beyond the last one repeats the last one).
    // d_voff[j][y]: per-lane byte offset from the step's scalar base for filter row y. Input rows are
    // clamped into the image instead of being skipped: an entry whose true source is outside the
    // image is never read unredirected, so it may hold any in-bounds data.
    unsigned d_voff[LPS][KS];
    unsigned d_lds[LPS];      // wave-uniform LDS byte offset inside a stage
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int k = min(j * NW + wave, C::NAI + C::NBI - 1);
        if (k < C::NAI) {
            const int dc = k / (ENTP / 16), chunk = k - dc * (ENTP / 16);
            const int e = chunk * 16 + (lane >> 2);
            const int quad = (lane & 3) ^ ((e >> 1) & 3);
            const int fb = m0 + e - a.pl;
            const bool ok = e < ENT && fb >= 0 && fb < a.M;
            const int fbc = ok ? fb : 0;
            const int n = a.dHW.div(fbc), pix = fbc - n * a.HW;
            const int hb = a.dW.div(pix), wb = pix - hb * a.W;
#pragma unroll
            for (int y = 0; y < KS; ++y) {
                const int row = min(max(hb + y - a.pt, 0), a.H - 1);
                d_voff[j][y] = (unsigned)((((n * a.nCib + dc) * a.H + row) * a.W + wb) * 16 + quad * 4) * 4u;
            }
            d_lds[j] = (unsigned)((dc * ENTP + chunk * 16) * 64);
        } else {
            const int kb = k - C::NAI;
            const int slab = kb / NSUB, sub = kb - slab * NSUB;
            const int dc = slab / KS, x = slab - dc * KS;
            const int row = lane >> 2, ci = 4 * (row & 3) + (row >> 2);
            const int cob = min(cob0 + sub, a.nCob - 1);
            const unsigned off = (unsigned)((((cob * a.nCib + dc) * KS) * KS + x) * 256 + ci * 16 + (lane & 3) * 4) * 4u;
#pragma unroll
            for (int y = 0; y < KS; ++y) d_voff[j][y] = off;
            d_lds[j] = (unsigned)(C::A_BYTES + (slab * NSUB + sub) * 1024);
        }
    }
    // scalar bases of a step: input + (first Ci block) planes, filter + (first Ci block, row y) slabs
    auto issue_one = [&](int j, int y, const char *baseA, const char *baseB, unsigned stage_lds) {
        const bool isA = min(j * NW + wave, C::NAI + C::NBI - 1) < C::NAI;     // wave-uniform
        dma16(isA ? baseA : baseB, d_voff[j][y], stage_lds + d_lds[j]);
    };

    if (tid < STAGES) lds[(tid * C::STAGE_BYTES + C::ZERO_REL) / 16] = floatx4{0.f, 0.f, 0.f, 0.f};

    // ---- per-lane fragment addresses relative to a stage, one per (pixel tile, filter row, tap):
    // the real entry, or the stage's zero entry when the tap is outside the image.
    unsigned p_addr[WM][KS][KS];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int px = (wave_m * WM + i) * 16 + lp;
        const int m = min(m0 + px, a.M - 1);
        const int n = a.dHW.div(m), pix = m - n * a.HW;
        const int oh = a.dW.div(pix), ow = pix - oh * a.W;
#pragma unroll
        for (int y = 0; y < KS; ++y)
#pragma unroll
            for (int x = 0; x < KS; ++x) {
                const int e = px + x;
                const bool ok = (unsigned)(oh + y - a.pt) < (unsigned)a.H && (unsigned)(ow + x - a.pl) < (unsigned)a.W;
                p_addr[i][y][x] = (ok || KS == 1) ? (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16) : (unsigned)C::ZERO_REL;
            }
    }
    const unsigned b_addr = (unsigned)(C::A_BYTES + wave_n * WN * 1024 + lane * 4);

    floatx4 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    // ---- reduction
    const int nsteps = (a.nCib / NA) * KS;
    const char *in_c = reinterpret_cast<const char *>(a.in);
    const char *filt_c = reinterpret_cast<const char *>(a.filt);
    const size_t planeA = (size_t)a.HW * 64 * NA;          // bytes between the inputs of consecutive steps' Ci blocks
    constexpr size_t rowB = (size_t)KS * 1024;             // bytes between filter rows; a Ci block is KS rows
    // loads of step t: bases in_c + (t / KS) * planeA and filt_c + ((t / KS) * NA * KS + t % KS) * rowB
    auto issue_step = [&](int t, int y, int slot) {
        const int cstep = t / KS;
        const char *baseA = in_c + (size_t)cstep * planeA;
        const char *baseB = filt_c + ((size_t)cstep * NA * KS + y) * rowB;
        const unsigned stage_lds = lds_base + (unsigned)slot * C::STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < LPS; ++j) issue_one(j, y, baseA, baseB, stage_lds);
    };
#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t)
        if (t < nsteps) issue_step(t, t % KS, t % STAGES);
    __syncthreads();                                      // the zero entries are visible to every wave

    auto load_frags = [&](floatx4 *fa, float (*fb)[4], int slot, int y, int sl) {
        const int dc = sl / KS, x = sl - dc * KS;
        const char *bs = lds_c + b_addr + slot * C::STAGE_BYTES + sl * NSUB * 1024;
#pragma unroll
        for (int j = 0; j < WN; ++j)
#pragma unroll
            for (int r = 0; r < 4; ++r) fb[j][r] = *reinterpret_cast<const float *>(bs + j * 1024 + r * 256);
#pragma unroll
        for (int i = 0; i < WM; ++i)
            fa[i] = *reinterpret_cast<const floatx4 *>(lds_c + p_addr[i][y][x] + slot * C::STAGE_BYTES + dc * (ENTP * 64));
    };

    for (int ks0 = 0; ks0 < nsteps; ks0 += C::UNROLL) {
#pragma unroll
        for (int u = 0; u < C::UNROLL; ++u) {
            const int ks = ks0 + u;
            if (ks >= nsteps) break;
            const int slot = u % STAGES, y = u % KS;                       // compile-time after unrolling
            const int tn = ks + STAGES - 1;                                // step whose loads are issued now
            const int slot_n = (u + STAGES - 1) % STAGES, y_n = (u + STAGES - 1) % KS;
            // step ks has landed once at most the loads of the steps issued after it are outstanding
            if (nsteps - 1 - ks >= STAGES - 2) wait_vmcnt<(STAGES - 2) * LPS>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            const bool more = tn < nsteps;
            const int cstep_n = tn / KS;
            const char *baseA = in_c + (size_t)cstep_n * planeA;
            const char *baseB = filt_c + ((size_t)cstep_n * NA * KS + y_n) * rowB;
            const unsigned stage_lds = lds_base + (unsigned)slot_n * C::STAGE_BYTES;

            // Fragments of slab s + 1 are requested before the matrix instructions of slab s are issued
            // (two register sets); the loads of step tn are issued between the matrix instructions of slab 0.
            floatx4 fa[2][WM];
            float fb[2][WN][4];
            load_frags(fa[0], fb[0], slot, y, 0);
#pragma unroll
            for (int sl = 0; sl < NS; ++sl) {
                if (sl + 1 < NS) load_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], slot, y, sl + 1);
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    if (sl == 0 && more) {
#pragma unroll
                        for (int j = r * LPS / 4; j < (r + 1) * LPS / 4; ++j) issue_one(j, y_n, baseA, baseB, stage_lds);
                    }
#pragma unroll
                    for (int i = 0; i < WM; ++i)
#pragma unroll
                        for (int j = 0; j < WN; ++j)
                            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fb[sl & 1][j][r], fa[sl & 1][i][r], acc[i][j], 0, 0, 0);
                }
            }
        }
    }

    // ---- STORE phase
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int m = m0 + (wave_m * WM + i) * 16 + lp;
        if (m >= a.M) continue;
        const int n = a.dHW.div(m), rem = m - n * a.HW;
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cob = cob0 + wave_n * WN + j;
            if (cob >= a.nCob) continue;
            const size_t o = ((size_t)(n * a.nCob + cob) * a.HW + rem) * 16 + lq * 4;
            *reinterpret_cast<floatx4 *>(a.out + o) = epi4(acc[i][j], a.epilogue, a.res + o);
        }
    }
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA>
hipError_t launch_cfg(SameArgs a, hipStream_t s)
{
    // three ring slots when they fit comfortably (at least two workgroups per compute unit), else two
    constexpr int kStages = 3 * SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, 3>::STAGE_BYTES <= 80 * 1024 ? 3 : 2;
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages>;
    auto kern = conv16_same<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages>;
    if (C::LDS_BYTES > 64 * 1024) {
        static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(kern),
                                                     hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (attr != hipSuccess) return attr;
    }
    a.n_mtiles = (a.M + C::TM - 1) / C::TM;
    const unsigned co_tiles = (unsigned)((a.nCob + C::NSUB - 1) / C::NSUB);
    a.n_cotiles = (int)co_tiles;
    a.dHW = make_fastdiv(a.HW); a.dW = make_fastdiv(a.W);
    a.dMt = make_fastdiv(a.n_mtiles); a.dCt = make_fastdiv(a.n_cotiles);
    hipLaunchKernelGGL(kern, dim3((unsigned)a.n_mtiles * co_tiles), dim3(C::NT), C::LDS_BYTES, s, a);
    return hipGetLastError();
}

template <int KW, int NA>
hipError_t launch_tile(int tile, const SameArgs &a, hipStream_t s)
{
    switch (tile) {
        case SAME_128x128: return launch_cfg<2, 2, 4, 4, KW, NA>(a, s);
        case SAME_64x128: return launch_cfg<1, 4, 4, 2, KW, NA>(a, s);
        case SAME_128x64: return launch_cfg<2, 2, 4, 2, KW, NA>(a, s);
        case SAME_64x64: return launch_cfg<2, 2, 2, 2, KW, NA>(a, s);
        case SAME_128x32: return launch_cfg<4, 1, 2, 2, KW, NA>(a, s);
        case SAME_64x32: return launch_cfg<4, 1, 1, 2, KW, NA>(a, s);
        case SAME_128x16: return launch_cfg<4, 1, 2, 1, KW, NA>(a, s);
        case SAME_32x64: return launch_cfg<2, 2, 1, 2, KW, NA>(a, s);
        case SAME_32x32: return launch_cfg<2, 2, 1, 1, KW, NA>(a, s);
        case SAME_256x16: return launch_cfg<4, 1, 4, 1, KW, NA>(a, s);
        default: return launch_cfg<4, 1, 1, 1, KW, NA>(a, s);
    }
}

}  // namespace

bool conv_same_eligible(const LayerGeom &g)
{
    // the last pixel's byte offset must fit the 32-bit per-lane offset of the load instruction
    const bool small_enough = (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30) &&
                              (size_t)g.Co * g.Ci * g.kh * g.kw < ((size_t)1 << 30);
    return g.Cib == 16 && g.Cob == 16 && g.stride == 1 && g.Ho == g.H && g.Wo == g.W && g.kh == g.kw &&
           (g.kw == 1 || g.kw == 3) && g.pl < g.kw && g.pt < g.kh && small_enough;
}

int conv_same_planes(const LayerGeom &g)
{
    if (g.kw != 1) return 1;
    const int nCib = g.Ci / 16;
    return nCib % 2 == 0 ? 2 : 1;
}

hipError_t launch_conv_same(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                            int tile, int epilogue, hipStream_t s)
{
    SameArgs a;
    a.in = in; a.filt = filt; a.out = out; a.res = (epilogue & EPI_ADD) ? res : out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.HW = g.H * g.W;
    a.nCib = g.Ci / 16; a.nCob = g.Co / 16;
    a.kh = g.kh; a.pt = g.pt; a.pl = g.pl;
    a.M = g.N * a.HW;
    a.n_mtiles = 0; a.n_cotiles = 0;
    // Consecutive workgroups run on one XCD and share its 4 MB L2: when the whole filter fits there, walk the
    // channel tiles of one pixel tile first (the input is then fetched from HBM once, not once per channel
    // tile); a larger filter is kept resident tile by tile instead.
    a.co_fast = (size_t)g.Co * g.Ci * g.kh * g.kw * 4 <= (size_t)3 << 20;
    a.epilogue = epilogue;
    if (g.kw == 3) return launch_tile<3, 1>(tile, a, s);
    if (conv_same_planes(g) == 2) return launch_tile<1, 2>(tile, a, s);
    return launch_tile<1, 1>(tile, a, s);
}

}  // namespace small
