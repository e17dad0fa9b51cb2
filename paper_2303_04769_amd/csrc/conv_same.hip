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

#include <type_traits>

namespace small {

namespace {

struct SameArgs {
    const float *in;
    const float *filt;
    float *out;
    const float *res;
    const float *bn;            // EPI_BN: scale[0 .. Co) then shift[0 .. Co)
    int N, H, W, HW;            // input image
    int Ho, Wo, HWo, stride;    // output image
    int nCib, nCob;             // input blocks of a reduction, output blocks of the tensor
    // group convolution (partial-channel reduction): output blocks [j * gk, (j + 1) * gk) reduce the nCib input blocks
    // from block j * gs on; in_blocks: channel blocks of an input image in memory. A plain convolution is one group:
    // gk = nCob, gs = 0, in_blocks = nCib.
    int in_blocks, gk, gs;
    int kh, pt, pl;
    int M;          // N * Ho * Wo
    int n_mtiles, n_cotiles;
    FastDiv dHWo, dWo, dMt, dCt;   // divisions by Ho*Wo, Wo, n_mtiles, n_cotiles
    int co_fast;    // workgroup order: channel tile fastest (input tile shared in L2) or pixel tile fastest (filter shared)
    int epilogue;
    // image-aligned persistent variant only: n_mtiles counts the pixel tiles of ONE image; a workgroup owns one
    // (pixel tile, channel tile) position and walks the images g, g + n_groups, g + 2 n_groups, ...
    int n_groups;
    FastDiv dGP;    // division by n_groups * n_mtiles
};

// bn_c: scale of this lane's four channels; bn_c + Co floats: their shifts
__device__ __forceinline__ floatx4 epi4(floatx4 v, int epi, const float *res, const float *bn_c = nullptr, int Co = 0)
{
    if (epi & EPI_BN) {
        const floatx4 sc = *reinterpret_cast<const floatx4 *>(bn_c), sh = *reinterpret_cast<const floatx4 *>(bn_c + Co);
        v.x = fmaf(v.x, sc.x, sh.x); v.y = fmaf(v.y, sc.y, sh.y); v.z = fmaf(v.z, sc.z, sh.z); v.w = fmaf(v.w, sc.w, sh.w);
    }
    if (epi & EPI_ADD) v += *reinterpret_cast<const floatx4 *>(res);
    if (epi & EPI_RELU) {
        v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
        v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
    }
    return v;
}

constexpr int gcd_(int a, int b) { return b == 0 ? a : gcd_(b, a % b); }

// KS: square filter size (1 or 3). NA: Ci blocks staged per reduction step (1 for 3x3). ES: staged entries
// per output pixel step (1: stride 1, or any stride with a 1x1 filter; 2: 3x3 filter with stride 2).
template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int STAGES, int ES = 1>
struct SameCfg {
    static constexpr int NW = WAVES_M * WAVES_N;
    static constexpr int NT = 64 * NW;
    static constexpr int TM = WAVES_M * WM * 16;
    static constexpr int TN = WAVES_N * WN * 16;
    static constexpr int NSUB = TN / 16;
    static constexpr int ENT = ES * (TM - 1) + KS;           // staged input pixels per plane
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
    static_assert(ES == 1 || (ES == 2 && KS == 3), "two entries per pixel only for the strided 3x3 filter");
};

template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int STAGES, int ES>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) conv16_same(SameArgs a)
{
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, STAGES, ES>;
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
    const int cib0 = (cob0 / a.gk) * a.gs;                 // first input block of this tile's group
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
    unsigned d_lds[LPS];      // wave-uniform LDS byte offset inside a stage (held in scalar registers)
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int k = min(j * NW + wave, C::NAI + C::NBI - 1);
        if (k < C::NAI) {
            const int dc = k / (ENTP / 16), chunk = k - dc * (ENTP / 16);
            const int e = chunk * 16 + (lane >> 2);
            const int quad = (lane & 3) ^ ((e >> 1) & 3);
            // Source pixel of entry e for filter row 0. Stride-1 3x3: entries are consecutive input pixels
            // (the flat order of input and output pixels is the same). Otherwise entry e belongs to output
            // pixel e / ES and holds its tap e % ES (the last entry: tap KS - 1 of the last pixel).
            int n, hb, wb;
            if constexpr (KS == 3 && ES == 1) {
                const int fb = m0 + e - a.pl;
                const bool ok = e < ENT && fb >= 0 && fb < a.M;
                const int fbc = ok ? fb : 0;
                n = a.dHWo.div(fbc);
                const int pix = fbc - n * a.HWo;
                hb = a.dWo.div(pix);
                wb = pix - hb * a.Wo;
            } else {
                const int pxe = min(e / ES, TM - 1), xe = min(e - pxe * ES, KS - 1);
                const int mo = min(m0 + pxe, a.M - 1);
                n = a.dHWo.div(mo);
                const int pix = mo - n * a.HWo;
                const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
                hb = oh * a.stride;
                wb = min(max(ow * a.stride + xe - a.pl, 0), a.W - 1);
            }
#pragma unroll
            for (int y = 0; y < KS; ++y) {
                const int row = min(max(hb + y - a.pt, 0), a.H - 1);
                d_voff[j][y] = (unsigned)((((n * a.in_blocks + cib0 + dc) * a.H + row) * a.W + wb) * 16 + quad * 4) * 4u;
            }
            d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)((dc * ENTP + chunk * 16) * 64));
        } else {
            const int kb = k - C::NAI;
            const int slab = kb / NSUB, sub = kb - slab * NSUB;
            const int dc = slab / KS, x = slab - dc * KS;
            const int row = lane >> 2, ci = 4 * (row & 3) + (row >> 2);
            const int cob = min(cob0 + sub, a.nCob - 1);
            const unsigned off = (unsigned)((((cob * a.nCib + dc) * KS) * KS + x) * 256 + ci * 16 + (lane & 3) * 4) * 4u;
#pragma unroll
            for (int y = 0; y < KS; ++y) d_voff[j][y] = off;
            d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)(C::A_BYTES + (slab * NSUB + sub) * 1024));
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
    unsigned o_off[WM];       // byte offset of (pixel, channel block 0, this lane's 4 channels) in the output
    bool o_ok[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int px = (wave_m * WM + i) * 16 + lp;
        o_ok[i] = m0 + px < a.M;
        const int m = min(m0 + px, a.M - 1);
        const int n = a.dHWo.div(m), pix = m - n * a.HWo;
        const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
        o_off[i] = (unsigned)((n * a.nCob * a.HWo + pix) * 16 + lq * 4) * 4u;
        bool row_ok[KS], col_ok[KS];
        unsigned real[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            row_ok[t] = (unsigned)(oh * a.stride + t - a.pt) < (unsigned)a.H;
            col_ok[t] = (unsigned)(ow * a.stride + t - a.pl) < (unsigned)a.W;
            const int e = px * ES + t;
            real[t] = (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16);
        }
#pragma unroll
        for (int y = 0; y < KS; ++y)
#pragma unroll
            for (int x = 0; x < KS; ++x)
                p_addr[i][y][x] = ((row_ok[y] && col_ok[x]) || KS == 1) ? real[x] : (unsigned)C::ZERO_REL;
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
            const int cstep_n = tn / KS;
            const char *baseA = in_c + (size_t)cstep_n * planeA;
            const char *baseB = filt_c + ((size_t)cstep_n * NA * KS + y_n) * rowB;
            const unsigned stage_lds = lds_base + (unsigned)slot_n * C::STAGE_BYTES;

            // Fragments of slab s + 1 are requested before the matrix instructions of slab s are issued
            // (two register sets); the loads of step tn are issued between the matrix instructions of slab 0.
            // Two copies of the body, with and without loads, so that no branch sits between the matrix instructions.
            auto body = [&](auto more) __attribute__((always_inline)) {
                floatx4 fa[2][WM];
                float fb[2][WN][4];
                load_frags(fa[0], fb[0], slot, y, 0);
#pragma unroll
                for (int sl = 0; sl < NS; ++sl) {
                    if (sl + 1 < NS) load_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], slot, y, sl + 1);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (decltype(more)::value) {
                            if (sl == 0) {
#pragma unroll
                                for (int j = r * LPS / 4; j < (r + 1) * LPS / 4; ++j) issue_one(j, y_n, baseA, baseB, stage_lds);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < WM; ++i)
#pragma unroll
                            for (int j = 0; j < WN; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fb[sl & 1][j][r], fa[sl & 1][i][r], acc[i][j], 0, 0, 0);
                    }
                }
            };
            if (tn < nsteps) body(std::true_type{});
            else body(std::false_type{});
        }
    }

    // ---- STORE phase: scalar base per output channel block + the per-lane offset kept from the set-up
    char *out_c = reinterpret_cast<char *>(a.out);
    const char *res_c = reinterpret_cast<const char *>(a.res);
#pragma unroll
    for (int j = 0; j < WN; ++j) {
        const int cob = cob0 + wave_n * WN + j;
        if (cob >= a.nCob) continue;
        const size_t cb = (size_t)cob * a.HWo * 64;
        const float *bn_c = a.bn + cob * 16 + lq * 4;
#pragma unroll
        for (int i = 0; i < WM; ++i) {
            if (!o_ok[i]) continue;
            *reinterpret_cast<floatx4 *>(out_c + cb + o_off[i]) =
                epi4(acc[i][j], a.epilogue, reinterpret_cast<const float *>(res_c + cb + o_off[i]), bn_c, a.nCob * 16);
        }
    }
}

// Image-aligned persistent variant. Pixel tiles do not cross image boundaries, and a workgroup keeps one
// (pixel tile, channel tile) position while it walks over images. Everything that depends on the lane
// (load descriptors, fragment addresses, edge masks, output offsets) is then the same for all of its
// tiles and is computed once; moving to the next image only adds to scalar base addresses. The ring of
// LDS stages runs on across tiles: the first loads of the next image are in flight while the last steps
// of the current one are computed and stored. The step loop is one endless sequence over all tiles of
// the workgroup, unrolled by UNROLL = lcm(STAGES, KS): a tile has a multiple of KS steps, so (ring slot,
// filter row) of unrolled step u are compile-time whatever the number of steps per tile; the end of a tile
// is a run-time check after every step.
template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int STAGES, int ES>
__global__ void __launch_bounds__(64 * WAVES_M * WAVES_N) conv16_img(SameArgs a)
{
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, STAGES, ES>;
    constexpr int NW = C::NW, TM = C::TM, NSUB = C::NSUB, ENT = C::ENT, ENTP = C::ENTP, LPS = C::LPS, NS = C::NS;

    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    const char *lds_c = reinterpret_cast<const char *>(lds);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int wave_m = wave % WAVES_M, wave_n = wave / WAVES_M;
    const int lp = lane & 15, lq = lane >> 4;

    // workgroup -> (channel tile, image group, pixel tile of the image); neighbours in this order share L2 lines
    const int wg = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    int co_tile, grp, m_tile;
    if (a.co_fast) {
        const int t = a.dCt.div(wg);
        co_tile = wg - t * a.n_cotiles;
        grp = a.dMt.div(t);
        m_tile = t - grp * a.n_mtiles;
    } else {
        co_tile = a.dGP.div(wg);
        const int t = wg - co_tile * (a.n_groups * a.n_mtiles);
        grp = a.dMt.div(t);
        m_tile = t - grp * a.n_mtiles;
    }
    const int m0 = m_tile * TM;            // first pixel of the tile inside its image
    const int cob0 = co_tile * NSUB;
    const int cib0 = (cob0 / a.gk) * a.gs;                 // first input block of this tile's group

    // ---- load descriptors, relative to the start of an image (see conv16_same for the scheme)
    unsigned d_voff[LPS][KS];
    unsigned d_lds[LPS];
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int k = min(j * NW + wave, C::NAI + C::NBI - 1);
        if (k < C::NAI) {
            const int dc = k / (ENTP / 16), chunk = k - dc * (ENTP / 16);
            const int e = chunk * 16 + (lane >> 2);
            const int quad = (lane & 3) ^ ((e >> 1) & 3);
            int hb, wb;                       // source pixel of entry e for filter row 0 (see conv16_same)
            if constexpr (KS == 3 && ES == 1) {
                const int fb = m0 + e - a.pl;
                const bool ok = e < ENT && fb >= 0 && fb < a.HWo;
                const int pix = ok ? fb : 0;
                hb = a.dWo.div(pix);
                wb = pix - hb * a.Wo;
            } else {
                const int pxe = min(e / ES, TM - 1), xe = min(e - pxe * ES, KS - 1);
                const int pix = min(m0 + pxe, a.HWo - 1);
                const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
                hb = oh * a.stride;
                wb = min(max(ow * a.stride + xe - a.pl, 0), a.W - 1);
            }
#pragma unroll
            for (int y = 0; y < KS; ++y) {
                const int row = min(max(hb + y - a.pt, 0), a.H - 1);
                d_voff[j][y] = (unsigned)((((dc * a.H + row) * a.W + wb) * 16 + quad * 4) * 4);
            }
            d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)((dc * ENTP + chunk * 16) * 64));
        } else {
            const int kb = k - C::NAI;
            const int slab = kb / NSUB, sub = kb - slab * NSUB;
            const int dc = slab / KS, x = slab - dc * KS;
            const int row = lane >> 2, ci = 4 * (row & 3) + (row >> 2);
            const int cob = min(cob0 + sub, a.nCob - 1);
            const unsigned off = (unsigned)((((cob * a.nCib + dc) * KS) * KS + x) * 256 + ci * 16 + (lane & 3) * 4) * 4u;
#pragma unroll
            for (int y = 0; y < KS; ++y) d_voff[j][y] = off;
            d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)(C::A_BYTES + (slab * NSUB + sub) * 1024));
        }
    }
    auto issue_one = [&](int j, int y, const char *baseA, const char *baseB, unsigned stage_lds) __attribute__((always_inline)) {
        const bool isA = min(j * NW + wave, C::NAI + C::NBI - 1) < C::NAI;     // wave-uniform
        dma16(isA ? baseA : baseB, d_voff[j][y], stage_lds + d_lds[j]);
    };

    if (tid < STAGES) lds[(tid * C::STAGE_BYTES + C::ZERO_REL) / 16] = floatx4{0.f, 0.f, 0.f, 0.f};

    // ---- fragment addresses and output offsets of this lane's pixels (the same in every image)
    unsigned p_addr[WM][KS][KS];
    unsigned o_off[WM];
    bool o_ok[WM];
#pragma unroll
    for (int i = 0; i < WM; ++i) {
        const int px = (wave_m * WM + i) * 16 + lp;
        o_ok[i] = m0 + px < a.HWo;
        const int pix = min(m0 + px, a.HWo - 1);
        const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
        o_off[i] = (unsigned)(pix * 16 + lq * 4) * 4u;
        bool row_ok[KS], col_ok[KS];
        unsigned real[KS];
#pragma unroll
        for (int t = 0; t < KS; ++t) {
            row_ok[t] = (unsigned)(oh * a.stride + t - a.pt) < (unsigned)a.H;
            col_ok[t] = (unsigned)(ow * a.stride + t - a.pl) < (unsigned)a.W;
            const int e = px * ES + t;
            real[t] = (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16);
        }
#pragma unroll
        for (int y = 0; y < KS; ++y)
#pragma unroll
            for (int x = 0; x < KS; ++x)
                p_addr[i][y][x] = ((row_ok[y] && col_ok[x]) || KS == 1) ? real[x] : (unsigned)C::ZERO_REL;
    }
    const unsigned b_addr = (unsigned)(C::A_BYTES + wave_n * WN * 1024 + lane * 4);

    // ---- issue side of the pipeline: (image, step) of the next step to load, STAGES - 1 steps ahead
    const int nsteps = (a.nCib / NA) * KS;
    const char *in_c = reinterpret_cast<const char *>(a.in);
    const char *filt_c = reinterpret_cast<const char *>(a.filt);
    char *out_c = reinterpret_cast<char *>(a.out);
    const char *res_c = reinterpret_cast<const char *>(a.res);
    const size_t planeA = (size_t)a.HW * 64 * NA;          // bytes between the inputs of consecutive steps' Ci blocks
    const size_t imgA = (size_t)a.in_blocks * a.HW * 64;   // bytes of one input image
    const size_t imgO = (size_t)a.nCob * a.HWo * 64;       // bytes of one output image
    constexpr size_t rowB = (size_t)KS * 1024;             // bytes between filter rows; a Ci block is KS rows
    int i_n = grp, i_step = 0;                             // i_n >= N: nothing left to load
    int ahead = 0;                                         // steps issued and not yet computed
    auto issue_bases = [&](const char *&baseA, const char *&baseB, int y) __attribute__((always_inline)) {
        const int cstep = i_step / KS;
        baseA = in_c + (size_t)i_n * imgA + (size_t)cib0 * a.HW * 64 + (size_t)cstep * planeA;
        baseB = filt_c + ((size_t)cstep * NA * KS + y) * rowB;
    };
    auto issue_done = [&]() __attribute__((always_inline)) {
        ++ahead;
        if (++i_step == nsteps) { i_step = 0; i_n += a.n_groups; }
    };
#pragma unroll
    for (int t = 0; t < STAGES - 1; ++t) {
        if (i_n < a.N) {
            const char *baseA, *baseB;
            issue_bases(baseA, baseB, t % KS);
            const unsigned stage_lds = lds_base + (unsigned)(t % STAGES) * C::STAGE_BYTES;
#pragma unroll
            for (int j = 0; j < LPS; ++j) issue_one(j, t % KS, baseA, baseB, stage_lds);
            issue_done();
        }
    }
    __syncthreads();                                      // the zero entries are visible to every wave

    auto load_frags = [&](floatx4 *fa, float (*fb)[4], int slot, int y, int sl) __attribute__((always_inline)) {
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

    floatx4 acc[WM][WN];
#pragma unroll
    for (int i = 0; i < WM; ++i)
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};

    int n = grp, c_step = 0;                               // image and step being computed
    for (;;) {
#pragma unroll
        for (int u = 0; u < C::UNROLL; ++u) {
            const int slot = u % STAGES, y = u % KS;                       // compile-time after unrolling
            const int slot_n = (u + STAGES - 1) % STAGES, y_n = (u + STAGES - 1) % KS;
            // the step to compute has landed once at most the loads of the steps issued after it are outstanding
            // (stores of the previous tile issued in between only make this wait stricter)
            if (ahead > STAGES - 2) wait_vmcnt<(STAGES - 2) * LPS>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            --ahead;
            const char *baseA, *baseB;
            issue_bases(baseA, baseB, y_n);
            const unsigned stage_lds = lds_base + (unsigned)slot_n * C::STAGE_BYTES;

            // Two copies of the body, with and without loads, so that no branch sits between the matrix instructions.
            auto body = [&](auto more) __attribute__((always_inline)) {
                floatx4 fa[2][WM];
                float fb[2][WN][4];
                load_frags(fa[0], fb[0], slot, y, 0);
#pragma unroll
                for (int sl = 0; sl < NS; ++sl) {
                    if (sl + 1 < NS) load_frags(fa[(sl + 1) & 1], fb[(sl + 1) & 1], slot, y, sl + 1);
#pragma unroll
                    for (int r = 0; r < 4; ++r) {
                        if constexpr (decltype(more)::value) {
                            if (sl == 0) {
#pragma unroll
                                for (int j = r * LPS / 4; j < (r + 1) * LPS / 4; ++j) issue_one(j, y_n, baseA, baseB, stage_lds);
                            }
                        }
#pragma unroll
                        for (int i = 0; i < WM; ++i)
#pragma unroll
                            for (int j = 0; j < WN; ++j)
                                acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fb[sl & 1][j][r], fa[sl & 1][i][r], acc[i][j], 0, 0, 0);
                    }
                }
            };
            if (i_n < a.N) { body(std::true_type{}); issue_done(); }
            else body(std::false_type{});

            if (++c_step == nsteps) {
                // ---- STORE phase of this image's tile
#pragma unroll
                for (int j = 0; j < WN; ++j) {
                    const int cob = cob0 + wave_n * WN + j;
                    if (cob < a.nCob) {
                        const size_t cb = (size_t)n * imgO + (size_t)cob * a.HWo * 64;
                        const float *bn_c = a.bn + cob * 16 + lq * 4;
#pragma unroll
                        for (int i = 0; i < WM; ++i) {
                            if (o_ok[i])
                                *reinterpret_cast<floatx4 *>(out_c + cb + o_off[i]) =
                                    epi4(acc[i][j], a.epilogue, reinterpret_cast<const float *>(res_c + cb + o_off[i]), bn_c,
                                         a.nCob * 16);
                        }
                    }
                }
#pragma unroll
                for (int i = 0; i < WM; ++i)
#pragma unroll
                    for (int j = 0; j < WN; ++j) acc[i][j] = floatx4{0.f, 0.f, 0.f, 0.f};
                c_step = 0;
                n += a.n_groups;
                if (n >= a.N) return;                          // uniform: every wave of the workgroup leaves here
            }
        }
    }
}

// three ring slots when they fit comfortably (at least two workgroups per compute unit), else two
template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int ES>
constexpr int stages_of = 3 * SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, 3, ES>::STAGE_BYTES <= 80 * 1024 ? 3 : 2;

// Images per workgroup for the image-aligned persistent variant, or 0 for the flat one-tile-per-workgroup
// kernel. Host arithmetic only. The persistent variant wastes the lanes of each image's last tile, so it
// is taken when that waste is small; the
// number of images per workgroup trades the per-workgroup set-up (paid once) against balance over the
// compute units and against keeping at least 4 workgroups per compute unit to hide latencies.
template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int ES>
int images_per_workgroup(int N, int HW, int nCib, int nCob)     // HW: pixels of an OUTPUT image
{
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, stages_of<WAVES_M, WAVES_N, WM, WN, KS, NA, ES>, ES>;
    const int nsteps = (nCib / NA) * KS;
    const long tpi = (HW + C::TM - 1) / C::TM;
    if (KS == 1 || tpi * C::TM * 100 > (long)HW * 108 || N < 2) return 0;   // measured: no gain for 1x1 filters
    const long positions = tpi * ((nCob + C::NSUB - 1) / C::NSUB);
    const long kCUs = device_cus();
    constexpr long kMinPerCU = 4;
    const double t_tile = (double)nsteps * C::NS * 4 * WM * WN * 32;   // matrix-pipe cycles of one wave per tile
    const double t_setup = 2500;                                       // set-up, launch and first-load latency, cycles
    int best = 0;
    double best_cost = 0;
    for (int t = 1; t <= N && t <= 64; ++t) {
        const long groups = (N + t - 1) / t;
        const int per_wg = (int)((N + groups - 1) / groups);
        const long wgs = positions * groups;
        if (t > 1 && wgs < kMinPerCU * kCUs) break;
        const double cost = (double)((wgs + kCUs - 1) / kCUs) * (per_wg * t_tile + t_setup);
        if (best == 0 || cost < best_cost * 0.98) { best = per_wg; best_cost = cost; }
    }
    return best > 1 ? best : 0;
}

template <int WAVES_M, int WAVES_N, int WM, int WN, int KS, int NA, int ES>
hipError_t launch_cfg(SameArgs a, hipStream_t s)
{
    constexpr int kStages = stages_of<WAVES_M, WAVES_N, WM, WN, KS, NA, ES>;
    using C = SameCfg<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages, ES>;
    const int per_wg = images_per_workgroup<WAVES_M, WAVES_N, WM, WN, KS, NA, ES>(a.N, a.HWo, a.nCib, a.nCob);
    auto kern = per_wg ? conv16_img<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages, ES> : conv16_same<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages, ES>;
    if (C::LDS_BYTES > 64 * 1024) {
        static hipError_t attr_img = hipFuncSetAttribute(reinterpret_cast<const void *>(conv16_img<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages, ES>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        static hipError_t attr_flat = hipFuncSetAttribute(reinterpret_cast<const void *>(conv16_same<WAVES_M, WAVES_N, WM, WN, KS, NA, kStages, ES>),
                                                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)C::LDS_BYTES);
        if (attr_img != hipSuccess) return attr_img;
        if (attr_flat != hipSuccess) return attr_flat;
    }
    const unsigned co_tiles = (unsigned)((a.nCob + C::NSUB - 1) / C::NSUB);
    a.n_cotiles = (int)co_tiles;
    a.dHWo = make_fastdiv(a.HWo); a.dWo = make_fastdiv(a.Wo);
    a.dCt = make_fastdiv(a.n_cotiles);
    unsigned grid;
    if (per_wg) {
        a.n_mtiles = (a.HWo + C::TM - 1) / C::TM;
        a.n_groups = (a.N + per_wg - 1) / per_wg;
        a.dGP = make_fastdiv(a.n_groups * a.n_mtiles);
        grid = (unsigned)a.n_mtiles * (unsigned)a.n_groups * co_tiles;
    } else {
        a.n_mtiles = (a.M + C::TM - 1) / C::TM;
        a.n_groups = 1;
        a.dGP = make_fastdiv(a.n_mtiles);
        grid = (unsigned)a.n_mtiles * co_tiles;
    }
    a.dMt = make_fastdiv(a.n_mtiles);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), C::LDS_BYTES, s, a);
    return hipGetLastError();
}

// calls f.template operator()<WAVES_M, WAVES_N, WM, WN>() for the tile id
template <class F>
auto with_tile(int tile, F &&f)
{
    switch (tile) {
        case SAME_128x128: return f.template operator()<2, 2, 4, 4>();
        case SAME_64x128: return f.template operator()<1, 4, 4, 2>();
        case SAME_128x64: return f.template operator()<2, 2, 4, 2>();
        case SAME_64x64: return f.template operator()<2, 2, 2, 2>();
        case SAME_128x32: return f.template operator()<4, 1, 2, 2>();
        case SAME_64x32: return f.template operator()<4, 1, 1, 2>();
        case SAME_128x16: return f.template operator()<4, 1, 2, 1>();
        case SAME_32x64: return f.template operator()<2, 2, 1, 2>();
        case SAME_32x32: return f.template operator()<2, 2, 1, 1>();
        case SAME_256x16: return f.template operator()<4, 1, 4, 1>();
        default: return f.template operator()<4, 1, 1, 1>();
    }
}

template <int KW, int NA, int ES>
struct LaunchTile {
    const SameArgs &a;
    hipStream_t s;
    template <int WAVES_M, int WAVES_N, int WM, int WN>
    hipError_t operator()() const { return launch_cfg<WAVES_M, WAVES_N, WM, WN, KW, NA, ES>(a, s); }
};

template <int KW, int NA, int ES>
struct PlanTile {
    int N, HWo, nCib, nCob;
    template <int WAVES_M, int WAVES_N, int WM, int WN>
    int operator()() const { return images_per_workgroup<WAVES_M, WAVES_N, WM, WN, KW, NA, ES>(N, HWo, nCib, nCob); }
};

}  // namespace

bool conv_same_eligible(const LayerGeom &g)
{
    // the last pixel's byte offset must fit the 32-bit per-lane offset of the load and store instructions
    const bool small_enough = (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30) &&
                              (size_t)g.N * g.Co * g.Ho * g.Wo < ((size_t)1 << 30) &&
                              (size_t)g.Co * g.Ci * g.kh * g.kw < ((size_t)1 << 30);
    if (g.Cib != 16 || g.Cob != 16 || g.kh != g.kw || !small_enough) return false;
    if (g.kw == 1)                                                          // every tap must be inside the image
        return g.pt == 0 && g.pl == 0 && g.stride >= 1 && (g.Ho - 1) * g.stride < g.H && (g.Wo - 1) * g.stride < g.W;
    if (g.kw != 3 || g.pl >= 3 || g.pt >= 3) return false;
    if (g.stride == 1) return g.Ho == g.H && g.Wo == g.W;                   // output pixels in input order
    // stride 2: taps 0, 1 of a pixel are its own staged entries, tap 2 is the next pixel's tap 0, which is
    // only right if a row's last pixel has no tap 2 inside the image
    return g.stride == 2 && 2 * (g.Wo - 1) + 2 - g.pl >= g.W;
}

int conv_same_planes(const LayerGeom &g)
{
    if (g.kw != 1) return 1;
    const int nCib = g.Ci / 16;
    return nCib % 2 == 0 ? 2 : 1;
}

namespace {

// calls f(LaunchTile / PlanTile functor type selector) for the layer's (filter size, planes per step, entry stride)
template <template <int, int, int> class F, class... Args>
auto with_shape(const LayerGeom &g, int tile, Args &&...args)
{
    if (g.kw == 3) {
        if (g.stride == 2) return with_tile(tile, F<3, 1, 2>{args...});
        return with_tile(tile, F<3, 1, 1>{args...});
    }
    if (conv_same_planes(g) == 2) return with_tile(tile, F<1, 2, 1>{args...});
    return with_tile(tile, F<1, 1, 1>{args...});
}

}  // namespace

hipError_t launch_conv_same(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                            int tile, int epilogue, hipStream_t s, int F_C, int S_C, int K, const float *bn)
{
    SameArgs a;
    a.in = in; a.filt = filt; a.out = out; a.res = (epilogue & EPI_ADD) ? res : out;
    a.bn = (epilogue & EPI_BN) ? bn : filt;        // (a valid address when unused)
    a.N = g.N; a.H = g.H; a.W = g.W; a.HW = g.H * g.W;
    a.Ho = g.Ho; a.Wo = g.Wo; a.HWo = g.Ho * g.Wo; a.stride = g.stride;
    a.nCib = g.Ci / 16; a.nCob = g.Co / 16;
    a.in_blocks = a.nCib; a.gk = a.nCob; a.gs = 0;
    if (F_C) { a.nCib = F_C / 16; a.gk = K / 16; a.gs = S_C / 16; }
    a.kh = g.kh; a.pt = g.pt; a.pl = g.pl;
    a.M = g.N * a.HWo;
    a.n_mtiles = 0; a.n_cotiles = 0;
    // Consecutive workgroups run on one XCD and share its 4 MB L2: when the whole filter fits there, walk the
    // channel tiles of one pixel tile first (the input is then fetched from HBM once, not once per channel
    // tile); a larger filter is kept resident tile by tile instead.
    a.co_fast = (size_t)g.Co * (F_C ? F_C : g.Ci) * g.kh * g.kw * 4 <= (size_t)3 << 20;
    a.epilogue = epilogue;
    a.n_groups = 1;
    if (F_C) {
        LayerGeom gg = g;
        gg.Ci = F_C;                     // what the kernel variants are chosen by: the reduction of one group
        return with_shape<LaunchTile>(gg, tile, a, s);
    }
    return with_shape<LaunchTile>(g, tile, a, s);
}

int conv_same_images_per_workgroup(const LayerGeom &g, int tile)
{
    return with_shape<PlanTile>(g, tile, g.N, g.Ho * g.Wo, g.Ci / 16, g.Co / 16);
}

}  // namespace small
