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
// the 3 x 3 and 2 x 2 layers at the end of a network still fill their lanes:
//   1. depthwise phase, one step per (channel block, filter row): the input pixels of that row are staged
//      global -> LDS (ring of STAGES steps, loads run STAGES - 1 steps ahead); lane (pixel p, quad q) reads
//      its three taps as float4 (channels 4q .. 4q + 3), multiplies by the filter taps held in LDS and
//      accumulates; after the third row the (ReLU'd) float4 goes to the "mid" tile in LDS (one float4 per
//      lane and channel block: it is also the float4 this lane feeds to the matrix instructions);
//   2. pointwise phase: 16x16x4 fp32 MFMAs, filter slabs resident in LDS for the whole kernel
//      (loaded once per workgroup), pixel operand = mid tile; accumulators -> (ReLU) -> global.
// Taps outside the image are redirected to an all-zero LDS entry, as in the convolution kernels.
#include "small_internal.h"

#include <algorithm>

namespace small {

namespace {

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
    FastDiv dWo, dHWo, dMt, dCt;
    int relu_mid, relu_out;
};

// ES: staged entries per output pixel (1: stride 1, 2: stride 2). WN: 16-channel output blocks per workgroup.
template <int WN, int ES, int STAGES>
struct DwPwCfg {
    static constexpr int NW = 4, NT = 256, TM = 64, KS = 3;
    static constexpr int ENT = ES * (TM - 1) + KS;
    static constexpr int ENTP = (ENT + 15) / 16 * 16;
    static constexpr int ZERO_REL = ENTP * 64;
    static constexpr int STAGE_BYTES = ZERO_REL + 16;
    static constexpr int NAI = ENTP / 16;                  // wave load instructions per step
    static constexpr int LPS = (NAI + NW - 1) / NW;        // ... per wave
    static constexpr int RING_BYTES = (STAGES * STAGE_BYTES + 255) / 256 * 256;
    static_assert(STAGES == 3, "(ring slot, filter row) of an unrolled step are compile-time because STAGES == KS");
    static_assert((STAGES - 2) * LPS < 64, "too many loads in flight for vmcnt");
    // LDS: ring | mid tile (nCb x 64 pixels x 64 B) | pointwise filter slabs (nCb x WN KiB) | depthwise taps (nCb x 576 B)
    static size_t lds_bytes(int nCb) { return (size_t)RING_BYTES + (size_t)nCb * (TM * 64 + WN * 1024 + 9 * 64); }
};

template <int WN, int ES, int STAGES>
__global__ void __launch_bounds__(256) dwpw16_img(DwPwArgs a)
{
    using C = DwPwCfg<WN, ES, STAGES>;
    constexpr int NW = C::NW, TM = C::TM, KS = 3, ENT = C::ENT, LPS = C::LPS;

    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    char *lds_c = reinterpret_cast<char *>(lds);
    const int mid_off = C::RING_BYTES;
    const int pwf_off = mid_off + a.nCb * (TM * 64);
    const int dwf_off = pwf_off + a.nCb * (WN * 1024);

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 15, lq = lane >> 4;

    // workgroup -> (image group, pixel tile of the image, channel tile), channel tile fastest
    const int wg = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int t = a.dCt.div(wg);
    const int co_tile = wg - t * a.n_cotiles;
    const int grp = a.dMt.div(t);
    const int m_tile = t - grp * a.n_mtiles;
    const int m0 = m_tile * TM;            // first pixel of the tile inside its tile group
    const int cob0 = co_tile * WN;
    const size_t planeA = (size_t)a.HW * 64;
    const size_t imgA = (size_t)a.nCb * planeA;
    const size_t imgO = (size_t)a.nCob * a.HWo * 64;

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
        for (int e = tid; e < ndw; e += C::NT)
            *reinterpret_cast<floatx4 *>(lds_c + dwf_off + e * 16) = reinterpret_cast<const floatx4 *>(a.dwf)[e];
        if (tid < STAGES) *reinterpret_cast<floatx4 *>(lds_c + tid * C::STAGE_BYTES + C::ZERO_REL) = floatx4{0.f, 0.f, 0.f, 0.f};
        wait_vmcnt<0>();
        __syncthreads();
    }

    // ---- load descriptors of the input steps, relative to the start of an image and a channel block
    unsigned d_voff[LPS][KS];
    unsigned d_lds[LPS];
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int chunk = min(j * NW + wave, C::NAI - 1);
        const int e = chunk * 16 + (lane >> 2);
        const int quad = (lane & 3) ^ ((e >> 1) & 3);
        int img, hb, wb;                         // image in the tile group and source pixel of entry e for filter row 0
        if constexpr (ES == 1) {                 // consecutive input pixels (input and output pixel order agree)
            const int fb = m0 + e - a.pl;
            const bool ok = e < ENT && fb >= 0 && fb < a.GHW;
            const int f = ok ? fb : 0;
            img = a.dHWo.div(f);
            const int pix = f - img * a.HWo;
            hb = a.dWo.div(pix);
            wb = pix - hb * a.Wo;
        } else {                                 // entry e: tap e % 2 of output pixel e / 2 (last entry: tap 2 of the last pixel)
            const int pxe = min(e / ES, TM - 1), xe = min(e - pxe * ES, KS - 1);
            const int f = min(m0 + pxe, a.GHW - 1);
            img = a.dHWo.div(f);
            const int pix = f - img * a.HWo;
            const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
            hb = oh * a.stride;
            wb = min(max(ow * a.stride + xe - a.pl, 0), a.W - 1);
        }
#pragma unroll
        for (int y = 0; y < KS; ++y) {
            const int row = min(max(hb + y - a.pt, 0), a.H - 1);
            d_voff[j][y] = (unsigned)(img * imgA) + (unsigned)(((row * a.W + wb) * 16 + quad * 4) * 4);
        }
        d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)(chunk * 16 * 64));
    }

    // ---- this lane's pixel: tap addresses in a stage, mid-tile address, output offset
    const int px = wave * 16 + lp;
    const bool o_ok = m0 + px < a.GHW;
    unsigned p_addr[KS][KS];
    unsigned o_off;
    {
        const int f = min(m0 + px, a.GHW - 1);
        const int img = a.dHWo.div(f), pix = f - img * a.HWo;
        const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
        o_off = (unsigned)(img * imgO) + (unsigned)((pix * 16 + lq * 4) * 4);
        bool row_ok[KS], col_ok[KS];
        unsigned real[KS];
#pragma unroll
        for (int k = 0; k < KS; ++k) {
            row_ok[k] = (unsigned)(oh * a.stride + k - a.pt) < (unsigned)a.H;
            col_ok[k] = (unsigned)(ow * a.stride + k - a.pl) < (unsigned)a.W;
            const int e = px * ES + k;
            real[k] = (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16);
        }
#pragma unroll
        for (int y = 0; y < KS; ++y)
#pragma unroll
            for (int x = 0; x < KS; ++x) p_addr[y][x] = (row_ok[y] && col_ok[x]) ? real[x] : (unsigned)C::ZERO_REL;
    }
    // mid tile of channel block cb: pixel-major entries of 64 B, quads swizzled like a staged input chunk
    const unsigned mid_addr = (unsigned)(mid_off + (px * 4 + (lq ^ ((px >> 1) & 3))) * 16);
    const unsigned b_addr = (unsigned)(pwf_off + lane * 4);
    const unsigned w_addr = (unsigned)(dwf_off + lq * 16);

    // ---- issue side of the input pipeline: (image, channel block, filter row) of the next step to load
    const int nsteps = a.nCb * KS;
    const char *in_c = reinterpret_cast<const char *>(a.in);
    char *out_c = reinterpret_cast<char *>(a.out);
    // tile group q covers images first_image(q) .. + ipt - 1
    auto first_image = [&](int q) __attribute__((always_inline)) { return min(q * a.ipt, a.N - a.ipt); };
    int i_n = grp, i_step = 0, ahead = 0;                  // i_n, n: tile groups
    auto issue_step = [&](int y, int slot) __attribute__((always_inline)) {
        const char *base = in_c + (size_t)first_image(i_n) * imgA + (size_t)(i_step / KS) * planeA;
        const unsigned stage_lds = lds_base + (unsigned)slot * C::STAGE_BYTES;
#pragma unroll
        for (int j = 0; j < LPS; ++j) dma16(base, d_voff[j][y], stage_lds + d_lds[j]);
        ++ahead;
        if (++i_step == nsteps) { i_step = 0; i_n += a.n_groups; }
    };
#pragma unroll
    for (int s = 0; s < STAGES - 1; ++s)
        if (i_n < a.n_igroups) issue_step(s % KS, s % STAGES);

    floatx4 dw = floatx4{0.f, 0.f, 0.f, 0.f};
    int cb = 0;                                            // channel block being reduced
    for (int n = grp; n < a.n_igroups;) {
#pragma unroll
        for (int u = 0; u < KS; ++u) {                     // ring slot == filter row == u (STAGES == KS)
            if (ahead > STAGES - 2) wait_vmcnt<(STAGES - 2) * LPS>();
            else wait_vmcnt<0>();
            __builtin_amdgcn_s_barrier();
            asm volatile("" ::: "memory");
            --ahead;
            if (i_n < a.n_igroups) issue_step((u + STAGES - 1) % KS, (u + STAGES - 1) % STAGES);
            const char *stage = lds_c + u * C::STAGE_BYTES;
            const char *wrow = lds_c + w_addr + (cb * 9 + u * 3) * 64;
#pragma unroll
            for (int x = 0; x < KS; ++x) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(stage + p_addr[u][x]);
                const floatx4 w = *reinterpret_cast<const floatx4 *>(wrow + x * 64);
                dw.x = fmaf(v.x, w.x, dw.x); dw.y = fmaf(v.y, w.y, dw.y);
                dw.z = fmaf(v.z, w.z, dw.z); dw.w = fmaf(v.w, w.w, dw.w);
            }
        }
        if (a.relu_mid) {
            dw.x = dw.x > 0.f ? dw.x : 0.f; dw.y = dw.y > 0.f ? dw.y : 0.f;
            dw.z = dw.z > 0.f ? dw.z : 0.f; dw.w = dw.w > 0.f ? dw.w : 0.f;
        }
        *reinterpret_cast<floatx4 *>(lds_c + mid_addr + cb * (TM * 64)) = dw;
        dw = floatx4{0.f, 0.f, 0.f, 0.f};
        if (++cb < a.nCb) continue;
        cb = 0;

        // ---- pointwise phase. The matrix instruction's pixel operand of lane (p, q) is channels 4q .. 4q + 3 of
        // pixel p: exactly the float4s this lane wrote, so no barrier is needed between the two phases.
        floatx4 acc[WN];
#pragma unroll
        for (int j = 0; j < WN; ++j) acc[j] = floatx4{0.f, 0.f, 0.f, 0.f};
        for (int c = 0; c < a.nCb; ++c) {
            const floatx4 fa = *reinterpret_cast<const floatx4 *>(lds_c + mid_addr + c * (TM * 64));
            const char *bs = lds_c + b_addr + c * (WN * 1024);
            float fb[WN][4];
#pragma unroll
            for (int j = 0; j < WN; ++j)
#pragma unroll
                for (int r = 0; r < 4; ++r) fb[j][r] = *reinterpret_cast<const float *>(bs + j * 1024 + r * 256);
#pragma unroll
            for (int r = 0; r < 4; ++r)
#pragma unroll
                for (int j = 0; j < WN; ++j) acc[j] = __builtin_amdgcn_mfma_f32_16x16x4f32(fb[j][r], fa[r], acc[j], 0, 0, 0);
        }
#pragma unroll
        for (int j = 0; j < WN; ++j) {
            const int cob = cob0 + j;
            if (cob < a.nCob && o_ok) {
                floatx4 v = acc[j];
                if (a.relu_out) {
                    v.x = v.x > 0.f ? v.x : 0.f; v.y = v.y > 0.f ? v.y : 0.f;
                    v.z = v.z > 0.f ? v.z : 0.f; v.w = v.w > 0.f ? v.w : 0.f;
                }
                *reinterpret_cast<floatx4 *>(out_c + (size_t)first_image(n) * imgO + (size_t)cob * a.HWo * 64 + o_off) = v;
            }
        }
        n += a.n_groups;
    }
}

template <int WN, int ES>
hipError_t launch_cfg(DwPwArgs a, hipStream_t s)
{
    using C = DwPwCfg<WN, ES, 3>;
    auto kern = dwpw16_img<WN, ES, 3>;
    const size_t lds = C::lds_bytes(a.nCb);
    static size_t lds_allowed = 64 * 1024;
    if (lds > lds_allowed) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kern), hipFuncAttributeMaxDynamicSharedMemorySize,
                                                 (int)kDwPwMaxLds);
        if (e != hipSuccess) return e;
        lds_allowed = kDwPwMaxLds;
    }
    a.ipt = a.HWo <= 32 ? std::max(1, std::min(a.N, C::TM / a.HWo)) : 1;
    a.GHW = a.ipt * a.HWo;
    a.n_igroups = (a.N + a.ipt - 1) / a.ipt;
    a.n_mtiles = (a.GHW + C::TM - 1) / C::TM;
    a.n_cotiles = (a.nCob + WN - 1) / WN;
    // tile groups per workgroup: enough workgroups to fill the chip (as many as LDS lets be resident, at most 4
    // per compute unit), the rest of the batch is walked by each workgroup with its set-up paid once
    const long positions = (long)a.n_mtiles * a.n_cotiles;
    const long resident = 256 * std::max<long>(1, std::min<long>(4, (long)(160 * 1024 / lds)));
    const long per_wg = std::max<long>(1, std::min<long>(a.n_igroups, (positions * a.n_igroups + resident - 1) / resident));
    a.n_groups = (int)((a.n_igroups + per_wg - 1) / per_wg);
    a.dWo = make_fastdiv(a.Wo);
    a.dHWo = make_fastdiv(a.HWo);
    a.dMt = make_fastdiv(a.n_mtiles);
    a.dCt = make_fastdiv(a.n_cotiles);
    const unsigned grid = (unsigned)(positions * a.n_groups);
    hipLaunchKernelGGL(kern, dim3(grid), dim3(C::NT), lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool dwpw_eligible(int C, int Co, int Cb, int Cob_pw, int kh, int kw, int stride, int pw_kh, int pw_kw, int pw_stride)
{
    if (Cb != 16 || Cob_pw != 16 || kh != 3 || kw != 3 || (stride != 1 && stride != 2)) return false;
    if (pw_kh != 1 || pw_kw != 1 || pw_stride != 1 || C % 16 || Co % 16) return false;
    const int wn = std::min(4, Co / 16);
    const size_t lds = (size_t)(stride == 1 ? 16 * 1024 : 28 * 1024) + (size_t)(C / 16) * (64 * 64 + wn * 1024 + 9 * 64);
    return lds <= kDwPwMaxLds;
}

bool dwpw_geom_ok(const LayerGeom &g)
{
    const bool small_enough = (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30) && (size_t)g.Ci * g.H * g.W < ((size_t)1 << 26);
    if (!small_enough || g.pt >= 3 || g.pl >= 3) return false;
    // several small images per tile: their offsets are part of the 32-bit per-lane offsets
    if ((size_t)64 * g.Ci * g.H * g.W * 4 >= ((size_t)1 << 31) && g.Ho * g.Wo <= 32) return false;
    if (g.stride == 1) return g.Ho == g.H && g.Wo == g.W;
    return g.stride == 2 && 2 * (g.Wo - 1) + 2 - g.pl >= g.W;    // see conv_same_eligible
}

hipError_t launch_dwpw(const float *in, const float *dw_filt, const float *pw_filt, float *out, const LayerGeom &g, int Co,
                       int relu_mid, int relu_out, hipStream_t s)
{
    DwPwArgs a;
    a.in = in; a.dwf = dw_filt; a.pwf = pw_filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.HW = g.H * g.W;
    a.Ho = g.Ho; a.Wo = g.Wo; a.HWo = g.Ho * g.Wo; a.stride = g.stride;
    a.nCb = g.Ci / 16; a.nCob = Co / 16;
    a.pt = g.pt; a.pl = g.pl;
    a.relu_mid = relu_mid; a.relu_out = relu_out;
    const int wn = std::min(4, a.nCob);
    if (g.stride == 1) {
        switch (wn) {
            case 1: return launch_cfg<1, 1>(a, s);
            case 2: return launch_cfg<2, 1>(a, s);
            case 3: return launch_cfg<3, 1>(a, s);
            default: return launch_cfg<4, 1>(a, s);
        }
    }
    switch (wn) {
        case 1: return launch_cfg<1, 2>(a, s);
        case 2: return launch_cfg<2, 2>(a, s);
        case 3: return launch_cfg<3, 2>(a, s);
        default: return launch_cfg<4, 2>(a, s);
    }
}

}  // namespace small
