// Depthwise 3x3 convolution for 16-channel blocks with its input staged global -> LDS by the load unit
// (gfx950): the single-channel-reduction layer of Table 1 on the shared blocked layout, HBM-bound.
//
// A workgroup (4 waves) keeps one tile position, R whole output rows of an image (or several whole
// small images), and walks over (image, channel block) planes with all per-lane state fixed: load
// descriptors, the nine tap addresses of each of its pixels, output offsets. One step per plane:
// the input rows the tile's windows touch are copied as whole rows into a ring of LDS stages with
// global_load_lds_dwordx4, several steps ahead of their use, tracked by hand with s_waitcnt vmcnt(n);
// lane (pixel p, quad q) gathers its taps as float4 (channels 4q .. 4q + 3), multiplies by the filter taps
// held in LDS, applies the optional ReLU and stores 16 bytes; four lanes cover the 64 bytes of a pixel.
// Taps outside the image are redirected to an all-zero LDS entry. Compared with a load / barrier /
// compute / store sequence per workgroup, loads, LDS reads and stores of consecutive planes overlap
// inside one workgroup and the set-up is paid once.
#include "small_internal.h"

#include <algorithm>

namespace small {

namespace {

constexpr int kMaxStages = 8;

struct RowsArgs {
    const float *in;
    const float *filt;   // [C/16][3][3][16]
    float *out;
    int N, H, W, HW;
    int Ho, Wo, HWo, stride;
    int nCb;
    int pt, pl;
    int ipt;             // images per tile group (whole small images side by side), else 1
    int GHW;             // output pixels of a tile group: ipt * Ho * Wo
    int tile_px;         // output pixels per tile: whole rows, at most 64 * PXL
    int n_igroups;       // tile groups in the batch: ceil(N / ipt); the last one is shifted back to end at image N - 1
    int n_mtiles;        // tiles per tile group
    int n_groups;        // workgroups along the (tile group, channel block) planes
    int n_planes;        // n_igroups * nCb
    int stages, stage_bytes;
    FastDiv dW, dH, dWo, dHWo, dMt, dCb;
    int relu;
};

// Input rows (numbered through the images of a tile group: image * H + row) that output pixels [m0, m0 + npx) touch.
__host__ __device__ inline void tile_rows(int m0, int npx, int GHW, int HWo, int Wo, int H, int stride, int pt, int &lo, int &hi)
{
    const int f0 = m0, f1 = (m0 + npx - 1 < GHW - 1) ? m0 + npx - 1 : GHW - 1;
    const int img0 = f0 / HWo, oh0 = (f0 - img0 * HWo) / Wo;
    const int img1 = f1 / HWo, oh1 = (f1 - img1 * HWo) / Wo;
    int r0 = oh0 * stride - pt, r1 = oh1 * stride - pt + 2;
    r0 = r0 < 0 ? 0 : (r0 > H - 1 ? H - 1 : r0);
    r1 = r1 < 0 ? 0 : (r1 > H - 1 ? H - 1 : r1);
    lo = img0 * H + r0;
    hi = img1 * H + r1;
}

// PXL: output pixels per lane (a tile has up to 64 * PXL pixels). LPS: load instructions per wave and step.
template <int PXL, int LPS>
__global__ void __launch_bounds__(256) dw16_rows(RowsArgs a)
{
    constexpr int NW = 4, NT = 256;
    static_assert((kMaxStages - 1) * LPS < 64, "too many loads in flight for vmcnt");

    extern __shared__ floatx4 lds[];
    const unsigned lds_base = (unsigned)(uintptr_t)(__attribute__((address_space(3))) void *)lds;
    char *lds_c = reinterpret_cast<char *>(lds);
    const int zero_rel = a.stage_bytes - 16;
    const int dwf_off = (a.stages * a.stage_bytes + 255) & ~255;

    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lp = lane & 15, lq = lane >> 4;

    // workgroup -> (plane group, tile of the tile group), tiles fastest: neighbours share halo rows in L2
    const int wg = (int)xcd_contiguous(blockIdx.x, gridDim.x);
    const int grp = a.dMt.div(wg);
    const int m_tile = wg - grp * a.n_mtiles;
    const int m0 = m_tile * a.tile_px;
    const size_t planeA = (size_t)a.HW * 64, planeO = (size_t)a.HWo * 64;
    const size_t imgA = (size_t)a.nCb * planeA, imgO = (size_t)a.nCb * planeO;
    int row_lo, row_hi;
    tile_rows(m0, a.tile_px, a.GHW, a.HWo, a.Wo, a.H, a.stride, a.pt, row_lo, row_hi);

    // ---- load descriptors of a step, relative to the first image of the tile group and to the channel block.
    // Chunks past the tile's rows repeat its last row.
    unsigned d_voff[LPS];
    unsigned d_lds[LPS];
    const int n_chunks = (a.stage_bytes - 16) / 1024;
#pragma unroll
    for (int j = 0; j < LPS; ++j) {
        const int chunk = min(j * NW + wave, n_chunks - 1);
        const int e = chunk * 16 + (lane >> 2);
        const int quad = (lane & 3) ^ ((e >> 1) & 3);
        const int er = a.dW.div(e);
        const int R = min(row_lo + er, row_hi), col = e - er * a.W;
        const int img = a.dH.div(R), row = R - img * a.H;
        d_voff[j] = (unsigned)(img * imgA) + (unsigned)(((row * a.W + col) * 16 + quad * 4) * 4);
        d_lds[j] = __builtin_amdgcn_readfirstlane((unsigned)(chunk * 1024));
    }

    // ---- this lane's pixels: tap addresses in a stage, output offsets
    unsigned p_addr[PXL][9];
    unsigned o_off[PXL];
    bool o_ok[PXL];
    const int m_end = min(m0 + a.tile_px, a.GHW);
#pragma unroll
    for (int i = 0; i < PXL; ++i) {
        const int px = i * 64 + wave * 16 + lp;
        o_ok[i] = m0 + px < m_end;
        const int f = min(m0 + px, m_end - 1);
        const int img = a.dHWo.div(f), pix = f - img * a.HWo;
        const int oh = a.dWo.div(pix), ow = pix - oh * a.Wo;
        o_off[i] = (unsigned)(img * imgO) + (unsigned)((pix * 16 + lq * 4) * 4);
#pragma unroll
        for (int y = 0; y < 3; ++y)
#pragma unroll
            for (int x = 0; x < 3; ++x) {
                const int ir = oh * a.stride + y - a.pt, ic = ow * a.stride + x - a.pl;
                const bool ok = (unsigned)ir < (unsigned)a.H && (unsigned)ic < (unsigned)a.W;
                const int e = (img * a.H + ir - row_lo) * a.W + ic;
                p_addr[i][y * 3 + x] = ok ? (unsigned)((e * 4 + (lq ^ ((e >> 1) & 3))) * 16) : (unsigned)zero_rel;
            }
    }
    const unsigned w_addr = (unsigned)(dwf_off + lq * 16);

    // ---- issue side of the input pipeline. Plane q: channel block q % nCb of tile group q / nCb, which covers
    // images first_image .. + ipt - 1
    const char *in_c = reinterpret_cast<const char *>(a.in);
    char *out_c = reinterpret_cast<char *>(a.out);
    auto first_image = [&](int ig) __attribute__((always_inline)) { return min(ig * a.ipt, a.N - a.ipt); };
    int i_q = grp, i_slot = 0, ahead = 0;
    auto issue_step = [&]() __attribute__((always_inline)) {
        const int ig = a.dCb.div(i_q), cb = i_q - ig * a.nCb;
        const char *base = in_c + (size_t)first_image(ig) * imgA + (size_t)cb * planeA;
        const unsigned stage_lds = lds_base + (unsigned)(i_slot * a.stage_bytes);
#pragma unroll
        for (int j = 0; j < LPS; ++j) dma16(base, d_voff[j], stage_lds + d_lds[j]);
        ++ahead;
        if (++i_slot == a.stages) i_slot = 0;
        i_q += a.n_groups;
    };
    for (int s = 0; s < a.stages - 1; ++s)
        if (i_q < a.n_planes) issue_step();

    // ---- filter taps of every channel block, zero entries
    {
        const int ndw = a.nCb * 9 * 4;                                   // float4s
        for (int e = tid; e < ndw; e += NT)
            *reinterpret_cast<floatx4 *>(lds_c + dwf_off + e * 16) = reinterpret_cast<const floatx4 *>(a.filt)[e];
        if (tid < a.stages) *reinterpret_cast<floatx4 *>(lds_c + tid * a.stage_bytes + zero_rel) = floatx4{0.f, 0.f, 0.f, 0.f};
        __syncthreads();
    }

    int slot = 0;
    for (int q = grp; q < a.n_planes; q += a.n_groups) {
        // the step to compute has landed once at most the loads of the steps issued after it are outstanding
        // (stores issued in between only make this wait stricter)
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
        if (i_q < a.n_planes) issue_step();                // into the slot that was computed one step ago
        const int ig = a.dCb.div(q), cb = q - ig * a.nCb;
        const char *stage = lds_c + slot * a.stage_bytes;
        const char *wrow = lds_c + w_addr + cb * (9 * 64);
        floatx4 w[9];
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = *reinterpret_cast<const floatx4 *>(wrow + k * 64);
        char *obase = out_c + (size_t)first_image(ig) * imgO + (size_t)cb * planeO;
#pragma unroll
        for (int i = 0; i < PXL; ++i) {
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int k = 0; k < 9; ++k) {
                const floatx4 v = *reinterpret_cast<const floatx4 *>(stage + p_addr[i][k]);
                acc.x = fmaf(v.x, w[k].x, acc.x); acc.y = fmaf(v.y, w[k].y, acc.y);
                acc.z = fmaf(v.z, w[k].z, acc.z); acc.w = fmaf(v.w, w[k].w, acc.w);
            }
            if (a.relu) {
                acc.x = acc.x > 0.f ? acc.x : 0.f; acc.y = acc.y > 0.f ? acc.y : 0.f;
                acc.z = acc.z > 0.f ? acc.z : 0.f; acc.w = acc.w > 0.f ? acc.w : 0.f;
            }
            if (o_ok[i]) __builtin_nontemporal_store(acc, reinterpret_cast<floatx4 *>(obase + o_off[i]));
        }
        if (++slot == a.stages) slot = 0;
    }
}

struct RowsPlan {
    int ipt, GHW, tile_px, n_mtiles, chunks, stage_bytes, stages, lps, pxl;
    size_t lds;
    bool ok;
};

RowsPlan make_plan(const LayerGeom &g)
{
    RowsPlan p = {};
    const int HWo = g.Ho * g.Wo, nCb = g.Ci / 16;
    // pixels per lane: 4 (256-pixel tiles) keeps the halo rows a small part of what is staged
    p.pxl = 4;
    const int TM = 64 * p.pxl;
    p.ipt = HWo * 2 <= TM ? std::max(1, std::min(g.N, TM / HWo)) : 1;
    p.GHW = p.ipt * HWo;
    if (p.GHW <= TM) p.tile_px = p.GHW;                       // whole image(s)
    else if (g.Wo <= TM) {                                    // whole rows, the same number in every tile
        const int rmax = TM / g.Wo, tiles = (g.Ho + rmax - 1) / rmax;
        p.tile_px = ((g.Ho + tiles - 1) / tiles) * g.Wo;
    }
    else p.tile_px = TM;
    p.n_mtiles = (p.GHW + p.tile_px - 1) / p.tile_px;
    int ent = 0;
    for (int m = 0; m < p.n_mtiles; ++m) {
        int lo, hi;
        tile_rows(m * p.tile_px, p.tile_px, p.GHW, HWo, g.Wo, g.H, g.stride, g.pt, lo, hi);
        ent = std::max(ent, (hi - lo + 1) * g.W);
    }
    p.chunks = (ent + 15) / 16;
    p.stage_bytes = p.chunks * 1024 + 16;
    p.lps = (p.chunks + 3) / 4;
    p.lps = p.lps <= 2 ? 2 : p.lps <= 4 ? 4 : p.lps <= 6 ? 6 : 8;
    const size_t fixed = (size_t)nCb * 9 * 64 + 256;
    // ring depth 2 (measured on the layer sweep: a third stage costs a resident workgroup per compute unit and
    // loses more than the deeper prefetch gains)
    const size_t budget = 64 * 1024 - fixed;
    p.stages = (int)std::min<size_t>({(size_t)2, budget / (size_t)p.stage_bytes, (size_t)(63 / p.lps + 1)});
    p.lds = (size_t)((p.stages * p.stage_bytes + 255) & ~255) + (size_t)nCb * 9 * 64;
    p.ok = p.chunks <= 32 && p.stages >= 2;
    return p;
}

template <int PXL, int LPS>
hipError_t launch_cfg(RowsArgs a, const RowsPlan &p, hipStream_t s)
{
    a.ipt = p.ipt;
    a.GHW = p.GHW;
    a.tile_px = p.tile_px;
    a.n_igroups = (a.N + a.ipt - 1) / a.ipt;
    a.n_planes = a.n_igroups * a.nCb;
    a.n_mtiles = p.n_mtiles;
    a.stages = p.stages;
    a.stage_bytes = p.stage_bytes;
    // planes per workgroup: as many workgroups as are resident at once (LDS-limited, at most 8 per compute unit)
    const long resident = device_cus() * std::max<long>(1, std::min<long>(8, (long)(160 * 1024 / p.lds)));
    const long per_wg = std::max<long>(1, ((long)a.n_mtiles * a.n_planes + resident - 1) / resident);
    a.n_groups = (int)((a.n_planes + per_wg - 1) / per_wg);
    a.dW = make_fastdiv(a.W);
    a.dH = make_fastdiv(a.H);
    a.dWo = make_fastdiv(a.Wo);
    a.dHWo = make_fastdiv(a.HWo);
    a.dMt = make_fastdiv(a.n_mtiles);
    a.dCb = make_fastdiv(a.nCb);
    const unsigned grid = (unsigned)((long)a.n_mtiles * a.n_groups);
    hipLaunchKernelGGL((dw16_rows<PXL, LPS>), dim3(grid), dim3(256), p.lds, s, a);
    return hipGetLastError();
}

}  // namespace

bool dw_rows_eligible(const LayerGeom &g)
{
    if (g.Cib != 16 || g.kh != 3 || g.kw != 3 || g.pt >= 3 || g.pl >= 3) return false;
    const bool small_enough = (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 30) &&
                              (size_t)256 * g.Ci * g.H * g.W * 4 < ((size_t)1 << 31) &&
                              (size_t)256 * g.Ci * g.Ho * g.Wo * 4 < ((size_t)1 << 31);
    // below about 40 MB of traffic the kernel is a few microseconds long and the plain LDS-tiled kernel, with more
    // and shorter workgroups, is as fast or faster (measured on the layer sweep)
    const bool large = ((size_t)g.N * g.Ci * g.H * g.W + (size_t)g.N * g.Ci * g.Ho * g.Wo) * 4 >= ((size_t)40 << 20);
    return small_enough && large && make_plan(g).ok;
}

hipError_t launch_dw_rows(const float *in, const float *filt, float *out, const LayerGeom &g, int relu, hipStream_t s)
{
    RowsArgs a = {};
    a.in = in; a.filt = filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.HW = g.H * g.W;
    a.Ho = g.Ho; a.Wo = g.Wo; a.HWo = g.Ho * g.Wo; a.stride = g.stride;
    a.nCb = g.Ci / 16;
    a.pt = g.pt; a.pl = g.pl;
    a.relu = relu;
    const RowsPlan p = make_plan(g);
    if (!p.ok) return hipErrorInvalidValue;
    switch (p.lps) {
        case 2: return launch_cfg<4, 2>(a, p, s);
        case 4: return launch_cfg<4, 4>(a, p, s);
        case 6: return launch_cfg<4, 6>(a, p, s);
        default: return launch_cfg<4, 8>(a, p, s);
    }
}

}  // namespace small
