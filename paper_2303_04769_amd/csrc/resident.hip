// A run of layers in one kernel, one image per workgroup, every tensor between them in LDS.
//
// The small networks of Section "MLPerf:Tiny Inference Models" have activations of a few tens of kilobytes per
// image: 16 x 32 x 32 floats are 64 KB, and a compute unit of this chip has 160 KB of LDS. So a workgroup can
// take one image through a whole run of layers and touch HBM only for the run's input, its last output and the
// filters (which all workgroups share through L2): a first convolution on fewer than 16 input channels, then
// convolutions on 16-channel blocks (with their folded ReLU / residual add, Table 2; a 1x1 projection shortcut
// becomes extra reduction rounds of the convolution it is added to) and depthwise convolutions, closed by an
// average pooling over the whole image + fully connected layer. This is the abstract fused layer of the paper's
// "Conclusion & Future Directions" taken across layers of the partial-reduction class of Table 1, where a pixel tile
// cannot be carried from layer to layer because of the halo: the whole image is the tile. What it removes is
// per-launch cost (ramp, drain, the gap between dependent kernels), which dominates layer-by-layer runs of these
// networks at a batch of a few hundred images.
//
// LDS layout. Every tensor of the run lives in LDS as [C/16][4][rows][pixels][4]: a 16-channel block is split into
// four planes of 4 channels, so that the 16 lanes which read 16 neighbouring pixels' float4 touch 256 contiguous
// bytes (with all 16 channels of a pixel together they would be 64 bytes apart and share LDS banks). Zero-padded
// by as many rows / columns as its consumers' windows reach outside the image (left and right padding share their
// columns, see clear_border), so that the reduction loop reads with no bounds test at all: the address of an input
// value is (tile base) + (tap, input block offset), the second term wave-uniform. The padding of a layer's result
// is cleared by the waves that finish the layer early; a barrier separates layers. Regions are handed out by the
// host from the tensors' lifetimes (first fit); the result of a convolution with a residual add overwrites the
// residual in place when nothing else reads it (each lane reads exactly the elements it then writes), which is
// what lets the 16-channel stage of the residual CNN (three live 70 KB tensors in the table) fit. The top 8 KB
// are the waves' private kilobytes for filter blocks in transit.
//
// Work split. 8 waves (two per SIMD, 256 registers each). A wave takes (output channel block, group of T 16-pixel
// tiles) pairs; per reduction step (input block, tap) it reads T float4 B operands from LDS, takes the step's 4 A
// operands (a 16 x 16 filter block, requested from global memory one round of taps ahead as one coalesced float4
// per lane and transposed through the wave's LDS kilobyte one step ahead) and issues 4 T matrix instructions:
//   A (filter):  lane (p = l % 16, q = l / 16) in MFMA j supplies filt[ci = 4q + j][co = p];
//   B (input):   lane (p, q) supplies channels 4q .. 4q + 3 of pixel p as one float4 (MFMA j takes element j);
//   D (output):  lane (p, q) receives channels 4q .. 4q + 3 of pixel p: the B layout again, stored as one float4.
#include "small_internal.h"

#include <string.h>

namespace small {
namespace {

#ifdef SMALL_RES_TIMING
__device__ unsigned long long g_res_t[2 * 8 * 64];
#define RES_STAMP(slot_) do { if (tblk >= 0 && lane == 0) g_res_t[(tblk * 8 + w) * 64 + (slot_)] = __builtin_readcyclecounter(); } while (0)
#else
#define RES_STAMP(slot_) do { } while (0)
#endif

constexpr int kResWaves = 8;
constexpr int kResThreads = kResWaves * 64;
constexpr int kResLdsBytes = 160 * 1024;
constexpr int kResSlotBytes = kResWaves * 1024;       // per wave: one 16 x 16 filter block in transit
constexpr int kResTensorBytes = kResLdsBytes - kResSlotBytes;
constexpr int kResMaxTaps = 9;
constexpr int kResMaxProj = 4;       // input blocks of a projection shortcut folded into a convolution
constexpr int kResMaxIds = 40;      // logical buffer ids + 2, as the runner numbers them

// A tensor in LDS, in float4 units: element (channel block cb, channels 4q .. 4q + 3, padded pixel x) is at
// off + (4 cb + q) * plane + x.
struct ResTensorDev {
    int off;      // first padded pixel of plane 0
    int Wp;       // padded row length
    int plane;    // padded pixels per plane
    int org;      // index inside a plane of image pixel (0, 0)
};

enum : int { RES_CONV = 0, RES_STEM = 1, RES_HEAD = 2, RES_DW = 3 };
constexpr int kStemMaxK = 40;        // reduction length of a first layer (input channels x taps), 10 steps of 4

struct ResLayerDev {
    int kind;                       // RES_CONV; RES_DW: depthwise convolution (at most 9 taps); RES_STEM: the first
                                    // layer on an input of fewer than 16 channels (LDS holds it as [C][rows][pixels]
                                    // floats); RES_HEAD: average pooling over the whole image + fully connected layer
    int K;                          // STEM: Ci * kh * kw; HEAD: channels
    int Co, Cob;                    // HEAD: outputs and their block
    const float *filt;
    const float *filt2;             // CONV: a 1x1 convolution of a second tensor (in2) summed into the same result:
    ResTensorDev in2;               // the projection shortcut of a residual block as extra reduction rounds
    int nCib2, stride2, win2;       // (nCib2 = 0: none)
    int rows3;                      // CONV with nine taps: they are a 3 x 3 window
    ResTensorDev in, out, res;      // out.off < 0: the run's last layer, the result goes to HBM
    int Wo, HoWo, nCib, nCob, stride, taps;
    int win0;                       // index inside an input plane of the window origin of output pixel (0, 0)
    int epilogue, T, nTg, nGroups;  // nTg: tile groups per output block; nGroups = nCob * nTg
    int tapoff[kResMaxTaps];        // dy * in.Wp + dx
    int oH, oW, opt, opb, opc;      // the output tensor's image size and padding (border clearing)
    FastDiv div_Wo, div_nTg;
};

struct ResArgs {
    const float *in;
    float *out;
    int N, n_layers;
    ResTensorDev src;               // where the run's input goes
    int sH, sW, snCb, spt, spb, spc;
    int in_floats, out_floats;      // floats per image of the run's input and output in HBM
    int stem_in;                    // the input has sC < 16 channels: 0 no, 1 blocked [H][W][sC], 2 plain [sC][H][W]
    int sC;
    FastDiv div_skw;                // STEM: division by the filter width
    int slot;                       // float4 index of the waves' private kilobytes (filter blocks in transit)
    FastDiv div_sW, div_sH, div_sC;
    ResLayerDev layer[kResMaxLayers];
};

typedef const __attribute__((address_space(4))) ResArgs *ResKernArgs;

// Clears the padding of the planes of a tensor (float4 planes of 4 channels, or float planes of one channel for a
// first layer's input): wave w takes planes w, w + 8, ...; no divisions (vector-ALU time is matrix-pipe time
// here). A plane is pt padding rows, H image rows, pb padding rows, every row pc padding pixels followed by W
// pixels, and pc more padding pixels at the very end: the pixel to the right of a row's last one is the next
// row's first padding pixel, so left and right padding share their columns (34 x 33 + 1 instead of 34 x 34 pixels
// for a 32 x 32 image padded by one).
template <typename E>
__device__ __forceinline__ void clear_border(E *tensor, int n_planes, int H, int W, int pt, int pb, int pc, int w, int lane,
                                             int n_waves = kResWaves)
{
    const int Wp = pc + W, plane = (pt + H + pb) * Wp + pc;
    const int top = pt * Wp, bot = pb * Wp + pc;
    const E zero = E{};
    for (int k = w; k < n_planes; k += n_waves) {
        E *t = tensor + k * plane;
        for (int r = lane; r < top; r += 64) t[r] = zero;
        for (int r = lane; r < bot; r += 64) t[(pt + H) * Wp + r] = zero;
        if (pc) {
            for (int row = lane; row < H; row += 64) {
                E *line = t + (pt + row) * Wp;
                for (int x = 0; x < pc; ++x) line[x] = zero;
            }
        }
    }
}

typedef const __attribute__((address_space(1))) floatx4 *GlobalFloat4s;

// Division by a launch constant without a branch: the quotient by multiplication is always computed and a divisor of
// 1 (for which that form has no 32-bit constant) selected afterwards. The two-way form in the shared header turns
// into a branch per use here, and the set-up code of a tile group has a dozen of them.
__device__ __forceinline__ int fdiv(const FastDiv &f, int n)
{
    const unsigned q = __umulhi((unsigned)n, f.magic) >> f.shift;
    return f.d == 1 ? n : (int)q;
}

// Position in a wave's sequence of reduction rounds: (group, input block).
struct Round { int g, cib; };

__device__ __forceinline__ Round next_round(Round r, int nCib, int nGroups)
{
    if (r.cib + 1 < nCib) return Round{r.g, r.cib + 1};
    if (r.g + kResWaves < nGroups) return Round{r.g + kResWaves, 0};
    return r;       // past the wave's last round: the same block again (a request that is never used)
}

// This lane's float4 of tap 0 of the round's filter block (f0: the filter's first float4 of this lane).
template <int TAPS>
__device__ __forceinline__ GlobalFloat4s round_block(GlobalFloat4s f0, Round r, const FastDiv &div_nTg, int nCib)
{
    return f0 + ((size_t)fdiv(div_nTg, r.g) * nCib + r.cib) * (TAPS * 64);
}

// Filter values as they come from memory: a (cob, cib, tap) block is 16 x 16 floats [ci][co]; lane l requests
// float4 l of it (row ci = l / 4, columns 4 (l % 4) ..), one fully coalesced 1 KB request per wave and block.
// The matrix instruction wants lane (p, q) to hold [ci = 4q + j][co = p] for j = 0 .. 3, so a block passes through
// 1 KB of LDS private to the wave: written as float4 with row ci at row 4 (ci % 4) + ci / 4, read back as four
// conflict-free 32-bit reads (rows 4j + q, column p).

// Requests the filter blocks of wave w's first round of layer li (every tap) into ar: issued before the barrier
// that ends the previous layer, so that they are under way while the waves meet.
__device__ __forceinline__ void prefetch_first(ResKernArgs ka, int li, int w, int lane, floatx4 (&ar)[kResMaxTaps])
{
    {
        // the layer's descriptor (four cache lines of kernel arguments) into the scalar cache ahead of its use
        const int touch = ka->layer[li].win2 + ka->layer[li].HoWo + ka->layer[li].tapoff[kResMaxTaps - 1] + (int)ka->layer[li].div_nTg.d;
        asm volatile("" : : "s"(touch));
    }
    if (ka->layer[li].kind != RES_CONV || w >= ka->layer[li].nGroups) return;
    const int taps = ka->layer[li].taps, nCib = ka->layer[li].nCib;
    FastDiv div_nTg;
    div_nTg.magic = ka->layer[li].div_nTg.magic; div_nTg.shift = ka->layer[li].div_nTg.shift; div_nTg.d = ka->layer[li].div_nTg.d;
    const int cob = fdiv(div_nTg, w);
    GlobalFloat4s fa = (GlobalFloat4s)(ka->layer[li].filt + (size_t)cob * nCib * taps * 256) + lane;
    asm volatile("" : "+v"(fa));
    if (taps == kResMaxTaps) {
#pragma unroll
        for (int tap = 0; tap < kResMaxTaps; ++tap) ar[tap] = fa[tap * 64];
    } else {
        ar[0] = fa[0];
    }
}

// ar: on entry the filter blocks of this wave's first round (prefetch_first). Ring entry x > 0 holds tap x of the
// current round until step x - 1 passes it on to LDS, and is then refilled with tap x of the next round; entry 0
// is passed on in a round's last step (for the next round's first) and refilled from the round after that.
// ROWS3: the nine taps are a 3 x 3 window: per round the three row bases of every tile are formed once and the
// column offsets travel as immediates of the LDS reads, instead of one address addition per read.
template <int T, int TAPS, bool ROWS3>
__device__ __forceinline__ void resident_conv(ResKernArgs ka, int li, floatx4 *lds, floatx4 *gout, int w, int lane,
                                              floatx4 (&ar)[kResMaxTaps], int slot)
{
    const int p = lane & 15, q = lane >> 4;
    const float *const filt = ka->layer[li].filt;
    const int in_off = ka->layer[li].in.off, in_Wp = ka->layer[li].in.Wp, in_plane = ka->layer[li].in.plane;
    const int out_off = ka->layer[li].out.off, out_Wp = ka->layer[li].out.Wp, out_plane = ka->layer[li].out.plane,
              out_org = ka->layer[li].out.org;
    const int res_off = ka->layer[li].res.off, res_Wp = ka->layer[li].res.Wp, res_plane = ka->layer[li].res.plane,
              res_org = ka->layer[li].res.org;
    const int Wo = ka->layer[li].Wo, HoWo = ka->layer[li].HoWo, nCib = ka->layer[li].nCib, stride = ka->layer[li].stride;
    const int win0 = ka->layer[li].win0, epilogue = ka->layer[li].epilogue;
    const int nTg = ka->layer[li].nTg, nGroups = ka->layer[li].nGroups;
    const int nCib2 = ka->layer[li].nCib2, stride2 = ka->layer[li].stride2, win2 = ka->layer[li].win2;
    const int in2_off = ka->layer[li].in2.off, in2_Wp = ka->layer[li].in2.Wp, in2_plane = ka->layer[li].in2.plane;
    const float *const filt2 = ka->layer[li].filt2;
    FastDiv div_Wo, div_nTg;
    div_Wo.magic = ka->layer[li].div_Wo.magic; div_Wo.shift = ka->layer[li].div_Wo.shift; div_Wo.d = ka->layer[li].div_Wo.d;
    div_nTg.magic = ka->layer[li].div_nTg.magic; div_nTg.shift = ka->layer[li].div_nTg.shift; div_nTg.d = ka->layer[li].div_nTg.d;
    int tapoff[TAPS];
#pragma unroll
    for (int t = 0; t < TAPS; ++t) tapoff[t] = ka->layer[li].tapoff[t];
    if (w >= nGroups) return;

    // the wave's LDS kilobyte: where this lane writes its float4 of a block, where it reads its four values
    floatx4 *const slot_w = lds + slot + w * 64 + (((lane >> 2) & 3) * 4 + (lane >> 4)) * 4 + (lane & 3);
    const float *const slot_r = reinterpret_cast<const float *>(lds + slot + w * 64) + q * 16 + p;
    const GlobalFloat4s f0 = (GlobalFloat4s)filt + lane;

    // the first step's filter values
    float a_cur[4];
    {
        *slot_w = ar[0];
#pragma unroll
        for (int j = 0; j < 4; ++j) a_cur[j] = slot_r[j * 64];
        GlobalFloat4s p1 = round_block<TAPS>(f0, next_round(Round{w, 0}, nCib, nGroups), div_nTg, nCib);
        asm volatile("" : "+v"(p1));
        ar[0] = p1[0];
    }

    // A wave's next group often is the same tiles a whole number of image rows further down (same output block, no
    // ragged tile): its indices then follow from the previous group's by additions.
    constexpr int kStepPixels = kResWaves * T * 16;
    const int step_rows = fdiv(div_Wo, kStepPixels);
    const bool by_rows = step_rows * Wo == kStepPixels;
    const int d_base = step_rows * stride * in_Wp, d_base2 = step_rows * stride2 * in2_Wp, d_res = step_rows * res_Wp;
    const int d_out = out_off >= 0 ? step_rows * out_Wp : kStepPixels * 4;
    int base[T], base2[T], m[T], o_at[T], r_at[T];   // where the tile's values are read, stored, the residual read
    bool inside_before = false;
    for (int g = w; g < nGroups; g += kResWaves) {
        // Index arithmetic and stores of one wave compete with the matrix instructions of the wave that shares its
        // SIMD, and lose: without a higher priority a wave's set-up takes several times longer, and the two waves
        // end up running their reduction loops one after the other instead of side by side.
        __builtin_amdgcn_s_setprio(3);
        const int cob = fdiv(div_nTg, g), tg = g - cob * nTg;
        // a folded projection: its filter blocks of this output block, requested now, used after the main rounds
        floatx4 proj[kResMaxProj];
        if (nCib2) {
            GlobalFloat4s f2 = (GlobalFloat4s)filt2 + (size_t)cob * nCib2 * 64 + lane;
#pragma unroll
            for (int c = 0; c < kResMaxProj; ++c) proj[c] = f2[(c < nCib2 ? c : 0) * 64];
        }
        const bool inside = (tg * T + T) * 16 <= HoWo;
        const bool step = g != w && by_rows && inside_before && inside && tg >= kResWaves;
        inside_before = inside;
        if (step) {
#pragma unroll
            for (int t = 0; t < T; ++t) {
                base[t] += d_base; base2[t] += d_base2; m[t] += kStepPixels; o_at[t] += d_out; r_at[t] += d_res;
            }
        } else
#pragma unroll
        for (int t = 0; t < T; ++t) {
            m[t] = (tg * T + t) * 16 + p;
            const int mc = m[t] < HoWo ? m[t] : HoWo - 1;
            const int oy = fdiv(div_Wo, mc), ox = mc - oy * Wo;
            base[t] = in_off + q * in_plane + win0 + oy * stride * in_Wp + ox * stride;
            base2[t] = in2_off + q * in2_plane + win2 + oy * stride2 * in2_Wp + ox * stride2;
            {
                // (a select by mask: as a two-way expression this becomes a branch per tile)
                const int gm = out_off >> 31;        // all ones when the result goes to HBM
                const int o_lds = out_off + (cob * 4 + q) * out_plane + out_org + oy * out_Wp + ox, o_glb = (cob * HoWo + mc) * 4 + q;
                o_at[t] = (o_lds & ~gm) | (o_glb & gm);
            }
            r_at[t] = res_off + (cob * 4 + q) * res_plane + res_org + oy * res_Wp + ox;
        }
        floatx4 acc[T], b[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
            b[t] = lds[base[t] + tapoff[0]];
        }
        __builtin_amdgcn_s_setprio(0);

        for (int cib = 0; cib < nCib; ++cib) {
            const int coff = cib * 4 * in_plane;
            const Round r1 = next_round(Round{g, cib}, nCib, nGroups), r2 = next_round(r1, nCib, nGroups);
            // the compiler must not see that these are the addresses later rounds read: it would turn the requests
            // made a round ahead into requests made at the point of use
            GlobalFloat4s p1 = round_block<TAPS>(f0, r1, div_nTg, nCib), p2 = round_block<TAPS>(f0, r2, div_nTg, nCib);
            asm volatile("" : "+v"(p1), "+v"(p2));
            int rowb[T][3];
            if (ROWS3) {
#pragma unroll
                for (int t = 0; t < T; ++t)
#pragma unroll
                    for (int r = 0; r < 3; ++r) rowb[t][r] = base[t] + coff + r * in_Wp;
            }
#pragma unroll
            for (int tap = 0; tap < TAPS; ++tap) {
                constexpr int kLast = TAPS - 1;
                const int x = tap == kLast ? 0 : tap + 1;
                // the next step's operands: its filter block through the wave's LDS kilobyte, its input values
                float a_nxt[4];
                floatx4 b_nxt[T];
                *slot_w = ar[x];
#pragma unroll
                for (int j = 0; j < 4; ++j) a_nxt[j] = slot_r[j * 64];
                ar[x] = x ? p1[x * 64] : p2[0];
                if (tap < kLast) {
                    if (ROWS3) {
#pragma unroll
                        for (int t = 0; t < T; ++t) b_nxt[t] = lds[rowb[t][(tap + 1) / 3] + (tap + 1) % 3];
                    } else {
#pragma unroll
                        for (int t = 0; t < T; ++t) b_nxt[t] = lds[base[t] + coff + tapoff[tap + 1]];
                    }
                } else if (cib + 1 < nCib) {
#pragma unroll
                    for (int t = 0; t < T; ++t) b_nxt[t] = lds[base[t] + coff + 4 * in_plane + tapoff[0]];
                } else {
#pragma unroll
                    for (int t = 0; t < T; ++t) b_nxt[t] = b[t];      // the group ends: the next one reads its own
                }
                __builtin_amdgcn_sched_barrier(0);     // the requests above stay ahead of the arithmetic below
#pragma unroll
                for (int j = 0; j < 4; ++j)
#pragma unroll
                    for (int t = 0; t < T; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a_cur[j], b[t][j], acc[t], 0, 0, 0);
#pragma unroll
                for (int j = 0; j < 4; ++j) a_cur[j] = a_nxt[j];
#pragma unroll
                for (int t = 0; t < T; ++t) b[t] = b_nxt[t];
            }
        }

        if (nCib2) {
            // a_cur holds the next group's first filter values by now: the projection takes registers of its own
#pragma unroll
            for (int c = 0; c < kResMaxProj; ++c) {
                if (c < nCib2) {
                    float a2[4];
                    floatx4 b2[T];
                    *slot_w = proj[c];
#pragma unroll
                    for (int j = 0; j < 4; ++j) a2[j] = slot_r[j * 64];
#pragma unroll
                    for (int t = 0; t < T; ++t) b2[t] = lds[base2[t] + c * 4 * in2_plane];
#pragma unroll
                    for (int j = 0; j < 4; ++j)
#pragma unroll
                        for (int t = 0; t < T; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(a2[j], b2[t][j], acc[t], 0, 0, 0);
                }
            }
        }
        __builtin_amdgcn_s_setprio(3);
#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (m[t] >= HoWo) continue;
            floatx4 v = acc[t];
            if (epilogue & EPI_ADD) v += lds[r_at[t]];
            if (epilogue & EPI_RELU) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
            }
            if (out_off >= 0) lds[o_at[t]] = v;
            else gout[o_at[t]] = v;
        }
    }
}

// The first layer: an input of fewer than 16 channels, held in LDS as zero-padded [C][rows][pixels] floats. The
// reduction runs over k = tap * C + ci (the order of the filter's [kh][kw][Cib] dimensions) in steps of 4: lane
// (p, q) supplies filt[k = 4t + q][co = p] and the input value of pixel p for that k, whose offset inside the tensor
// follows from (ci, dy, dx). Four 16-pixel tiles at a time. fa: the filter values of the wave's first group
// (stem_filter), requested before the image arrives.
constexpr int kStemSteps = kStemMaxK / 4;

__device__ __forceinline__ void stem_filter(ResKernArgs ka, int cob, int lane, float (&fa)[kStemSteps])
{
    const int p = lane & 15, q = lane >> 4, K = ka->layer[0].K;
    const float *const filt = ka->layer[0].filt;
#pragma unroll
    for (int t = 0; t < kStemSteps; ++t) fa[t] = 4 * t + q < K ? filt[((size_t)cob * K + 4 * t + q) * 16 + p] : 0.f;
}

__device__ __forceinline__ void resident_stem(ResKernArgs ka, floatx4 *lds, floatx4 *gout, int w, int lane,
                                              float (&fa)[kStemSteps])
{
    constexpr int li = 0, kSteps = kStemSteps, T = 4;
    const int p = lane & 15, q = lane >> 4;
    const int K = ka->layer[li].K, steps = (K + 3) >> 2;
    const int in_off = ka->layer[li].in.off, in_Wp = ka->layer[li].in.Wp, in_plane = ka->layer[li].in.plane;
    const int out_off = ka->layer[li].out.off, out_Wp = ka->layer[li].out.Wp, out_plane = ka->layer[li].out.plane,
              out_org = ka->layer[li].out.org;
    const int Wo = ka->layer[li].Wo, HoWo = ka->layer[li].HoWo, stride = ka->layer[li].stride, win0 = ka->layer[li].win0;
    const int epilogue = ka->layer[li].epilogue, nTg = ka->layer[li].nTg, nGroups = ka->layer[li].nGroups;
    FastDiv div_Wo, div_nTg;
    div_Wo.magic = ka->layer[li].div_Wo.magic; div_Wo.shift = ka->layer[li].div_Wo.shift; div_Wo.d = ka->layer[li].div_Wo.d;
    div_nTg.magic = ka->layer[li].div_nTg.magic; div_nTg.shift = ka->layer[li].div_nTg.shift; div_nTg.d = ka->layer[li].div_nTg.d;
    const float *const ldsf = reinterpret_cast<const float *>(lds) + in_off * 4;
    FastDiv div_C, div_kw;
    div_C.magic = ka->div_sC.magic; div_C.shift = ka->div_sC.shift; div_C.d = ka->div_sC.d;
    div_kw.magic = ka->div_skw.magic; div_kw.shift = ka->div_skw.shift; div_kw.d = ka->div_skw.d;
    const int sC = ka->sC, kw = (int)div_kw.d;
    int koff[kSteps];
#pragma unroll
    for (int t = 0; t < kSteps; ++t) {
        const int k = 4 * t + q, tap = fdiv(div_C, k), ci = k - tap * sC, dy = fdiv(div_kw, tap), dx = tap - dy * kw;
        koff[t] = k < K ? ci * in_plane + dy * in_Wp + dx : 0;
    }

    __builtin_amdgcn_s_setprio(3);
    if (w >= nGroups) return;
    int cob_held = fdiv(div_nTg, w);
    for (int g = w; g < nGroups; g += kResWaves) {
        const int cob = fdiv(div_nTg, g), tg = g - cob * nTg;
        if (cob != cob_held) {
            stem_filter(ka, cob, lane, fa);
            cob_held = cob;
        }
        int base[T], m[T], o_at[T];
#pragma unroll
        for (int t = 0; t < T; ++t) {
            m[t] = (tg * T + t) * 16 + p;
            const int mc = m[t] < HoWo ? m[t] : HoWo - 1;
            const int oy = fdiv(div_Wo, mc), ox = mc - oy * Wo;
            base[t] = win0 + oy * stride * in_Wp + ox * stride;
            {
                // (a select by mask: as a two-way expression this becomes a branch per tile)
                const int gm = out_off >> 31;        // all ones when the result goes to HBM
                const int o_lds = out_off + (cob * 4 + q) * out_plane + out_org + oy * out_Wp + ox, o_glb = (cob * HoWo + mc) * 4 + q;
                o_at[t] = (o_lds & ~gm) | (o_glb & gm);
            }
        }
        floatx4 acc[T];
#pragma unroll
        for (int t = 0; t < T; ++t) acc[t] = floatx4{0.f, 0.f, 0.f, 0.f};
        // every input value of the group is requested before the first matrix instruction (steps past the
        // reduction read offset 0 and meet a zero filter value): one LDS latency per group, not one per step
        float b[kSteps][T];
#pragma unroll
        for (int k = 0; k < kSteps; ++k)
#pragma unroll
            for (int t = 0; t < T; ++t) b[k][t] = ldsf[base[t] + koff[k]];
        __builtin_amdgcn_sched_barrier(0);
#pragma unroll
        for (int k = 0; k < kSteps; ++k) {
            if (k < steps) {
#pragma unroll
                for (int t = 0; t < T; ++t) acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(fa[k], b[k][t], acc[t], 0, 0, 0);
            }
        }
#pragma unroll
        for (int t = 0; t < T; ++t) {
            if (m[t] >= HoWo) continue;
            floatx4 v = acc[t];
            if (epilogue & EPI_RELU) {
#pragma unroll
                for (int r = 0; r < 4; ++r) v[r] = v[r] > 0.f ? v[r] : 0.f;
            }
            if (out_off >= 0) lds[o_at[t]] = v;
            else gout[o_at[t]] = v;
        }
    }
}

// Depthwise convolution (Table 1's layer class with one filter per channel; at most 9 taps): plain vector
// arithmetic, a four-channel plane per wave at a time, a lane per output pixel; the plane's filter values (one
// float4 per tap) are the same for the whole wave.
__device__ __forceinline__ void resident_dw(ResKernArgs ka, int li, floatx4 *lds, floatx4 *gout, int w, int lane)
{
    const float *const filt = ka->layer[li].filt;
    const int in_off = ka->layer[li].in.off, in_Wp = ka->layer[li].in.Wp, in_plane = ka->layer[li].in.plane;
    const int out_off = ka->layer[li].out.off, out_Wp = ka->layer[li].out.Wp, out_plane = ka->layer[li].out.plane,
              out_org = ka->layer[li].out.org;
    const int Wo = ka->layer[li].Wo, HoWo = ka->layer[li].HoWo, nCb = ka->layer[li].nCob, stride = ka->layer[li].stride;
    const int win0 = ka->layer[li].win0, epilogue = ka->layer[li].epilogue, taps = ka->layer[li].taps;
    FastDiv div_Wo;
    div_Wo.magic = ka->layer[li].div_Wo.magic; div_Wo.shift = ka->layer[li].div_Wo.shift; div_Wo.d = ka->layer[li].div_Wo.d;
    int tapoff[kResMaxTaps];
#pragma unroll
    for (int t = 0; t < kResMaxTaps; ++t) tapoff[t] = t < taps ? ka->layer[li].tapoff[t] : 0;
    __builtin_amdgcn_s_setprio(3);
    for (int k = w; k < nCb * 4; k += kResWaves) {
        const int cb = k >> 2, qq = k & 3;
        floatx4 f[kResMaxTaps];
#pragma unroll
        for (int t = 0; t < kResMaxTaps; ++t)
            f[t] = t < taps ? *reinterpret_cast<const floatx4 *>(filt + ((size_t)(cb * taps + t) * 16 + 4 * qq))
                            : floatx4{0.f, 0.f, 0.f, 0.f};
        for (int m = lane; m < HoWo; m += 64) {
            const int oy = fdiv(div_Wo, m), ox = m - oy * Wo;
            const int src = in_off + k * in_plane + win0 + oy * stride * in_Wp + ox * stride;
            floatx4 acc = floatx4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int t = 0; t < kResMaxTaps; ++t) acc += lds[src + tapoff[t]] * f[t];
            if (epilogue & EPI_RELU) {
#pragma unroll
                for (int r = 0; r < 4; ++r) acc[r] = acc[r] > 0.f ? acc[r] : 0.f;
            }
            if (out_off >= 0) lds[out_off + k * out_plane + out_org + oy * out_Wp + ox] = acc;
            else gout[(cb * HoWo + m) * 4 + qq] = acc;
        }
    }
}

// Average pooling over the whole image + fully connected layer on the run's last tensor. Pooling: a thread takes
// one channel and a quarter of the pixels (independent LDS reads, no long shuffle chain), the four quarters meet by
// two quad shuffles, the means go to LDS (`scratch`, 64 float4). Dot products: 16 lanes over the outputs x 32 parts
// over the channels, the filter values requested before the pooling starts; summed across the four parts of a wave
// by shuffles and across the waves through LDS.
__device__ __forceinline__ void resident_head(ResKernArgs ka, int li, floatx4 *lds, float *gout, int scratch, int w, int lane)
{
    constexpr int kParts = kResThreads / 16, kMaxPer = 256 / kParts;       // channels per part: at most 8
    const int in_off = ka->layer[li].in.off, in_Wp = ka->layer[li].in.Wp, in_plane = ka->layer[li].in.plane,
              in_org = ka->layer[li].in.org;
    const int W = ka->layer[li].Wo, HW = ka->layer[li].HoWo, nCib = ka->layer[li].nCib, C = nCib * 16;
    const int Co = ka->layer[li].Co, Cob = ka->layer[li].Cob;
    const float *const filt = ka->layer[li].filt;
    FastDiv div_W;
    div_W.magic = ka->layer[li].div_Wo.magic; div_W.shift = ka->layer[li].div_Wo.shift; div_W.d = ka->layer[li].div_Wo.d;

    const int co = lane & 15, part = (int)threadIdx.x >> 4;
    float fv[kMaxPer];
    {
        const int cob = co < Co ? co / Cob : 0, cc = co < Co ? co - cob * Cob : 0;
#pragma unroll
        for (int k = 0; k < kMaxPer; ++k) {
            const int c = part + k * kParts;
            fv[k] = (co < Co && c < C) ? filt[((size_t)(cob * nCib + (c >> 4)) * 16 + (c & 15)) * Cob + cc] : 0.f;
        }
    }

    const float *t = reinterpret_cast<const float *>(lds + in_off);
    float *mean = reinterpret_cast<float *>(lds + scratch);
    const float inv = 1.0f / (float)HW;
    for (int idx = (int)threadIdx.x; idx < C * 4; idx += kResThreads) {
        const int c = idx >> 2, quarter = idx & 3;            // channel c = 4 plane + element
        const float *src = t + ((c >> 2) * in_plane + in_org) * 4 + (c & 3);
        float sum = 0.f;
        for (int m = quarter; m < HW; m += 4) {
            const int y = fdiv(div_W, m), x = m - y * W;
            sum += src[(y * in_Wp + x) * 4];
        }
        sum += __shfl_xor(sum, 1, 64);
        sum += __shfl_xor(sum, 2, 64);
        if (quarter == 0) mean[c] = sum * inv;
    }
    __syncthreads();
    float *partial = mean + 256;
    float acc = 0.f;
#pragma unroll
    for (int k = 0; k < kMaxPer; ++k) {
        const int c = part + k * kParts;
        if (c < C) acc += mean[c] * fv[k];
    }
    acc += __shfl_xor(acc, 16, 64);
    acc += __shfl_xor(acc, 32, 64);
    if (lane < 16) partial[w * 16 + lane] = acc;
    __syncthreads();
    if ((int)threadIdx.x < Co) {
        float sum = 0.f;
#pragma unroll
        for (int k = 0; k < kResWaves; ++k) sum += partial[k * 16 + (int)threadIdx.x];
        gout[threadIdx.x] = sum;
    }
}

// One workgroup per compute unit (LDS): two waves per SIMD, 256 vector registers each.
__global__ void __launch_bounds__(kResThreads) __attribute__((amdgpu_waves_per_eu(2, 2))) resident_run(ResArgs args)
{
    (void)args;
    const ResKernArgs ka = (ResKernArgs)__builtin_amdgcn_kernarg_segment_ptr();
    extern __shared__ floatx4 lds[];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
    const int N = ka->N, n_layers = ka->n_layers, in_floats = ka->in_floats, out_floats = ka->out_floats;
    const int stem_in = ka->stem_in, sC = ka->sC;
    const int s_off = ka->src.off, s_Wp = ka->src.Wp, s_plane = ka->src.plane, s_org = ka->src.org;
    const int sH = ka->sH, sW = ka->sW;
    FastDiv div_sW, div_sH;
    div_sW.magic = ka->div_sW.magic; div_sW.shift = ka->div_sW.shift; div_sW.d = ka->div_sW.d;
    div_sH.magic = ka->div_sH.magic; div_sH.shift = ka->div_sH.shift; div_sH.d = ka->div_sH.d;

#ifdef SMALL_RES_TIMING
    const int tblk = blockIdx.x == 0 ? 0 : (blockIdx.x == 100 ? 1 : -1);
#endif
    RES_STAMP(0);
    const int slot = ka->slot;
    floatx4 a_pre[kResMaxTaps];
#pragma unroll
    for (int tap = 0; tap < kResMaxTaps; ++tap) a_pre[tap] = floatx4{0.f, 0.f, 0.f, 0.f};
    if ((int)blockIdx.x < N) prefetch_first(ka, 0, w, lane, a_pre);
    for (int n = (int)blockIdx.x; n < N; n += (int)gridDim.x) {
        // the image's input tensor: HBM -> its padded place in LDS
        float stem_fa[kStemSteps];
        if (stem_in) {
            // the first layer's filter values of this wave's first group, under way while the image arrives
            if (w < ka->layer[0].nGroups) {
                FastDiv d0;
                d0.magic = ka->layer[0].div_nTg.magic; d0.shift = ka->layer[0].div_nTg.shift; d0.d = ka->layer[0].div_nTg.d;
                stem_filter(ka, fdiv(d0, w), lane, stem_fa);
            }
            // fewer than 16 channels, blocked [y][x][c] or plain [c][y][x]: float planes [c][rows][pixels] in LDS
            const float *gin = ka->in + (size_t)n * in_floats;
            float *t = reinterpret_cast<float *>(lds + s_off);
            FastDiv div_sC;
            div_sC.magic = ka->div_sC.magic; div_sC.shift = ka->div_sC.shift; div_sC.d = ka->div_sC.d;
#pragma unroll 4
            for (int i = (int)threadIdx.x; i < in_floats; i += kResThreads) {
                int c, y, x;
                if (stem_in == 2) {
                    const int row = fdiv(div_sW, i);          // c * H + y
                    x = i - row * sW;
                    c = fdiv(div_sH, row);
                    y = row - c * sH;
                } else {
                    const int pixel = fdiv(div_sC, i);
                    c = i - pixel * sC;
                    y = fdiv(div_sW, pixel);
                    x = pixel - y * sW;
                }
                t[c * s_plane + s_org + y * s_Wp + x] = gin[i];
            }
            clear_border(t, sC, sH, sW, ka->spt, ka->spb, ka->spc, w, lane);
        } else {
            const floatx4 *gin = reinterpret_cast<const floatx4 *>(ka->in + (size_t)n * in_floats);
#pragma unroll 4
            for (int i = (int)threadIdx.x; i < (in_floats >> 2); i += kResThreads) {
                const int pixel = i >> 2;
                const int cbrow = fdiv(div_sW, pixel), x = pixel - cbrow * sW;
                const int cb = fdiv(div_sH, cbrow), y = cbrow - cb * sH;
                lds[s_off + (cb * 4 + (i & 3)) * s_plane + s_org + y * s_Wp + x] = gin[i];
            }
            clear_border(lds + s_off, ka->snCb * 4, sH, sW, ka->spt, ka->spb, ka->spc, w, lane);
        }
        __syncthreads();
        RES_STAMP(1);

        float *gout_f = ka->out + (size_t)n * out_floats;
        floatx4 *gout = reinterpret_cast<floatx4 *>(gout_f);
        for (int li = 0; li < n_layers; ++li) {
            // (a_pre holds this wave's first filter values of layer li)
            const int T = ka->layer[li].T, taps = ka->layer[li].taps, kind = ka->layer[li].kind;
            RES_STAMP(2 + 4 * li);
            // The padding of the result is cleared by the upper four waves BEFORE they start on the layer (nobody
            // reads or writes it during the layer): the two waves of a SIMD then run half a set-up apart, and one's
            // set-up and store phases fall into the other's matrix loop instead of coinciding with its own.
            
            if (kind == RES_STEM) {
                resident_stem(ka, lds, gout, w, lane, stem_fa);
            } else if (kind == RES_HEAD) {
                resident_head(ka, li, lds, gout_f, slot, w, lane);
            } else if (kind == RES_DW) {
                resident_dw(ka, li, lds, gout, w, lane);
            } else if (taps == 9 && ka->layer[li].rows3) {
                if (T == 4) resident_conv<4, 9, true>(ka, li, lds, gout, w, lane, a_pre, slot);
                else if (T == 2) resident_conv<2, 9, true>(ka, li, lds, gout, w, lane, a_pre, slot);
                else resident_conv<1, 9, true>(ka, li, lds, gout, w, lane, a_pre, slot);
            } else if (taps == 9) {
                resident_conv<1, 9, false>(ka, li, lds, gout, w, lane, a_pre, slot);      // (1 x 9, 9 x 1: one tile at a time)
            } else {
                if (T == 4) resident_conv<4, 1, false>(ka, li, lds, gout, w, lane, a_pre, slot);
                else if (T == 2) resident_conv<2, 1, false>(ka, li, lds, gout, w, lane, a_pre, slot);
                else resident_conv<1, 1, false>(ka, li, lds, gout, w, lane, a_pre, slot);
            }
            RES_STAMP(3 + 4 * li);
            // the padding of the result (nobody reads it before the barrier; a wave that is done early does this
            // while the others still compute)
            if (kind != RES_HEAD && ka->layer[li].out.off >= 0)
                clear_border(lds + ka->layer[li].out.off, ka->layer[li].nCob * 4, ka->layer[li].oH, ka->layer[li].oW,
                             ka->layer[li].opt, ka->layer[li].opb, ka->layer[li].opc, w, lane);
            if (li + 1 < n_layers) prefetch_first(ka, li + 1, w, lane, a_pre);
            else if (n + (int)gridDim.x < N) prefetch_first(ka, 0, w, lane, a_pre);
            RES_STAMP(4 + 4 * li);
            __syncthreads();   // the layer's output is complete, its input may be overwritten
            RES_STAMP(5 + 4 * li);
            }
    }
}

// ------------------------------------------------------------------------------------------------ host side

struct Pads { int t, b, l, r; };

struct Instance {          // one tensor of the run
    int C, H, W;
    bool planar;           // a first layer's input: [C][rows][pixels] floats instead of four-channel float4 planes
    Pads pad;
    int last_use;          // last group that reads it (-1: none)
    int off, bytes;        // LDS region
};

inline int imax(int a, int b) { return a > b ? a : b; }

// First fit over the regions in use (at most a handful).
int first_fit(const int (*used)[2], int n_used, int bytes, int capacity)
{
    int at = 0;
    for (;;) {
        bool moved = false;
        for (int k = 0; k < n_used; ++k) {
            if (at < used[k][0] + used[k][1] && used[k][0] < at + bytes) {
                at = used[k][0] + used[k][1];
                moved = true;
            }
        }
        if (!moved) break;
    }
    return at + bytes <= capacity ? at : -1;
}

bool group_ok(const ResGroup &g, int position)
{
    const int taps = g.kh * g.kw;
    const bool ids = g.src + 2 >= 0 && g.src + 2 < kResMaxIds && g.dst + 2 >= 0 && g.dst + 2 < kResMaxIds &&
                     (!(g.epilogue & EPI_ADD) || (g.res + 2 >= 0 && g.res + 2 < kResMaxIds));
    if (!ids || !g.filt || g.Ci <= 0 || g.Co <= 0 || g.Ho <= 0 || g.Wo <= 0) return false;
    if (g.kind == RESIDENT_STEM)
        return position == 0 && g.Ci < 16 && g.Cib == g.Ci && g.Cob == 16 && g.Co % 16 == 0 && g.Ci * taps <= kStemMaxK &&
               taps >= 1 && g.stride >= 1 && g.pt >= 0 && g.pl >= 0 && !(g.epilogue & EPI_ADD);
    if (g.kind == RESIDENT_DW)
        return g.Cib == 16 && g.Cob == 16 && g.Ci == g.Co && g.Ci % 16 == 0 && taps >= 1 && taps <= kResMaxTaps &&
               g.stride >= 1 && g.pt >= 0 && g.pl >= 0 && !(g.epilogue & EPI_ADD) && ((uintptr_t)g.filt & 15u) == 0;
    if (g.kind == RESIDENT_HEAD)
        return position > 0 && g.Cib == 16 && g.Ci % 16 == 0 && g.Ci <= 256 && g.Co <= 16 && g.Cob > 0 && g.Co % g.Cob == 0 &&
               g.kh == g.H && g.kw == g.W && g.pt == 0 && g.pl == 0 && g.Ho == 1 && g.Wo == 1 && g.epilogue == EPI_NONE;
    return g.Cib == 16 && g.Cob == 16 && g.Ci % 16 == 0 && g.Co % 16 == 0 && (taps == 1 || taps == 9) && g.stride >= 1 &&
           g.pt >= 0 && g.pl >= 0;
}

// Plans groups [0, n) as one run; false when a tensor is read that the run does not hold, or LDS does not fit.
bool plan_prefix(const ResGroup *g_in, int n_in, ResArgs &a, int &lds_bytes)
{
    // A 1x1 convolution that is added onto the result of the convolution before it (the projection shortcut of a
    // residual block: y = relu(conv3x3(a) + conv1x1(x))) becomes extra reduction rounds of that convolution: one
    // pass over the layer, and the tensor between the two is never formed.
    ResGroup g[kResMaxLayers];
    const ResGroup *pj[kResMaxLayers];
    int n = 0;
    for (int k = 0; k < n_in; ++k) {
        g[n] = g_in[k];
        pj[n] = nullptr;
        if (k + 1 < n_in) {
            const ResGroup &c = g_in[k], &s2 = g_in[k + 1];
            if (c.kind == RESIDENT_CONV && s2.kind == RESIDENT_CONV && c.epilogue == EPI_NONE && (s2.epilogue & EPI_ADD) &&
                s2.kh * s2.kw == 1 && s2.pt == 0 && s2.pl == 0 && s2.res == c.dst && s2.dst == c.dst && s2.src != c.dst &&
                s2.Co == c.Co && s2.Ho == c.Ho && s2.Wo == c.Wo && s2.Ci % 16 == 0 && s2.Ci / 16 <= kResMaxProj && s2.filt) {
                pj[n] = &s2;
                g[n].epilogue = s2.epilogue & ~EPI_ADD;
                ++k;
            }
        }
        ++n;
    }
    if (n < 1) return false;
    Instance inst[kResMaxLayers + 1];
    int in_i[kResMaxLayers], res_i[kResMaxLayers], out_i[kResMaxLayers], in2_i[kResMaxLayers];
    bool alias[kResMaxLayers];
    int cur[kResMaxIds];
    for (int k = 0; k < kResMaxIds; ++k) cur[k] = -1;
    int n_inst = 1;
    inst[0] = Instance{g[0].Ci, g[0].H, g[0].W, g[0].kind == RESIDENT_STEM, Pads{0, 0, 0, 0}, -1, -1, 0};
    cur[g[0].src + 2] = 0;
    for (int k = 0; k < n; ++k) {
        const ResGroup &c = g[k];
        in_i[k] = cur[c.src + 2];
        res_i[k] = (c.epilogue & EPI_ADD) ? cur[c.res + 2] : -1;
        if (in_i[k] < 0 || ((c.epilogue & EPI_ADD) && res_i[k] < 0)) return false;
        const Instance &x = inst[in_i[k]];
        if (x.C != c.Ci || x.H != c.H || x.W != c.W || x.planar != (c.kind == RESIDENT_STEM)) return false;
        if (c.kind == RESIDENT_HEAD && k + 1 != n) return false;
        if (res_i[k] >= 0 && (inst[res_i[k]].C != c.Co || inst[res_i[k]].H != c.Ho || inst[res_i[k]].W != c.Wo)) return false;
        // rows / columns outside the image that the windows really reach
        Pads &pd = inst[in_i[k]].pad;
        pd.t = imax(pd.t, c.pt);
        pd.l = imax(pd.l, c.pl);
        pd.b = imax(pd.b, (c.Ho - 1) * c.stride - c.pt + c.kh - c.H);
        pd.r = imax(pd.r, (c.Wo - 1) * c.stride - c.pl + c.kw - c.W);
        inst[in_i[k]].last_use = k;
        if (res_i[k] >= 0) inst[res_i[k]].last_use = k;
        in2_i[k] = -1;
        if (pj[k]) {
            in2_i[k] = cur[pj[k]->src + 2];
            if (in2_i[k] < 0) return false;
            const Instance &x2 = inst[in2_i[k]];
            if (x2.planar || x2.C != pj[k]->Ci || x2.H != pj[k]->H || x2.W != pj[k]->W) return false;
            inst[in2_i[k]].last_use = k;
        }
        out_i[k] = n_inst;
        inst[n_inst++] = Instance{c.Co, c.Ho, c.Wo, false, Pads{0, 0, 0, 0}, -1, -1, 0};
        cur[c.dst + 2] = out_i[k];
    }
    // a residual that nothing else reads afterwards is overwritten in place: both tensors then share one padding
    for (int k = 0; k < n; ++k) alias[k] = k + 1 < n && res_i[k] >= 0 && res_i[k] != in_i[k] && inst[res_i[k]].last_use == k;
    for (int round = 0; round < n; ++round) {
        for (int k = 0; k < n; ++k) {
            if (!alias[k]) continue;
            Pads &x = inst[res_i[k]].pad, &y = inst[out_i[k]].pad;
            x.t = y.t = imax(x.t, y.t);
            x.b = y.b = imax(x.b, y.b);
            x.l = y.l = imax(x.l, y.l);
            x.r = y.r = imax(x.r, y.r);
        }
    }
    for (int k = 0; k < n_inst; ++k) {
        const Pads &pd = inst[k].pad;
        const int pc = imax(pd.l, pd.r);       // left and right padding share their columns
        const int padded = (pd.t + inst[k].H + pd.b) * (pc + inst[k].W) + pc;
        inst[k].bytes = inst[k].planar ? (inst[k].C * padded * 4 + 63) / 64 * 64 : (inst[k].C / 16) * padded * 64;
    }
    // regions, in the order of the run
    int used[kResMaxLayers + 1][2], used_inst[kResMaxLayers + 1], n_used = 0, peak = 0;
    auto take = [&](int i, int off) {
        inst[i].off = off;
        used[n_used][0] = off;
        used[n_used][1] = inst[i].bytes;
        used_inst[n_used++] = i;
        peak = imax(peak, off + inst[i].bytes);
    };
    auto release = [&](int i) {
        for (int k = 0; k < n_used; ++k) {
            if (used_inst[k] == i) {
                --n_used;
                used[k][0] = used[n_used][0];
                used[k][1] = used[n_used][1];
                used_inst[k] = used_inst[n_used];
                return;
            }
        }
    };
    if (inst[0].bytes > kResTensorBytes) return false;
    // a first layer's small input lives only during that layer: at the top, so that it does not split the space
    take(0, inst[0].planar ? kResTensorBytes - inst[0].bytes : 0);
    for (int k = 0; k < n; ++k) {
        const int o = out_i[k];
        if (k + 1 < n) {
            if (alias[k]) {
                inst[o].off = inst[res_i[k]].off;
                for (int u = 0; u < n_used; ++u)
                    if (used_inst[u] == res_i[k]) used_inst[u] = o;       // the region changes hands
            } else {
                const int off = first_fit(used, n_used, inst[o].bytes, kResTensorBytes);
                if (off < 0) return false;
                take(o, off);
            }
        }
        if (inst[in_i[k]].last_use == k) release(in_i[k]);
        if (in2_i[k] >= 0 && in2_i[k] != in_i[k] && inst[in2_i[k]].last_use == k) release(in2_i[k]);
        if (res_i[k] >= 0 && !alias[k] && inst[res_i[k]].last_use == k) release(res_i[k]);
        if (k + 1 < n && inst[o].last_use < 0) release(o);
    }
    lds_bytes = peak + kResSlotBytes;

    auto dev = [&](int i) {
        const Instance &t = inst[i];
        const int pc = imax(t.pad.l, t.pad.r), Wp = pc + t.W;
        return ResTensorDev{t.off / 16, Wp, (t.pad.t + t.H + t.pad.b) * Wp + pc, t.pad.t * Wp + pc};
    };
    memset(&a, 0, sizeof(a));
    a.n_layers = n;
    a.slot = peak / 16;
    a.src = dev(0);
    a.sH = inst[0].H; a.sW = inst[0].W; a.snCb = inst[0].C / 16; a.sC = inst[0].C;
    a.spt = inst[0].pad.t; a.spb = inst[0].pad.b; a.spc = imax(inst[0].pad.l, inst[0].pad.r);
    a.stem_in = g[0].kind == RESIDENT_STEM ? (g[0].plain_input ? 2 : 1) : 0;
    a.in_floats = inst[0].C * a.sH * a.sW;
    a.out_floats = g[n - 1].Co * g[n - 1].Ho * g[n - 1].Wo;
    a.div_sW = make_fastdiv(a.sW);
    a.div_sH = make_fastdiv(a.sH);
    a.div_sC = make_fastdiv(a.sC);
    for (int k = 0; k < n; ++k) {
        const ResGroup &c = g[k];
        ResLayerDev &d = a.layer[k];
        const Instance &x = inst[in_i[k]], &y = inst[out_i[k]];
        d.filt = c.filt;
        d.kind = c.kind == RESIDENT_STEM ? RES_STEM : (c.kind == RESIDENT_HEAD ? RES_HEAD : (c.kind == RESIDENT_DW ? RES_DW : RES_CONV));
        d.K = c.kind == RESIDENT_STEM ? c.Ci * c.kh * c.kw : c.Ci;
        d.Co = c.Co; d.Cob = c.Cob;
        d.in = dev(in_i[k]);
        d.out = k + 1 < n ? dev(out_i[k]) : ResTensorDev{-1, 0, 0, 0};
        d.res = res_i[k] >= 0 ? dev(res_i[k]) : ResTensorDev{0, 0, 0, 0};
        d.Wo = c.Wo; d.HoWo = c.Ho * c.Wo; d.nCib = c.Ci / 16; d.nCob = c.Co / 16; d.stride = c.stride; d.taps = c.kh * c.kw;
        d.win0 = (x.pad.t - c.pt) * d.in.Wp + (imax(x.pad.l, x.pad.r) - c.pl);
        if (pj[k]) {
            const Instance &x2 = inst[in2_i[k]];
            d.filt2 = pj[k]->filt;
            d.in2 = dev(in2_i[k]);
            d.nCib2 = pj[k]->Ci / 16;
            d.stride2 = pj[k]->stride;
            d.win2 = x2.pad.t * d.in2.Wp + imax(x2.pad.l, x2.pad.r);
        }
        d.epilogue = c.epilogue;
        // tiles per wave and step: the split that needs the fewest rounds of the 8 waves, the larger group on a tie
        const int tiles = (d.HoWo + 15) / 16;
        int best_cost = 1 << 30;
        for (int T = 4; T >= 1; T >>= 1) {
            const int groups = d.nCob * ((tiles + T - 1) / T);
            const int cost = ((groups + kResWaves - 1) / kResWaves) * T;
            if (cost < best_cost) {
                best_cost = cost;
                d.T = T;
            }
        }
        if (d.kind == RES_STEM) d.T = 4;
        d.rows3 = d.kind == RES_CONV && d.taps == 9 && c.kw == 3;
        if (d.kind == RES_CONV && d.taps == 9 && !d.rows3) d.T = 1;     // the kernel has that case for single tiles only
        d.nTg = (tiles + d.T - 1) / d.T;
        d.nGroups = d.nCob * d.nTg;
        if (d.kind == RES_CONV || d.kind == RES_DW)
            for (int t = 0; t < d.taps; ++t) d.tapoff[t] = (t / c.kw) * d.in.Wp + (t % c.kw);
        if (d.kind == RES_STEM) {
            a.div_skw = make_fastdiv(c.kw);
            d.taps = 0;
        }
        if (d.kind == RES_HEAD) {
            d.Wo = c.W;             // the pooled image
            d.HoWo = c.H * c.W;
            d.div_Wo = make_fastdiv(c.W);
            d.nCob = 1; d.T = 1; d.nTg = 1; d.nGroups = 1; d.taps = 0;
            continue;
        }
        d.oH = y.H; d.oW = y.W; d.opt = y.pad.t; d.opb = y.pad.b; d.opc = imax(y.pad.l, y.pad.r);
        d.div_Wo = make_fastdiv(c.Wo);
        d.div_nTg = make_fastdiv(d.nTg);
    }
    return true;
}

}  // namespace

#ifdef SMALL_RES_TIMING
extern "C" int small_debug_resident_timing(unsigned long long *host_out)
{
    return (int)hipMemcpyFromSymbol(host_out, HIP_SYMBOL(g_res_t), sizeof(unsigned long long) * 2 * 8 * 64);
}
#endif

int resident_groups(const ResGroup *g, int n, const bool *closed_after)
{
    if (n > kResMaxLayers) n = kResMaxLayers;
    int ok = 0;
    while (ok < n && group_ok(g[ok], ok)) ++ok;
    ResArgs local;
    for (int e = ok; e >= 2; --e) {
        int lds = 0;
        if (closed_after[e - 1] && plan_prefix(g, e, local, lds)) return e;
    }
    return 0;
}

hipError_t launch_resident(const ResGroup *g, int n, const float *in, float *out, int N, hipStream_t s)
{
    ResArgs a;
    int lds = 0;
    if (n < 2 || n > kResMaxLayers || !plan_prefix(g, n, a, lds)) return hipErrorInvalidValue;
    a.in = in;
    a.out = out;
    a.N = N;
    static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void *>(resident_run),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, kResLdsBytes);
    if (attr != hipSuccess) return attr;
    const int grid = N < device_cus() ? N : device_cus();       // one workgroup per compute unit; more images: further rounds
    hipLaunchKernelGGL(resident_run, dim3((unsigned)grid), dim3(kResThreads), (size_t)lds, s, a);
    return hipGetLastError();
}

}  // namespace small
