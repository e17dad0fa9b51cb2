// Quantized depthwise 3x3 convolution, stride 1, padding 1, 16-byte channel blocks: the uint8 counterpart of
// window_dpp.hip. uint8 codes in and out, exact int32 sums, the library's requantization rule; HBM traffic is a
// quarter of the fp32 layer's, so the bound is vector arithmetic, not memory.
//
// The mapping is window_dpp.hip's: a wave owns 16 neighbouring pixels of a strip of at most 7 rows of one plane
// (or several narrow planes side by side), lane = 16 q + l holding the four channels 4q .. 4q + 3 of pixel l --
// one 32-bit word of the pixel's 16-byte block. Every lane requests its nine input words at once (buffer
// addressing: lanes and rows outside the image read as the code zx); the left and right neighbours come from
// lanes l - 1 and l + 1 by lane shifts of the words (zero is shifted in at a band's ends: lanes 0 and 15 produce no
// output there, or the value is replaced). The sums are taken with four-byte signed dot products over the three
// taps of a window row (see the kernel), go through the requantization (the clamped 64-bit form: the host sends only
// layers whose scale allows it) and into their byte of the output word.
#include "small_internal.h"

namespace small {

namespace {

struct DppU8Args {
    const unsigned char *in;
    const unsigned char *filt;     // [C/16][3][3][16]
    unsigned char *out;
    int H, W, nCb;
    int n_planes;          // N * nCb
    int nb;                // bands per row
    int sp;                // row strips per plane
    int n_units;           // plane groups * sp * nb: one per wave
    int ppb;               // planes per band of 16 lanes (SEG 0), else unused
    unsigned bytes;        // of the input = of the output tensor (< 2^31)
    FastDiv by_nb, by_sp, by_nCb, by_W;
    QuantParams q;
};

// Output rows per strip (two more input rows prime the window). Strips of 13 rows, tried where they still leave two
// waves for every SIMD, save a tenth of the vector work and measure 10-30 % slower: a wave is one serial chain from
// its loads to its last row, and what hides it is the number of waves.
constexpr int kStripRowsU8 = 7;
constexpr int kStepsU8 = kStripRowsU8 + 2;

// SEG 16: a band is 16 neighbouring pixels of one plane (14 outputs). SEG 8: rows of at most 7 pixels, two planes
// side by side with a lane of padding on their left. SEG 0: rows of at most 5 pixels, floor(16 / W) planes back to
// back without padding lanes (three planes of the audio CNN's 5-pixel rows instead of two): the neighbour a plane's
// first and last pixel would take from the plane next to it is replaced by the code zx with a select.
template <int SEG, bool HAS_ZB>
__global__ void __launch_bounds__(256) dw16_dpp_u8(DppU8Args a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int unit = (int)blockIdx.x * 4 + wave;
    if (unit >= a.n_units) return;
    const int l = lane & 15, q = lane >> 4;

    const int t = a.by_nb.div(unit), band = unit - t * a.nb;
    const int pg = a.by_sp.div(t), strip = t - pg * a.sp;
    const int r0 = a.by_sp.div(strip * a.H), r1 = a.by_sp.div((strip + 1) * a.H);      // output rows r0 .. r1 - 1
    const int n_in = r1 - r0 + 2;

    int plane, x;
    bool lane_used = true;
    if (SEG == 16) {
        plane = pg;
        x = band * 14 - 1 + l;
    } else if (SEG == 8) {
        plane = pg * 2 + (l >> 3);
        x = (l & 7) - 1;
    } else {
        const int pi = a.by_W.div(l);
        plane = pg * a.ppb + pi;
        x = l - pi * a.W;
        lane_used = pi < a.ppb;
    }
    const bool col_in = lane_used && x >= 0 && x < a.W && plane < a.n_planes;
    const bool col_out = col_in && (SEG != 16 || (l >= 1 && l <= 14));
    const bool at_left = x == 0, at_right = x == a.W - 1;          // (SEG 0)
    const int row_bytes = a.W * 16;
    const unsigned at = (unsigned)plane * (unsigned)(a.H * row_bytes) + (unsigned)(x * 16 + q * 4);

    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.in), 0, a.bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.bytes, kRawBuffer);

    // the nine input words (codes), zx where there is no input
    const unsigned zx4 = (unsigned)a.q.zx * 0x01010101u;
    unsigned raw[kStepsU8];
#pragma unroll
    for (int j = 0; j < kStepsU8; ++j) {
        const int r = r0 - 1 + j;
        const bool have = col_in && r >= 0 && r < a.H && j < n_in;
        const unsigned v = __builtin_amdgcn_raw_buffer_load_b32(src, have ? at + (unsigned)(r * row_bytes) : kBeyond, 0, 0);
        raw[j] = have ? v : zx4;
    }
    // Everything below works on signed bytes x' = x - 128 and w' = w - 128 (one exclusive-or per word), whose products
    // the four-byte signed dot product sums exactly:
    //     sum (x - zx)(w - zw) = sum x' w' + b sum x' + a sum w' + 9 a b,   a = 128 - zx, b = 128 - zw,
    // over all nine taps, those outside the image carrying the code zx. A dot product wants the three taps of one
    // window row of ONE channel in a word, the tensor has the four channels of one pixel in a word: per input row the
    // words of the left neighbour, the pixel and the right neighbour (lane shifts of the raw words: two per row, not
    // eight) are transposed into four words [left, centre, right, 0], one per channel, with two byte permutes each;
    // every such word serves three output rows. The filter is transposed the same way once. Per output word: 2 lane
    // shifts, 8 permutes and 12 dot products, where the float form of this kernel had 8 shifts, 4 conversions and 36
    // multiply-adds; with zw = 128 (b = 0) the sum of the window's codes is not needed at all.
    const unsigned flip = 0x80808080u;
    const int za = 128 - a.q.zx, zb = 128 - a.q.zw;
    auto channel_words = [&](unsigned left, unsigned mid, unsigned right, unsigned (&t)[4]) __attribute__((always_inline)) {
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            const unsigned lm = __builtin_amdgcn_perm(mid, left, 0x0c0c0000u | (unsigned)((4 + c) << 8) | (unsigned)c);
            t[c] = __builtin_amdgcn_perm(right, lm, 0x0c000100u | (unsigned)((4 + c) << 16));
        }
    };
    unsigned wt[3][4];                                      // [window row][channel]: its three taps
    int cst[4];                                             // a sum w' + 9 a b per channel
    {
        const int pc = min(plane, a.n_planes - 1), cb = pc - a.by_nCb.div(pc) * a.nCb;
        const unsigned *tp = reinterpret_cast<const unsigned *>(a.filt) + cb * 36 + q;
#pragma unroll
        for (int c = 0; c < 4; ++c) cst[c] = 0;
#pragma unroll
        for (int r = 0; r < 3; ++r) {
            channel_words(tp[(3 * r) * 4] ^ flip, tp[(3 * r + 1) * 4] ^ flip, tp[(3 * r + 2) * 4] ^ flip, wt[r]);
#pragma unroll
            for (int c = 0; c < 4; ++c) cst[c] = __builtin_amdgcn_sdot4((int)wt[r][c], 0x00010101, cst[c], false);
        }
#pragma unroll
        for (int c = 0; c < 4; ++c) cst[c] = za * cst[c] + 9 * za * zb;
    }
    const long bias = requant_bias(a.q);
    const unsigned zxs = zx4 ^ flip;                        // the padding code as signed bytes

    unsigned tw[kStepsU8][4];                               // [input row][channel]: left, centre and right value
    int sx[kStepsU8][4];                                    // their sums (zb != 0 only)
#pragma unroll
    for (int j = 0; j < kStepsU8; ++j) {
        const unsigned mid = raw[j] ^ flip;
        unsigned left = (unsigned)__builtin_amdgcn_update_dpp(0, (int)mid, kRowShr1, 0xf, 0xf, true);
        unsigned right = (unsigned)__builtin_amdgcn_update_dpp(0, (int)mid, kRowShl1, 0xf, 0xf, true);
        // (zero is shifted in at the ends of a row of 16 lanes; where such a lane has an output, it wants zx there)
        if (SEG == 0) {
            left = at_left ? zxs : left;
            right = at_right ? zxs : right;
        } else if (SEG == 8) {
            right = l == 15 ? zxs : right;
        }
        channel_words(left, mid, right, tw[j]);
        if (HAS_ZB) {
#pragma unroll
            for (int c = 0; c < 4; ++c) sx[j][c] = __builtin_amdgcn_sdot4((int)tw[j][c], 0x00010101, 0, false);
        }
        if (j < 2) continue;
        unsigned y = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int acc = __builtin_amdgcn_sdot4((int)tw[j - 2][c], (int)wt[0][c], cst[c], false);
            acc = __builtin_amdgcn_sdot4((int)tw[j - 1][c], (int)wt[1][c], acc, false);
            acc = __builtin_amdgcn_sdot4((int)tw[j][c], (int)wt[2][c], acc, false);
            if (HAS_ZB) acc += zb * (sx[j - 2][c] + sx[j - 1][c] + sx[j][c]);
            y |= (unsigned)requant_clamped(acc, a.q, bias) << (8 * c);
        }
        const unsigned off = (col_out && j < n_in) ? at + (unsigned)((r0 + j - 2) * row_bytes) : kBeyond;
        __builtin_amdgcn_raw_buffer_store_b32(y, dst, off, 0, kNonTemporal);
    }
}

}  // namespace

bool dw_dpp_u8_eligible(const LayerGeom &g, const QuantParams &q, const void *in, const void *filt, const void *out)
{
    if (q.amax <= 0) return false;                            // (a scale too large for the clamped requantization)
    if (g.Cib != 16 || g.kh != 3 || g.kw != 3 || g.stride != 1 || g.pt != 1 || g.pl != 1) return false;
    if (g.Ho != g.H || g.Wo != g.W) return false;
    if ((((uintptr_t)in | (uintptr_t)filt | (uintptr_t)out) & 3u) != 0) return false;
    return (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 31);
}

hipError_t launch_dw_dpp_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                            const QuantParams &q, hipStream_t s)
{
    DppU8Args a;
    a.in = in; a.filt = filt; a.out = out;
    a.H = g.H; a.W = g.W; a.nCb = g.Ci / 16;
    a.n_planes = g.N * a.nCb;
    a.bytes = (unsigned)((size_t)g.N * g.Ci * g.H * g.W);
    a.q = q;
    const int seg = g.W <= 5 ? 0 : g.W <= 7 ? 8 : 16;
    a.ppb = seg == 0 ? 16 / g.W : seg == 8 ? 2 : 1;
    a.nb = seg == 16 ? (g.W + 13) / 14 : 1;
    const long groups = (a.n_planes + a.ppb - 1) / a.ppb;
    a.sp = (g.H + kStripRowsU8 - 1) / kStripRowsU8;
    a.n_units = (int)(groups * a.sp * a.nb);
    a.by_nb = make_fastdiv(a.nb);
    a.by_sp = make_fastdiv(a.sp);
    a.by_nCb = make_fastdiv(a.nCb);
    a.by_W = make_fastdiv(g.W);
    const dim3 grid((unsigned)((a.n_units + 3) / 4)), block(256);
    if (q.zw == 128) {
        if (seg == 0) hipLaunchKernelGGL((dw16_dpp_u8<0, false>), grid, block, 0, s, a);
        else if (seg == 8) hipLaunchKernelGGL((dw16_dpp_u8<8, false>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((dw16_dpp_u8<16, false>), grid, block, 0, s, a);
    } else {
        if (seg == 0) hipLaunchKernelGGL((dw16_dpp_u8<0, true>), grid, block, 0, s, a);
        else if (seg == 8) hipLaunchKernelGGL((dw16_dpp_u8<8, true>), grid, block, 0, s, a);
        else hipLaunchKernelGGL((dw16_dpp_u8<16, true>), grid, block, 0, s, a);
    }
    return hipGetLastError();
}

}  // namespace small
