// Quantized depthwise 3x3 convolution, stride 1, padding 1, 16-byte channel blocks: the uint8 counterpart of
// window_dpp.hip. uint8 codes in and out, exact sums, the library's requantization rule; HBM traffic is a quarter of
// the fp32 layer's, so the bound is vector arithmetic (36 multiply-adds, 8 conversions and 4 requantizations per
// 4 output bytes), not memory.
//
// The mapping is window_dpp.hip's: a wave owns 16 neighbouring pixels of a strip of at most 7 rows of one plane
// (or several narrow planes side by side), lane = 16 q + l holding the four channels 4q .. 4q + 3 of pixel l --
// one 32-bit word of the pixel's 16-byte block. Every lane requests its nine input words at once (buffer
// addressing: lanes and rows outside the image read as the code zx); the bytes become floats x, the left and right
// neighbours come from lanes l - 1 and l + 1 by lane shifts of those floats (zero is shifted in at a band's ends:
// lanes 0 and 15 produce no output there, except lane 15 of a pair of planes, whose sum is corrected), the nine
// taps w' = w - zw are floats in registers, and sum over all nine taps of x w' - zx sum w' -- the sum over the
// taps inside the image of (x - zx)(w - zw), since every other tap reads zx -- is exact in fp32 in any order
// (integers below 2^24). The sum goes back to int, through the requantization (the clamped 64-bit form: the host
// sends only layers whose scale allows it), into its byte of the output word. Vector arithmetic per output word:
// 36 multiply-adds, 8 lane shifts, 4 conversions, 4 requantizations of five instructions.
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

__device__ __forceinline__ float byte_of(unsigned w, int c) { return (float)((w >> (8 * c)) & 255u); }

// clamp(zy + floor((acc * mult + 2^(shift-1)) / 2^shift), lo, hi) for layers with q.amax > 0: the sum is clamped to
// +-amax first (beyond it the output saturates anyway, within it everything below fits), and bias =
// 2^(shift-1) + zy * 2^shift carries the rounding term and the zero point through the one shift.
__device__ __forceinline__ unsigned requant_clamped(float acc, const QuantParams &q, float amax, long bias)
{
    const int c = (int)__builtin_amdgcn_fmed3f(acc, -amax, amax);
    const int r = (int)(((long)c * (long)q.mult + bias) >> q.shift);
    return (unsigned)min(max(r, q.lo), q.hi);
}

// SEG 16: a band is 16 neighbouring pixels of one plane (14 outputs). SEG 8: rows of at most 7 pixels, two planes
// side by side with a lane of padding on their left. SEG 0: rows of at most 5 pixels, floor(16 / W) planes back to
// back without padding lanes (three planes of the audio CNN's 5-pixel rows instead of two): the neighbour a plane's
// first and last pixel would take from the plane next to it is replaced by the code zx with a select.
template <int SEG>
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
    // the plane's nine taps of this quad as floats w - zw
    const float zx = (float)a.q.zx, zw = (float)a.q.zw;
    floatx4 w[9];
    {
        const int pc = min(plane, a.n_planes - 1), cb = pc - a.by_nCb.div(pc) * a.nCb;
        const unsigned *tp = reinterpret_cast<const unsigned *>(a.filt) + cb * 36 + q;
#pragma unroll
        for (int k = 0; k < 9; ++k) {
            const unsigned wr = tp[k * 4];
            w[k] = floatx4{byte_of(wr, 0) - zw, byte_of(wr, 1) - zw, byte_of(wr, 2) - zw, byte_of(wr, 3) - zw};
        }
    }
    floatx4 wsum = w[0];
#pragma unroll
    for (int k = 1; k < 9; ++k) wsum += w[k];
    floatx4 acc0 = wsum * (-zx);                               // - zx * sum of the taps
    if (SEG == 8 && l == 15) acc0 += (w[2] + w[5] + w[8]) * zx;       // its right neighbours read 0, not zx
    const long bias = (a.q.shift > 0 ? 1L << (a.q.shift - 1) : 0L) + ((long)a.q.zy << a.q.shift);
    const float amax = (float)min(a.q.amax, 1 << 24);          // (sums stay below 2^24: a larger bound never binds)

    floatx4 row[kStepsU8], row_l[kStepsU8], row_r[kStepsU8];
#pragma unroll
    for (int j = 0; j < kStepsU8; ++j) {
        row[j] = floatx4{byte_of(raw[j], 0), byte_of(raw[j], 1), byte_of(raw[j], 2), byte_of(raw[j], 3)};
        row_l[j] = lane_shift<kRowShr1>(row[j]);
        row_r[j] = lane_shift<kRowShl1>(row[j]);
        if (SEG == 0) {
            row_l[j] = at_left ? floatx4{zx, zx, zx, zx} : row_l[j];
            row_r[j] = at_right ? floatx4{zx, zx, zx, zx} : row_r[j];
        }
        if (j < 2) continue;
        floatx4 acc = acc0;
        acc += row[j - 1] * w[4];
        acc += row[j - 2] * w[1];
        acc += row[j] * w[7];
        acc += row_l[j - 2] * w[0];
        acc += row_l[j - 1] * w[3];
        acc += row_l[j] * w[6];
        acc += row_r[j - 2] * w[2];
        acc += row_r[j - 1] * w[5];
        acc += row_r[j] * w[8];
        const unsigned y = requant_clamped(acc.x, a.q, amax, bias) | (requant_clamped(acc.y, a.q, amax, bias) << 8) |
                           (requant_clamped(acc.z, a.q, amax, bias) << 16) | (requant_clamped(acc.w, a.q, amax, bias) << 24);
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
    if (seg == 0) hipLaunchKernelGGL((dw16_dpp_u8<0>), grid, block, 0, s, a);
    else if (seg == 8) hipLaunchKernelGGL((dw16_dpp_u8<8>), grid, block, 0, s, a);
    else hipLaunchKernelGGL((dw16_dpp_u8<16>), grid, block, 0, s, a);
    return hipGetLastError();
}

}  // namespace small
