// Quantized (uint8) layers on the blocked byte layouts: activations [N][C/Cb][H][W][Cb], filters
// [Co/Cob][Ci/Cib][kh][kw][Cob][Cib] (input channel fastest, so the Cib bytes one output channel multiplies
// with one pixel's Cib bytes are one contiguous operand of the 8-bit matrix instruction), depthwise filters
// [C/Cb][kh][kw][Cb]. Inputs and outputs are uint8 codes, sums are int32 (Section "Memory Usage Comparison",
// Section "Quantized Inference"); the paper gives no requantization rule, the one used is stated in the
// public header: acc = sum over in-image taps of (x - zx)(w - zw),
// y = clamp(zy + ((int64)acc * mult + 2^(shift-1)) >> shift, lo, hi).
//
// conv_u8_mfma (16-byte blocks): v_mfma_i32_16x16x64_i8 multiplies signed bytes, 64 per lane row: lane
// (p = l % 16, g = l / 16) supplies 16 consecutive reduction elements of filter row co = p (A) and of pixel p (B).
// One such 16-byte operand is exactly one pixel's channel block at one filter tap, so lane group g takes
// reduction chunk 4t + g of step t, a chunk being (input block, tap). Codes become signed by flipping bit 7
// (x - 128); with a = zx - 128, b = zw - 128 and taps outside the image read as the code zx:
//   sum (x - zx)(w - zw) = sum xs ws - b sum xs - a sum ws + K a b        (over all K taps)
// where the two correction sums come from the same instruction with an all-ones operand: ones x B gives
// sum xs per pixel in every row, A x ones gives sum ws per output channel in every column, both already in
// the accumulator layout. They are skipped when b = 0 or a = 0.
#include "small_internal.h"

namespace small {
namespace {

typedef int intx4 __attribute__((ext_vector_type(4)));

struct QConvArgs {
    const unsigned char *in, *filt;
    unsigned char *out;
    int N, H, W, Ho, Wo, HoWo, M;
    int nCib, nCob, Cib, Cob, kh, kw, stride, pt, pl;
    int n_chunks;     // nCib * kh * kw (matrix-core kernel)
    FastDiv div_HoWo, div_Wo, div_taps, div_kw;
    const int *filt_sums;   // per output channel: sum of the filter's codes over the whole reduction, or null
    QuantParams q;
};

// Zero-point corrections and requantization of a wave's accumulators, four consecutive output channels
// (one 32-bit word of the blocked output) per lane and tile. acc_w: sum of the signed filter bytes per channel.
template <int WM, int WN>
__device__ __forceinline__ void store_tiles(const QConvArgs &a, const intx4 (&acc)[WM][WN], const intx4 (&acc_s)[WM],
                                            const intx4 (&acc_w)[WN], int tile0, int cob0, int p, int g)
{
    const int za = a.q.zx - 128, zb = a.q.zw - 128;
    const unsigned K = (unsigned)a.n_chunks * 16u;
    const unsigned kab = K * (unsigned)(za * zb);
    const bool narrow = a.q.amax > 0;                  // (uniform) the five-instruction requantization applies
    const long bias = requant_bias(a.q);
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        const int m = tile0 + wm * 16 + p;
        if (m >= a.M) continue;
        const int n = a.div_HoWo.div(m), pix = m - n * a.HoWo;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            unsigned packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // wrap-around arithmetic: the true sum fits 32 bits, the partial terms need not
                const unsigned v = (unsigned)acc[wm][wn][r] - (unsigned)zb * (unsigned)acc_s[wm][r] -
                                   (unsigned)za * (unsigned)acc_w[wn][r] + kab;
                packed |= (unsigned)(narrow ? requant_clamped((int)v, a.q, bias) : requant((int)v, a.q)) << (8 * r);
            }
            unsigned *o = reinterpret_cast<unsigned *>(a.out + (((size_t)n * a.nCob + cob0 + wn) * a.HoWo + pix) * 16 + g * 4);
            *o = packed;
        }
    }
}

// sum of the signed filter bytes of output channels 4g .. 4g+3 of block cob, from the caller's sums of codes
__device__ __forceinline__ intx4 signed_filter_sums(const QConvArgs &a, int cob, int g)
{
    const intx4 v = *reinterpret_cast<const intx4 *>(a.filt_sums + cob * 16 + 4 * g);
    const int k128 = a.n_chunks * 16 * 128;
    return intx4{v[0] - k128, v[1] - k128, v[2] - k128, v[3] - k128};
}

// ------------------------------------------------------------------------------------------------ layouts

__global__ void __launch_bounds__(256) pack_u8_kernel(const unsigned char *nchw, unsigned char *blk, int C, int HW, int Cb,
                                                      size_t total, int unpack)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index into the blocked tensor
    if (i >= total) return;
    const int c_in = (int)(i % Cb);
    const size_t t = i / Cb;
    const int pix = (int)(t % HW);
    const size_t t2 = t / HW;          // n * nCb + cb
    const int nCb = C / Cb;
    const int cb = (int)(t2 % nCb);
    const size_t n = t2 / nCb;
    const size_t j = (n * C + (size_t)cb * Cb + c_in) * HW + pix;
    if (unpack) const_cast<unsigned char *>(nchw)[j] = blk[i];
    else blk[i] = nchw[j];
}

__global__ void __launch_bounds__(256) pack_filter_u8_kernel(const unsigned char *oihw, unsigned char *blk, int Co, int Ci,
                                                             int khw, int Cob, int Cib, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index into the blocked filter
    if (i >= total) return;
    const int ci_in = (int)(i % Cib);
    size_t t = i / Cib;
    const int co_in = (int)(t % Cob);
    t /= Cob;
    const int tap = (int)(t % khw);
    t /= khw;
    const int nCib = Ci / Cib;
    const int cib = (int)(t % nCib);
    const int cob = (int)(t / nCib);
    const size_t co = (size_t)cob * Cob + co_in, ci = (size_t)cib * Cib + ci_in;
    blk[i] = oihw[(co * Ci + ci) * khw + tap];
}

// One lane per output channel: the sum of its codes over (input block, tap, input channel).
__global__ void __launch_bounds__(256) filter_sums_u8_kernel(const unsigned char *blk, int *sums, int Co, int nCib, int khw,
                                                             int Cob, int Cib)
{
    const int co = blockIdx.x * 256 + threadIdx.x;
    if (co >= Co) return;
    const int cob = co / Cob, co_in = co - cob * Cob;
    int sum = 0;
    for (int c = 0; c < nCib * khw; ++c) {
        const unsigned char *w = blk + (((size_t)cob * nCib * khw + c) * Cob + co_in) * Cib;
        for (int i = 0; i < Cib; ++i) sum += w[i];
    }
    sums[co] = sum;
}

// ------------------------------------------------------------------------------------------------ convolution

// Any block sizes: one lane per output code.
__global__ void __launch_bounds__(256) conv_u8_direct(QConvArgs a, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index into the blocked output
    if (i >= total) return;
    const int co_in = (int)(i % a.Cob);
    size_t t = i / a.Cob;
    const int pix = (int)(t % a.HoWo);
    t /= a.HoWo;
    const int cob = (int)(t % a.nCob);
    const int n = (int)(t / a.nCob);
    const int oh = pix / a.Wo, ow = pix - oh * a.Wo;
    int acc = 0;
    for (int cib = 0; cib < a.nCib; ++cib)
        for (int ky = 0; ky < a.kh; ++ky) {
            const int ih = oh * a.stride + ky - a.pt;
            if (ih < 0 || ih >= a.H) continue;
            for (int kx = 0; kx < a.kw; ++kx) {
                const int iw = ow * a.stride + kx - a.pl;
                if (iw < 0 || iw >= a.W) continue;
                const unsigned char *x = a.in + ((((size_t)n * a.nCib + cib) * a.H + ih) * a.W + iw) * a.Cib;
                const unsigned char *w =
                    a.filt + ((((((size_t)cob * a.nCib + cib) * a.kh + ky) * a.kw + kx) * a.Cob) + co_in) * a.Cib;
                for (int c = 0; c < a.Cib; ++c) acc += ((int)x[c] - a.q.zx) * ((int)w[c] - a.q.zw);
            }
        }
    a.out[i] = (unsigned char)requant(acc, a.q);
}

// Each wave: WM groups of 16 output pixels x WN blocks of 16 output channels (blockIdx.y counts groups of WN blocks).
// CORR: which zero-point correction sums the loop takes with all-ones operands: 0 none, 1 the pixel sums
// (zw != 128), 2 the pixel sums and the filter sums (zx != 128 and the caller gave no filter sums).
template <int WM, int WN, int CORR>
__global__ void __launch_bounds__(256) conv_u8_mfma(QConvArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const int HW = a.H * a.W;
    const int za = a.q.zx - 128, zb = a.q.zw - 128;
    constexpr bool use_s = CORR >= 1, mfma_w = CORR == 2;
    const bool use_w = za != 0;

    int ih0[WM], iw0[WM];
    size_t img[WM];       // 16-byte pixel index of the image's first block
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        int m = tile0 + wm * 16 + p;
        m = m < a.M ? m : a.M - 1;
        const int n = a.div_HoWo.div(m), rem = m - n * a.HoWo;
        const int oh = a.div_Wo.div(rem), ow = rem - oh * a.Wo;
        ih0[wm] = oh * a.stride - a.pt;
        iw0[wm] = ow * a.stride - a.pl;
        img[wm] = (size_t)n * a.nCib * HW;
    }
    // this lane group's reduction chunk: c = (cib * kh + ky) * kw + kx, advanced by 4 per step
    int c = g;
    int kx = c % a.kw, ky = (c / a.kw) % a.kh, cib = c / (a.kw * a.kh);
    const intx4 *filt = reinterpret_cast<const intx4 *>(a.filt) + (size_t)cob0 * a.n_chunks * 16 + p;
    const size_t cob_stride = (size_t)a.n_chunks * 16;
    const intx4 *in = reinterpret_cast<const intx4 *>(a.in);
    const int flip = (int)0x80808080u;
    const int zx4 = a.q.zx * 0x01010101;
    const intx4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const intx4 zero = {0, 0, 0, 0};

    intx4 acc[WM][WN], acc_s[WM], acc_w[WN];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        acc_s[wm] = zero;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = zero;
    }
#pragma unroll
    for (int wn = 0; wn < WN; ++wn) acc_w[wn] = zero;

    // operands of one step: this lane group's chunk c = (cib, ky, kx); chunks past the end read as zero
    auto load = [&](intx4 (&fa)[WN], intx4 (&fb)[WM]) __attribute__((always_inline)) {
        const bool live = c < a.n_chunks;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            fa[wn] = zero;
            if (live) fa[wn] = filt[wn * cob_stride + (size_t)c * 16] ^ flip;
        }
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            const int ih = ih0[wm] + ky, iw = iw0[wm] + kx;
            const bool inside = live && ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            // always a load from a valid address (no branch around it), then the choice
            const intx4 v = in[inside ? img[wm] + (size_t)cib * HW + ih * a.W + iw : img[wm]];
#pragma unroll
            for (int k = 0; k < 4; ++k) fb[wm][k] = live ? (inside ? v[k] ^ flip : zx4 ^ flip) : 0;
        }
        c += 4;
        kx += 4;
        while (kx >= a.kw) { kx -= a.kw; ++ky; }
        while (ky >= a.kh) { ky -= a.kh; ++cib; }
    };
    auto multiply = [&](const intx4 (&fa)[WN], const intx4 (&fb)[WM]) __attribute__((always_inline)) {
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int wn = 0; wn < WN; ++wn)
                acc[wm][wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], fb[wm], acc[wm][wn], 0, 0, 0);
            if (use_s) acc_s[wm] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, fb[wm], acc_s[wm], 0, 0, 0);
        }
        if (mfma_w) {
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) acc_w[wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], ones, acc_w[wn], 0, 0, 0);
        }
    };

    // two operand sets in turn: the loads of step t + 1 are in flight while step t multiplies
    const int steps = (a.n_chunks + 3) >> 2;
    intx4 fa0[WN], fb0[WM], fa1[WN], fb1[WM];
    load(fa0, fb0);
    for (int t = 0; t < steps; t += 2) {
        load(fa1, fb1);               // step t + 1 (all zero past the end)
        multiply(fa0, fb0);
        load(fa0, fb0);               // step t + 2
        multiply(fa1, fb1);
    }

    if (use_w && a.filt_sums) {
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc_w[wn] = signed_filter_sums(a, cob0 + wn, g);
    }
    store_tiles<WM, WN>(a, acc, acc_s, acc_w, tile0, cob0, p, g);
}

// The same tile for short reductions (at most 4 * STEPS chunks: 16 or 32 input channels under a 3x3 window, up to 64
// under 1x1): every operand of the whole reduction is requested before the first matrix instruction, from addresses that
// are always valid (chunks past the end and taps outside the image are replaced afterwards), so a wave waits for memory
// once instead of once per step, which is what these launches' time consists of.
template <int WM, int WN, int CORR, int STEPS>
__global__ void __launch_bounds__(256) conv_u8_mfma_short(QConvArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const int HW = a.H * a.W;
    const int za = a.q.zx - 128;
    constexpr bool use_s = CORR >= 1, mfma_w = CORR == 2;
    const bool use_w = za != 0;

    int ih0[WM], iw0[WM];
    const intx4 *img[WM];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        int m = tile0 + wm * 16 + p;
        m = m < a.M ? m : a.M - 1;
        const int n = a.div_HoWo.div(m), rem = m - n * a.HoWo;
        const int oh = a.div_Wo.div(rem), ow = rem - oh * a.Wo;
        ih0[wm] = oh * a.stride - a.pt;
        iw0[wm] = ow * a.stride - a.pl;
        img[wm] = reinterpret_cast<const intx4 *>(a.in) + (size_t)n * a.nCib * HW;
    }
    const intx4 *filt = reinterpret_cast<const intx4 *>(a.filt) + (size_t)cob0 * a.n_chunks * 16 + p;
    const size_t cob_stride = (size_t)a.n_chunks * 16;
    const int flip = (int)0x80808080u;
    const int pad = (a.q.zx * 0x01010101) ^ flip;
    const intx4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const intx4 zero = {0, 0, 0, 0};

    intx4 ra[STEPS][WN], rb[STEPS][WM];
    bool live[STEPS], inside[STEPS][WM];
#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        // this lane group's chunk of step t: c = (cib * kh + ky) * kw + kx
        const int c_raw = 4 * t + g;
        live[t] = c_raw < a.n_chunks;
        const int c = live[t] ? c_raw : a.n_chunks - 1;
        const int cib = a.div_taps.div(c), tap = c - cib * a.kh * a.kw;
        const int ky = a.div_kw.div(tap), kx = tap - ky * a.kw;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) ra[t][wn] = filt[wn * cob_stride + (size_t)c * 16];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            const int ih = ih0[wm] + ky, iw = iw0[wm] + kx;
            inside[t][wm] = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            rb[t][wm] = img[wm][inside[t][wm] ? cib * HW + ih * a.W + iw : 0];
        }
    }

    intx4 acc[WM][WN], acc_s[WM], acc_w[WN];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        acc_s[wm] = zero;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = zero;
    }
#pragma unroll
    for (int wn = 0; wn < WN; ++wn) acc_w[wn] = zero;

#pragma unroll
    for (int t = 0; t < STEPS; ++t) {
        intx4 fa[WN], fb[WM];
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
#pragma unroll
            for (int k = 0; k < 4; ++k) fa[wn][k] = live[t] ? ra[t][wn][k] ^ flip : 0;
        }
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int k = 0; k < 4; ++k) fb[wm][k] = live[t] ? (inside[t][wm] ? rb[t][wm][k] ^ flip : pad) : 0;
        }
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
            for (int wn = 0; wn < WN; ++wn)
                acc[wm][wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], fb[wm], acc[wm][wn], 0, 0, 0);
            if (use_s) acc_s[wm] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, fb[wm], acc_s[wm], 0, 0, 0);
        }
        if (mfma_w) {
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) acc_w[wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], ones, acc_w[wn], 0, 0, 0);
        }
    }

    if (use_w && a.filt_sums) {
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc_w[wn] = signed_filter_sums(a, cob0 + wn, g);
    }
    store_tiles<WM, WN>(a, acc, acc_s, acc_w, tile0, cob0, p, g);
}

// The same tile for layers whose input has a multiple of four 16-channel blocks: one matrix instruction takes one
// filter tap of four consecutive input blocks (lane group g = block 4j + g), so the tap, its bounds test and the
// operand addresses are per-tap values and the walk over j only adds constants. Steps (tap, j) run through a ring
// of DEPTH register sets: the loads of step s + DEPTH - 1 are issued before step s multiplies, every load is
// unconditional (out-of-image taps read the image's first pixel and are replaced afterwards), so a wave keeps
// DEPTH - 1 steps of operands in flight instead of waiting for each step's loads in turn.
template <int WM, int WN, int CORR, int DEPTH>
__global__ void __launch_bounds__(256) conv_u8_mfma4(QConvArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const int HW = a.H * a.W;
    const int za = a.q.zx - 128;
    constexpr bool use_s = CORR >= 1, mfma_w = CORR == 2;
    const bool use_w = za != 0;
    const int taps = a.kh * a.kw;

    int ih0[WM], iw0[WM];
    const intx4 *img[WM];       // this lane group's first input block of the pixel's image
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        int m = tile0 + wm * 16 + p;
        m = m < a.M ? m : a.M - 1;
        const int n = a.div_HoWo.div(m), rem = m - n * a.HoWo;
        const int oh = a.div_Wo.div(rem), ow = rem - oh * a.Wo;
        ih0[wm] = oh * a.stride - a.pt;
        iw0[wm] = ow * a.stride - a.pl;
        img[wm] = reinterpret_cast<const intx4 *>(a.in) + ((size_t)n * a.nCib + g) * HW;
    }
    // filter block (cob, cib, tap) holds 16 rows of 16 bytes: row p of block (cob0, g, 0)
    const intx4 *filt = reinterpret_cast<const intx4 *>(a.filt) + ((size_t)cob0 * a.n_chunks + (size_t)g * taps) * 16 + p;
    const size_t cob_stride = (size_t)a.n_chunks * 16;
    const int flip = (int)0x80808080u;
    const int pad = (a.q.zx * 0x01010101) ^ flip;
    const intx4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const intx4 zero = {0, 0, 0, 0};

    intx4 acc[WM][WN], acc_s[WM], acc_w[WN];
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        acc_s[wm] = zero;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = zero;
    }
#pragma unroll
    for (int wn = 0; wn < WN; ++wn) acc_w[wn] = zero;

    const int groups = a.nCib >> 2;
    const int total = taps * groups;
    // request cursor
    int r_s = 0, r_j = 0, r_ky = 0, r_kx = 0, r_tap = 0;
    const intx4 *bp[WM], *ap = filt;
    int inside[WM];
    auto enter_tap = [&]() __attribute__((always_inline)) {
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            const int ih = ih0[wm] + r_ky, iw = iw0[wm] + r_kx;
            inside[wm] = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            bp[wm] = img[wm] + (inside[wm] ? ih * a.W + iw : 0);
        }
        ap = filt + (size_t)r_tap * 16;
    };
    intx4 ra[DEPTH][WN], rb[DEPTH][WM];
    int rin[DEPTH][WM];
    auto request = [&](int d) __attribute__((always_inline)) {
        if (r_s >= total) return;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) ra[d][wn] = ap[wn * cob_stride];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            rb[d][wm] = *bp[wm];
            rin[d][wm] = inside[wm];
            bp[wm] += (size_t)4 * HW;
        }
        ap += (size_t)4 * taps * 16;
        ++r_s;
        if (++r_j == groups) {
            r_j = 0;
            ++r_tap;
            if (++r_kx == a.kw) { r_kx = 0; ++r_ky; }
            enter_tap();
        }
    };
    enter_tap();
#pragma unroll
    for (int d = 0; d < DEPTH - 1; ++d) request(d);

    for (int s0 = 0; s0 < total; s0 += DEPTH) {
#pragma unroll
        for (int d = 0; d < DEPTH; ++d) {
            if (s0 + d < total) {
                request((d + DEPTH - 1) % DEPTH);      // the set used in the step before this one
                intx4 fa[WN], fb[WM];
#pragma unroll
                for (int wn = 0; wn < WN; ++wn) fa[wn] = ra[d][wn] ^ flip;
#pragma unroll
                for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) fb[wm][k] = rin[d][wm] ? rb[d][wm][k] ^ flip : pad;
                }
#pragma unroll
                for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
                    for (int wn = 0; wn < WN; ++wn)
                        acc[wm][wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], fb[wm], acc[wm][wn], 0, 0, 0);
                    if (use_s) acc_s[wm] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, fb[wm], acc_s[wm], 0, 0, 0);
                }
                if (mfma_w) {
#pragma unroll
                    for (int wn = 0; wn < WN; ++wn)
                        acc_w[wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], ones, acc_w[wn], 0, 0, 0);
                }
            }
        }
    }

    if (use_w && a.filt_sums) {
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) acc_w[wn] = signed_filter_sums(a, cob0 + wn, g);
    }
    store_tiles<WM, WN>(a, acc, acc_s, acc_w, tile0, cob0, p, g);
}

// Pointwise layers (1x1 window, stride 1, no padding) on 64 or 128 input channels: the kernel above is one or two steps
// per workgroup there -- load, multiply, requantize, store, every wave of a round in the same phase at the same time,
// and a launch is a few rounds of load latencies (13.6 us for 26 MB at the sweep's 64-channel shape). Here a wave keeps
// the filter operands of its WN output blocks in registers (a pointwise filter is all of 4 or 8 matrix operands per
// output block) and walks tiles of 16 * WM pixels: the next tile's pixels are requested before the current tile is
// multiplied and requantized, so the vector work of one tile hides the load latency of the next.
template <int WM, int WN, int CORR, int GROUPS>
__global__ void __launch_bounds__(256) pw_u8_stream(QConvArgs a, int n_tiles, int n_waves)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int wv = (int)blockIdx.x * 4 + wave;
    if (wv >= n_waves) return;
    const int za = a.q.zx - 128;
    constexpr bool use_s = CORR >= 1, mfma_w = CORR == 2;
    const bool use_w = za != 0;
    const int flip = (int)0x80808080u;
    const intx4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const intx4 zero = {0, 0, 0, 0};

    // filter block (cob, cib) holds 16 rows of 16 bytes: row p of blocks (cob0 + wn, 4j + g)
    intx4 fa[GROUPS][WN], acc_w[WN];
    {
        const intx4 *filt = reinterpret_cast<const intx4 *>(a.filt) + ((size_t)cob0 * a.nCib + g) * 16 + p;
#pragma unroll
        for (int j = 0; j < GROUPS; ++j)
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) fa[j][wn] = filt[((size_t)wn * a.nCib + 4 * j) * 16] ^ flip;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            acc_w[wn] = zero;
            if (mfma_w) {
#pragma unroll
                for (int j = 0; j < GROUPS; ++j) acc_w[wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[j][wn], ones, acc_w[wn], 0, 0, 0);
            }
        }
        if (use_w && a.filt_sums) {
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) acc_w[wn] = signed_filter_sums(a, cob0 + wn, g);
        }
    }
    const size_t group_stride = (size_t)4 * a.HoWo;      // four input blocks further, in 16-byte units
    auto request = [&](int tile, intx4 (&rb)[GROUPS][WM]) __attribute__((always_inline)) {
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            int m = tile * (16 * WM) + wm * 16 + p;
            m = m < a.M ? m : a.M - 1;
            const int n = a.div_HoWo.div(m), pix = m - n * a.HoWo;
            const intx4 *px = reinterpret_cast<const intx4 *>(a.in) + ((size_t)n * a.nCib + g) * a.HoWo + pix;
#pragma unroll
            for (int j = 0; j < GROUPS; ++j) rb[j][wm] = px[j * group_stride];
        }
    };
    intx4 cur[GROUPS][WM];
    request(wv, cur);
    for (int tile = wv; tile < n_tiles; tile += n_waves) {
        intx4 nxt[GROUPS][WM];
        request(tile + n_waves < n_tiles ? tile + n_waves : tile, nxt);
        __builtin_amdgcn_sched_barrier(0);             // the requests above stay ahead of the arithmetic below
        intx4 acc[WM][WN], acc_s[WM];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            acc_s[wm] = zero;
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = zero;
        }
#pragma unroll
        for (int j = 0; j < GROUPS; ++j)
#pragma unroll
            for (int wm = 0; wm < WM; ++wm) {
                const intx4 fb = cur[j][wm] ^ flip;
#pragma unroll
                for (int wn = 0; wn < WN; ++wn) acc[wm][wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[j][wn], fb, acc[wm][wn], 0, 0, 0);
                if (use_s) acc_s[wm] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, fb, acc_s[wm], 0, 0, 0);
            }
        store_tiles<WM, WN>(a, acc, acc_s, acc_w, tile * (16 * WM), cob0, p, g);
#pragma unroll
        for (int j = 0; j < GROUPS; ++j)
#pragma unroll
            for (int wm = 0; wm < WM; ++wm) cur[j][wm] = nxt[j][wm];
    }
}

// ------------------------------------------------------------------------------------------------ single channel

struct QWindowArgs {
    const unsigned char *in, *filt;
    unsigned char *out;
    int N, H, W, Ho, Wo, nCb, Cb, kh, kw, stride, pt, pl;
    int mode;   // 0 depthwise, 1 max, 2 average
    FastDiv div_groups, div_Wo, div_Ho, div_nCb;
    QuantParams q;
};

// VEC channels per lane (4: one 32-bit word of a pixel's block; 1: any block size)
template <int VEC>
__global__ void __launch_bounds__(256) window_u8(QWindowArgs a, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index of a VEC-channel group of the blocked output
    if (i >= total) return;
    // i < 2^31 (the host checks the tensor size): divisions by launch constants
    const int groups = a.Cb / VEC;
    int t = a.div_groups.div((int)i);
    const int cg = (int)i - t * groups;
    int t2 = a.div_Wo.div(t);
    const int ow = t - t2 * a.Wo;
    t = a.div_Ho.div(t2);   // n * nCb + cb
    const int oh = t2 - t * a.Ho;
    const int cb = t - a.div_nCb.div(t) * a.nCb;
    int acc[VEC], cnt = 0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0;
    for (int ky = 0; ky < a.kh; ++ky) {
        const int ih = oh * a.stride + ky - a.pt;
        if (ih < 0 || ih >= a.H) continue;
        for (int kx = 0; kx < a.kw; ++kx) {
            const int iw = ow * a.stride + kx - a.pl;
            if (iw < 0 || iw >= a.W) continue;
            const unsigned char *x = a.in + (((size_t)t * a.H + ih) * a.W + iw) * a.Cb + cg * VEC;
            int xv[VEC], wv[VEC];
            if (VEC == 4) {
                const unsigned xw = *reinterpret_cast<const unsigned *>(x);
#pragma unroll
                for (int v = 0; v < VEC; ++v) xv[v] = (int)((xw >> (8 * v)) & 255u);
            } else {
                xv[0] = x[0];
            }
            if (a.mode == 0) {
                const unsigned char *w = a.filt + (((size_t)cb * a.kh + ky) * a.kw + kx) * a.Cb + cg * VEC;
                if (VEC == 4) {
                    const unsigned ww = *reinterpret_cast<const unsigned *>(w);
#pragma unroll
                    for (int v = 0; v < VEC; ++v) wv[v] = (int)((ww >> (8 * v)) & 255u);
                } else {
                    wv[0] = w[0];
                }
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] += (xv[v] - a.q.zx) * (wv[v] - a.q.zw);
            } else if (a.mode == 1) {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] = xv[v] > acc[v] ? xv[v] : acc[v];
            } else {
#pragma unroll
                for (int v = 0; v < VEC; ++v) acc[v] += xv[v];
            }
            ++cnt;
        }
    }
    unsigned packed = 0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) {
        int y;
        if (a.mode == 0) y = requant(acc[v], a.q);
        else if (a.mode == 1) y = acc[v];
        else y = cnt > 0 ? (acc[v] + cnt / 2) / cnt : 0;
        packed |= (unsigned)y << (8 * v);
    }
    unsigned char *o = a.out + i * VEC;
    if (VEC == 4) *reinterpret_cast<unsigned *>(o) = packed;
    else o[0] = (unsigned char)packed;
}

// Depthwise 3x3 on 16-byte blocks: a lane owns four channels (one 32-bit word of the block) of four output pixels
// 64 apart, so the nine filter words are unpacked to (w - zw) once per lane and every access of a wave is one
// contiguous kilobyte. Taps outside the image read a valid address and are replaced by the code zx, so that
// sum over all nine taps of x (w - zw) - zx * sum (w - zw) is the sum over the taps inside the image of (x - zx)(w - zw).
struct QDw3Args {
    const unsigned *in, *filt;
    unsigned *out;
    int H, W, Ho, Wo, HoWo, nCb, stride, pt, pl;
    FastDiv div_Wo, div_nCb;
    QuantParams q;
};

__global__ void __launch_bounds__(256) dw3x3_u8(QDw3Args a)
{
    const int cg = threadIdx.x & 3, pl64 = threadIdx.x >> 2;
    const int plane = blockIdx.y;                               // n * nCb + cb
    const int cb = plane - a.div_nCb.div(plane) * a.nCb;
    int wq[9][4], wsum[4] = {0, 0, 0, 0};
#pragma unroll
    for (int t = 0; t < 9; ++t) {
        const unsigned w = a.filt[(cb * 9 + t) * 4 + cg];
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            wq[t][c] = (int)((w >> (8 * c)) & 255u) - a.q.zw;
            wsum[c] += wq[t][c];
        }
    }
    const unsigned *img = a.in + (size_t)plane * a.H * a.W * 4 + cg;
    unsigned *dst = a.out + (size_t)plane * a.HoWo * 4 + cg;
    const unsigned zx4 = (unsigned)a.q.zx * 0x01010101u;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const int pix = (int)blockIdx.x * 256 + i * 64 + pl64;
        if (pix >= a.HoWo) break;
        const int oh = a.div_Wo.div(pix), ow = pix - oh * a.Wo;
        const int ih0 = oh * a.stride - a.pt, iw0 = ow * a.stride - a.pl;
        unsigned x[9];
#pragma unroll
        for (int ky = 0; ky < 3; ++ky)
#pragma unroll
            for (int kx = 0; kx < 3; ++kx) {
                const int ih = ih0 + ky, iw = iw0 + kx;
                const bool inside = (unsigned)ih < (unsigned)a.H && (unsigned)iw < (unsigned)a.W;
                const unsigned v = img[inside ? (ih * a.W + iw) * 4 : 0];
                x[ky * 3 + kx] = inside ? v : zx4;
            }
        unsigned packed = 0;
#pragma unroll
        for (int c = 0; c < 4; ++c) {
            int acc = -a.q.zx * wsum[c];
#pragma unroll
            for (int t = 0; t < 9; ++t) acc += (int)((x[t] >> (8 * c)) & 255u) * wq[t][c];
            packed |= (unsigned)requant(acc, a.q) << (8 * c);
        }
        dst[(size_t)pix * 4] = packed;
    }
}

__global__ void __launch_bounds__(256) relu_u8_kernel(const unsigned char *in, unsigned char *out, size_t n, int z)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = in[i] > z ? in[i] : (unsigned char)z;
}

typedef unsigned short ushortx2 __attribute__((ext_vector_type(2)));

// Byte-wise unsigned maximum of two words, as two packed 16-bit maxima over the even and the odd bytes.
struct SplitBytes { ushortx2 even, odd; };
__device__ __forceinline__ SplitBytes split_bytes(unsigned w)
{
    return SplitBytes{__builtin_bit_cast(ushortx2, w & 0x00ff00ffu), __builtin_bit_cast(ushortx2, (w >> 8) & 0x00ff00ffu)};
}
__device__ __forceinline__ SplitBytes max_bytes(SplitBytes a, SplitBytes b)
{
    return SplitBytes{__builtin_elementwise_max(a.even, b.even), __builtin_elementwise_max(a.odd, b.odd)};
}
__device__ __forceinline__ unsigned join_bytes(SplitBytes a)
{
    return __builtin_bit_cast(unsigned, a.even) | (__builtin_bit_cast(unsigned, a.odd) << 8);
}

// 16 bytes per lane, streaming loads and stores
__global__ void __launch_bounds__(256) relu_u8_vec16(const uintx4 *in, uintx4 *out, size_t n_vec, int z)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vec) return;
    const uintx4 v = __builtin_nontemporal_load(in + i);
    const SplitBytes zz = split_bytes((unsigned)z * 0x01010101u);
    uintx4 y;
    y.x = join_bytes(max_bytes(split_bytes(v.x), zz));
    y.y = join_bytes(max_bytes(split_bytes(v.y), zz));
    y.z = join_bytes(max_bytes(split_bytes(v.z), zz));
    y.w = join_bytes(max_bytes(split_bytes(v.w), zz));
    __builtin_nontemporal_store(y, out + i);
}

__device__ __forceinline__ unsigned add_one_u8(unsigned a, unsigned b, const AddQuantParams &q)
{
    long v = (long)((int)a - q.za) * (long)q.mult_a + (long)((int)b - q.zb) * (long)q.mult_b;
    if (q.shift > 0) v = (v + (1L << (q.shift - 1))) >> q.shift;
    v += q.zy;
    v = v < q.lo ? q.lo : v;
    v = v > q.hi ? q.hi : v;
    return (unsigned)v;
}

__global__ void __launch_bounds__(256) add_u8_kernel(const unsigned char *a, const unsigned char *b, unsigned char *out, size_t n,
                                                     AddQuantParams q)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = (unsigned char)add_one_u8(a[i], b[i], q);
}

__global__ void __launch_bounds__(256) add_u8_vec16(const uintx4 *a, const uintx4 *b, uintx4 *out, size_t n_vec, AddQuantParams q)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_vec) return;
    const uintx4 va = __builtin_nontemporal_load(a + i), vb = __builtin_nontemporal_load(b + i);
    uintx4 y;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        unsigned r = 0;
#pragma unroll
        for (int k = 0; k < 4; ++k) r |= add_one_u8((va[w] >> (8 * k)) & 255u, (vb[w] >> (8 * k)) & 255u, q) << (8 * k);
        y[w] = r;
    }
    __builtin_nontemporal_store(y, out + i);
}

// Max pooling on 16-byte blocks: a lane owns one output pixel's block and reads the 16 bytes of every tap inside the
// image (taps outside are skipped, as the layer's definition says); the running maximum stays split into even and
// odd bytes, so a tap costs three instructions to split and two packed maxima per word.
struct QPool16Args {
    const uintx4 *in;
    uintx4 *out;
    int H, W, Ho, Wo, kh, kw, stride, pt, pl;
    FastDiv div_Wo, div_Ho;
};

__global__ void __launch_bounds__(256) maxpool_u8_16(QPool16Args a, int total)
{
    const int i = (int)blockIdx.x * 256 + (int)threadIdx.x;          // output pixel over (plane, row, column)
    if (i >= total) return;
    const int t = a.div_Wo.div(i), ow = i - t * a.Wo;
    const int plane = a.div_Ho.div(t), oh = t - plane * a.Ho;
    const uintx4 *img = a.in + (size_t)plane * a.H * a.W;
    SplitBytes m[4];
#pragma unroll
    for (int w = 0; w < 4; ++w) m[w] = split_bytes(0u);
    for (int ky = 0; ky < a.kh; ++ky) {
        const int ih = oh * a.stride + ky - a.pt;
        if (ih < 0 || ih >= a.H) continue;
        for (int kx = 0; kx < a.kw; ++kx) {
            const int iw = ow * a.stride + kx - a.pl;
            if (iw < 0 || iw >= a.W) continue;
            const uintx4 v = img[ih * a.W + iw];
#pragma unroll
            for (int w = 0; w < 4; ++w) m[w] = max_bytes(m[w], split_bytes(v[w]));
        }
    }
    uintx4 y;
#pragma unroll
    for (int w = 0; w < 4; ++w) y[w] = join_bytes(m[w]);
    __builtin_nontemporal_store(y, a.out + i);
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

// Pixel groups (wm) and output blocks (wn) per wave: an input operand serves wn matrix instructions and a filter
// operand wm of them, and the sign flips of both cost vector instructions, which is what bounds these kernels:
// two pixel groups and as many output blocks (up to four) as divide the layer measured best at the sweep shapes,
// also where that leaves fewer workgroups than compute units.
// A reduction of at most eight chunks (pointwise layers on up to 128 channels) is one or two steps: load, multiply,
// requantize, store, with every wave of the launch in the same phase at the same time. Two output blocks per
// workgroup instead of four then give twice the waves to overlap those phases (10.7 -> 9.9 us on the audio CNN's
// pointwise layers at batch 1024, 14.9 -> 13.6 and 9.9 -> 8.9 us at the sweep's 64- and 128-channel shapes; with 16
// chunks it loses, 7.1 -> 7.5 us; one block per workgroup: slower again, the input is then read four times).
void pick_conv_tile(int nCob, int n_chunks, int &wm, int &wn)
{
    wm = 2;
    wn = nCob % 4 == 0 ? 4 : (nCob % 2 == 0 ? 2 : 1);
    if (wn == 4 && n_chunks <= 8) wn = 2;
}

QConvArgs conv_args(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                    const QuantParams &q, const int *filt_sums)
{
    QConvArgs a;
    a.in = in; a.filt = filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.HoWo = g.Ho * g.Wo; a.M = g.N * a.HoWo;
    a.nCib = g.Ci / g.Cib; a.nCob = g.Co / g.Cob; a.Cib = g.Cib; a.Cob = g.Cob;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    a.n_chunks = a.nCib * g.kh * g.kw;
    a.div_HoWo = make_fastdiv(a.HoWo);
    a.div_Wo = make_fastdiv(g.Wo);
    a.div_taps = make_fastdiv(g.kh * g.kw);
    a.div_kw = make_fastdiv(g.kw);
    a.filt_sums = filt_sums;
    a.q = q;
    return a;
}

}  // namespace

hipError_t launch_pack_u8(const unsigned char *nchw, unsigned char *blk, int N, int C, int H, int W, int Cb, bool unpack,
                          hipStream_t s)
{
    const size_t total = (size_t)N * C * H * W;
    hipLaunchKernelGGL(pack_u8_kernel, dim3(blocks_for(total)), dim3(256), 0, s, nchw, blk, C, H * W, Cb, total, unpack ? 1 : 0);
    return hipGetLastError();
}

hipError_t launch_pack_filter_u8(const unsigned char *oihw, unsigned char *blk, int Co, int Ci, int kh, int kw, int Cob,
                                 int Cib, hipStream_t s)
{
    const size_t total = (size_t)Co * Ci * kh * kw;
    hipLaunchKernelGGL(pack_filter_u8_kernel, dim3(blocks_for(total)), dim3(256), 0, s, oihw, blk, Co, Ci, kh * kw, Cob, Cib, total);
    return hipGetLastError();
}

hipError_t launch_filter_sums_u8(const unsigned char *filt, int *sums, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                                 hipStream_t s)
{
    hipLaunchKernelGGL(filter_sums_u8_kernel, dim3(blocks_for((size_t)Co)), dim3(256), 0, s, filt, sums, Co, Ci / Cib, kh * kw,
                       Cob, Cib);
    return hipGetLastError();
}

bool conv_u8_uses_mfma(const LayerGeom &g, const void *in, const void *filt, const void *out)
{
    const bool aligned = ((((uintptr_t)in | (uintptr_t)filt) & 15u) == 0) && (((uintptr_t)out & 3u) == 0);
    return aligned && g.Cib == 16 && g.Cob == 16;
}

hipError_t launch_conv_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                          const QuantParams &q, const int *filt_sums, hipStream_t s)
{
    if (conv_first_u8_eligible(g, out)) return launch_conv_first_u8(in, filt, out, g, q, s);
    if (dense_u8_eligible(g, in, filt)) return launch_dense_u8(in, filt, out, g, q, s);
    const QConvArgs a = conv_args(in, filt, out, g, q, filt_sums);
    if (conv_u8_uses_mfma(g, in, filt, out)) {
        const int corr = (q.zx != 128 && !filt_sums) ? 2 : (q.zw != 128 ? 1 : 0);
        // pointwise layers on 64 or 128 channels with enough pixels for a round of waves: the streaming kernel
        if (g.kh == 1 && g.kw == 1 && g.stride == 1 && g.pt == 0 && g.pl == 0 && g.Ho == g.H && g.Wo == g.W &&
            (a.nCib == 4 || a.nCib == 8) && a.nCob % 2 == 0 && (long)a.M >= 32L * 4 * device_cus()) {
            const int n_tiles = (a.M + 31) / 32;
            const int resident = 16 * device_cus();                                 // waves per output-block pair
            const int per_wave = (n_tiles + resident - 1) / resident;
            const int n_waves = (n_tiles + per_wave - 1) / per_wave;
            const dim3 grid((unsigned)((n_waves + 3) / 4), (unsigned)(a.nCob / 2));
#define SMALL_PW_CASE(C_, G_)                                                                                \
    if (corr == C_ && a.nCib == 4 * G_) hipLaunchKernelGGL((pw_u8_stream<2, 2, C_, G_>), grid, dim3(256), 0, s, a, n_tiles, n_waves);
            SMALL_PW_CASE(0, 1) SMALL_PW_CASE(1, 1) SMALL_PW_CASE(2, 1) SMALL_PW_CASE(0, 2) SMALL_PW_CASE(1, 2) SMALL_PW_CASE(2, 2)
#undef SMALL_PW_CASE
            return hipGetLastError();
        }
        int wm = 4, wn = 4;
        pick_conv_tile(a.nCob, a.n_chunks, wm, wn);
        const dim3 grid((unsigned)((a.M + 64 * wm - 1) / (64 * wm)), (unsigned)(a.nCob / wn));
#define SMALL_U8_CASE(M_, N_, C_)                                                                            \
    if (wm == M_ && wn == N_ && corr == C_) {                                                                \
        if (a.nCib % 4 == 0) hipLaunchKernelGGL((conv_u8_mfma4<M_, N_, C_, 3>), grid, dim3(256), 0, s, a);   \
        else if (a.n_chunks <= 4) hipLaunchKernelGGL((conv_u8_mfma_short<M_, N_, C_, 1>), grid, dim3(256), 0, s, a);  \
        else if (a.n_chunks <= 12) hipLaunchKernelGGL((conv_u8_mfma_short<M_, N_, C_, 3>), grid, dim3(256), 0, s, a); \
        else if (a.n_chunks <= 20) hipLaunchKernelGGL((conv_u8_mfma_short<M_, N_, C_, 5>), grid, dim3(256), 0, s, a); \
        else hipLaunchKernelGGL((conv_u8_mfma<M_, N_, C_>), grid, dim3(256), 0, s, a);                       \
    }
#define SMALL_U8_TILE(M_, N_) SMALL_U8_CASE(M_, N_, 0) SMALL_U8_CASE(M_, N_, 1) SMALL_U8_CASE(M_, N_, 2)
        SMALL_U8_TILE(2, 4) SMALL_U8_TILE(2, 2) SMALL_U8_TILE(2, 1)
#undef SMALL_U8_TILE
#undef SMALL_U8_CASE
        return hipGetLastError();
    }
    const size_t total = (size_t)a.M * g.Co;
    hipLaunchKernelGGL(conv_u8_direct, dim3(blocks_for(total)), dim3(256), 0, s, a, total);
    return hipGetLastError();
}

hipError_t launch_window_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                            int mode, const QuantParams &q, hipStream_t s)
{
    QWindowArgs a;
    a.in = in; a.filt = filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.nCb = g.Ci / g.Cib; a.Cb = g.Cib;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    a.mode = mode;
    a.q = q;
    if (mode == 0 && dw_dpp_u8_eligible(g, q, in, filt, out)) return launch_dw_dpp_u8(in, filt, out, g, q, s);
    if (pool_dpp_u8_eligible(g, mode, in, out)) return launch_pool_dpp_u8(in, out, g, s);
    if (avgpool_global_u8_eligible(g, mode, in, out)) return launch_avgpool_global_u8(in, out, g, s);
    if (mode == 0 && g.Cib == 16 && g.kh == 3 && g.kw == 3 &&
        ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)filt) & 3u) == 0) && (size_t)g.N * a.nCb <= 65535) {
        QDw3Args d;
        d.in = reinterpret_cast<const unsigned *>(in); d.filt = reinterpret_cast<const unsigned *>(filt);
        d.out = reinterpret_cast<unsigned *>(out);
        d.H = g.H; d.W = g.W; d.Ho = g.Ho; d.Wo = g.Wo; d.HoWo = g.Ho * g.Wo; d.nCb = a.nCb;
        d.stride = g.stride; d.pt = g.pt; d.pl = g.pl;
        d.div_Wo = make_fastdiv(g.Wo); d.div_nCb = make_fastdiv(a.nCb);
        d.q = q;
        hipLaunchKernelGGL(dw3x3_u8, dim3((unsigned)((d.HoWo + 255) / 256), (unsigned)(g.N * a.nCb)), dim3(256), 0, s, d);
        return hipGetLastError();
    }
    const size_t n_out = (size_t)g.N * g.Ci * g.Ho * g.Wo;
    if (mode == 1 && g.Cib == 16 && ((((uintptr_t)in | (uintptr_t)out) & 15u) == 0) && n_out / 16 < ((size_t)1 << 31) &&
        (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 31)) {
        QPool16Args p;
        p.in = reinterpret_cast<const uintx4 *>(in); p.out = reinterpret_cast<uintx4 *>(out);
        p.H = g.H; p.W = g.W; p.Ho = g.Ho; p.Wo = g.Wo; p.kh = g.kh; p.kw = g.kw; p.stride = g.stride; p.pt = g.pt; p.pl = g.pl;
        p.div_Wo = make_fastdiv(g.Wo); p.div_Ho = make_fastdiv(g.Ho);
        const int total = (int)(n_out / 16);
        hipLaunchKernelGGL(maxpool_u8_16, dim3(blocks_for((size_t)total)), dim3(256), 0, s, p, total);
        return hipGetLastError();
    }
    const bool words4 = g.Cib % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)(filt ? filt : in)) & 3u) == 0);
    a.div_groups = make_fastdiv(words4 ? g.Cib / 4 : g.Cib);
    a.div_Wo = make_fastdiv(g.Wo);
    a.div_Ho = make_fastdiv(g.Ho);
    a.div_nCb = make_fastdiv(a.nCb);
    const bool words = g.Cib % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)(filt ? filt : in)) & 3u) == 0);
    if (words) hipLaunchKernelGGL((window_u8<4>), dim3(blocks_for(n_out / 4)), dim3(256), 0, s, a, n_out / 4);
    else hipLaunchKernelGGL((window_u8<1>), dim3(blocks_for(n_out)), dim3(256), 0, s, a, n_out);
    return hipGetLastError();
}

hipError_t launch_relu_u8(const unsigned char *in, unsigned char *out, size_t n, int z, hipStream_t s)
{
    if (n % 16 == 0 && ((((uintptr_t)in | (uintptr_t)out) & 15u) == 0))
        hipLaunchKernelGGL(relu_u8_vec16, dim3(blocks_for(n / 16)), dim3(256), 0, s, reinterpret_cast<const uintx4 *>(in),
                           reinterpret_cast<uintx4 *>(out), n / 16, z);
    else hipLaunchKernelGGL(relu_u8_kernel, dim3(blocks_for(n)), dim3(256), 0, s, in, out, n, z);
    return hipGetLastError();
}

hipError_t launch_add_u8(const unsigned char *a, const unsigned char *b, unsigned char *out, size_t n, const AddQuantParams &q,
                         hipStream_t s)
{
    if (n % 16 == 0 && ((((uintptr_t)a | (uintptr_t)b | (uintptr_t)out) & 15u) == 0))
        hipLaunchKernelGGL(add_u8_vec16, dim3(blocks_for(n / 16)), dim3(256), 0, s, reinterpret_cast<const uintx4 *>(a),
                           reinterpret_cast<const uintx4 *>(b), reinterpret_cast<uintx4 *>(out), n / 16, q);
    else hipLaunchKernelGGL(add_u8_kernel, dim3(blocks_for(n)), dim3(256), 0, s, a, b, out, n, q);
    return hipGetLastError();
}

}  // namespace small
