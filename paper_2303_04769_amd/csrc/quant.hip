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

__device__ __forceinline__ int requant(int acc, const QuantParams &q)
{
    long v = (long)acc * (long)q.mult;
    if (q.shift > 0) v = (v + (1L << (q.shift - 1))) >> q.shift;
    v += q.zy;
    v = v < q.lo ? q.lo : v;
    v = v > q.hi ? q.hi : v;
    return (int)v;
}

struct QConvArgs {
    const unsigned char *in, *filt;
    unsigned char *out;
    int N, H, W, Ho, Wo, HoWo, M;
    int nCib, nCob, Cib, Cob, kh, kw, stride, pt, pl;
    int n_chunks;     // nCib * kh * kw (matrix-core kernel)
    QuantParams q;
};

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
template <int WM, int WN>
__global__ void __launch_bounds__(256) conv_u8_mfma(QConvArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const int HW = a.H * a.W;
    const int za = a.q.zx - 128, zb = a.q.zw - 128;
    const bool use_s = zb != 0, use_w = za != 0;

    int ih0[WM], iw0[WM];
    size_t img[WM];       // 16-byte pixel index of the image's first block
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        int m = tile0 + wm * 16 + p;
        m = m < a.M ? m : a.M - 1;
        const int n = m / a.HoWo, rem = m - n * a.HoWo;
        const int oh = rem / a.Wo, ow = rem - oh * a.Wo;
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
            fb[wm] = intx4{zx4, zx4, zx4, zx4};
            if (inside) fb[wm] = in[img[wm] + (size_t)cib * HW + ih * a.W + iw];
            fb[wm] ^= flip;
            if (!live) fb[wm] = zero;
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
        if (use_w) {
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

    // lane (p, g) holds output channels 4g .. 4g+3 of pixel p: four consecutive bytes of the blocked output
    const unsigned K = (unsigned)a.n_chunks * 16u;
    const unsigned kab = K * (unsigned)(za * zb);
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        const int m = tile0 + wm * 16 + p;
        if (m >= a.M) continue;
        const int n = m / a.HoWo, pix = m - n * a.HoWo;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            unsigned packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                // wrap-around arithmetic: the true sum fits 32 bits, the partial terms need not
                const unsigned v = (unsigned)acc[wm][wn][r] - (unsigned)zb * (unsigned)acc_s[wm][r] -
                                   (unsigned)za * (unsigned)acc_w[wn][r] + kab;
                packed |= (unsigned)requant((int)v, a.q) << (8 * r);
            }
            unsigned *o = reinterpret_cast<unsigned *>(a.out + (((size_t)n * a.nCob + cob0 + wn) * a.HoWo + pix) * 16 + g * 4);
            *o = packed;
        }
    }
}

// The same tile for layers whose input has a multiple of four 16-channel blocks: one matrix instruction takes one
// filter tap of four consecutive input blocks (lane group g = block 4j + g), so the tap, its bounds test and the
// operand addresses are per-tap values and the walk over j only adds constants.
template <int WM, int WN>
__global__ void __launch_bounds__(256) conv_u8_mfma4(QConvArgs a)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int p = lane & 15, g = lane >> 4;
    const int cob0 = blockIdx.y * WN;
    const int tile0 = ((int)blockIdx.x * 4 + wave) * (16 * WM);
    const int HW = a.H * a.W;
    const int za = a.q.zx - 128, zb = a.q.zw - 128;
    const bool use_s = zb != 0, use_w = za != 0;
    const int taps = a.kh * a.kw;

    int ih0[WM], iw0[WM];
    const intx4 *img[WM];       // this lane group's first input block of the pixel's image
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        int m = tile0 + wm * 16 + p;
        m = m < a.M ? m : a.M - 1;
        const int n = m / a.HoWo, rem = m - n * a.HoWo;
        const int oh = rem / a.Wo, ow = rem - oh * a.Wo;
        ih0[wm] = oh * a.stride - a.pt;
        iw0[wm] = ow * a.stride - a.pl;
        img[wm] = reinterpret_cast<const intx4 *>(a.in) + ((size_t)n * a.nCib + g) * HW;
    }
    // filter block (cob, cib, tap) holds 16 rows of 16 bytes: row p of block (cob0, g, 0)
    const intx4 *filt = reinterpret_cast<const intx4 *>(a.filt) + ((size_t)cob0 * a.n_chunks + (size_t)g * taps) * 16 + p;
    const size_t cob_stride = (size_t)a.n_chunks * 16;
    const int flip = (int)0x80808080u;
    const int zx4 = a.q.zx * 0x01010101;
    const intx4 ones = {0x01010101, 0x01010101, 0x01010101, 0x01010101};
    const intx4 zero = {0, 0, 0, 0};
    const intx4 pad = {zx4 ^ flip, zx4 ^ flip, zx4 ^ flip, zx4 ^ flip};

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
    int ky = 0, kx = 0;
    for (int tap = 0; tap < taps; ++tap) {
        const intx4 *bp[WM];
        bool inside[WM];
#pragma unroll
        for (int wm = 0; wm < WM; ++wm) {
            const int ih = ih0[wm] + ky, iw = iw0[wm] + kx;
            inside[wm] = ih >= 0 && ih < a.H && iw >= 0 && iw < a.W;
            bp[wm] = img[wm] + (inside[wm] ? ih * a.W + iw : 0);
        }
        const intx4 *ap = filt + (size_t)tap * 16;
        for (int j = 0; j < groups; ++j) {
            intx4 fa[WN], fb[WM];
#pragma unroll
            for (int wn = 0; wn < WN; ++wn) fa[wn] = ap[wn * cob_stride] ^ flip;
#pragma unroll
            for (int wm = 0; wm < WM; ++wm) {
                fb[wm] = pad;
                if (inside[wm]) fb[wm] = *bp[wm] ^ flip;
                bp[wm] += (size_t)4 * HW;
            }
            ap += (size_t)4 * taps * 16;
#pragma unroll
            for (int wm = 0; wm < WM; ++wm) {
#pragma unroll
                for (int wn = 0; wn < WN; ++wn)
                    acc[wm][wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], fb[wm], acc[wm][wn], 0, 0, 0);
                if (use_s) acc_s[wm] = __builtin_amdgcn_mfma_i32_16x16x64_i8(ones, fb[wm], acc_s[wm], 0, 0, 0);
            }
            if (use_w) {
#pragma unroll
                for (int wn = 0; wn < WN; ++wn)
                    acc_w[wn] = __builtin_amdgcn_mfma_i32_16x16x64_i8(fa[wn], ones, acc_w[wn], 0, 0, 0);
            }
        }
        if (++kx == a.kw) { kx = 0; ++ky; }
    }

    const unsigned K = (unsigned)a.n_chunks * 16u;
    const unsigned kab = K * (unsigned)(za * zb);
#pragma unroll
    for (int wm = 0; wm < WM; ++wm) {
        const int m = tile0 + wm * 16 + p;
        if (m >= a.M) continue;
        const int n = m / a.HoWo, pix = m - n * a.HoWo;
#pragma unroll
        for (int wn = 0; wn < WN; ++wn) {
            unsigned packed = 0;
#pragma unroll
            for (int r = 0; r < 4; ++r) {
                const unsigned v = (unsigned)acc[wm][wn][r] - (unsigned)zb * (unsigned)acc_s[wm][r] -
                                   (unsigned)za * (unsigned)acc_w[wn][r] + kab;
                packed |= (unsigned)requant((int)v, a.q) << (8 * r);
            }
            unsigned *o = reinterpret_cast<unsigned *>(a.out + (((size_t)n * a.nCob + cob0 + wn) * a.HoWo + pix) * 16 + g * 4);
            *o = packed;
        }
    }
}

// ------------------------------------------------------------------------------------------------ single channel

struct QWindowArgs {
    const unsigned char *in, *filt;
    unsigned char *out;
    int N, H, W, Ho, Wo, nCb, Cb, kh, kw, stride, pt, pl;
    int mode;   // 0 depthwise, 1 max, 2 average
    QuantParams q;
};

// VEC channels per lane (4: one 32-bit word of a pixel's block; 1: any block size)
template <int VEC>
__global__ void __launch_bounds__(256) window_u8(QWindowArgs a, size_t total)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;   // index of a VEC-channel group of the blocked output
    if (i >= total) return;
    const int groups = a.Cb / VEC;
    const int cg = (int)(i % groups);
    size_t t = i / groups;
    const int ow = (int)(t % a.Wo);
    t /= a.Wo;
    const int oh = (int)(t % a.Ho);
    t /= a.Ho;   // n * nCb + cb
    const int cb = (int)(t % a.nCb);
    int acc[VEC], cnt = 0;
#pragma unroll
    for (int v = 0; v < VEC; ++v) acc[v] = 0;
    for (int ky = 0; ky < a.kh; ++ky) {
        const int ih = oh * a.stride + ky - a.pt;
        if (ih < 0 || ih >= a.H) continue;
        for (int kx = 0; kx < a.kw; ++kx) {
            const int iw = ow * a.stride + kx - a.pl;
            if (iw < 0 || iw >= a.W) continue;
            const unsigned char *x = a.in + ((t * a.H + ih) * a.W + iw) * a.Cb + cg * VEC;
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

__global__ void __launch_bounds__(256) relu_u8_kernel(const unsigned char *in, unsigned char *out, size_t n, int z)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i < n) out[i] = in[i] > z ? in[i] : (unsigned char)z;
}

__global__ void __launch_bounds__(256) relu_u8_words(const unsigned *in, unsigned *out, size_t n_words, int z)
{
    const size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (i >= n_words) return;
    const unsigned w = in[i];
    unsigned y = 0;
#pragma unroll
    for (int v = 0; v < 4; ++v) {
        const unsigned b = (w >> (8 * v)) & 255u;
        y |= (b > (unsigned)z ? b : (unsigned)z) << (8 * v);
    }
    out[i] = y;
}

inline unsigned blocks_for(size_t n) { return (unsigned)((n + 255) / 256); }

// Pixel groups (wm) and output blocks (wn) per wave: an input operand serves wn matrix instructions and a filter
// operand wm of them. Four output blocks and two pixel groups measured best at the sweep shapes; smaller tiles
// when the grid would otherwise have fewer than two workgroups per compute unit.
void pick_conv_tile(int M, int nCob, int &wm, int &wn)
{
    wn = nCob % 4 == 0 ? 4 : (nCob % 2 == 0 ? 2 : 1);
    wm = 2;
    auto wgs = [&](int m, int n) { return ((long)M + 64 * m - 1) / (64 * m) * (nCob / n); };
    if (wgs(wm, wn) < 512) wm = 1;
    if (wgs(wm, wn) < 512 && wn == 4) wn = 2;
}

QConvArgs conv_args(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                    const QuantParams &q)
{
    QConvArgs a;
    a.in = in; a.filt = filt; a.out = out;
    a.N = g.N; a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.HoWo = g.Ho * g.Wo; a.M = g.N * a.HoWo;
    a.nCib = g.Ci / g.Cib; a.nCob = g.Co / g.Cob; a.Cib = g.Cib; a.Cob = g.Cob;
    a.kh = g.kh; a.kw = g.kw; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    a.n_chunks = a.nCib * g.kh * g.kw;
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

bool conv_u8_uses_mfma(const LayerGeom &g, const void *in, const void *filt, const void *out)
{
    const bool aligned = ((((uintptr_t)in | (uintptr_t)filt) & 15u) == 0) && (((uintptr_t)out & 3u) == 0);
    return aligned && g.Cib == 16 && g.Cob == 16;
}

hipError_t launch_conv_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                          const QuantParams &q, hipStream_t s)
{
    const QConvArgs a = conv_args(in, filt, out, g, q);
    if (conv_u8_uses_mfma(g, in, filt, out)) {
        int wm = 4, wn = 4;
        pick_conv_tile(a.M, a.nCob, wm, wn);
        const dim3 grid((unsigned)((a.M + 64 * wm - 1) / (64 * wm)), (unsigned)(a.nCob / wn));
#define SMALL_U8_CASE(M_, N_)                                                                         \
    if (wm == M_ && wn == N_) {                                                                       \
        if (a.nCib % 4 == 0) hipLaunchKernelGGL((conv_u8_mfma4<M_, N_>), grid, dim3(256), 0, s, a);   \
        else hipLaunchKernelGGL((conv_u8_mfma<M_, N_>), grid, dim3(256), 0, s, a);                    \
    }
        SMALL_U8_CASE(2, 4); SMALL_U8_CASE(2, 2); SMALL_U8_CASE(2, 1);
        SMALL_U8_CASE(1, 4); SMALL_U8_CASE(1, 2); SMALL_U8_CASE(1, 1);
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
    const size_t n_out = (size_t)g.N * g.Ci * g.Ho * g.Wo;
    const bool words = g.Cib % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out | (uintptr_t)(filt ? filt : in)) & 3u) == 0);
    if (words) hipLaunchKernelGGL((window_u8<4>), dim3(blocks_for(n_out / 4)), dim3(256), 0, s, a, n_out / 4);
    else hipLaunchKernelGGL((window_u8<1>), dim3(blocks_for(n_out)), dim3(256), 0, s, a, n_out);
    return hipGetLastError();
}

hipError_t launch_relu_u8(const unsigned char *in, unsigned char *out, size_t n, int z, hipStream_t s)
{
    if (n % 4 == 0 && ((((uintptr_t)in | (uintptr_t)out) & 3u) == 0))
        hipLaunchKernelGGL(relu_u8_words, dim3(blocks_for(n / 4)), dim3(256), 0, s, reinterpret_cast<const unsigned *>(in),
                           reinterpret_cast<unsigned *>(out), n / 4, z);
    else hipLaunchKernelGGL(relu_u8_kernel, dim3(blocks_for(n)), dim3(256), 0, s, in, out, n, z);
    return hipGetLastError();
}

}  // namespace small
