// The two ends of a quantized network (Section "Quantized Inference": whole models on uint8 tensors with int32
// partial sums): the first convolution on an input of one or three channels (and the pointwise convolution on the
// eight channels such a layer may produce), the global average pooling and the
// small fully connected layer that close it. None of them has the 16 x 16 channel blocks the 8-bit matrix-core
// kernel needs, and all of them are small: plain vector code around the four-byte dot product (v_dot4_u32_u8),
// with the zero points taken out afterwards,
//     sum (x - zx)(w - zw) = sum x w - zx sum w - zw sum x + K zx zw,
// where a tap outside the image carries the code zx (its term is then zero) and K counts all taps.
#include "small_internal.h"

namespace small {

namespace {

constexpr unsigned kOnes = 0x01010101u;

__device__ __forceinline__ unsigned dot4(unsigned a, unsigned b, unsigned c) { return __builtin_amdgcn_udot4(a, b, c, false); }

// ------------------------------------------------------------------------------------------------ first convolution

struct FirstU8Args {
    const unsigned char *in, *filt;
    unsigned char *out;
    int H, W, Ho, Wo, HoWo, M, nCob, stride, pt, pl;
    unsigned in_bytes;
    FastDiv div_HoWo, div_Wo;
    QuantParams q;
};

// One lane per (output pixel, block of COB output channels; blockIdx.y counts the blocks): it gathers its window
// (K = KH * KW * CIB bytes, reduction index k = tap * CIB + channel, padded with zeros to KD words) into registers
// and walks the block's channels; the block's filters sit in LDS as one row of KD words per output channel (all lanes
// read the same word: a broadcast) beside their sums. A lane stores the COB codes of its pixel at once, so a wave's
// store is one contiguous run.
template <int KH, int KW, int CIB, int COB>
__global__ void __launch_bounds__(256) conv_first_u8(FirstU8Args a)
{
    constexpr int K = KH * KW * CIB, KD = (K + 15) / 16 * 4;
    __shared__ __attribute__((aligned(16))) unsigned wl[COB * KD];
    __shared__ int sw[COB];
    const int tid = threadIdx.x, cob = blockIdx.y;
    for (int i = tid; i < COB * KD; i += 256) {
        const int co = i / KD, kd = i - co * KD;
        unsigned w = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int k = 4 * kd + b;
            if (k < K) w |= (unsigned)a.filt[((cob * KH * KW + k / CIB) * COB + co) * CIB + k % CIB] << (8 * b);
        }
        wl[i] = w;
    }
    __syncthreads();
    if (tid < COB) {
        unsigned s = 0;
#pragma unroll
        for (int kd = 0; kd < KD; ++kd) s = dot4(wl[tid * KD + kd], kOnes, s);
        sw[tid] = (int)s;
    }

    const int m_raw = (int)blockIdx.x * 256 + tid;
    const bool live = m_raw < a.M;
    const int m = live ? m_raw : a.M - 1;
    const int n = a.div_HoWo.div(m), pix = m - n * a.HoWo;
    const int oh = a.div_Wo.div(pix), ow = pix - oh * a.Wo;
    // The window, row by row: a row's KW * CIB bytes are contiguous in memory and, in reduction order, contiguous in
    // the K-byte string x, so a row is NDW unaligned 32-bit loads (a load per byte, with its clamps, select and shift,
    // was two thirds of this kernel's vector instructions). Bytes of columns outside the image and whole rows outside
    // it become the code zx; bytes past the row's window become zero.
    constexpr int NB = KW * CIB, NDW = (NB + 3) / 4;
    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.in), 0, a.in_bytes, kRawBuffer);
    const int ih0 = oh * a.stride - a.pt, iw0 = ow * a.stride - a.pl;
    const unsigned zx4 = (unsigned)a.q.zx * kOnes;
    unsigned keep[NDW], fill[NDW];          // byte masks of a row's words: inside the image; outside it but inside the window
#pragma unroll
    for (int d = 0; d < NDW; ++d) {
        keep[d] = 0; fill[d] = 0;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const int j = 4 * d + b;
            if (j < NB) {
                const int col = iw0 + j / CIB;
                if (col >= 0 && col < a.W) keep[d] |= 0xffu << (8 * b);
                else fill[d] |= 0xffu << (8 * b);
            }
        }
        fill[d] &= zx4;
    }
    const int first = n * a.H * a.W * CIB + (ih0 * a.W + iw0) * CIB;        // byte offset of the window's first row
    // A 32-bit access that straddles either end of the tensor reads zero as a whole, also its bytes inside: where a
    // wave has such an access, words are read from the nearest offset inside and shifted into place.
    const int lim = (int)a.in_bytes - 4;
    const int last = first + (KH - 1) * a.W * CIB + 4 * (NDW - 1);
    const bool at_an_end = __builtin_amdgcn_ballot_w64(first < 0 || last > lim) != 0;
    unsigned x[KD];
#pragma unroll
    for (int kd = 0; kd < KD; ++kd) x[kd] = 0;
#pragma unroll
    for (int ky = 0; ky < KH; ++ky) {
        const bool row_in = (unsigned)(ih0 + ky) < (unsigned)a.H;
        unsigned r[NDW];
#pragma unroll
        for (int d = 0; d < NDW; ++d) {
            const int off = first + ky * a.W * CIB + 4 * d;
            unsigned v;
            if (!at_an_end) {
                v = __builtin_amdgcn_raw_buffer_load_b32(src, row_in ? (unsigned)off : kBeyond, 0, 0);
            } else {
                const int inside = min(max(off, 0), lim), by = off - inside;       // by < 0: the word lies before the tensor
                const unsigned w = __builtin_amdgcn_raw_buffer_load_b32(src, row_in ? (unsigned)inside : kBeyond, 0, 0);
                v = by == 0 ? w : (by < 0 ? (by > -4 ? w << (-8 * by) : 0u) : (by < 4 ? w >> (8 * by) : 0u));
            }
            // (a row outside the image: zx in every byte of the window)
            const unsigned window = 4 * d + 4 <= NB ? 0xffffffffu : (NB > 4 * d ? (1u << (8 * (NB - 4 * d))) - 1u : 0u);
            r[d] = row_in ? ((v & keep[d]) | fill[d]) : (zx4 & window);
        }
        const int at = ky * NB;                    // the row's place in x, in bytes (a constant once unrolled)
#pragma unroll
        for (int d = 0; d < NDW; ++d) {
            const int word = (at + 4 * d) / 4, sh = 8 * ((at + 4 * d) % 4);
            if (word < KD) x[word] |= r[d] << sh;
            if (sh != 0 && word + 1 < KD) x[word + 1] |= r[d] >> (32 - sh);
        }
    }
    unsigned sx = 0;
#pragma unroll
    for (int kd = 0; kd < KD; ++kd) sx = dot4(x[kd], kOnes, sx);
    const int base = K * a.q.zx * a.q.zw - a.q.zw * (int)sx;
    __syncthreads();                                     // the filter sums

    const bool narrow = a.q.amax > 0;                    // (uniform) the five-instruction requantization applies
    const long bias = requant_bias(a.q);
    unsigned packed[COB / 4];
#pragma unroll
    for (int j = 0; j < COB / 4; ++j) packed[j] = 0;
#pragma unroll
    for (int co = 0; co < COB; ++co) {
        unsigned dot = 0;
#pragma unroll
        for (int kd = 0; kd < KD; ++kd) dot = dot4(x[kd], wl[co * KD + kd], dot);
        const int acc = (int)dot - a.q.zx * sw[co] + base;
        packed[co / 4] |= (unsigned)(narrow ? requant_clamped(acc, a.q, bias) : requant(acc, a.q)) << (8 * (co % 4));
    }
    if (live) {
        unsigned char *o = a.out + ((size_t)(n * a.nCob + cob) * a.HoWo + pix) * COB;
        if constexpr (COB == 16) *reinterpret_cast<uintx4 *>(o) = uintx4{packed[0], packed[1], packed[2], packed[3]};
        else *reinterpret_cast<uint2 *>(o) = uint2{packed[0], packed[1]};
    }
}

// ------------------------------------------------------------------------------------------------ global average

struct AvgU8Args {
    const uintx4 *in;
    uintx4 *out;
    int planes, HW;
    FastDiv by_HW;
};

// A wave per (image, 16-byte block): lanes take the pixels 64 apart, sixteen 32-bit sums each (a dot product with a
// one-byte mask adds one byte of a word), then the wave's sums meet by exchanges between lanes; the mean is
// (sum + count / 2) / count, the rule of the windowed average.
__global__ void __launch_bounds__(256) avgpool_global_u8(AvgU8Args a)
{
    const int lane = threadIdx.x & 63;
    const int plane = (int)blockIdx.x * 4 + ((int)threadIdx.x >> 6);
    if (plane >= a.planes) return;
    const uintx4 *p = a.in + (size_t)plane * a.HW;
    unsigned s[16];
#pragma unroll
    for (int c = 0; c < 16; ++c) s[c] = 0;
    for (int i = lane; i < a.HW; i += 64) {
        const uintx4 v = p[i];
        const unsigned w0 = v.x, w1 = v.y, w2 = v.z, w3 = v.w;
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            s[b] = dot4(w0, 1u << (8 * b), s[b]);
            s[4 + b] = dot4(w1, 1u << (8 * b), s[4 + b]);
            s[8 + b] = dot4(w2, 1u << (8 * b), s[8 + b]);
            s[12 + b] = dot4(w3, 1u << (8 * b), s[12 + b]);
        }
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1)
#pragma unroll
        for (int c = 0; c < 16; ++c) s[c] += (unsigned)__shfl_xor((int)s[c], off, 64);
    if (lane == 0) {
        unsigned y[4] = {0, 0, 0, 0};
#pragma unroll
        for (int c = 0; c < 16; ++c) y[c / 4] |= (unsigned)a.by_HW.div((int)s[c] + a.HW / 2) << (8 * (c % 4));
        a.out[plane] = uintx4{y[0], y[1], y[2], y[3]};
    }
}

// ------------------------------------------------------------------------------------------------ fully connected

struct DenseU8Args {
    const uintx4 *in, *filt;
    unsigned char *out;
    int N, nCib, nCob, Cob;
    QuantParams q;
};

// A wave per (image, block of at most 16 outputs): lane = 16 part + output; the four parts split the input blocks,
// each step being 16 input codes against the 16 filter codes of the lane's output (four dot products), with the
// sums of both operands taken on the way; the parts meet by two exchanges.
__global__ void __launch_bounds__(256) dense_u8(DenseU8Args a)
{
    const int lane = threadIdx.x & 63, co = lane & 15, part = lane >> 4;
    const int unit = (int)blockIdx.x * 4 + ((int)threadIdx.x >> 6);
    if (unit >= a.N * a.nCob) return;
    const int n = unit / a.nCob, cob = unit - n * a.nCob;
    const bool mine = co < a.Cob;
    const uintx4 *x = a.in + (size_t)n * a.nCib;
    const uintx4 *w = a.filt + ((size_t)cob * a.nCib * a.Cob + (mine ? co : 0));
    unsigned dot = 0, sx = 0, sw = 0;
    for (int cib = part; cib < a.nCib; cib += 4) {
        const uintx4 xv = x[cib], wv = w[(size_t)cib * a.Cob];
        const unsigned x0 = xv.x, x1 = xv.y, x2 = xv.z, x3 = xv.w, w0 = wv.x, w1 = wv.y, w2 = wv.z, w3 = wv.w;
        dot = dot4(x0, w0, dot); dot = dot4(x1, w1, dot); dot = dot4(x2, w2, dot); dot = dot4(x3, w3, dot);
        sx = dot4(x0, kOnes, sx); sx = dot4(x1, kOnes, sx); sx = dot4(x2, kOnes, sx); sx = dot4(x3, kOnes, sx);
        sw = dot4(w0, kOnes, sw); sw = dot4(w1, kOnes, sw); sw = dot4(w2, kOnes, sw); sw = dot4(w3, kOnes, sw);
    }
#pragma unroll
    for (int off = 32; off >= 16; off >>= 1) {
        dot += (unsigned)__shfl_xor((int)dot, off, 64);
        sx += (unsigned)__shfl_xor((int)sx, off, 64);
        sw += (unsigned)__shfl_xor((int)sw, off, 64);
    }
    if (mine && part == 0) {
        const int K = a.nCib * 16;
        const int acc = (int)dot - a.q.zx * (int)sw - a.q.zw * (int)sx + K * a.q.zx * a.q.zw;
        a.out[(size_t)unit * a.Cob + co] = (unsigned char)requant(acc, a.q);
    }
}

template <int KH, int KW, int CIB>
hipError_t launch_first(const FirstU8Args &a, int Cob, hipStream_t s)
{
    const dim3 grid((unsigned)((a.M + 255) / 256), (unsigned)a.nCob);
    if (Cob == 16) hipLaunchKernelGGL((conv_first_u8<KH, KW, CIB, 16>), grid, dim3(256), 0, s, a);
    else hipLaunchKernelGGL((conv_first_u8<KH, KW, CIB, 8>), grid, dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace

bool conv_first_u8_eligible(const LayerGeom &g, const void *out)
{
    const bool shape = (g.kh == 3 && g.kw == 3 && g.Cib == 3) || (g.kh == 10 && g.kw == 4 && g.Cib == 1) ||
                       (g.kh == 1 && g.kw == 1 && g.Cib == 8);
    if (!shape || g.Ci != g.Cib || (g.Cob != 16 && g.Cob != 8) || g.Co / g.Cob > 65535) return false;
    if (((uintptr_t)out & (uintptr_t)(g.Cob - 1)) != 0) return false;
    return (size_t)g.N * g.Ho * g.Wo < ((size_t)1 << 31) && (size_t)g.N * g.H * g.W * g.Ci < ((size_t)1 << 31) &&
           (size_t)g.N * g.H * g.W * g.Ci >= 4;
}

hipError_t launch_conv_first_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                                const QuantParams &q, hipStream_t s)
{
    FirstU8Args a;
    a.in = in; a.filt = filt; a.out = out;
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo; a.HoWo = g.Ho * g.Wo; a.M = g.N * a.HoWo;
    a.nCob = g.Co / g.Cob; a.stride = g.stride; a.pt = g.pt; a.pl = g.pl;
    a.in_bytes = (unsigned)((size_t)g.N * g.H * g.W * g.Ci);
    a.div_HoWo = make_fastdiv(a.HoWo);
    a.div_Wo = make_fastdiv(g.Wo);
    a.q = q;
    if (g.Cib == 8) return launch_first<1, 1, 8>(a, g.Cob, s);
    return g.Cib == 3 ? launch_first<3, 3, 3>(a, g.Cob, s) : launch_first<10, 4, 1>(a, g.Cob, s);
}

bool avgpool_global_u8_eligible(const LayerGeom &g, int mode, const void *in, const void *out)
{
    if (mode != 2 || g.Cib != 16 || g.Ho != 1 || g.Wo != 1 || g.kh != g.H || g.kw != g.W || g.pt != 0 || g.pl != 0) return false;
    if ((((uintptr_t)in | (uintptr_t)out) & 15u) != 0) return false;
    return (size_t)g.H * g.W < ((size_t)1 << 23) && (size_t)g.N * (g.Ci / 16) < ((size_t)1 << 31);      // sums below 2^31
}

hipError_t launch_avgpool_global_u8(const unsigned char *in, unsigned char *out, const LayerGeom &g, hipStream_t s)
{
    AvgU8Args a;
    a.in = reinterpret_cast<const uintx4 *>(in); a.out = reinterpret_cast<uintx4 *>(out);
    a.planes = g.N * (g.Ci / 16); a.HW = g.H * g.W;
    a.by_HW = make_fastdiv(a.HW);
    hipLaunchKernelGGL(avgpool_global_u8, dim3((unsigned)((a.planes + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

bool dense_u8_eligible(const LayerGeom &g, const void *in, const void *filt)
{
    if (g.H != 1 || g.W != 1 || g.kh != 1 || g.kw != 1 || g.Ho != 1 || g.Wo != 1 || g.Cib != 16 || g.Cob >= 16) return false;
    if ((((uintptr_t)in | (uintptr_t)filt) & 15u) != 0) return false;
    return (size_t)g.N * (g.Co / g.Cob) < ((size_t)1 << 31);
}

hipError_t launch_dense_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                           const QuantParams &q, hipStream_t s)
{
    DenseU8Args a;
    a.in = reinterpret_cast<const uintx4 *>(in); a.filt = reinterpret_cast<const uintx4 *>(filt); a.out = out;
    a.N = g.N; a.nCib = g.Ci / 16; a.nCob = g.Co / g.Cob; a.Cob = g.Cob;
    a.q = q;
    hipLaunchKernelGGL(dense_u8, dim3((unsigned)((g.N * a.nCob + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace small
