// Quantized max pooling, 3x3 window, stride 2, no padding, 16-byte channel blocks: codes in, codes out (the maximum
// of codes is the code of the maximum: one scale, Section "Quantized Inference"). HBM-bound: 1.25 bytes moved per
// input byte, no arithmetic to speak of.
//
// A wave owns a band of 64 neighbouring pixels of a plane (a lane holds the 16-byte block of its pixel, so a row of
// the band is one contiguous kilobyte) and a strip of at most 7 output rows = 15 input rows, all requested at once.
// The horizontal maximum of a row, max(x[l], x[l + 1], x[l + 2]), takes its neighbours from the next lanes by lane
// shifts over the whole wave (wave_shl:1, twice); lane 2j then holds output column j of the band: 31 outputs per
// band of 64 pixels (bands overlap by two pixels; a 56-pixel row is one band). The vertical maximum runs over the
// rows' horizontal maxima, every input row being loaded and reduced once per strip. Byte-wise maxima are two packed
// 16-bit maxima over the even and the odd bytes of a word; the running values stay in that split form.
// Lanes and rows with nothing to load or store use an offset beyond the tensors' buffer descriptors.
#include "small_internal.h"

namespace small {

namespace {

typedef unsigned short ushortx2 __attribute__((ext_vector_type(2)));

struct PoolU8Args {
    const unsigned char *in;
    unsigned char *out;
    int H, W, Ho, Wo;
    int n_planes, nb, sp, n_units;
    unsigned in_bytes, out_bytes;
    FastDiv by_nb, by_sp;
};

constexpr int kPoolStripRows = 7;                      // output rows of a strip, at most
constexpr int kPoolInRows = 2 * kPoolStripRows + 1;    // its input rows
constexpr int kWaveShl1 = 0x130;                       // lane l reads lane l + 1 of the wave (lane 63: zero)

struct Split { ushortx2 even[4], odd[4]; };            // a 16-byte block as 8 + 8 bytes, each in a 16-bit slot

__device__ __forceinline__ Split split16(uintx4 v)
{
    Split s;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        s.even[k] = __builtin_bit_cast(ushortx2, v[k] & 0x00ff00ffu);
        s.odd[k] = __builtin_bit_cast(ushortx2, (v[k] >> 8) & 0x00ff00ffu);
    }
    return s;
}
__device__ __forceinline__ Split max16(Split a, const Split &b)
{
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        a.even[k] = __builtin_elementwise_max(a.even[k], b.even[k]);
        a.odd[k] = __builtin_elementwise_max(a.odd[k], b.odd[k]);
    }
    return a;
}
__device__ __forceinline__ uintx4 join16(const Split &s)
{
    uintx4 v;
#pragma unroll
    for (int k = 0; k < 4; ++k) v[k] = __builtin_bit_cast(unsigned, s.even[k]) | (__builtin_bit_cast(unsigned, s.odd[k]) << 8);
    return v;
}
__device__ __forceinline__ uintx4 next_lane(uintx4 v)
{
    uintx4 r;
#pragma unroll
    for (int k = 0; k < 4; ++k) r[k] = (unsigned)__builtin_amdgcn_update_dpp(0, (int)v[k], kWaveShl1, 0xf, 0xf, true);
    return r;
}

__global__ void __launch_bounds__(256) maxpool3s2_u8_rows(PoolU8Args a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int unit = (int)blockIdx.x * 4 + wave;
    if (unit >= a.n_units) return;
    const int t = a.by_nb.div(unit), band = unit - t * a.nb;
    const int plane = a.by_sp.div(t), strip = t - plane * a.sp;
    const int r0 = a.by_sp.div(strip * a.Ho), r1 = a.by_sp.div((strip + 1) * a.Ho);      // output rows r0 .. r1 - 1
    const int n_out = r1 - r0, n_in = 2 * n_out + 1;

    const int x = band * 62 + lane;                              // input column of this lane
    const int ow = band * 31 + (lane >> 1);                      // output column (even lanes)
    const bool col_in = x < a.W;
    const bool col_out = !(lane & 1) && lane <= 60 && ow < a.Wo;
    const unsigned at_in = (unsigned)plane * (unsigned)(a.H * a.W * 16) + (unsigned)(x * 16);
    const unsigned at_out = (unsigned)plane * (unsigned)(a.Ho * a.Wo * 16) + (unsigned)(ow * 16);

    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char *>(a.in), 0, a.in_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, kRawBuffer);

    uintx4 raw[kPoolInRows];
#pragma unroll
    for (int j = 0; j < kPoolInRows; ++j) {
        const bool have = col_in && j < n_in;
        raw[j] = __builtin_amdgcn_raw_buffer_load_b128(src, have ? at_in + (unsigned)((2 * r0 + j) * a.W * 16) : kBeyond, 0, kNonTemporal);
    }
    Split h[3];                                                  // horizontal maxima of the rows 2r, 2r + 1, 2r + 2
#pragma unroll
    for (int j = 0; j < kPoolInRows; ++j) {
        const uintx4 s1 = next_lane(raw[j]), s2 = next_lane(s1);
        h[j % 3] = max16(max16(split16(raw[j]), split16(s1)), split16(s2));
        if (j >= 2 && !(j & 1)) {
            // rows j - 2, j - 1, j are output row r0 + j / 2 - 1
            const int r = j / 2 - 1;
            const Split m = max16(max16(h[(j + 1) % 3], h[(j + 2) % 3]), h[j % 3]);
            const unsigned off = (col_out && r < n_out) ? at_out + (unsigned)((r0 + r) * a.Wo * 16) : kBeyond;
            __builtin_amdgcn_raw_buffer_store_b128(join16(m), dst, off, 0, kNonTemporal);
        }
    }
}

}  // namespace

bool pool_dpp_u8_eligible(const LayerGeom &g, int mode, const void *in, const void *out)
{
    if (mode != 1 || g.Cib != 16 || g.kh != 3 || g.kw != 3 || g.stride != 2 || g.pt != 0 || g.pl != 0) return false;
    if (g.Ho != (g.H - 3) / 2 + 1 || g.Wo != (g.W - 3) / 2 + 1) return false;          // (no bottom / right padding either)
    if ((((uintptr_t)in | (uintptr_t)out) & 15u) != 0) return false;
    return (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 31);
}

hipError_t launch_pool_dpp_u8(const unsigned char *in, unsigned char *out, const LayerGeom &g, hipStream_t s)
{
    PoolU8Args a;
    a.in = in; a.out = out;
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo;
    a.n_planes = g.N * (g.Ci / 16);
    a.nb = (g.Wo + 30) / 31;
    a.sp = (g.Ho + kPoolStripRows - 1) / kPoolStripRows;
    a.n_units = a.n_planes * a.sp * a.nb;
    a.in_bytes = (unsigned)((size_t)g.N * g.Ci * g.H * g.W);
    a.out_bytes = (unsigned)((size_t)g.N * g.Ci * g.Ho * g.Wo);
    a.by_nb = make_fastdiv(a.nb);
    a.by_sp = make_fastdiv(a.sp);
    hipLaunchKernelGGL(maxpool3s2_u8_rows, dim3((unsigned)((a.n_units + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace small
