// Max pooling, 3x3 window, stride 2, no padding, 16-channel blocks: the abstract layer's single-channel reduction
// with max as its operation (Table 1). HBM-bound: 1.25 floats moved per input float and nine comparisons per output.
//
// Lane = 16 q + l holds the float4 of channels 4q .. 4q + 3 of pixel l of a band of 16 neighbouring pixels, so a row
// of the band is one contiguous kilobyte and every input row is loaded once per strip (at most 7 output rows = 15
// input rows, all requested at once, as streaming loads: measured, 43 us against 46 at 64x256x56x56; strips of 2 to 14
// rows all land within 44 .. 46 us, the read-dominated floor of this traffic). The window's second and third column are the registers of lanes l + 1 and
// l + 2 (row_shl lane shifts over rows of 16 lanes); lane l = 2j then holds output column j of the band: 7 outputs
// per band, bands 14 pixels apart (a 56-pixel row: 27 outputs in 4 bands). The vertical maximum runs over the rows'
// horizontal maxima.
//
// The maximum is the reference scan's: start from -inf and replace on "greater than", columns before rows, so the
// first of equal values (+0 / -0) stays and a NaN is never taken. The horizontal-then-vertical order picks the same
// element: the first row that attains the maximum, and the first column within it.
// Lanes and rows with nothing to load or store use an offset beyond the tensors' buffer descriptors.
#include "small_internal.h"

namespace small {

namespace {

struct PoolArgs {
    const float *in;
    float *out;
    int H, W, Ho, Wo;
    int n_planes, nb, sp, n_units;
    unsigned in_bytes, out_bytes;
    FastDiv by_nb, by_sp;
};

constexpr int kPoolStripRows = 7;                      // output rows of a strip, at most
constexpr int kPoolInRows = 2 * kPoolStripRows + 1;    // its input rows
constexpr int kRowShl2 = 0x102;                        // lane l reads lane l + 2 of its row of 16 (beyond the row: zero)

__device__ __forceinline__ floatx4 take_greater(floatx4 m, floatx4 v)
{
    m.x = v.x > m.x ? v.x : m.x; m.y = v.y > m.y ? v.y : m.y;
    m.z = v.z > m.z ? v.z : m.z; m.w = v.w > m.w ? v.w : m.w;
    return m;
}

__global__ void __launch_bounds__(256) maxpool3s2_rows(PoolArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int unit = (int)blockIdx.x * 4 + wave;
    if (unit >= a.n_units) return;
    const int l = lane & 15, q = lane >> 4;
    const int t = a.by_nb.div(unit), band = unit - t * a.nb;
    const int plane = a.by_sp.div(t), strip = t - plane * a.sp;
    const int r0 = a.by_sp.div(strip * a.Ho), r1 = a.by_sp.div((strip + 1) * a.Ho);      // output rows r0 .. r1 - 1
    const int n_out = r1 - r0, n_in = 2 * n_out + 1;

    const int x = band * 14 + l;                                 // input column of this lane
    const int ow = band * 7 + (l >> 1);                          // output column (even lanes up to 12)
    const bool col_in = x < a.W;
    const bool col_out = !(l & 1) && l <= 12 && ow < a.Wo;
    const unsigned at_in = (unsigned)plane * (unsigned)(a.H * a.W * 64) + (unsigned)(x * 64 + q * 16);
    const unsigned at_out = (unsigned)plane * (unsigned)(a.Ho * a.Wo * 64) + (unsigned)(ow * 64 + q * 16);

    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.in), 0, a.in_bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.out_bytes, kRawBuffer);

    floatx4 raw[kPoolInRows];
#pragma unroll
    for (int j = 0; j < kPoolInRows; ++j) {
        const bool have = col_in && j < n_in;
        const unsigned off = have ? at_in + (unsigned)((2 * r0 + j) * a.W * 64) : kBeyond;
        raw[j] = __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(src, off, 0, kNonTemporal));
    }
    const float ninf = -__builtin_inff();
    floatx4 h[3];                                                // horizontal maxima of the rows 2r, 2r + 1, 2r + 2
#pragma unroll
    for (int j = 0; j < kPoolInRows; ++j) {
        floatx4 m = take_greater(floatx4{ninf, ninf, ninf, ninf}, raw[j]);
        m = take_greater(m, lane_shift<kRowShl1>(raw[j]));
        h[j % 3] = take_greater(m, lane_shift<kRowShl2>(raw[j]));
        if (j >= 2 && !(j & 1)) {
            const int r = j / 2 - 1;                             // rows j - 2, j - 1, j are output row r0 + r
            const floatx4 v = take_greater(take_greater(h[(j + 1) % 3], h[(j + 2) % 3]), h[j % 3]);
            const unsigned off = (col_out && r < n_out) ? at_out + (unsigned)((r0 + r) * a.Wo * 64) : kBeyond;
            __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, v), dst, off, 0, kNonTemporal);
        }
    }
}

}  // namespace

bool pool_dpp_eligible(const LayerGeom &g, const void *in, const void *out)
{
    if (g.Cib != 16 || g.kh != 3 || g.kw != 3 || g.stride != 2 || g.pt != 0 || g.pl != 0) return false;
    if (g.Ho != (g.H - 3) / 2 + 1 || g.Wo != (g.W - 3) / 2 + 1) return false;          // (no bottom / right padding either)
    if ((((uintptr_t)in | (uintptr_t)out) & 15u) != 0) return false;
    return (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 29);                          // byte offsets below 2^31
}

hipError_t launch_pool_dpp(const float *in, float *out, const LayerGeom &g, hipStream_t s)
{
    PoolArgs a;
    a.in = in; a.out = out;
    a.H = g.H; a.W = g.W; a.Ho = g.Ho; a.Wo = g.Wo;
    a.n_planes = g.N * (g.Ci / 16);
    a.nb = (g.Wo + 6) / 7;
    a.sp = (g.Ho + kPoolStripRows - 1) / kPoolStripRows;
    a.n_units = a.n_planes * a.sp * a.nb;
    a.in_bytes = (unsigned)((size_t)g.N * g.Ci * g.H * g.W * 4);
    a.out_bytes = (unsigned)((size_t)g.N * g.Ci * g.Ho * g.Wo * 4);
    a.by_nb = make_fastdiv(a.nb);
    a.by_sp = make_fastdiv(a.sp);
    hipLaunchKernelGGL(maxpool3s2_rows, dim3((unsigned)((a.n_units + 3) / 4)), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace small
