// Depthwise 3x3 convolution, stride 1, padding 1 (output size = input size), 16-channel blocks: the single-channel
// reduction of Table 1 on the shared blocked layout, HBM-bound (8 bytes per output value against 18 flop). Written
// like an element-wise kernel: no LDS, no barrier, every input row loaded once per wave straight into registers.
//
// A wave owns a band of 16 neighbouring pixels of a row times the 16 channels of the block -- lane = 16 q + l holds
// the float4 of channels 4q .. 4q + 3 of pixel l -- and walks down a strip of rows. One 1 KB load brings a row of
// the band in; the window's left and right neighbours are the same registers of lanes l - 1 and l + 1 (row_shr /
// row_shl lane shifts over rows of 16 lanes, zero shifted in at the ends), and the rows above and below are the
// registers of the two previous steps. So a row costs one load, eight lane shifts, 36 multiply-adds and one store.
// Lanes 0 and 15 of a band are halo: a band yields 14 output pixels (rows of 56, 28 and 14 pixels are 4, 2 and 1
// bands exactly). Rows of at most 7 pixels put two planes side by side in the 16 lanes (8 lanes each: one zero lane
// + 7 pixels), the zero lane being both the left edge of one and the right edge of the other.
//
// Memory is addressed through buffer descriptors of the two tensors: a lane that has nothing to load (a pixel or a
// row outside the image: the zero padding, which so exists in registers only) or nothing to store (halo lanes, the
// two steps that only bring in a strip's first rows, steps past the strip's end) gets an offset beyond the
// descriptor's size, for which the hardware returns zeros / drops the store. The steps therefore have no branch and
// no select, and every step issues exactly one store, so the wait the compiler places before a row is used covers
// that row's load alone (vmcnt counts loads and stores alike, in order): later rows and all stores stay in flight.
//
// A strip has at most 7 output rows = 9 input rows, all requested at once into nine registers before the first
// step (the kernel is as deep in flight as an element-wise one; measured, a streaming ring of rows for taller
// strips was no faster), and the nine steps are straight-line code. Where a plane has more than two strips its
// strips are on neighbouring workgroups of one XCD, so the halo rows they share meet in that L2; with one or two
// strips per plane the workgroups run in memory order.
#include "small_internal.h"

namespace small {

namespace {

struct DppArgs {
    const float *in;
    const float *filt;     // [C/16][3][3][16]
    float *out;
    int H, W, nCb;
    int n_planes;          // N * nCb
    int nb;                // bands per row
    int sp;                // row strips per plane
    FastDiv by_nb, by_sp, by_nCb;
    int xcd_remap;         // strips of a plane on one XCD
    int n_units;           // plane groups * sp * nb: one per wave
    unsigned bytes;        // of the input = of the output tensor (< 2^31)
};


// SEG: lanes per plane in a row of 16 lanes (16: one plane, bands of 14 output pixels with a halo lane on each
// side; 8: two planes of at most 7 pixels, each behind one zero lane).
constexpr int kStripRows = 7;                  // output rows of a strip, at most
constexpr int kSteps = kStripRows + 2;         // its input rows = steps

template <int SEG, bool RELU>
__global__ void __launch_bounds__(256) dw16_dpp(DppArgs a)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane((int)threadIdx.x >> 6);
    const int unit = (int)(a.xcd_remap ? xcd_contiguous(blockIdx.x, gridDim.x) : blockIdx.x) * 4 + wave;
    if (unit >= a.n_units) return;
    const int l = lane & 15, q = lane >> 4;

    // unit -> (plane group, row strip, band)
    const int t = a.by_nb.div(unit), band = unit - t * a.nb;
    const int pg = a.by_sp.div(t), strip = t - pg * a.sp;
    const int r0 = a.by_sp.div(strip * a.H), r1 = a.by_sp.div((strip + 1) * a.H);      // output rows r0 .. r1 - 1

    int plane, x;
    if (SEG == 16) {
        plane = pg;
        x = band * 14 - 1 + l;
    } else {
        plane = pg * 2 + (l >> 3);
        x = (l & 7) - 1;
    }
    const bool col_in = x >= 0 && x < a.W && plane < a.n_planes;               // this lane holds an image pixel
    const bool col_out = col_in && (SEG == 8 || (l >= 1 && l <= 14));           // ... and computes an output
    const int row_bytes = a.W * 64;
    // byte offsets of this lane's 16 bytes in row 0 of its plane (beyond the tensor where it has none)
    const unsigned at = (unsigned)plane * (unsigned)(a.H * row_bytes) + (unsigned)(x * 64 + q * 16);
    const unsigned at_in = col_in ? at : kBeyond, at_out = col_out ? at : kBeyond;

    const __amdgpu_buffer_rsrc_t src = __builtin_amdgcn_make_buffer_rsrc(const_cast<float *>(a.in), 0, a.bytes, kRawBuffer);
    const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(a.out, 0, a.bytes, kRawBuffer);

    floatx4 w[9];
    {
        const int pc = min(plane, a.n_planes - 1), cb = pc - a.by_nCb.div(pc) * a.nCb;
        const floatx4 *tp = reinterpret_cast<const floatx4 *>(a.filt) + cb * 36 + q;
#pragma unroll
        for (int k = 0; k < 9; ++k) w[k] = tp[k * 4];
    }

    // input rows r0 - 1 .. r1 of the image are steps j = 0 .. n_in - 1; step j >= 2 completes output row r0 + j - 2
    const int n_in = r1 - r0 + 2;
    auto load_row = [&](int j) {
        const int r = r0 - 1 + j;
        const bool row_in = r >= 0 && r < a.H && j < n_in;                      // (uniform)
        const unsigned off = row_in ? at_in + (unsigned)(r * row_bytes) : kBeyond;
        return __builtin_bit_cast(floatx4, __builtin_amdgcn_raw_buffer_load_b128(src, off, 0, 0));
    };

    floatx4 row[kSteps], row_l[kSteps], row_r[kSteps];
#pragma unroll
    for (int j = 0; j < kSteps; ++j) row[j] = load_row(j);
#pragma unroll
    for (int j = 0; j < kSteps; ++j) {
        row_l[j] = lane_shift<kRowShr1>(row[j]);
        row_r[j] = lane_shift<kRowShl1>(row[j]);
        if (j < 2) continue;
        floatx4 acc = row[j - 1] * w[4];
        acc += row[j - 2] * w[1];
        acc += row[j] * w[7];
        acc += row_l[j - 2] * w[0];
        acc += row_l[j - 1] * w[3];
        acc += row_l[j] * w[6];
        acc += row_r[j - 2] * w[2];
        acc += row_r[j - 1] * w[5];
        acc += row_r[j] * w[8];
        if (RELU) {
            acc.x = acc.x > 0.f ? acc.x : 0.f; acc.y = acc.y > 0.f ? acc.y : 0.f;
            acc.z = acc.z > 0.f ? acc.z : 0.f; acc.w = acc.w > 0.f ? acc.w : 0.f;
        }
        const unsigned off = j < n_in ? at_out + (unsigned)((r0 + j - 2) * row_bytes) : kBeyond;      // (uniform)
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(uintx4, acc), dst, off, 0, kNonTemporal);
    }
}

template <int SEG>
hipError_t launch_dpp_seg(const DppArgs &a, int relu, hipStream_t s)
{
    const unsigned wgs = (unsigned)((a.n_units + 3) / 4);
    if (relu) hipLaunchKernelGGL((dw16_dpp<SEG, true>), dim3(wgs), dim3(256), 0, s, a);
    else hipLaunchKernelGGL((dw16_dpp<SEG, false>), dim3(wgs), dim3(256), 0, s, a);
    return hipGetLastError();
}

}  // namespace

bool dw_dpp_eligible(const LayerGeom &g)
{
    if (g.Cib != 16 || g.kh != 3 || g.kw != 3 || g.stride != 1 || g.pt != 1 || g.pl != 1) return false;
    if (g.Ho != g.H || g.Wo != g.W) return false;
    return (size_t)g.N * g.Ci * g.H * g.W < ((size_t)1 << 29);          // byte offsets below 2^31
}

hipError_t launch_dw_dpp(const float *in, const float *filt, float *out, const LayerGeom &g, int relu, hipStream_t s)
{
    DppArgs a;
    a.in = in; a.filt = filt; a.out = out;
    a.H = g.H; a.W = g.W; a.nCb = g.Ci / 16;
    a.n_planes = g.N * a.nCb;
    a.bytes = (unsigned)((size_t)g.N * g.Ci * g.H * g.W * 4);
    const bool pairs = g.W <= 7;
    a.nb = pairs ? 1 : (g.W + 13) / 14;
    const long groups = pairs ? (a.n_planes + 1) / 2 : a.n_planes;
    a.sp = (g.H + kStripRows - 1) / kStripRows;
    a.n_units = (int)(groups * a.sp * a.nb);
    a.by_nb = make_fastdiv(a.nb);
    a.by_sp = make_fastdiv(a.sp);
    a.by_nCb = make_fastdiv(a.nCb);
    a.xcd_remap = a.sp > 2;
    return pairs ? launch_dpp_seg<8>(a, relu, s) : launch_dpp_seg<16>(a, relu, s);
}

}  // namespace small
