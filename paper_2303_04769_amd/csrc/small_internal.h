// Internal declarations shared by the HIP translation units of libsmall_hip (gfx950 only).
// Host-side launchers validate nothing: the C-ABI layer in small_api.hip has already
// checked shapes, block sizes and aliasing before any launcher is called.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace small {

typedef float floatx4 __attribute__((ext_vector_type(4)));

// Geometry of one windowed layer on the blocked layout (conv, depthwise, pooling).
struct LayerGeom {
    int N, H, W, Ho, Wo;
    int Ci, Co;          // channels (pool / depthwise: Ci == Co)
    int Cib, Cob;        // channel blocks in memory
    int kh, kw, stride, pt, pl;
};

// MI355X dispatches consecutive workgroup ids round-robin over its 8 XCDs, each with a private L2.
// This maps the hardware id b of an n-workgroup 1-D grid to a logical id such that each XCD works
// on one contiguous range of logical ids, so neighbouring tiles (which share halo rows or filter
// slabs) meet in the same L2.
__device__ __forceinline__ unsigned xcd_contiguous(unsigned b, unsigned n)
{
    const unsigned q = n >> 3, r = n & 7u, xcd = b & 7u, idx = b >> 3;
    return xcd * q + (xcd < r ? xcd : r) + idx;
}

// Division of a non-negative int < 2^31 by a positive launch constant: q = mulhi(n, magic) >> shift with
// magic = ceil(2^(31 + l) / d), l = ceil(log2 d), shift = l - 1 (exact for every n < 2^31). An integer
// division costs ~25 vector-ALU instructions per lane, and vector-ALU time is matrix-pipe time on this chip.
struct FastDiv {
    unsigned magic, shift, d;
    __host__ __device__ __forceinline__ int div(int n) const
    {
#ifdef __HIP_DEVICE_COMPILE__
        return d == 1 ? n : (int)(__umulhi((unsigned)n, magic) >> shift);
#else
        return n / (int)d;
#endif
    }
};
inline FastDiv make_fastdiv(int d)
{
    FastDiv f;
    f.d = (unsigned)d;
    unsigned l = 0;
    while ((1ull << l) < (unsigned long long)d) ++l;
    f.shift = l ? l - 1 : 0;
    f.magic = d > 1 ? (unsigned)(((1ull << (31 + l)) + (unsigned)d - 1) / (unsigned)d) : 0u;
    return f;
}

// Compute units of the current device (asked once; 256 -- an MI355X -- when no device can be asked, so that the
// host-only planning calls give the same answers on a machine without a GPU). Launch shapes, tile choices and the
// batch windows of image-resident runs are derived from it.
int device_cus();

// Direct global -> LDS loads, issued from inline assembly so that the compiler does not serialise them
// against every LDS read; the issuing kernel tracks them by hand with wait_vmcnt.
// 64 lanes x 16 B: global (base + per-lane byte offset) -> LDS (wave-uniform byte address + 16 * lane).
__device__ __forceinline__ void dma16(const void *gbase, unsigned lane_off_bytes, unsigned lds_addr_uniform)
{
    asm volatile("s_mov_b32 m0, %2\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %0, %1"
                 :
                 : "v"(lane_off_bytes), "s"(gbase), "s"(__builtin_amdgcn_readfirstlane(lds_addr_uniform))
                 : "memory");
}

template <int N>
__device__ __forceinline__ void wait_vmcnt()
{
    static_assert(N >= 0 && N < 64, "vmcnt is a 6-bit counter");
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// Lane shifts over rows of 16 lanes (DPP): lane l reads lane l - 1 (kRowShr1) or l + 1 (kRowShl1) of its row; zero is
// shifted in at the row's ends. The depthwise kernels take a window's left and right neighbours this way.
typedef unsigned uintx4 __attribute__((ext_vector_type(4)));
constexpr int kRowShr1 = 0x111;
constexpr int kRowShl1 = 0x101;
template <int CTRL>
__device__ __forceinline__ float lane_shift1(float v)
{
    return __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), CTRL, 0xf, 0xf, true));
}
template <int CTRL>
__device__ __forceinline__ floatx4 lane_shift(floatx4 v)
{
    const float x = v.x, y = v.y, z = v.z, w = v.w;      // (scalars first: the builtin takes values, not vector elements)
    return floatx4{lane_shift1<CTRL>(x), lane_shift1<CTRL>(y), lane_shift1<CTRL>(z), lane_shift1<CTRL>(w)};
}
// Buffer-descriptor addressing (raw buffers over a whole tensor): an offset at or beyond the descriptor's size reads
// zeros and drops stores, which serves as a branch-free mask. kBeyond: an offset no tensor of less than 2 GiB reaches.
constexpr unsigned kBeyond = 0x80000000u;
constexpr int kRawBuffer = 0x00020000;         // descriptor word 3: untyped 32-bit data, no swizzle, no stride
constexpr int kNonTemporal = 2;

// Epilogue fused into the convolution's STORE phase (the paper's "abstract fused layer" direction).
// ADD: accumulate onto the tensor `res` (same layout as out). BN: y = y * scale[c] + shift[c] first (batch normalization
// folded behind the reduction; parameters: scale[0 .. C) then shift[0 .. C), 16-byte aligned). Order: BN, ADD, RELU.
enum : int { EPI_NONE = 0, EPI_RELU = 1, EPI_ADD = 2, EPI_BN = 4 };

hipError_t launch_relu(const float *in, float *out, size_t n, hipStream_t s);
hipError_t launch_add(const float *a, const float *b, float *out, size_t n, hipStream_t s);

hipError_t launch_pack(const float *nchw, float *blk, int N, int C, int H, int W, int Cb, bool unpack, hipStream_t s);
hipError_t launch_pack_filter(const float *oihw, float *blk, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                              hipStream_t s);

hipError_t launch_dwconv(const float *in, const float *filt, float *out, const LayerGeom &g, int epilogue, hipStream_t s);
hipError_t launch_pool(const float *in, float *out, const LayerGeom &g, int mode, hipStream_t s);
// depthwise 3x3, 16-channel blocks, input rows staged by the load unit (window_rows.hip); pointers 16-byte aligned
bool dw_rows_eligible(const LayerGeom &g);
hipError_t launch_dw_rows(const float *in, const float *filt, float *out, const LayerGeom &g, int relu, hipStream_t s);
// depthwise 3x3, stride 1, padding 1, 16-channel blocks: rows through registers, neighbours by lane shifts
// (window_dpp.hip); pointers 16-byte aligned
bool dw_dpp_eligible(const LayerGeom &g);
hipError_t launch_dw_dpp(const float *in, const float *filt, float *out, const LayerGeom &g, int relu, hipStream_t s);

// Global average pooling + fully connected layer in one launch (network heads): in [N][C/16][HW][16] (16-byte
// aligned), filt [Co/Cob][C/16][1][1][16][Cob], out [N][Co]; C <= 256, Co <= 16.
bool avgpool_dense_eligible(int C, int Cb, int Co, int Cob);
hipError_t launch_avgpool_dense(const float *in, const float *filt, float *out, int N, int C, int HW, int Co, int Cob,
                                hipStream_t s);

// res: tensor added to the result when epilogue has EPI_ADD (may be `out` itself: each lane reads the
// elements it is about to write), else ignored.
hipError_t launch_conv(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                       int epilogue, hipStream_t s, bool plain_input = false, const float *bn = nullptr);
// true when the kernel launch_conv picks for this layer applies EPI_BN itself; otherwise the caller launches the
// normalization after the convolution
bool conv_epilogue_takes_bn(const LayerGeom &g, const void *in, const void *filt, const void *out, const void *res,
                            const void *bn);
// plain_input: `in` is a plain [N][Ci][H][W] tensor instead of a blocked one. Only the first-layer matrix-core kernel
// takes that (one input block of fewer than 16 channels, a reduction of 5..8, 25..28 or 37..40 values, at least
// 16384 output pixels, 16-byte aligned pointers); conv_takes_plain_input tells, and launch_conv fails otherwise.
bool conv_takes_plain_input(const LayerGeom &g, const void *in, const void *filt, const void *out, const void *res);
// A run of convolutions (with their folded epilogues) in one kernel, one image per workgroup, all tensors between
// them in LDS (resident.hip). A group is one convolution as the runner launches it: logical buffer ids of its
// input, residual (EPI_ADD only) and result, geometry, epilogue.
constexpr int kResMaxLayers = 12;
// kind: RESIDENT_CONV (16-channel blocks in and out); RESIDENT_STEM: a first layer on fewer than 16 input channels
// (only as group 0; plain_input: its input tensor is a plain [N][Ci][H][W] one, else blocked with Cib = Ci);
// RESIDENT_HEAD: average pooling over the whole image followed by a fully connected layer (only as the last group;
// filt, Co, Cob are the fully connected layer's, kh = H, kw = W the pooling window, dst its result [N][Co]);
// RESIDENT_DW: depthwise convolution, 16-channel blocks, at most 9 taps, filter 16-byte aligned.
enum : int { RESIDENT_CONV = 0, RESIDENT_STEM = 1, RESIDENT_HEAD = 2, RESIDENT_DW = 3 };
struct ResGroup {
    const float *filt;
    int src, res, dst;
    int Ci, Co, Cib, Cob, H, W, Ho, Wo, kh, kw, stride, pt, pl;
    int epilogue;
    int kind, plain_input;
};
// How many of the groups g[0..n) (a prefix, 0 or at least 2) one launch takes: 16-channel blocks, 1 or 9 taps (a
// stem: a reduction of at most 40 values), every
// tensor read is the first group's input or produced inside, the live tensors fit 160 KB of LDS per image, and
// closed_after[k - 1] holds (after group k - 1 nothing produced inside but its result is needed any more).
int resident_groups(const ResGroup *g, int n, const bool *closed_after);
// in: the first group's input tensor, out: the last group's result, both blocked, 16-byte aligned.
hipError_t launch_resident(const ResGroup *g, int n, const float *in, float *out, int N, hipStream_t s);

// Name of the kernel launch_conv picks for this geometry when all pointers are 16-byte aligned.
const char *conv_kernel_name(const LayerGeom &g);

// Workgroup tiles (output pixels x output channels) of the matrix-core convolutions.
enum : int { SAME_128x128, SAME_64x128, SAME_128x64, SAME_64x64, SAME_128x32, SAME_64x32, SAME_128x16, SAME_64x16,
              SAME_32x64, SAME_32x32, SAME_256x16, SAME_NUM_TILES };
bool conv_same_eligible(const LayerGeom &g);     // stride 1, output size == input size, kw in {1, 3}, 16-blocks
int conv_same_planes(const LayerGeom &g);        // Ci blocks staged per reduction step (1x1 filters)
// images each workgroup walks in the image-aligned persistent variant, 0 = flat variant (host arithmetic only)
int conv_same_images_per_workgroup(const LayerGeom &g, int tile);
// F_C > 0: a group convolution (partial-channel reduction) on the same kernels: g.Ci, g.Co are all input / output
// channels, group j = output channels [j K, (j + 1) K) reduces input channels [j S_C, j S_C + F_C); F_C, S_C, K
// multiples of 16 and the tile's output channels a divisor of K.
hipError_t launch_conv_same(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                            int tile, int epilogue, hipStream_t s, int F_C = 0, int S_C = 0, int K = 0,
                            const float *bn = nullptr);
// tile (SAME_*) for a group convolution that launch_conv_same takes, or -1: geometry of conv_same_eligible, channel
// counts as above
int group_conv_same_tile(const LayerGeom &g, int F_C, int S_C, int K);

// Pointwise (1x1, stride 1, unpadded) convolution with the filter resident on the compute unit and autonomous
// waves that stream 16-pixel groups (conv_pw.hip): 64 -> 64 and 128 -> 128 channels, at least 32768 pixels, 16-byte
// aligned pointers.
bool conv_pw_eligible(const LayerGeom &g);
const char *conv_pw_kernel_name(const LayerGeom &g);
hipError_t launch_conv_pw(const float *in, const float *filt, float *out, const float *res, const LayerGeom &g,
                          int epilogue, hipStream_t s, const float *bn = nullptr);

// Depthwise 3x3 (+ ReLU) followed by pointwise 1x1 (+ ReLU) in one launch, 16-channel blocks. dwpw_eligible looks
// at what a layer table states (channels, blocks, windows, strides); dwpw_geom_ok at the image geometry.
constexpr size_t kDwPwMaxLds = 160 * 1024;
bool dwpw_eligible(int C, int Co, int Cb, int Cob_pw, int kh, int kw, int stride, int pw_kh, int pw_kw, int pw_stride);
bool dwpw_geom_ok(const LayerGeom &dw_geom, int Co);
hipError_t launch_dwpw(const float *in, const float *dw_filt, const float *pw_filt, float *out, const LayerGeom &dw_geom,
                       int Co, int relu_mid, int relu_out, hipStream_t s);

// A run of pointwise layers (dense on 1x1 images, 1x1 stride-1 unpadded convolution), each with an optional ReLU,
// in one launch (chain.hip). Tensors of the run have a multiple of 16 channels (at most 16 * kChainMaxBlocks) in
// 16-channel blocks; tensors inside the run may instead have 8 channels in one 8-channel block. The run's input must
// be smaller than 4 GiB and may not overlap its output; all pointers 16-byte aligned.
constexpr int kChainMaxLayers = 16;
constexpr int kChainMaxBlocks = 8;
struct ChainLayer { const float *filt; int Ci, Co, relu; };
bool chain_layer_eligible(int Ci, int Co, int Cib, int Cob);
hipError_t launch_dense_chain(const float *in, float *out, const ChainLayer *layers, int n_layers, long M, int HW,
                              hipStream_t s);

// A run of [depthwise 3x3, any stride and padding (+ ReLU)] -> [1x1 convolution Cin -> Cout (+ ReLU)] blocks on 16-channel
// blocks, every tensor of the run an image of at most 256 pixels (and few enough pixel groups per output block: see
// dwpw_run_eligible), each block reading what the one before wrote, in one
// launch (dwpw_run.hip). out may not overlap in, except that a run whose blocks all keep the shape may work in place (a
// workgroup reads its images before it writes them); pointers 16-byte aligned; tensors smaller than 4 GiB.
constexpr int kDwpwChainMaxBlocks = 12;
constexpr int kDwpwRunMaxPixels = 256;       // per image, for every tensor of a run
constexpr int kDwpwRunMaxValues = 6144;      // ... and values per image
struct DwpwRunBlock {
    const float *dw, *pw;
    int dw_relu, pw_relu;
    int Cin, Cout, Hi, Wi, Ho, Wo, stride, pt, pl;
};
bool dwpw_run_eligible(const DwpwRunBlock *blocks, int n_blocks);      // shapes only
int dwpw_run_images(const DwpwRunBlock *blocks, int n_blocks, int N);  // images per workgroup of the launch at batch N
// head.filt != null: the run closes with the mean over the last result's pixels and a fully connected layer on it
// (at most 16 outputs, filter [Co/Cob][C/16][1][1][16][Cob]); out is then [N][Co] and the last result is not written.
struct DwpwRunHead { const float *filt; int Co, Cob; };
hipError_t launch_dwpw_run(const float *in, float *out, const DwpwRunBlock *blocks, int n_blocks, int N, const DwpwRunHead &head,
                           hipStream_t s);

// Remaining Table 2 layers (table2.hip): y = x * scale[c] + shift[c]; nearest-neighbour upsampling by integer
// factors; group convolution (geometry in g with g.Ci = all input channels, g.Co = G * K, g.Cib the activation block).
hipError_t launch_batchnorm(const float *in, const float *scale, const float *shift, float *out, int N, int C, int H, int W,
                            int Cb, hipStream_t s, bool relu = false);
hipError_t launch_upsample(const float *in, float *out, int N, int C, int H, int W, int fh, int fw, int Cb, hipStream_t s);
hipError_t launch_group_conv(const float *in, const float *filt, float *out, const LayerGeom &g, int F_C, int S_C, int K,
                             int F_Cb, hipStream_t s);

// Quantized (uint8) layers (quant.hip). acc = sum over in-image taps of (x - zx)(w - zw) in int32;
// y = clamp(zy + ((int64)acc * mult + 2^(shift-1)) >> shift, lo, hi) (no rounding term when shift == 0).
// amax: host-derived clamp of the sum that makes the 32-bit requantization path exact (0 = not available).
struct QuantParams { int zx, zw, zy, mult, shift, lo, hi, amax; };
// q.amax > 0: sums beyond +-amax saturate the output anyway (|amax * mult / 2^shift| >= 512) and within it the
// scaled value fits 32 bits, so one clamp of the sum replaces 64-bit compares and selects after the product
// (the host derives amax; 0 = scale too large for that, take the wide path). Same codes either way.
__device__ __forceinline__ int requant(int acc, const QuantParams &q)
{
    if (q.amax > 0) {
        const int c = acc < -q.amax ? -q.amax : (acc > q.amax ? q.amax : acc);
        long v = (long)c * (long)q.mult;
        if (q.shift > 0) v = (v + (1L << (q.shift - 1))) >> q.shift;
        int r = (int)v + q.zy;
        r = r < q.lo ? q.lo : r;
        return r > q.hi ? q.hi : r;
    }
    long v = (long)acc * (long)q.mult;
    if (q.shift > 0) v = (v + (1L << (q.shift - 1))) >> q.shift;
    v += q.zy;
    v = v < q.lo ? q.lo : v;
    v = v > q.hi ? q.hi : v;
    return (int)v;
}

// The same for layers with q.amax > 0, in five instructions: the sum is clamped to +-amax first (beyond it the output
// saturates anyway, within it everything below fits), and bias = 2^(shift-1) + zy * 2^shift (requant_bias) carries the
// rounding term and the zero point through the one shift.
__device__ __forceinline__ long requant_bias(const QuantParams &q)
{
    return (q.shift > 0 ? 1L << (q.shift - 1) : 0L) + ((long)q.zy << q.shift);
}
__device__ __forceinline__ int requant_clamped(int acc, const QuantParams &q, long bias)
{
    const int c = min(max(acc, -q.amax), q.amax);
    const int r = (int)(((long)c * (long)q.mult + bias) >> q.shift);
    return min(max(r, q.lo), q.hi);
}

hipError_t launch_pack_u8(const unsigned char *nchw, unsigned char *blk, int N, int C, int H, int W, int Cb, bool unpack,
                          hipStream_t s);
hipError_t launch_pack_filter_u8(const unsigned char *oihw, unsigned char *blk, int Co, int Ci, int kh, int kw, int Cob,
                                 int Cib, hipStream_t s);
// true when the 8-bit matrix-core kernel takes the layer (16-byte blocks, aligned pointers), else one lane per output
bool conv_u8_uses_mfma(const LayerGeom &g, const void *in, const void *filt, const void *out);
// filt_sums: per output channel the sum of the filter's codes over its whole reduction (launch_filter_sums_u8), or
// null: the kernels then take these sums themselves, with one more matrix instruction per filter operand.
hipError_t launch_conv_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                          const QuantParams &q, const int *filt_sums, hipStream_t s);
hipError_t launch_filter_sums_u8(const unsigned char *filt, int *sums, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                                 hipStream_t s);
// mode 0: depthwise (filt [C/Cb][kh][kw][Cb]), 1: max pooling, 2: average pooling (filt unused, may be null)
hipError_t launch_window_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                            int mode, const QuantParams &q, hipStream_t s);
hipError_t launch_relu_u8(const unsigned char *in, unsigned char *out, size_t n, int z, hipStream_t s);
// the ends of a quantized network (quant_ends.hip): the first convolution on a 3-channel (3x3) or 1-channel (10x4) input
// or a 1x1 convolution on 8 channels, with 8 or 16 output channels per block, global average pooling on 16-byte blocks (mode 2 = average), a fully connected
// layer with fewer than 16 outputs per block
bool conv_first_u8_eligible(const LayerGeom &g, const void *out);
hipError_t launch_conv_first_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                                const QuantParams &q, hipStream_t s);
bool avgpool_global_u8_eligible(const LayerGeom &g, int mode, const void *in, const void *out);
hipError_t launch_avgpool_global_u8(const unsigned char *in, unsigned char *out, const LayerGeom &g, hipStream_t s);
bool dense_u8_eligible(const LayerGeom &g, const void *in, const void *filt);
hipError_t launch_dense_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                           const QuantParams &q, hipStream_t s);
// max pooling 3x3, stride 2, no padding, 16-channel blocks, 16-byte aligned pointers (pool_dpp.hip)
bool pool_dpp_eligible(const LayerGeom &g, const void *in, const void *out);
hipError_t launch_pool_dpp(const float *in, float *out, const LayerGeom &g, hipStream_t s);
// quantized max pooling 3x3, stride 2, no padding, 16-byte blocks, 16-byte aligned pointers (pool_dpp_u8.hip); mode 1 = max
bool pool_dpp_u8_eligible(const LayerGeom &g, int mode, const void *in, const void *out);
hipError_t launch_pool_dpp_u8(const unsigned char *in, unsigned char *out, const LayerGeom &g, hipStream_t s);
// quantized depthwise 3x3, stride 1, padding 1, 16-byte blocks, 4-byte aligned pointers (window_dpp_u8.hip)
bool dw_dpp_u8_eligible(const LayerGeom &g, const QuantParams &q, const void *in, const void *filt, const void *out);
hipError_t launch_dw_dpp_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, const LayerGeom &g,
                            const QuantParams &q, hipStream_t s);
// y = clamp(zy + floor(((a - za) mult_a + (b - zb) mult_b + 2^(shift-1)) / 2^shift), lo, hi); out may be a or b
struct AddQuantParams { int za, zb, zy, mult_a, mult_b, shift, lo, hi; };
hipError_t launch_add_u8(const unsigned char *a, const unsigned char *b, unsigned char *out, size_t n, const AddQuantParams &q,
                         hipStream_t s);

}  // namespace small
