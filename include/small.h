/*
 * small.h -- C ABI of libsmall_hip: the SMaLL abstract-layer hot path on one MI355X (gfx950).
 *
 * Every layer is an instance of one loop nest (paper Algorithm 1) over one shared,
 * channel-blocked data format (paper Section 4.4 "Common Data Format"), so the output
 * of any layer is the input of the next with no reformatting:
 *
 *   activations  [N][C/Cb][H][W][Cb]                     Cb fastest, batch outermost
 *   filters      [Co/Cob][Ci/Cib][kh][kw][Cib][Cob]      Cob fastest (loop order of Algorithm 1)
 *   dw filters   [C/Cb][kh][kw][Cb]                      (the same layout with F_Cb = 1, G_b = Cb)
 *
 * All data are IEEE fp32. Block sizes are run-time arguments; a tensor with C channels
 * is stored with any block Cb that divides C (the tuned kernels expect Cb = 16 and fall
 * back to a generic kernel otherwise; callers normally use min(16, C)).
 *
 * Conventions for every entry point unless stated otherwise:
 *   - every pointer is a DEVICE pointer owned by the caller, valid until the enqueued
 *     work has finished; the library allocates nothing, frees nothing and never
 *     synchronises. Work is enqueued on `stream` (a hipStream_t passed as void*; NULL is
 *     the default stream);
 *   - `in` and `out` must not overlap, except small_relu, small_add and small_batchnorm where out
 *     may equal an input exactly (in place);
 *   - padding is explicit zero padding, 4-sided; output size per side is
 *     floor((in + lo + hi - k) / stride) + 1 (the paper's output-size equation of
 *     Section 3.1.2 extended with padding and floor). Every padding must be smaller than the
 *     window on its axis (pad.t, pad.b < kh; pad.l, pad.r < kw), so that no window lies entirely
 *     in the padding (a maximum or an average over no element has no value): SMALL_ERR_SHAPE otherwise;
 *   - return value: SMALL_OK (0) or an error code below. When an error is returned
 *     nothing has been enqueued. No exception crosses this boundary.
 */
#ifndef SMALL_H
#define SMALL_H

#include <stddef.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SMALL_OK = 0,
    SMALL_ERR_NULL = 1,   /* a required pointer is NULL */
    SMALL_ERR_SHAPE = 2,  /* non-positive dim, window larger than the padded input, padding >= window, C % Cb != 0,
                             size overflow */
    SMALL_ERR_BLOCK = 3,  /* block size with no kernel (Cb > 64) */
    SMALL_ERR_ALIAS = 4,  /* in/out overlap where it is not allowed */
    SMALL_ERR_LAUNCH = 5, /* the HIP runtime refused the launch */
    SMALL_ERR_WORKSPACE = 6, /* workspace too small or misaligned (small_network_run) */
    SMALL_ERR_LAYER = 7,  /* malformed layer table (bad op, bad buffer id, block mismatch between layers) */
    SMALL_ERR_QUANT = 8,  /* quantization parameters out of range, or a reduction too long for int32 sums */
    SMALL_ERR_STATIC = 9  /* small_network_run_static: the run needs more than SMALL_STATIC_WORKSPACE_BYTES */
};

typedef struct { int t, b, l, r; } small_pad; /* zero padding: top, bottom, left, right */

/* floor((in + pad_lo + pad_hi - k) / stride) + 1, or 0 when the window does not fit. Host only. */
int small_out_dim(int in, int k, int stride, int pad_lo, int pad_hi);

const char *small_strerror(int code);

/* ---- layout conversion at the network boundary (Section 4.4). Bit-exact copies. ----
 * small_pack:   plain [N][C][H][W]  ->  blocked [N][C/Cb][H][W][Cb];  small_unpack is its inverse.
 * small_pack_filter:    plain [Co][Ci][kh][kw] -> [Co/Cob][Ci/Cib][kh][kw][Cib][Cob].
 * small_pack_dw_filter: plain [C][1][kh][kw]   -> [C/Cb][kh][kw][Cb].
 * Both buffers hold exactly N*C*H*W (resp. Co*Ci*kh*kw, C*kh*kw) floats. */
int small_pack(const float *nchw, float *blocked, int N, int C, int H, int W, int Cb, void *stream);
int small_unpack(const float *blocked, float *nchw, int N, int C, int H, int W, int Cb, void *stream);
int small_pack_filter(const float *oihw, float *blocked, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                      void *stream);
int small_pack_dw_filter(const float *c1hw, float *blocked, int C, int kh, int kw, int Cb, void *stream);

/* ---- full-channel reduction: convolution (Table 1 row "Full Channel Reduction": F_C = I_C,
 * K = O_C, G = 1; Table 2: reduction = FMA).
 *   out[n,co,oh,ow] = sum_{ci,y,x} in[n,ci,oh*stride+y-pad.t, ow*stride+x-pad.l] * filt[co,ci,y,x],
 * taps outside the input contribute 0. in: [N][Ci/Cib][H][W][Cib]; filt: blocked filter;
 * out: [N][Co/Cob][Ho][Wo][Cob]. Cib = Cob = 16 runs on the fp32 matrix cores; any other
 * block sizes (<= 64) run a generic kernel. fp32 accumulation, summation order unspecified. */
int small_conv2d(const float *in, const float *filt, float *out, int N, int Ci, int Co, int H, int W, int kh,
                 int kw, int stride, small_pad pad, int Cib, int Cob, void *stream);

/* Host only, enqueues nothing: the name of the kernel small_conv2d launches for this shape (for example
 * "conv16_mfma<4,1,2,1>" = 4x1 wavefronts of 2x1 16x16 matrix-core tiles, or "conv_direct"), so that a
 * profile's per-kernel rows can be matched to layers. Returns NULL when the arguments are invalid. */
const char *small_conv2d_kernel(int N, int Ci, int Co, int H, int W, int kh, int kw, int stride, small_pad pad,
                                int Cib, int Cob);

/* ---- single-channel reduction with weights: depthwise convolution (Table 1 row "Single
 * Channel Reduction": F_C = 1, K = 1, G = I_C; Section 3.2 item 2).
 *   out[n,c,oh,ow] = sum_{y,x} in[n,c,oh*stride+y-pad.t, ow*stride+x-pad.l] * filt[c,y,x]. */
int small_dwconv2d(const float *in, const float *filt, float *out, int N, int C, int H, int W, int kh, int kw,
                   int stride, small_pad pad, int Cb, void *stream);

/* ---- single-channel reduction without weights: pooling (Section 3.2 item 2; Table 2 "Max Pooling").
 * mode SMALL_POOL_MAX: m = -inf; taps visited row-major; m = v when v > m; taps outside the
 *   input are skipped (bit-exact, ties keep the first value seen, NaN is never selected).
 * mode SMALL_POOL_AVG: sum of the in-range taps divided by their count (the paper names only
 *   "pooling"; average pooling is the Add reduction of the same class). */
enum { SMALL_POOL_MAX = 0, SMALL_POOL_AVG = 1 };
int small_pool2d(const float *in, float *out, int N, int C, int H, int W, int kh, int kw, int stride,
                 small_pad pad, int Cb, int mode, void *stream);

/* ---- single-element reductions (Table 1 row "Single Element Reduction"; Table 2 "Activation (ReLU)":
 * reduction = Max; Section 3.2 item 1 names addition). Layout-agnostic over n_elems floats.
 *   small_relu: out[i] = in[i] > 0 ? in[i] : +0   (so -0 -> +0 and NaN -> +0), bit-exact.
 *   small_add:  out[i] = a[i] + b[i]  (one IEEE fp32 addition), used for residual connections
 *               (Section "MLPerf:Tiny Inference Models": the block input is accumulated with its output). */
int small_relu(const float *in, float *out, size_t n_elems, void *stream);
int small_add(const float *a, const float *b, float *out, size_t n_elems, void *stream);

/* ---- full reduction: dense / fully connected (Table 1 row "Full Reduction") on a 1x1 image.
 *   out[n,o] = sum_i in[n,i] * filt[o,i];  in: [N][Ci/Cib][1][1][Cib] (= [N][Ci]),
 *   filt: [Co/Cob][Ci/Cib][1][1][Cib][Cob], out: [N][Co/Cob][1][1][Cob] (= [N][Co]).
 * A dense layer over an H x W image is small_conv2d with kh = H, kw = W and no padding. */
int small_dense(const float *in, const float *filt, float *out, int N, int Ci, int Co, int Cib, int Cob,
                void *stream);

/* ---- the remaining layers of Table 2 (also ops of small_network_run's layer table, see below).
 * small_batchnorm: batch normalization as the single-element FMA of Table 2, statistics folded by the
 *   caller: out[n,c,h,w] = in[n,c,h,w] * scale[c] + shift[c] (one fused multiply-add). scale, shift: C floats
 *   in plain channel order. out may equal in exactly (in place).
 * small_upsample: nearest-neighbour interpolation (Table 2 "Upsample") by integer factors:
 *   out[n,c,oh,ow] = in[n,c,oh / fh,ow / fw]; out is [N][C/Cb][H*fh][W*fw][Cb]. Bit-exact copy.
 * small_group_conv2d: partial-channel reduction (Section 3.2 item 3, Table 2 "Group Convolutions").
 *   G = (Ci - F_C) / S_C + 1 groups (the division must be exact); group g reduces input channels
 *   g * S_C .. g * S_C + F_C - 1 with K filters; output channel g * K + k (Section 3.1.2: O_C = K * G).
 *   S_C = F_C gives the usual disjoint groups; S_C < F_C overlapping ones.
 *   in: [N][Ci/Cib][H][W][Cib]; out: [N][Co/Cob][Ho][Wo][Cob] with Co = G * K;
 *   filt: the plain tensor [Co][F_C][kh][kw] in the general filter layout [Co/Cob][F_C/F_Cb][kh][kw][F_Cb][Cob]
 *   (small_pack_filter with Ci = F_C, Cib = F_Cb). */
int small_batchnorm(const float *in, const float *scale, const float *shift, float *out, int N, int C, int H, int W, int Cb,
                    void *stream);
int small_upsample(const float *in, float *out, int N, int C, int H, int W, int fh, int fw, int Cb, void *stream);
int small_group_conv2d(const float *in, const float *filt, float *out, int N, int Ci, int F_C, int S_C, int K, int H, int W,
                       int kh, int kw, int stride, small_pad pad, int Cib, int F_Cb, int Cob, void *stream);

/* ---- quantized layers: uint8 codes in and out, int32 sums (Section "Memory Usage Comparison": inputs and
 * outputs of the quantized models are uint8, partial results are accumulated in int32; Section "Quantized
 * Inference"). The paper gives no rule for turning the sum back into a code; this library uses the usual
 * integer-only affine rule, with real value = scale * (code - zero point):
 *   acc = sum over the taps inside the image of (x - zx) * (w - zw)                       (int32, exact)
 *   y   = clamp(zy + floor((acc * mult + 2^(shift-1)) / 2^shift), lo, hi)                 (64-bit product,
 *         ties round up; no rounding term when shift == 0)
 * 0 <= zx, zw, zy <= 255; 0 <= mult <= 2^31 - 1; 0 <= shift <= 31; 0 <= lo <= hi <= 255 (a ReLU after the layer
 * is lo = zy). The reduction length K = Ci*kh*kw (kh*kw for depthwise) must satisfy K * 255 * 255 < 2^31.
 * Layouts (bytes): activations [N][C/Cb][H][W][Cb] as for fp32; convolution filters
 * [Co/Cob][Ci/Cib][kh][kw][Cob][Cib] -- the two innermost dimensions are swapped with respect to the fp32
 * filter layout, because the 8-bit matrix instruction multiplies runs of consecutive reduction elements:
 * the Cib bytes of one output channel must be contiguous (Section 4.4 chooses the layout for the machine's
 * kernel); depthwise filters [C/Cb][kh][kw][Cb]. Results are bit-exact (integer arithmetic).
 * small_conv2d_u8: Cib = Cob = 16 with in and filt 16-byte aligned and out 4-byte aligned runs on the int8
 *   matrix cores, anything else one lane per output. small_dense_u8 is the window = image case on a 1x1 image.
 * small_pool2d_u8: SMALL_POOL_MAX compares codes and skips taps outside the image; SMALL_POOL_AVG is
 *   floor((sum + n/2) / n) over the n taps inside the image. small_relu_u8: out = max(in, z). */
typedef struct { int zx, zw, zy, mult, shift, lo, hi; } small_quant;
int small_pack_u8(const unsigned char *nchw, unsigned char *blocked, int N, int C, int H, int W, int Cb, void *stream);
int small_unpack_u8(const unsigned char *blocked, unsigned char *nchw, int N, int C, int H, int W, int Cb, void *stream);
int small_pack_filter_u8(const unsigned char *oihw, unsigned char *blocked, int Co, int Ci, int kh, int kw, int Cob,
                         int Cib, void *stream);
/* small_filter_sums_u8: sums[co] = sum of the codes of output channel co's filter over its whole reduction
 * (Ci*kh*kw values), from the blocked filter; Co ints. small_conv2d_u8 / small_dense_u8 take it as filt_sums
 * (16-byte aligned, or NULL): the term zx-dependent part of the sum, (zx - 128) * sum(w - 128), is the same for
 * every pixel, so a caller that keeps the filter keeps these sums with it; with NULL the kernels take the sums
 * themselves on every call (same results, more matrix instructions). */
int small_filter_sums_u8(const unsigned char *filt, int *sums, int Co, int Ci, int kh, int kw, int Cob, int Cib,
                         void *stream);
int small_conv2d_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int Ci, int Co, int H,
                    int W, int kh, int kw, int stride, small_pad pad, int Cib, int Cob, const small_quant *q,
                    const int *filt_sums, void *stream);
int small_dwconv2d_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int C, int H, int W,
                      int kh, int kw, int stride, small_pad pad, int Cb, const small_quant *q, void *stream);
int small_dense_u8(const unsigned char *in, const unsigned char *filt, unsigned char *out, int N, int Ci, int Co, int Cib,
                   int Cob, const small_quant *q, const int *filt_sums, void *stream);
int small_pool2d_u8(const unsigned char *in, unsigned char *out, int N, int C, int H, int W, int kh, int kw, int stride,
                    small_pad pad, int Cb, int mode, void *stream);
int small_relu_u8(const unsigned char *in, unsigned char *out, size_t n_elems, int z, void *stream);

/* Addition of two quantized tensors (the residual blocks of Section "MLPerf:Tiny Inference Models" on codes). The
 * operands have scales and zero points of their own; the paper gives no rule, this library brings both to the
 * output's scale with a multiplier each and one common shift, rounding once:
 *   acc = (a - za) * mult_a + (b - zb) * mult_b                                          (64-bit, exact)
 *   y   = clamp(zy + floor((acc + 2^(shift-1)) / 2^shift), lo, hi)                       (no rounding term when shift == 0)
 * so mult_a / 2^shift stands for scale_a / scale_y, mult_b / 2^shift for scale_b / scale_y. 0 <= za, zb, zy <= 255;
 * 0 <= mult_a, mult_b <= 2^31 - 1; 0 <= shift <= 31; 0 <= lo <= hi <= 255. Element-wise on n_elems bytes (any layout,
 * the same for all three tensors); out may be a or b (in place), other overlaps: SMALL_ERR_ALIAS. Bit-exact. */
typedef struct { int za, zb, zy, mult_a, mult_b, shift, lo, hi; } small_quant_add;
int small_add_u8(const unsigned char *a, const unsigned char *b, unsigned char *out, size_t n_elems, const small_quant_add *q,
                 void *stream);

/* A whole quantized network (Section "Quantized Inference" runs entire models on uint8 tensors): a table of layers
 * over shared buffers as for small_network_run below -- same buffer ids, same sizing rule (bytes instead of floats),
 * the same checks before anything is enqueued -- with the ops SMALL_OP_CONV, DWCONV, MAXPOOL, AVGPOOL, RELU, ADD and
 * DENSE (others: SMALL_ERR_LAYER). q: parameters of CONV / DWCONV / DENSE (q.zx must be the source tensor's zero
 * point); RELU uses q.zy as the tensor's zero point and nothing else of q; qa: parameters of ADD (src = a, src2 = b);
 * the pools have none (codes in, codes out, same scale). filt: blocked uint8 filter in the layout of
 * small_conv2d_u8 / small_dwconv2d_u8, filt_sums: optional, as for small_conv2d_u8. Layers run one after the other
 * through the entry points above, except that an in-place ReLU directly after a CONV / DWCONV / DENSE / ADD goes
 * into that layer's lower clamp (lo = max(lo, z): the same codes). Results are bit-exact.
 * small_network_workspace_u8: bytes of workspace (host only). small_network_run_u8: in_blocked [N][C0/Cb0][H0][W0][Cb0]
 * bytes with Cb0 = layers[0].Cib; out_blocked receives every write to SMALL_BUF_OUT; workspace 256-byte aligned. */
typedef struct {
    int op;
    int Ci, Co, kh, kw, stride;
    small_pad pad;
    int Cib, Cob;
    int src, src2, dst;
    const unsigned char *filt;
    const int *filt_sums;
    small_quant q;
    small_quant_add qa;
} small_layer_u8;
int small_network_workspace_u8(const small_layer_u8 *layers, int n_layers, int N, int C0, int H0, int W0, size_t *bytes);
int small_network_run_u8(const small_layer_u8 *layers, int n_layers, const unsigned char *in_blocked,
                         unsigned char *out_blocked, void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0,
                         void *stream);

/* ---- a whole network: a table of layers over shared buffers (Section "Memory Usage
 * Comparison": buffers are shared across layers; nothing is reformatted between layers).
 * Logical buffer ids: SMALL_BUF_IN = the caller's blocked input (read-only), SMALL_BUF_OUT = the
 * caller's blocked output, 0..SMALL_MAX_SLOTS-1 = slots carved out of the workspace. Each slot is
 * sized for the largest tensor any layer writes to it.
 * For op RELU / ADD / MAXPOOL / AVGPOOL, Ci is the channel count and Co must equal Ci.
 * For ADD, src2 is the second operand. For DENSE, kh/kw must equal the input H/W.
 * filt is the layer's blocked device filter (NULL for layers without weights).
 * The remaining rows of Table 2 as ops:
 *   SMALL_OP_BATCHNORM  y = x * scale[c] + shift[c]; Co = Ci, Cob = Cib; filt: 2 * Ci floats, scale[0 .. Ci) then
 *                       shift[0 .. Ci), plain channel order; dst may equal src (in place).
 *   SMALL_OP_UPSAMPLE   nearest neighbour by the integer factors kh (rows) and kw (columns); Co = Ci, Cob = Cib.
 *   SMALL_OP_GROUPCONV  small_group_conv2d: Ci, Co all input / output channels, F_C, S_C the group's window and stride
 *                       over the channels, K = Co / ((Ci - F_C) / S_C + 1) filters per group; the filter's channel
 *                       block F_Cb is min(16, F_C) and must divide F_C. F_C and S_C are ignored by every other op. */
enum { SMALL_OP_CONV = 0, SMALL_OP_DWCONV = 1, SMALL_OP_MAXPOOL = 2, SMALL_OP_AVGPOOL = 3, SMALL_OP_RELU = 4,
       SMALL_OP_ADD = 5, SMALL_OP_DENSE = 6, SMALL_OP_BATCHNORM = 7, SMALL_OP_UPSAMPLE = 8, SMALL_OP_GROUPCONV = 9 };
enum { SMALL_BUF_IN = -1, SMALL_BUF_OUT = -2, SMALL_MAX_SLOTS = 8 };

typedef struct {
    int op;
    int Ci, Co, kh, kw, stride;
    small_pad pad;
    int Cib, Cob;
    int src, src2, dst;
    const float *filt;
    int F_C, S_C;
} small_layer;

/* Bytes of workspace small_network_run needs for this table and input shape (host only, enqueues nothing).
 * Slots are 256-byte aligned. */
int small_network_workspace(const small_layer *layers, int n_layers, int N, int C0, int H0, int W0,
                            size_t *bytes);

/* Enqueues every layer of the table, in order, on `stream`. `layers` is a HOST array (read during the
 * call only). in_blocked: [N][C0/Cb0][H0][W0][Cb0] with Cb0 = layers[0].Cib. out_blocked receives every
 * write to SMALL_BUF_OUT. workspace: device memory, 256-byte aligned, workspace_bytes >= the size
 * reported by small_network_workspace. The table is validated completely before anything is enqueued. */
int small_network_run(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                      void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, void *stream);

/* small_network_run_plain: the same run from a plain [N][C0][H0][W0] input: the layout change of the network boundary
 * (Section 4.4: formats are converted only where the network meets the outside) happens inside the first layer's
 * kernel instead of in a small_pack launch of its own. Only for tables whose input is read by layer 0 alone, a
 * convolution with one input block of fewer than 16 channels and a reduction Ci*kh*kw of 5..8, 25..28 or 37..40
 * values (the first layers of the CNNs here) producing at least 16384 output pixels; otherwise SMALL_ERR_LAYER and
 * nothing is enqueued (pack the input and call small_network_run). Same results as small_pack + small_network_run. */
int small_network_run_plain(const small_layer *layers, int n_layers, const float *in_nchw, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, void *stream);

/* small_network_run_opt: small_network_run with options (flags, a sum of SMALL_RUN_*; unknown bits: SMALL_ERR_SHAPE).
 *   SMALL_RUN_PLAIN_INPUT   `in` is a plain [N][C0][H0][W0] tensor: exactly small_network_run_plain.
 *   SMALL_RUN_RESIDENT_OFF  never use image-resident runs (below); SMALL_RUN_RESIDENT_ON: use them at any batch size.
 *   SMALL_RUN_PLAIN_OUTPUT  the caller reads `out_blocked` as a plain [N][C][H][W] tensor (the layout change at the
 *                           network's other boundary). Accepted when blocked and plain layout coincide, i.e. the
 *                           result has one pixel per image and one channel block (H = W = 1, C = Cb: the logits of a
 *                           classifier head); then no small_unpack is needed. Otherwise SMALL_ERR_LAYER, nothing
 *                           enqueued: run without the flag and call small_unpack.
 * Image-resident runs: consecutive layers whose per-image tensors fit 152 KB of LDS together run as ONE launch,
 * one image per workgroup (one workgroup per compute unit, further images in further rounds): optionally a first convolution on
 * fewer than 16 input channels that reads the network input (Ci * kh * kw <= 40), then convolutions with 16-channel
 * blocks in and out (1 or 9 filter taps, any stride and padding, with their folded ReLU / residual add), optionally
 * closed by an average pooling over the whole image + fully connected layer (C <= 256, Co <= 16). Only the run's
 * input, its last result and the filters touch HBM; the tensors between them are never written (allowed only when
 * nothing outside the run reads them, as for every fusion here). This is the fused layer of the paper's
 * "Conclusion & Future Directions" across layers of Table 1's partial-reduction class. Depthwise convolutions
 * (16-channel blocks, at most 9 taps, filter 16-byte aligned) may stand inside a run, and a 1x1 convolution added onto
 * the convolution before it (a projection shortcut) is folded into that one. Without either RESIDENT flag such runs
 * are used when the batch is 9/16 .. 1 or 1 3/4 .. 2 rounds of one image per compute unit (on the 256 compute units of
 * an MI355X: 144 <= N <= 256 or 448 <= N <= 512; measured break-even points against the layer-by-layer kernels) and
 * the run averages at least
 * 250000 (one round) or 500000 (two rounds) multiply-adds per layer and image (below that the per-layer cost inside
 * a workgroup outweighs the launches saved: measured on the depthwise-separable CNNs); small_network_run,
 * small_network_run_plain and small_network_run_range follow that rule too (small_network_run_plain then also
 * accepts tables whose first layer only the run's own first-layer code can take from a plain tensor). Results
 * agree with the layer-by-layer kernels within the conv tolerance, not bit for bit (another summation order).
 * small_network_launches_at: the first layer of every launch that a run with these N, C0, H0, W0 and flags makes
 * (small_network_launches: the list that depends on the table alone: without image-resident runs and without the
 * runs of depthwise + pointwise blocks below, which depend on the image size). Host-only, no GPU needed. */
enum { SMALL_RUN_PLAIN_INPUT = 1, SMALL_RUN_RESIDENT_OFF = 2, SMALL_RUN_RESIDENT_ON = 4, SMALL_RUN_PLAIN_OUTPUT = 8 };
int small_network_run_opt(const small_layer *layers, int n_layers, const float *in, float *out_blocked, void *workspace,
                          size_t workspace_bytes, int N, int C0, int H0, int W0, unsigned flags, void *stream);
int small_network_launches_at(const small_layer *layers, int n_layers, int N, int C0, int H0, int W0, unsigned flags,
                              int *first_layer, int *n_launches);

/* Cross-layer fusion. small_network_run folds layers that only touch a convolution's output element by
 * element into that convolution's store phase (the direction the paper's conclusion calls an abstract
 * "fused" layer, possible because every layer shares one layout): a ReLU in place on the output of a
 * convolution or depthwise convolution, and an addition of the convolution's output to another buffer
 * (residual connection), optionally followed by an in-place ReLU. Results are bit-identical to the
 * unfused sequence and every buffer that is read later holds what the table says.
 * An in-place batch normalization directly after a convolution or fully connected layer (before the addition and the
 * ReLU, the order of a residual block: conv, norm, add, ReLU) is folded the same way -- one fused multiply-add per
 * element in the store phase, the same operation the separate layer performs -- where the convolution's kernel has
 * that epilogue (16-channel blocks, 16-byte aligned parameters); elsewhere the runner launches the convolution and
 * then the normalization (with the ReLU, if one follows) over its result. A ReLU in place after a batch
 * normalization that stands alone runs in the normalization's kernel.
 * A depthwise 3x3 convolution (16-channel blocks, stride 1 or 2, optional in-place ReLU) whose output is read
 * only by an unpadded stride-1 1x1 convolution (optional in-place ReLU) runs with it in one kernel: the
 * depthwise result stays on the compute unit and its buffer is never written (allowed only when no later
 * layer reads that buffer before it is rewritten). The depthwise sum is then taken in a different order
 * than by small_dwconv2d: results agree within the tolerance of the two layers, not bit for bit.
 * Two to twelve such pairs in a row -- any strides, paddings and channel counts (multiples of 16), each pair reading
 * what the pair before wrote, every tensor of the run a small image (at most 256 pixels and 6144 values; with one image
 * per workgroup only up to one round of workgroups: the launch list depends on the batch) --
 * run in ONE kernel from the first pair's source to the last pair's destination: a workgroup keeps whole images on
 * the compute unit through all pairs. Every buffer the table writes inside the run except that destination is
 * never written (same liveness rule); the destination may be the run's own source buffer (when the pairs change the
 * tensor's shape, the runner then writes into the memory of the last depthwise layer's buffer and lets the two
 * workspace slots change places, as for a single pair). When the run is followed by an average pooling over the whole
 * image and a fully connected layer of at most 16 outputs that alone read its result, these close the same kernel: the
 * run's last tensor is then never written (same liveness rule) and the launch writes the logits. Same tolerance.
 * A run of two to sixteen pointwise layers (SMALL_OP_DENSE on 1x1 images, unpadded stride-1 1x1 SMALL_OP_CONV;
 * at most 128 channels per tensor, in 16-channel blocks, or 8 channels in one 8-channel block for tensors
 * inside the run), each optionally followed by an in-place ReLU and each read only by the next, runs in one
 * kernel from the first layer's source to the last layer's destination: the tensors between them stay on
 * the compute unit and their buffers are never written (same liveness rule as above; the run never ends in
 * the buffer it starts from). The fully connected autoencoder of Section "MLPerf:Tiny Inference Models"
 * is one such run. Results agree with the layer-by-layer run within the tolerance of the chained
 * reductions, not bit for bit.
 *
 * An average pooling over the whole image (no padding, 16-channel blocks, at most 256 channels) whose output only
 * the following SMALL_OP_DENSE layer (at most 16 outputs) reads runs with it in one kernel; the pooled tensor's
 * buffer is never written (same liveness rule).
 *
 * small_network_launches (host only): how many kernel launches the table becomes, and for each the index
 * of the first layer it covers (folded layers follow it directly). It sees the table only: where a
 * depthwise + 1x1 pair or a pointwise run cannot run in one kernel for reasons outside the table (unaligned
 * pointers, an image geometry the kernel does not take, a run input of 4 GiB or more), the run launches
 * the layers separately. first_layer may be NULL, else it must
 * have room for n_layers ints.
 * small_network_run_range: like small_network_run, but enqueues only the launches whose first layer index
 * lies in [first, first + count); buffers keep whatever earlier calls left in them (for per-layer timing
 * and debugging). */
int small_network_launches(const small_layer *layers, int n_layers, int *first_layer, int *n_launches);
int small_network_run_range(const small_layer *layers, int n_layers, const float *in_blocked, float *out_blocked,
                            void *workspace, size_t workspace_bytes, int N, int C0, int H0, int W0, int first,
                            int count, void *stream);

/* small_network_run_static: small_network_run_opt for callers that cannot allocate device memory or hand over a
 * workspace of their own -- code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc. The
 * layer workspace is an array of SMALL_STATIC_WORKSPACE_BYTES (64 MiB) inside the library's device image, one copy per
 * GPU, held until the process ends; the caller passes only the input and the output. Same kernels, same results
 * (bit for bit) as small_network_run_opt with a workspace of that size. The call allocates nothing and frees nothing
 * (the first call on a device looks the array's address up once; make that call outside a graph capture).
 * A table and batch whose small_network_workspace size exceeds SMALL_STATIC_WORKSPACE_BYTES: SMALL_ERR_STATIC, nothing
 * enqueued (64 MiB holds, for example, the residual CNN of 32x32x3 images up to batch 256). Every call on a GPU uses
 * that GPU's one array: calls that may overlap on one GPU (different streams, or replays of graphs that captured it)
 * race on it, and the array keeps the last call's tensors; nothing in it needs clearing, every layer writes its
 * result before a later layer reads it. in / out_blocked / flags as for small_network_run_opt. */
enum { SMALL_STATIC_WORKSPACE_BYTES = 64 * 1024 * 1024 };
int small_network_run_static(const small_layer *layers, int n_layers, const float *in, float *out_blocked, int N, int C0,
                             int H0, int W0, unsigned flags, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SMALL_H */
