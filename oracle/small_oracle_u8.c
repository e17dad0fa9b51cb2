/*
 * small_oracle_u8.c -- CPU oracle for the quantized (uint8) layers. TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow C on plain NCHW uint8 activations and OIHW uint8 filters; the product
 * library never links, loads or calls it and shares no code with it.
 *
 * What the paper fixes (Section "Memory Usage Comparison", Section "Quantized Inference"):
 * inputs and outputs of a quantized layer are uint8, partial results are accumulated in
 * int32. It gives no rule for turning the int32 sum back into uint8, so the rule below is
 * this build's own (the usual affine scheme, integer-only):
 *
 *   real value of a code q = scale * (q - zero_point)
 *   acc  = sum over the in-image taps of (x - zx) * (w - zw)            (int32, exact)
 *   y    = clamp(zy + floor((acc * mult + 2^(shift-1)) / 2^shift), lo, hi)   (int64 product;
 *          round half up; no rounding term when shift == 0)
 *
 * with 0 <= mult < 2^31, 0 <= shift <= 31, 0 <= lo <= hi <= 255. A ReLU after the layer is
 * lo = zy. Taps outside the image contribute nothing (the padding value is the zero point).
 * Max pooling compares codes (scale > 0 keeps the order) and skips out-of-image taps;
 * average pooling is floor((sum + n/2) / n) over the n in-image taps; ReLU is max(x, z).
 * Addition (the residual blocks of Section "MLPerf:Tiny Inference Models" on codes) takes two
 * tensors with scales and zero points of their own; both are brought to the output's scale by a
 * multiplier each and one common shift, with a single rounding:
 *
 *   acc = (a - za) * mult_a + (b - zb) * mult_b                          (int64, exact)
 *   y   = clamp(zy + floor((acc + 2^(shift-1)) / 2^shift), lo, hi)       (no rounding term when shift == 0)
 *
 * i.e. mult_a / 2^shift stands for scale_a / scale_y and mult_b / 2^shift for scale_b / scale_y.
 *
 * Parity pins (tests/test_oracle_u8.py): accumulators == a library fp64 convolution of the
 * zero-point-shifted tensors (exact for these magnitudes); requantization == exact rational
 * rounding, hand-worked values, identity for mult = 2^shift; pooling and ReLU == the fp32
 * oracle applied to the codes; layouts == the offset formulas of the layout statement;
 * addition == exact rational arithmetic on every pair of codes, plain integer addition for
 * equal unit scales, the real-valued sum within half an output step.
 */
#include <stddef.h>
#include <stdint.h>

static int out_dim(int in, int f, int s, int lo, int hi)
{
    int t = in + lo + hi - f;
    if (t < 0 || s <= 0) return 0;
    return t / s + 1;
}

/* floor(a / 2^k) for signed a, without relying on the shift of a negative value */
static int64_t floor_shift(int64_t a, int k)
{
    const int64_t d = (int64_t)1 << k;
    int64_t q = a / d;
    if (a % d != 0 && a < 0) --q;
    return q;
}

uint8_t sq_requant_one(int32_t acc, int zy, int32_t mult, int shift, int lo, int hi)
{
    int64_t v = (int64_t)acc * (int64_t)mult;
    if (shift > 0) v = floor_shift(v + ((int64_t)1 << (shift - 1)), shift);
    v += zy;
    if (v < lo) v = lo;
    if (v > hi) v = hi;
    return (uint8_t)v;
}

void sq_requant(const int32_t *acc, uint8_t *y, size_t n, int zy, int32_t mult, int shift, int lo, int hi)
{
    for (size_t i = 0; i < n; ++i) y[i] = sq_requant_one(acc[i], zy, mult, shift, lo, hi);
}

/* Full-channel reduction (Table 1 row 4) on codes: int32 accumulators. */
void sq_conv2d_acc(const uint8_t *x, const uint8_t *w, int32_t *acc, int N, int Ci, int Co, int H, int W, int kh, int kw,
                   int s, int pt, int pb, int pl, int pr, int zx, int zw)
{
    const int Ho = out_dim(H, kh, s, pt, pb), Wo = out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Co; ++co)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    int64_t a = 0;
                    for (int ci = 0; ci < Ci; ++ci)
                        for (int ky = 0; ky < kh; ++ky)
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                a += ((int)x[(((size_t)n * Ci + ci) * H + ih) * W + iw] - zx) *
                                     ((int)w[(((size_t)co * Ci + ci) * kh + ky) * kw + kx] - zw);
                            }
                    acc[(((size_t)n * Co + co) * Ho + oh) * Wo + ow] = (int32_t)a;
                }
}

/* Single-channel reduction with weights (Table 1 row 2); w is [C][1][kh][kw]. */
void sq_dwconv2d_acc(const uint8_t *x, const uint8_t *w, int32_t *acc, int N, int C, int H, int W, int kh, int kw, int s,
                     int pt, int pb, int pl, int pr, int zx, int zw)
{
    const int Ho = out_dim(H, kh, s, pt, pb), Wo = out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    int64_t a = 0;
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            a += ((int)x[(((size_t)n * C + c) * H + ih) * W + iw] - zx) *
                                 ((int)w[((size_t)c * kh + ky) * kw + kx] - zw);
                        }
                    acc[(((size_t)n * C + c) * Ho + oh) * Wo + ow] = (int32_t)a;
                }
}

/* Single-channel reduction without weights on codes. mode 0 = max, 1 = average (round half up). */
void sq_pool2d(const uint8_t *x, uint8_t *y, int N, int C, int H, int W, int kh, int kw, int s, int pt, int pb, int pl,
               int pr, int mode)
{
    const int Ho = out_dim(H, kh, s, pt, pb), Wo = out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    int m = 0, sum = 0, cnt = 0;
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const int v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (v > m) m = v;
                            sum += v;
                            ++cnt;
                        }
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] =
                        (uint8_t)(mode == 0 ? m : (cnt > 0 ? (sum + cnt / 2) / cnt : 0));
                }
}

/* Single-element layer with two inputs on codes (rule in the header). */
void sq_add(const uint8_t *a, const uint8_t *b, uint8_t *y, size_t n, int za, int zb, int zy, int32_t mult_a, int32_t mult_b,
            int shift, int lo, int hi)
{
    for (size_t i = 0; i < n; ++i) {
        int64_t v = (int64_t)((int)a[i] - za) * mult_a + (int64_t)((int)b[i] - zb) * mult_b;
        if (shift > 0) v = floor_shift(v + ((int64_t)1 << (shift - 1)), shift);
        v += zy;
        if (v < lo) v = lo;
        if (v > hi) v = hi;
        y[i] = (uint8_t)v;
    }
}

void sq_relu(const uint8_t *x, uint8_t *y, size_t n, int z)
{
    for (size_t i = 0; i < n; ++i) y[i] = x[i] > z ? x[i] : (uint8_t)z;
}

/* Section "Common Data Format" on bytes: activations [N][C/Cb][H][W][Cb]; filters
 * [Co/Cob][Ci/Cib][kh][kw][Cob][Cib] -- for the quantized path the two innermost filter
 * dimensions are swapped with respect to the fp32 layout, so that the Cib bytes one output
 * channel multiplies with one pixel's Cib bytes are contiguous. */
size_t sq_act_offset(int n, int c, int h, int w, int C, int H, int W, int Cb)
{
    return ((((size_t)n * (C / Cb) + c / Cb) * H + h) * W + w) * Cb + c % Cb;
}

size_t sq_filter_offset(int co, int ci, int ky, int kx, int Ci, int kh, int kw, int Cob, int Cib)
{
    return ((((((size_t)(co / Cob) * (Ci / Cib) + ci / Cib) * kh + ky) * kw + kx) * Cob) + co % Cob) * Cib + ci % Cib;
}

void sq_pack(const uint8_t *nchw, uint8_t *blk, int N, int C, int H, int W, int Cb, int unpack)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w) {
                    const size_t a = (((size_t)n * C + c) * H + h) * W + w, b = sq_act_offset(n, c, h, w, C, H, W, Cb);
                    if (unpack) ((uint8_t *)nchw)[a] = blk[b];
                    else blk[b] = nchw[a];
                }
}

void sq_pack_filter(const uint8_t *oihw, uint8_t *blk, int Co, int Ci, int kh, int kw, int Cob, int Cib)
{
    for (int co = 0; co < Co; ++co)
        for (int ci = 0; ci < Ci; ++ci)
            for (int ky = 0; ky < kh; ++ky)
                for (int kx = 0; kx < kw; ++kx)
                    blk[sq_filter_offset(co, ci, ky, kx, Ci, kh, kw, Cob, Cib)] =
                        oihw[(((size_t)co * Ci + ci) * kh + ky) * kw + kx];
}
