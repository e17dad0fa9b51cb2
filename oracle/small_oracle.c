/*
 * small_oracle.c -- CPU oracle for the SMaLL layer set. TEST INFRASTRUCTURE ONLY.
 *
 * Plain, slow, obviously-correct C. It is used by the tests, by the smoke check and
 * by the benchmark's CPU-baseline leg; the product library never links, loads or
 * calls it, and it shares no code, header or table with the HIP path.
 *
 * Two families:
 *   so_*   "O1": every layer written as its mathematical definition on plain
 *          NCHW activations / OIHW filters, each output accumulated in fp64 and
 *          rounded once to fp32 (paper Section 3.1 "Abstract DNN Layer", Section 3.2
 *          "Classes of layers", Table 1, Table 2).
 *   so_abstract_layer_blocked  "O2": the paper's Algorithm 1 loop nest, in its loop
 *          order and notation, on the channel-blocked layouts of Section 4.4
 *          "Common Data Format", with the kernel phases of Algorithm 2 (LOAD tile,
 *          COMPUTE over x, y, ii, STORE tile).
 *
 * Readings where the paper is silent (kept identical in the HIP library's contract):
 *   - batch is an outermost dimension, images independent (Section 3.1.1 allows I_B);
 *   - explicit zero padding (t, b, l, r); O = floor((I + lo + hi - F) / S) + 1;
 *     conv / depthwise: out-of-range taps contribute 0; max-pool: out-of-range taps
 *     are skipped; avg-pool: divisor = number of in-range taps;
 *   - ReLU is y = (x > 0) ? x : +0  (so -0 -> +0 and NaN -> +0);
 *   - max-pool starts from -inf and replaces on (v > m), taps visited row-major;
 *   - average pooling = Add reduction over the window, then divide by the count;
 *   - output channel of the abstract layer = group * K + filter-in-group.
 *
 * Parity pins (tests/test_oracle_*.py): hand-worked examples under tests/golden/,
 * delta / all-ones closed forms, 1x1 conv == GEMM, depthwise == block-diagonal
 * conv, dense == full-window conv, O2 == O1, pack/unpack offsets from the layout
 * statement; group convolution == per-group full convolutions == a library grouped
 * convolution == O2; batch normalization == a library's inference batch-norm with the
 * statistics folded; upsampling == element repetition. No function in this file is unpinned.
 */
#include <math.h>
#include <stddef.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

int so_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* Output-size equation of Section 3.1.2, extended with padding and floor. */
int so_out_dim(int in, int f, int s, int lo, int hi)
{
    int t = in + lo + hi - f;
    if (t < 0 || s <= 0) return 0;
    return t / s + 1;
}

/* ------------------------------------------------------------------ O1 layers */

/* Full-channel reduction (Table 1 row 4): O[n,co,oh,ow] = sum_{ci,ky,kx} I * W. */
void so_conv2d(const float *x, const float *w, float *y, int N, int Ci, int Co, int H, int W,
               int kh, int kw, int s, int pt, int pb, int pl, int pr)
{
    const int Ho = so_out_dim(H, kh, s, pt, pb), Wo = so_out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Co; ++co)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int ci = 0; ci < Ci; ++ci)
                        for (int ky = 0; ky < kh; ++ky)
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += (double)x[(((size_t)n * Ci + ci) * H + ih) * W + iw] *
                                       (double)w[(((size_t)co * Ci + ci) * kh + ky) * kw + kx];
                            }
                    y[(((size_t)n * Co + co) * Ho + oh) * Wo + ow] = (float)acc;
                }
}

/* Single-channel reduction with weights (Table 1 row 2, G = C, K = 1); w is [C][1][kh][kw]. */
void so_dwconv2d(const float *x, const float *w, float *y, int N, int C, int H, int W,
                 int kh, int kw, int s, int pt, int pb, int pl, int pr)
{
    const int Ho = so_out_dim(H, kh, s, pt, pb), Wo = so_out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            acc += (double)x[(((size_t)n * C + c) * H + ih) * W + iw] *
                                   (double)w[((size_t)c * kh + ky) * kw + kx];
                        }
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] = (float)acc;
                }
}

/* Single-channel reduction without weights. mode 0 = max, 1 = average. */
void so_pool2d(const float *x, float *y, int N, int C, int H, int W,
               int kh, int kw, int s, int pt, int pb, int pl, int pr, int mode)
{
    const int Ho = so_out_dim(H, kh, s, pt, pb), Wo = so_out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    float m = -INFINITY;
                    double sum = 0.0;
                    int cnt = 0;
                    for (int ky = 0; ky < kh; ++ky)
                        for (int kx = 0; kx < kw; ++kx) {
                            const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                            if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                            const float v = x[(((size_t)n * C + c) * H + ih) * W + iw];
                            if (v > m) m = v;
                            sum += (double)v;
                            ++cnt;
                        }
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] =
                        mode == 0 ? m : (float)(sum / (double)(cnt > 0 ? cnt : 1));
                }
}

/* Single-element reductions (Table 1 row 1). */
void so_relu(const float *x, float *y, size_t n)
{
    for (size_t i = 0; i < n; ++i) y[i] = (x[i] > 0.0f) ? x[i] : 0.0f;
}

void so_add(const float *a, const float *b, float *y, size_t n)
{
    for (size_t i = 0; i < n; ++i) y[i] = (float)((double)a[i] + (double)b[i]);
}

/* Batch normalization as the single-element FMA of Table 2: y = x * scale[c] + shift[c] (the layer's
 * statistics folded into one scale and one shift per channel), one rounding per output. */
void so_batchnorm(const float *x, const float *scale, const float *shift, float *y, int N, int C, int H, int W)
{
    const size_t HW = (size_t)H * W;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (size_t i = 0; i < HW; ++i) {
                const size_t o = ((size_t)n * C + c) * HW + i;
                y[o] = (float)((double)x[o] * (double)scale[c] + (double)shift[c]);
            }
}

/* Nearest-neighbour upsampling by integer factors (Table 2): output pixel (oh, ow) copies input pixel
 * (oh / fh, ow / fw). */
void so_upsample(const float *x, float *y, int N, int C, int H, int W, int fh, int fw)
{
    const int Ho = H * fh, Wo = W * fw;
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow)
                    y[(((size_t)n * C + c) * Ho + oh) * Wo + ow] = x[(((size_t)n * C + c) * H + oh / fh) * W + ow / fw];
}

/* Partial-channel reduction (Table 1 row 3, group convolution): G = (Ci - F_C) / S_C + 1 groups; group g reduces
 * input channels g * S_C .. g * S_C + F_C - 1 with K filters; output channel = g * K + k (Section 3.1.2).
 * w is [G * K][F_C][kh][kw]. */
void so_group_conv2d(const float *x, const float *w, float *y, int N, int Ci, int F_C, int S_C, int K, int H, int W,
                     int kh, int kw, int s, int pt, int pb, int pl, int pr)
{
    const int G = (Ci - F_C) / S_C + 1, Co = G * K;
    const int Ho = so_out_dim(H, kh, s, pt, pb), Wo = so_out_dim(W, kw, s, pl, pr);
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int co = 0; co < Co; ++co) {
            const int g = co / K;
            for (int oh = 0; oh < Ho; ++oh)
                for (int ow = 0; ow < Wo; ++ow) {
                    double acc = 0.0;
                    for (int fc = 0; fc < F_C; ++fc)
                        for (int ky = 0; ky < kh; ++ky)
                            for (int kx = 0; kx < kw; ++kx) {
                                const int ih = oh * s + ky - pt, iw = ow * s + kx - pl;
                                if (ih < 0 || ih >= H || iw < 0 || iw >= W) continue;
                                acc += (double)x[(((size_t)n * Ci + g * S_C + fc) * H + ih) * W + iw] *
                                       (double)w[(((size_t)co * F_C + fc) * kh + ky) * kw + kx];
                            }
                    y[(((size_t)n * Co + co) * Ho + oh) * Wo + ow] = (float)acc;
                }
        }
}

/* Full reduction (Table 1 row 5): x is [N][Ci][H][W], w is [Co][Ci][H][W], y is [N][Co]. */
void so_dense(const float *x, const float *w, float *y, int N, int Ci, int Co, int H, int W)
{
    const size_t L = (size_t)Ci * H * W;
#pragma omp parallel for collapse(2) schedule(static)
    for (int n = 0; n < N; ++n)
        for (int o = 0; o < Co; ++o) {
            double acc = 0.0;
            for (size_t i = 0; i < L; ++i) acc += (double)x[n * L + i] * (double)w[o * L + i];
            y[(size_t)n * Co + o] = (float)acc;
        }
}

/* ------------------------------------------------------------------ layouts
 * Activations: Cb fastest, then W, then H, then channel block (Section 4.4), batch outermost.
 * Filters: tiled in both channel dims, dimension order = loop order of Algorithm 1. */

size_t so_act_offset(int n, int c, int h, int w, int C, int H, int W, int Cb)
{
    return ((((size_t)n * (C / Cb) + c / Cb) * H + h) * W + w) * Cb + c % Cb;
}

size_t so_filter_offset(int co, int ci, int ky, int kx, int Ci, int kh, int kw, int Cob, int Cib)
{
    return (((((size_t)(co / Cob) * (Ci / Cib) + ci / Cib) * kh + ky) * kw + kx) * Cib + ci % Cib) * Cob +
           co % Cob;
}

void so_pack(const float *nchw, float *blk, int N, int C, int H, int W, int Cb)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    blk[so_act_offset(n, c, h, w, C, H, W, Cb)] =
                        nchw[(((size_t)n * C + c) * H + h) * W + w];
}

void so_unpack(const float *blk, float *nchw, int N, int C, int H, int W, int Cb)
{
    for (int n = 0; n < N; ++n)
        for (int c = 0; c < C; ++c)
            for (int h = 0; h < H; ++h)
                for (int w = 0; w < W; ++w)
                    nchw[(((size_t)n * C + c) * H + h) * W + w] =
                        blk[so_act_offset(n, c, h, w, C, H, W, Cb)];
}

void so_pack_filter(const float *oihw, float *blk, int Co, int Ci, int kh, int kw, int Cob, int Cib)
{
    for (int co = 0; co < Co; ++co)
        for (int ci = 0; ci < Ci; ++ci)
            for (int ky = 0; ky < kh; ++ky)
                for (int kx = 0; kx < kw; ++kx)
                    blk[so_filter_offset(co, ci, ky, kx, Ci, kh, kw, Cob, Cib)] =
                        oihw[(((size_t)co * Ci + ci) * kh + ky) * kw + kx];
}

/* Depthwise filters [C][1][kh][kw] -> [C/Cb][kh][kw][Cb] (general layout with F_Cb = 1, G_b = Cb). */
void so_pack_dw_filter(const float *c1hw, float *blk, int C, int kh, int kw, int Cb)
{
    for (int c = 0; c < C; ++c)
        for (int ky = 0; ky < kh; ++ky)
            for (int kx = 0; kx < kw; ++kx)
                blk[((((size_t)(c / Cb)) * kh + ky) * kw + kx) * Cb + c % Cb] =
                    c1hw[((size_t)c * kh + ky) * kw + kx];
}

/* ------------------------------------------------------------------ O2: Algorithm 1
 *
 * One loop nest for every layer class. Parameters in the paper's notation:
 *   window F_H x F_W x F_C, strides S_H, S_W, S_C, K filters per group,
 *   G = (I_C - F_C) / S_C + 1 groups, O_C = K * G,
 *   tile sizes G_b, K_b (output-channel block O_cb = G_b * K_b), F_Cb, O_wb.
 * op: 0 = FMA with weights, 1 = Max (no weights), 2 = Add then divide by tap count.
 * I  : [N][I_C/Icb][I_H][I_W][Icb]
 * Wt : [G/G_b][K/K_b][F_C/F_Cb][F_H][F_W][F_Cb][G_b][K_b]   (ignored for op != 0)
 * O  : [N][O_C/O_cb][O_H][O_W][O_cb]
 * The O tensor is held in fp64 between visits so the result equals the definition
 * rounded once. Returns 0, or a negative code for an indivisible tiling.
 */
int so_abstract_layer_blocked(int op, const float *I, const float *Wt, float *O, int N, int I_C, int I_H,
                              int I_W, int F_H, int F_W, int F_C, int S_H, int S_W, int S_C, int K, int pt,
                              int pb, int pl, int pr, int Icb, int G_b, int K_b, int F_Cb, int O_wb)
{
    if (S_C <= 0 || (I_C - F_C) % S_C) return -1;
    const int G = (I_C - F_C) / S_C + 1;
    const int O_C = K * G, O_cb = G_b * K_b;
    if (G % G_b || K % K_b || F_C % F_Cb || I_C % Icb || O_C % O_cb || O_wb <= 0) return -2;
    const int O_H = so_out_dim(I_H, F_H, S_H, pt, pb), O_W = so_out_dim(I_W, F_W, S_W, pl, pr);
    const size_t out_elems = (size_t)N * O_C * O_H * O_W;
    double *acc = (double *)malloc(sizeof(double) * (out_elems ? out_elems : 1));
    double *tile = (double *)malloc(sizeof(double) * (size_t)O_wb * G_b * K_b);
    if (!acc || !tile) { free(acc); free(tile); return -3; }

    for (int n = 0; n < N; ++n)
    for (int g = 0; g < G; g += G_b)                     /* "in parallel" in the paper */
    for (int k = 0; k < K; k += K_b)                     /* "in parallel" in the paper */
    for (int i = 0; i < F_C; i += F_Cb)
    for (int j = 0; j < O_H; ++j)
    for (int l = 0; l < O_W; l += O_wb) {
        /* ---- kernel, LOAD phase: first visit initialises, later visits reload */
        for (int ll = 0; ll < O_wb && l + ll < O_W; ++ll)
        for (int gg = 0; gg < G_b; ++gg)
        for (int kk = 0; kk < K_b; ++kk) {
            const int oc = (g + gg) * K + (k + kk);
            double *t = &tile[((size_t)ll * G_b + gg) * K_b + kk];
            if (i == 0) *t = (op == 1) ? -INFINITY : 0.0;
            else *t = acc[so_act_offset(n, oc, j, l + ll, O_C, O_H, O_W, O_cb)];
        }
        /* ---- COMPUTE phase */
        for (int x = 0; x < F_H; ++x)
        for (int y = 0; y < F_W; ++y)
        for (int ii = 0; ii < F_Cb; ++ii)
        for (int ll = 0; ll < O_wb && l + ll < O_W; ++ll)
        for (int gg = 0; gg < G_b; ++gg)
        for (int kk = 0; kk < K_b; ++kk) {
            const int ih = j * S_H + x - pt, iw = (l + ll) * S_W + y - pl;
            if (ih < 0 || ih >= I_H || iw < 0 || iw >= I_W) continue;   /* edge handling around the kernel */
            const int ic = (g + gg) * S_C + i + ii;
            const double v = (double)I[so_act_offset(n, ic, ih, iw, I_C, I_H, I_W, Icb)];
            double *t = &tile[((size_t)ll * G_b + gg) * K_b + kk];
            if (op == 0) {
                const size_t wo =
                    (((((((size_t)(g / G_b) * (K / K_b) + k / K_b) * (F_C / F_Cb) + i / F_Cb) * F_H + x) * F_W + y) *
                          F_Cb + ii) * G_b + gg) * K_b + kk;
                *t += v * (double)Wt[wo];
            } else if (op == 1) {
                if (v > *t) *t = v;
            } else {
                *t += v;
            }
        }
        /* ---- STORE phase */
        for (int ll = 0; ll < O_wb && l + ll < O_W; ++ll)
        for (int gg = 0; gg < G_b; ++gg)
        for (int kk = 0; kk < K_b; ++kk) {
            const int oc = (g + gg) * K + (k + kk);
            acc[so_act_offset(n, oc, j, l + ll, O_C, O_H, O_W, O_cb)] = tile[((size_t)ll * G_b + gg) * K_b + kk];
        }
    }

    /* round once; the Add reduction becomes an average over the in-range taps */
    for (int n = 0; n < N; ++n)
    for (int oc = 0; oc < O_C; ++oc)
    for (int j = 0; j < O_H; ++j)
    for (int l = 0; l < O_W; ++l) {
        const size_t o = so_act_offset(n, oc, j, l, O_C, O_H, O_W, O_cb);
        double v = acc[o];
        if (op == 2) {
            int cnt = 0;
            for (int x = 0; x < F_H; ++x)
                for (int y = 0; y < F_W; ++y) {
                    const int ih = j * S_H + x - pt, iw = l * S_W + y - pl;
                    if (ih >= 0 && ih < I_H && iw >= 0 && iw < I_W) ++cnt;
                }
            v /= (double)(cnt > 0 ? cnt * F_C : 1);
        }
        O[o] = (float)v;
    }
    free(acc);
    free(tile);
    return 0;
}
