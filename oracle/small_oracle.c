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
 *   so_abstract_layer_blocked  "O2": the blocked evaluation that Algorithm 1 defines,
 *          on the channel-blocked layouts of Section 4.4 "Common Data Format": register
 *          tiles of the output visited once per block of reduction channels, each visit
 *          being the three kernel phases of Algorithm 2.
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

/* ------------------------------------------------------------------ O2: the blocked evaluation
 *
 * One routine for every layer class, on the channel-blocked layouts of Section 4.4. It is the evaluation that
 * Algorithm 1 defines (the definition being checked here; tests require O2 == O1): the output is cut into register
 * tiles of O_wb pixels x (G_b * K_b) output channels; for every block of F_Cb reduction channels every tile of the
 * tensor is visited once, and a visit is Algorithm 2's three phases -- bring the tile in (start values on the first
 * reduction block, the partial results of the earlier blocks afterwards), reduce the window over this block's
 * channels into it, put it back. Written here as a tile descriptor plus one helper per phase.
 *
 * Parameters in the paper's notation: window F_H x F_W x F_C, strides S_H, S_W, S_C, K filters per group,
 * G = (I_C - F_C) / S_C + 1 groups, O_C = K * G, tile sizes G_b, K_b (output-channel block O_cb = G_b * K_b),
 * F_Cb, O_wb. op: 0 = FMA with weights, 1 = Max (no weights), 2 = Add then divide by tap count.
 * I  : [N][I_C/Icb][I_H][I_W][Icb]
 * Wt : [G/G_b][K/K_b][F_C/F_Cb][F_H][F_W][F_Cb][G_b][K_b]   (ignored for op != 0)
 * O  : [N][O_C/O_cb][O_H][O_W][O_cb]
 * Partial results are held in fp64 between visits so the result equals the definition rounded once.
 * Returns 0, or a negative code for an indivisible tiling.
 */
struct blocked_layer {
    int op;
    const float *I, *Wt;
    double *partial;                 /* the output tensor in its blocked layout, fp64 */
    int I_C, I_H, I_W, O_C, O_H, O_W;
    int F_H, F_W, F_C, S_H, S_W, S_C, K, G;
    int pt, pl;
    int Icb, G_b, K_b, F_Cb, O_wb, O_cb;
};

/* One visit: image, first group and first filter of the channel tile, first reduction channel, output row, first
 * output column; `width` pixels wide (O_wb, fewer at the right edge). */
struct tile_visit { int image, group0, filter0, red0, row, col0, width; };

static int tile_channel(const struct blocked_layer *a, const struct tile_visit *v, int dg, int dk)
{
    return (v->group0 + dg) * a->K + v->filter0 + dk;        /* output channel = group * K + filter in group */
}

static void tile_bring_in(const struct blocked_layer *a, const struct tile_visit *v, double *regs)
{
    for (int p = 0; p < v->width; ++p)
        for (int dg = 0; dg < a->G_b; ++dg)
            for (int dk = 0; dk < a->K_b; ++dk) {
                double *r = &regs[(p * a->G_b + dg) * a->K_b + dk];
                if (v->red0 == 0)
                    *r = a->op == 1 ? -INFINITY : 0.0;
                else
                    *r = a->partial[so_act_offset(v->image, tile_channel(a, v, dg, dk), v->row, v->col0 + p, a->O_C,
                                                  a->O_H, a->O_W, a->O_cb)];
            }
}

static void tile_put_back(const struct blocked_layer *a, const struct tile_visit *v, const double *regs)
{
    for (int p = 0; p < v->width; ++p)
        for (int dg = 0; dg < a->G_b; ++dg)
            for (int dk = 0; dk < a->K_b; ++dk)
                a->partial[so_act_offset(v->image, tile_channel(a, v, dg, dk), v->row, v->col0 + p, a->O_C, a->O_H,
                                         a->O_W, a->O_cb)] = regs[(p * a->G_b + dg) * a->K_b + dk];
}

/* Offset of a weight in [G/G_b][K/K_b][F_C/F_Cb][F_H][F_W][F_Cb][G_b][K_b]: tap (ty, tx), reduction channel
 * red0 + dc of the window, group group0 + dg, filter filter0 + dk. */
static size_t tile_weight(const struct blocked_layer *a, const struct tile_visit *v, int ty, int tx, int dc, int dg, int dk)
{
    size_t o = (size_t)(v->group0 / a->G_b);
    o = o * (size_t)(a->K / a->K_b) + (size_t)(v->filter0 / a->K_b);
    o = o * (size_t)(a->F_C / a->F_Cb) + (size_t)(v->red0 / a->F_Cb);
    o = (o * a->F_H + ty) * a->F_W + tx;
    return ((o * a->F_Cb + dc) * a->G_b + dg) * a->K_b + dk;
}

static void tile_reduce(const struct blocked_layer *a, const struct tile_visit *v, double *regs)
{
    for (int ty = 0; ty < a->F_H; ++ty)
        for (int tx = 0; tx < a->F_W; ++tx)
            for (int dc = 0; dc < a->F_Cb; ++dc)
                for (int p = 0; p < v->width; ++p) {
                    const int ih = v->row * a->S_H + ty - a->pt, iw = (v->col0 + p) * a->S_W + tx - a->pl;
                    if (ih < 0 || ih >= a->I_H || iw < 0 || iw >= a->I_W) continue;   /* taps in the padding */
                    for (int dg = 0; dg < a->G_b; ++dg) {
                        const int ic = (v->group0 + dg) * a->S_C + v->red0 + dc;      /* the group's window start + channel */
                        const double x = (double)a->I[so_act_offset(v->image, ic, ih, iw, a->I_C, a->I_H, a->I_W, a->Icb)];
                        for (int dk = 0; dk < a->K_b; ++dk) {
                            double *r = &regs[(p * a->G_b + dg) * a->K_b + dk];
                            if (a->op == 0) *r += x * (double)a->Wt[tile_weight(a, v, ty, tx, dc, dg, dk)];
                            else if (a->op == 1) { if (x > *r) *r = x; }
                            else *r += x;
                        }
                    }
                }
}

int so_abstract_layer_blocked(int op, const float *I, const float *Wt, float *O, int N, int I_C, int I_H,
                              int I_W, int F_H, int F_W, int F_C, int S_H, int S_W, int S_C, int K, int pt,
                              int pb, int pl, int pr, int Icb, int G_b, int K_b, int F_Cb, int O_wb)
{
    if (S_C <= 0 || (I_C - F_C) % S_C) return -1;
    struct blocked_layer a;
    a.op = op; a.I = I; a.Wt = Wt;
    a.I_C = I_C; a.I_H = I_H; a.I_W = I_W;
    a.F_H = F_H; a.F_W = F_W; a.F_C = F_C; a.S_H = S_H; a.S_W = S_W; a.S_C = S_C; a.K = K;
    a.G = (I_C - F_C) / S_C + 1;
    a.O_C = K * a.G;
    a.pt = pt; a.pl = pl;
    a.Icb = Icb; a.G_b = G_b; a.K_b = K_b; a.F_Cb = F_Cb; a.O_wb = O_wb; a.O_cb = G_b * K_b;
    if (a.G % G_b || K % K_b || F_C % F_Cb || I_C % Icb || a.O_C % a.O_cb || O_wb <= 0) return -2;
    a.O_H = so_out_dim(I_H, F_H, S_H, pt, pb);
    a.O_W = so_out_dim(I_W, F_W, S_W, pl, pr);
    const size_t out_elems = (size_t)N * a.O_C * a.O_H * a.O_W;
    a.partial = (double *)malloc(sizeof(double) * (out_elems ? out_elems : 1));
    double *regs = (double *)malloc(sizeof(double) * (size_t)O_wb * G_b * K_b);
    if (!a.partial || !regs) { free(a.partial); free(regs); return -3; }

    /* Visits in the order the loop nest prescribes: channel tiles (groups, filters; independent of each other),
     * then the reduction blocks, and inside a reduction block every row and column tile of the output. */
    struct tile_visit v;
    for (v.image = 0; v.image < N; ++v.image)
        for (v.group0 = 0; v.group0 < a.G; v.group0 += G_b)
            for (v.filter0 = 0; v.filter0 < K; v.filter0 += K_b)
                for (v.red0 = 0; v.red0 < F_C; v.red0 += F_Cb)
                    for (v.row = 0; v.row < a.O_H; ++v.row)
                        for (v.col0 = 0; v.col0 < a.O_W; v.col0 += O_wb) {
                            v.width = a.O_W - v.col0 < O_wb ? a.O_W - v.col0 : O_wb;
                            tile_bring_in(&a, &v, regs);
                            tile_reduce(&a, &v, regs);
                            tile_put_back(&a, &v, regs);
                        }

    /* round once; the Add reduction becomes an average over the taps inside the image */
    for (int n = 0; n < N; ++n)
        for (int oc = 0; oc < a.O_C; ++oc)
            for (int oh = 0; oh < a.O_H; ++oh)
                for (int ow = 0; ow < a.O_W; ++ow) {
                    const size_t o = so_act_offset(n, oc, oh, ow, a.O_C, a.O_H, a.O_W, a.O_cb);
                    double r = a.partial[o];
                    if (op == 2) {
                        int inside = 0;
                        for (int ty = 0; ty < F_H; ++ty)
                            for (int tx = 0; tx < F_W; ++tx) {
                                const int ih = oh * S_H + ty - pt, iw = ow * S_W + tx - pl;
                                if (ih >= 0 && ih < I_H && iw >= 0 && iw < I_W) ++inside;
                            }
                        r /= (double)(inside > 0 ? inside * F_C : 1);
                    }
                    O[o] = (float)r;
                }
    free(a.partial);
    free(regs);
    return 0;
}
