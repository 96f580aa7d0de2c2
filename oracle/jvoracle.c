/*
 * jvoracle.c -- CPU oracle for the JetViT token mixers.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain statement of what
 * the GPU library must compute.  It shares no code with the HIP path, is never
 * linked into it, and may be called only from tests, the smoke check and the
 * benchmark's CPU-baseline leg.
 *
 * Every routine writes the definition out as loops, accumulates in fp64, and
 * does no tiling, no online softmax and no reordering.  OpenMP only spreads
 * independent (batch, head) problems or independent rows over host cores; it
 * never splits a sum.
 *
 * Tensors: Q, K, V are contiguous [B, heads, N, d] float32 (bf16 test inputs
 * are widened exactly to float32 by the caller); outputs are float64 of the
 * same shape unless stated.  Tokens are the row-major raster of the H x W
 * grid: token n = r*W + c.
 *
 * Pins (tests/test_oracle_*.py): hand-worked cases under tests/golden/,
 * brute-force equivalences (state form vs quadratic form, window vs masked
 * full attention, whole-grid window vs full attention), closed forms (Q = 0
 * gives the mean of V, V = 1 gives 1, softmax rows sum to 1, key-shift and
 * positive-scale invariances), exhaustive index-map enumeration.
 *
 * Parity unpinned against the paper itself (the mathematics of every routine is pinned as
 * above): jvo_squeeze_kernel -- the paper describes the generator of the dynamic filters only
 * as a compact two-layer MLP with SiLU fed by the token average of V; where the activation
 * sits, the biases and the hidden width are this file's reading -- and the encoder routines in
 * the Python front end (pre-LN block, exact GELU, no final norm), which the paper leaves to the
 * pretrained model it inherits from.
 *
 * Return value: 0 on success, 1 on an invalid argument.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#define IDX4(b, h, n, H, N, d) ((((size_t)(b) * (H) + (h)) * (size_t)(N) + (n)) * (size_t)(d))

/* ------------------------------------------------------------------------
 * Full softmax attention, Eq. 1 of the paper: similarity exp(q.k/sqrt(d)),
 * normalised over the keys of the row, applied to V.
 * One query row:  s_j = scale * sum_c q_c k_jc ;  m = max_j s_j ;
 * p_j = exp(s_j - m) ;  o = sum_j p_j v_j / sum_j p_j.
 * `keys` lists the token indices the row may attend to (n_keys > 0).
 * ---------------------------------------------------------------------- */
static void softmax_row(const float *q_row, const float *k_bh, const float *v_bh,
                        const int *keys, int n_keys, int d, double scale,
                        double *logit /* scratch [n_keys] */, double *o_row)
{
    double m = -INFINITY;
    for (int t = 0; t < n_keys; ++t) {
        const float *k_row = k_bh + (size_t)keys[t] * d;
        double s = 0.0;
        for (int c = 0; c < d; ++c) s += (double)q_row[c] * (double)k_row[c];
        s *= scale;
        logit[t] = s;
        if (s > m) m = s;
    }
    double denom = 0.0;
    for (int c = 0; c < d; ++c) o_row[c] = 0.0;
    for (int t = 0; t < n_keys; ++t) {
        double p = exp(logit[t] - m);
        const float *v_row = v_bh + (size_t)keys[t] * d;
        denom += p;
        for (int c = 0; c < d; ++c) o_row[c] += p * (double)v_row[c];
    }
    for (int c = 0; c < d; ++c) o_row[c] /= denom;
}

int jvo_full_attn(const float *q, const float *k, const float *v, double *o,
                  int B, int heads, int N, int d, double scale)
{
    if (!q || !k || !v || !o || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
    int *all = (int *)malloc(sizeof(int) * (size_t)N);
    for (int j = 0; j < N; ++j) all[j] = j;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for collapse(2) schedule(dynamic, 16)
        for (int bh = 0; bh < B * heads; ++bh)
            for (int i = 0; i < N; ++i) {
                size_t base = (size_t)bh * N * d;
                softmax_row(q + base + (size_t)i * d, k + base, v + base, all, N, d, scale,
                            logit, o + base + (size_t)i * d);
            }
        free(logit);
    }
    free(all);
    return 0;
}

/* Selected rows of full attention: rows[3*r + {0,1,2}] = (b, head, i);
 * o_rows is [n_rows, d].  Same arithmetic as jvo_full_attn, row by row. */
int jvo_full_attn_rows(const float *q, const float *k, const float *v, double *o_rows,
                       int B, int heads, int N, int d, double scale,
                       const int64_t *rows, int n_rows)
{
    if (!q || !k || !v || !o_rows || !rows || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
    for (int r = 0; r < n_rows; ++r)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 ||
            rows[3 * r + 1] >= heads || rows[3 * r + 2] < 0 || rows[3 * r + 2] >= N)
            return 1;
    int *all = (int *)malloc(sizeof(int) * (size_t)N);
    for (int j = 0; j < N; ++j) all[j] = j;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)N);
#pragma omp for schedule(dynamic, 1)
        for (int r = 0; r < n_rows; ++r) {
            size_t base = IDX4(rows[3 * r], rows[3 * r + 1], 0, heads, N, d);
            softmax_row(q + base + (size_t)rows[3 * r + 2] * d, k + base, v + base, all, N, d,
                        scale, logit, o_rows + (size_t)r * d);
        }
        free(logit);
    }
    free(all);
    return 0;
}

/* Normalised attention probabilities of one head, p[i, j], [N, N] float64.
 * Exists so that a test can check that every row sums to one. */
int jvo_full_attn_probs(const float *q, const float *k, double *p, int N, int d, double scale)
{
    if (!q || !k || !p || N <= 0 || d <= 0) return 1;
    for (int i = 0; i < N; ++i) {
        double m = -INFINITY;
        for (int j = 0; j < N; ++j) {
            double s = 0.0;
            for (int c = 0; c < d; ++c) s += (double)q[(size_t)i * d + c] * (double)k[(size_t)j * d + c];
            s *= scale;
            p[(size_t)i * N + j] = s;
            if (s > m) m = s;
        }
        double denom = 0.0;
        for (int j = 0; j < N; ++j) {
            p[(size_t)i * N + j] = exp(p[(size_t)i * N + j] - m);
            denom += p[(size_t)i * N + j];
        }
        for (int j = 0; j < N; ++j) p[(size_t)i * N + j] /= denom;
    }
    return 0;
}

/* Full attention under an explicit 0/1 mask allow[i, j] ([N, N] uint8, shared
 * by all batches and heads): keys with allow = 0 are left out of the row.
 * A row with no allowed key is an error.  Used to pin window attention. */
int jvo_masked_attn(const float *q, const float *k, const float *v, double *o,
                    int B, int heads, int N, int d, double scale, const uint8_t *allow)
{
    if (!q || !k || !v || !o || !allow || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
    int bad = 0;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)N);
        int *keys = (int *)malloc(sizeof(int) * (size_t)N);
#pragma omp for collapse(2) schedule(dynamic, 16)
        for (int bh = 0; bh < B * heads; ++bh)
            for (int i = 0; i < N; ++i) {
                size_t base = (size_t)bh * N * d;
                int n_keys = 0;
                for (int j = 0; j < N; ++j)
                    if (allow[(size_t)i * N + j]) keys[n_keys++] = j;
                if (n_keys == 0) {
#pragma omp atomic write
                    bad = 1;
                    continue;
                }
                softmax_row(q + base + (size_t)i * d, k + base, v + base, keys, n_keys, d, scale,
                            logit, o + base + (size_t)i * d);
            }
        free(logit);
        free(keys);
    }
    return bad;
}

/* ------------------------------------------------------------------------
 * Window partition (Sec. 3.2.2: the feature map is cut into non-overlapping
 * windows).  The grid is extended at the bottom and the right to the next
 * multiple of the window; windows are anchored at (0, 0) and numbered
 * row-major; slots inside a window are numbered row-major.
 * ---------------------------------------------------------------------- */
int jvo_window_geometry(int H, int W, int wh, int ww, int *Hp, int *Wp, int *n_win)
{
    if (H <= 0 || W <= 0 || wh <= 0 || ww <= 0 || !Hp || !Wp || !n_win) return 1;
    *Hp = ((H + wh - 1) / wh) * wh;
    *Wp = ((W + ww - 1) / ww) * ww;
    *n_win = (*Hp / wh) * (*Wp / ww);
    return 0;
}

/* token_index [n_win * wh*ww] int32: real token r*W + c, or -1 for a pad cell;
 * pad_mask    [n_win * wh*ww] uint8: 1 real, 0 pad;
 * window_of_token [H*W] int32.   Any output may be NULL. */
int jvo_window_maps(int H, int W, int wh, int ww, int32_t *token_index, uint8_t *pad_mask,
                    int32_t *window_of_token)
{
    int Hp, Wp, n_win;
    if (jvo_window_geometry(H, W, wh, ww, &Hp, &Wp, &n_win)) return 1;
    int wins_per_row = Wp / ww;
    for (int r = 0; r < Hp; ++r)
        for (int c = 0; c < Wp; ++c) {
            int win = (r / wh) * wins_per_row + (c / ww);
            int slot = (r % wh) * ww + (c % ww);
            int real = (r < H && c < W);
            size_t at = (size_t)win * wh * ww + slot;
            if (token_index) token_index[at] = real ? r * W + c : -1;
            if (pad_mask) pad_mask[at] = real ? 1 : 0;
            if (real && window_of_token) window_of_token[r * W + c] = win;
        }
    return 0;
}

/* Collect the real tokens of the window that contains grid cell (r, c). */
static int window_keys(int r, int c, int H, int W, int wh, int ww, int *keys)
{
    int r0 = (r / wh) * wh, c0 = (c / ww) * ww, n = 0;
    for (int rr = r0; rr < r0 + wh; ++rr)
        for (int cc = c0; cc < c0 + ww; ++cc)
            if (rr < H && cc < W) keys[n++] = rr * W + cc;
    return n;
}

/* Window attention: each real token attends, with the full-attention formula
 * and the same scale, to the real tokens of its own window only.  Pad cells
 * are never read and produce no output.  O is [B, heads, H*W, d]. */
int jvo_window_attn(const float *q, const float *k, const float *v, double *o,
                    int B, int heads, int H, int W, int d, int wh, int ww, double scale)
{
    if (!q || !k || !v || !o || B <= 0 || heads <= 0 || H <= 0 || W <= 0 || d <= 0 ||
        wh <= 0 || ww <= 0)
        return 1;
    int N = H * W;
#pragma omp parallel
    {
        double *logit = (double *)malloc(sizeof(double) * (size_t)wh * ww);
        int *keys = (int *)malloc(sizeof(int) * (size_t)wh * ww);
#pragma omp for collapse(2) schedule(dynamic, 16)
        for (int bh = 0; bh < B * heads; ++bh)
            for (int i = 0; i < N; ++i) {
                size_t base = (size_t)bh * N * d;
                int n_keys = window_keys(i / W, i % W, H, W, wh, ww, keys);
                softmax_row(q + base + (size_t)i * d, k + base, v + base, keys, n_keys, d, scale,
                            logit, o + base + (size_t)i * d);
            }
        free(logit);
        free(keys);
    }
    return 0;
}

int jvo_window_attn_rows(const float *q, const float *k, const float *v, double *o_rows,
                         int B, int heads, int H, int W, int d, int wh, int ww, double scale,
                         const int64_t *rows, int n_rows)
{
    if (!q || !k || !v || !o_rows || !rows || B <= 0 || heads <= 0 || H <= 0 || W <= 0 ||
        d <= 0 || wh <= 0 || ww <= 0)
        return 1;
    int N = H * W;
    for (int r = 0; r < n_rows; ++r)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 ||
            rows[3 * r + 1] >= heads || rows[3 * r + 2] < 0 || rows[3 * r + 2] >= N)
            return 1;
    double *logit = (double *)malloc(sizeof(double) * (size_t)wh * ww);
    int *keys = (int *)malloc(sizeof(int) * (size_t)wh * ww);
    for (int r = 0; r < n_rows; ++r) {
        size_t base = IDX4(rows[3 * r], rows[3 * r + 1], 0, heads, N, d);
        int i = (int)rows[3 * r + 2];
        int n_keys = window_keys(i / W, i % W, H, W, wh, ww, keys);
        softmax_row(q + base + (size_t)i * d, k + base, v + base, keys, n_keys, d, scale, logit,
                    o_rows + (size_t)r * d);
    }
    free(logit);
    free(keys);
    return 0;
}

/* ------------------------------------------------------------------------
 * Linear attention with the ReLU feature map (Eq. 2; the block keeps ReLU),
 * normalised by the key sum.
 * Quadratic (reference) form, one query row:
 *   a_j = sum_c relu(q_c) relu(k_jc) ;  o = sum_j a_j v_j / (sum_j a_j + eps)
 * ---------------------------------------------------------------------- */
static inline double relu(double x) { return x > 0.0 ? x : 0.0; }

static void linear_row_quadratic(const float *q_row, const float *k_bh, const float *v_bh,
                                 int N, int d, double eps, double *o_row)
{
    double denom = 0.0;
    for (int c = 0; c < d; ++c) o_row[c] = 0.0;
    for (int j = 0; j < N; ++j) {
        double a = 0.0;
        for (int c = 0; c < d; ++c) a += relu(q_row[c]) * relu(k_bh[(size_t)j * d + c]);
        denom += a;
        for (int c = 0; c < d; ++c) o_row[c] += a * (double)v_bh[(size_t)j * d + c];
    }
    for (int c = 0; c < d; ++c) o_row[c] /= (denom + eps);
}

int jvo_linear_attn_quadratic(const float *q, const float *k, const float *v, double *o,
                              int B, int heads, int N, int d, double eps)
{
    if (!q || !k || !v || !o || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
#pragma omp parallel for collapse(2) schedule(dynamic, 16)
    for (int bh = 0; bh < B * heads; ++bh)
        for (int i = 0; i < N; ++i) {
            size_t base = (size_t)bh * N * d;
            linear_row_quadratic(q + base + (size_t)i * d, k + base, v + base, N, d, eps,
                                 o + base + (size_t)i * d);
        }
    return 0;
}

int jvo_linear_attn_rows(const float *q, const float *k, const float *v, double *o_rows,
                         int B, int heads, int N, int d, double eps,
                         const int64_t *rows, int n_rows)
{
    if (!q || !k || !v || !o_rows || !rows || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
    for (int r = 0; r < n_rows; ++r)
        if (rows[3 * r] < 0 || rows[3 * r] >= B || rows[3 * r + 1] < 0 ||
            rows[3 * r + 1] >= heads || rows[3 * r + 2] < 0 || rows[3 * r + 2] >= N)
            return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < n_rows; ++r) {
        size_t base = IDX4(rows[3 * r], rows[3 * r + 1], 0, heads, N, d);
        linear_row_quadratic(q + base + (size_t)rows[3 * r + 2] * d, k + base, v + base, N, d,
                             eps, o_rows + (size_t)r * d);
    }
    return 0;
}

/* State (reordered, O(N)) form:  S = sum_j relu(k_j)^T v_j  [d, d],
 * z = sum_j relu(k_j) [d],  o_i = relu(q_i) S / (relu(q_i).z + eps).
 * S is [B, heads, d, d] (row = key channel, column = value channel) and z is
 * [B, heads, d]; either may be NULL. */
int jvo_linear_attn_state(const float *q, const float *k, const float *v, double *o,
                          double *S_out, double *z_out, int B, int heads, int N, int d, double eps)
{
    if (!q || !k || !v || !o || B <= 0 || heads <= 0 || N <= 0 || d <= 0) return 1;
#pragma omp parallel for schedule(dynamic, 1)
    for (int bh = 0; bh < B * heads; ++bh) {
        size_t base = (size_t)bh * N * d;
        double *S = (double *)calloc((size_t)d * d, sizeof(double));
        double *z = (double *)calloc((size_t)d, sizeof(double));
        for (int j = 0; j < N; ++j)
            for (int a = 0; a < d; ++a) {
                double kf = relu(k[base + (size_t)j * d + a]);
                z[a] += kf;
                for (int c = 0; c < d; ++c) S[(size_t)a * d + c] += kf * (double)v[base + (size_t)j * d + c];
            }
        for (int i = 0; i < N; ++i) {
            double denom = 0.0;
            for (int a = 0; a < d; ++a) denom += relu(q[base + (size_t)i * d + a]) * z[a];
            for (int c = 0; c < d; ++c) {
                double num = 0.0;
                for (int a = 0; a < d; ++a) num += relu(q[base + (size_t)i * d + a]) * S[(size_t)a * d + c];
                o[base + (size_t)i * d + c] = num / (denom + eps);
            }
        }
        if (S_out) memcpy(S_out + (size_t)bh * d * d, S, sizeof(double) * (size_t)d * d);
        if (z_out) memcpy(z_out + (size_t)bh * d, z, sizeof(double) * (size_t)d);
        free(S);
        free(z);
    }
    return 0;
}

/* ========================================================================
 * Encoder pieces (pre-LN transformer block around a token mixer) and the
 * depth-wise-convolution branch of the linear-attention block.
 * ====================================================================== */

/* LayerNorm over the last axis: y = (x - mean) / sqrt(var + eps) * gamma + beta,
 * var = population variance.  x is [rows, cols] float64, gamma/beta float32. */
int jvo_layernorm(const double *x, const float *gamma, const float *beta, double *y,
                  int64_t rows, int cols, double eps)
{
    if (!x || !gamma || !beta || !y || rows <= 0 || cols <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t r = 0; r < rows; ++r) {
        const double *xr = x + r * cols;
        double mean = 0.0;
        for (int c = 0; c < cols; ++c) mean += xr[c];
        mean /= cols;
        double var = 0.0;
        for (int c = 0; c < cols; ++c) var += (xr[c] - mean) * (xr[c] - mean);
        var /= cols;
        double inv = 1.0 / sqrt(var + eps);
        for (int c = 0; c < cols; ++c)
            y[r * cols + c] = (xr[c] - mean) * inv * (double)gamma[c] + (double)beta[c];
    }
    return 0;
}

/* Linear layer y = a W^T + b: a [T, K] float64, W [N, K] float32, b [N] float32 or NULL. */
int jvo_linear(const double *a, const float *w, const float *b, double *y,
               int64_t T, int N, int K)
{
    if (!a || !w || !y || T <= 0 || N <= 0 || K <= 0) return 1;
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < T; ++t)
        for (int n = 0; n < N; ++n) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) s += a[t * K + k] * (double)w[(size_t)n * K + k];
            y[t * N + n] = s + (b ? (double)b[n] : 0.0);
        }
    return 0;
}

/* GELU(x) = x * 0.5 * (1 + erf(x / sqrt 2)), in place. */
int jvo_gelu(double *x, int64_t n)
{
    if (!x || n < 0) return 1;
    for (int64_t i = 0; i < n; ++i) x[i] = x[i] * 0.5 * (1.0 + erf(x[i] / sqrt(2.0)));
    return 0;
}

/* Depth-wise k x k cross-correlation of V on the H x W token grid (Eq. 4 of the paper: the
 * DWC(V) term), stride 1, zero padding k/2, no bias.  V is [B, heads, N, d] float32 and is
 * read as C = heads*d channel images, channel = head*d + c.  kernel is [kb, C, k, k]
 * float64 with kb = 1 (one static kernel) or kb = B (one kernel per image).
 * out[b, head, r*W + col, c] = sum_{i,j} kernel[.., ch, i, j] * V[b, head, (r+i-k/2)*W + (col+j-k/2), c]. */
int jvo_dwc(const float *v, const double *kernel, double *out, int B, int heads, int H, int W,
            int d, int k, int kb)
{
    if (!v || !kernel || !out || B <= 0 || heads <= 0 || H <= 0 || W <= 0 || d <= 0 || k <= 0 ||
        (k & 1) == 0 || (kb != 1 && kb != B))
        return 1;
    const int N = H * W, C = heads * d, pad = k / 2;
#pragma omp parallel for collapse(2) schedule(static)
    for (int b = 0; b < B; ++b)
        for (int hd = 0; hd < heads; ++hd)
            for (int r = 0; r < H; ++r)
                for (int col = 0; col < W; ++col)
                    for (int c = 0; c < d; ++c) {
                        const int ch = hd * d + c;
                        const double *kk = kernel + ((size_t)(kb == 1 ? 0 : b) * C + ch) * k * k;
                        double s = 0.0;
                        for (int i = 0; i < k; ++i)
                            for (int j = 0; j < k; ++j) {
                                int rr = r + i - pad, cc = col + j - pad;
                                if (rr < 0 || rr >= H || cc < 0 || cc >= W) continue;
                                s += kk[i * k + j] * (double)v[IDX4(b, hd, rr * W + cc, heads, N, d) + c];
                            }
                        out[IDX4(b, hd, r * W + col, heads, N, d) + c] = s;
                    }
    return 0;
}

/* Squeeze Dynamic Convolution kernel generator (Sec. 3.2.1): the depth-wise weights are
 * produced per image from the average of V over all tokens by a two-layer MLP with SiLU:
 *   g = mean_n V[b, :, n]  (C values);  u = SiLU(W1 g + b1)  (hidden values);
 *   kappa[b] = reshape(W2 u + b2, [C, k, k]);   SiLU(x) = x / (1 + exp(-x)).
 * W1 [hidden, C], b1 [hidden], W2 [C*k*k, hidden], b2 [C*k*k], all float32;
 * kappa is [B, C, k, k] float64. */
int jvo_squeeze_kernel(const float *v, const float *w1, const float *b1, const float *w2,
                       const float *b2, double *kappa, int B, int heads, int N, int d, int k,
                       int hidden)
{
    if (!v || !w1 || !b1 || !w2 || !b2 || !kappa || B <= 0 || heads <= 0 || N <= 0 || d <= 0 ||
        k <= 0 || hidden <= 0)
        return 1;
    const int C = heads * d, KK = C * k * k;
    for (int b = 0; b < B; ++b) {
        double *g = (double *)calloc((size_t)C, sizeof(double));
        double *u = (double *)calloc((size_t)hidden, sizeof(double));
        for (int hd = 0; hd < heads; ++hd)
            for (int n = 0; n < N; ++n)
                for (int c = 0; c < d; ++c) g[hd * d + c] += (double)v[IDX4(b, hd, n, heads, N, d) + c];
        for (int ch = 0; ch < C; ++ch) g[ch] /= N;
        for (int j = 0; j < hidden; ++j) {
            double s = (double)b1[j];
            for (int ch = 0; ch < C; ++ch) s += (double)w1[(size_t)j * C + ch] * g[ch];
            u[j] = s / (1.0 + exp(-s));
        }
        for (int o = 0; o < KK; ++o) {
            double s = (double)b2[o];
            for (int j = 0; j < hidden; ++j) s += (double)w2[(size_t)o * hidden + j] * u[j];
            kappa[(size_t)b * KK + o] = s;
        }
        free(g);
        free(u);
    }
    return 0;
}
