/*
 * Driver for the sanitizer build of the CPU oracle (tests/test_oracle_sanitize.py compiles this
 * file together with oracle/jvoracle.c under -fsanitize=address,undefined and runs it).
 *
 * Every routine of the oracle is called on heap buffers of exactly the size it is documented to
 * read and write, on ragged shapes (grids the window does not divide, one token, one channel),
 * so that an out-of-bounds access, a use of uninitialised index arithmetic or a signed overflow
 * stops the program.  The hand-worked values of the paper's definitions (Eq. 1: p = 1/4, 3/4 ->
 * o = 7; Eq. 2 with ReLU: the d = 2, N = 3 case; the 3 x 3 grid with 2 x 2 windows of
 * Sec. 3.2.2) are checked as well, so the run also shows that the sanitized build computes the
 * same numbers.  Test infrastructure only.
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

int jvo_full_attn(const float *, const float *, const float *, double *, int, int, int, int, double);
int jvo_full_attn_rows(const float *, const float *, const float *, double *, int, int, int, int, double,
                       const int64_t *, int);
int jvo_full_attn_probs(const float *, const float *, double *, int, int, double);
int jvo_masked_attn(const float *, const float *, const float *, double *, int, int, int, int, double,
                    const uint8_t *);
int jvo_window_geometry(int, int, int, int, int *, int *, int *);
int jvo_window_maps(int, int, int, int, int32_t *, uint8_t *, int32_t *);
int jvo_window_attn(const float *, const float *, const float *, double *, int, int, int, int, int, int, int,
                    double);
int jvo_window_attn_rows(const float *, const float *, const float *, double *, int, int, int, int, int, int,
                         int, double, const int64_t *, int);
int jvo_linear_attn_quadratic(const float *, const float *, const float *, double *, int, int, int, int, double);
int jvo_linear_attn_rows(const float *, const float *, const float *, double *, int, int, int, int, double,
                         const int64_t *, int);
int jvo_linear_attn_state(const float *, const float *, const float *, double *, double *, double *, int, int,
                          int, int, double);
int jvo_layernorm(const double *, const float *, const float *, double *, int64_t, int, double);
int jvo_linear(const double *, const float *, const float *, double *, int64_t, int, int);
int jvo_gelu(double *, int64_t);
int jvo_dwc(const float *, const double *, double *, int, int, int, int, int, int, int);
int jvo_squeeze_kernel(const float *, const float *, const float *, const float *, const float *, double *,
                       int, int, int, int, int, int);

static int failures = 0;
#define EXPECT(cond) do { if (!(cond)) { printf("FAILED line %d: %s\n", __LINE__, #cond); ++failures; } } while (0)
static int near(double a, double b) { return fabs(a - b) <= 1e-12 * (1.0 + fabs(b)); }

/* heap array of n floats filled from a small linear-congruential sequence in [-1, 1) */
static float *rnd(size_t n, unsigned seed) {
    float *p = (float *)malloc(n * sizeof(float));
    unsigned s = seed * 2654435761u + 12345u;
    for (size_t i = 0; i < n; ++i) {
        s = s * 1664525u + 1013904223u;
        p[i] = (float)((int)(s >> 8) % 2000 - 1000) / 1000.0f;
    }
    return p;
}
static double *out(size_t n) {
    double *p = (double *)malloc(n * sizeof(double));
    for (size_t i = 0; i < n; ++i) p[i] = NAN;
    return p;
}
static int all_finite(const double *p, size_t n) {
    for (size_t i = 0; i < n; ++i)
        if (!isfinite(p[i])) return 0;
    return 1;
}

static void hand_cases(void) {
    /* Eq. 1, d = 1, scale 1: q = 1, k = (0, ln 3), v = (4, 8): p = (1/4, 3/4), o = 7 */
    float q[2] = {1.f, 1.f}, k[2] = {0.f, logf(3.f)}, v[2] = {4.f, 8.f};   /* two equal queries */
    double o[2], p[4];
    EXPECT(jvo_full_attn(q, k, v, o, 1, 1, 2, 1, 1.0) == 0);
    /* the key is float(ln 3): compare with the same rounded value */
    double e = exp((double)k[1]);
    EXPECT(near(o[0], (4.0 + 8.0 * e) / (1.0 + e)));
    EXPECT(fabs(o[0] - 7.0) < 1e-6);
    EXPECT(o[1] == o[0]);
    EXPECT(jvo_full_attn_probs(q, k, p, 2, 1, 1.0) == 0);
    EXPECT(fabs(p[0] - 0.25) < 1e-6 && fabs(p[1] - 0.75) < 1e-6 && near(p[0] + p[1], 1.0));
    EXPECT(p[2] == p[0] && p[3] == p[1]);

    /* Eq. 2 with ReLU, d = 2, N = 3 */
    float lk[6] = {1, -1, 2, 0, -1, 3}, lv[6] = {1, 2, 3, 4, 5, 6}, lq[6] = {1, 2, -1, 1, -1, -2};
    double lo[6], S[4], z[2];
    EXPECT(jvo_linear_attn_state(lq, lk, lv, lo, S, z, 1, 1, 3, 2, 1e-30) == 0);
    EXPECT(S[0] == 7 && S[1] == 10 && S[2] == 15 && S[3] == 18 && z[0] == 3 && z[1] == 3);
    EXPECT(near(lo[0], 37.0 / 9) && near(lo[1], 46.0 / 9) && near(lo[2], 5) && near(lo[3], 6));
    EXPECT(lo[4] == 0 && lo[5] == 0);
    double lo2[6];
    EXPECT(jvo_linear_attn_quadratic(lq, lk, lv, lo2, 1, 1, 3, 2, 1e-30) == 0);
    for (int i = 0; i < 6; ++i) EXPECT(near(lo2[i], lo[i]));

    /* Sec. 3.2.2: 3 x 3 grid, 2 x 2 windows */
    int Hp, Wp, nw;
    EXPECT(jvo_window_geometry(3, 3, 2, 2, &Hp, &Wp, &nw) == 0 && Hp == 4 && Wp == 4 && nw == 4);
    int32_t *ti = (int32_t *)malloc(16 * sizeof(int32_t)), *wt = (int32_t *)malloc(9 * sizeof(int32_t));
    uint8_t *pm = (uint8_t *)malloc(16);
    EXPECT(jvo_window_maps(3, 3, 2, 2, ti, pm, wt) == 0);
    const int32_t ti_want[16] = {0, 1, 3, 4, 2, -1, 5, -1, 6, 7, -1, -1, 8, -1, -1, -1};
    const int32_t wt_want[9] = {0, 0, 1, 0, 0, 1, 2, 2, 3};
    for (int i = 0; i < 16; ++i) EXPECT(ti[i] == ti_want[i] && pm[i] == (ti_want[i] >= 0));
    for (int i = 0; i < 9; ++i) EXPECT(wt[i] == wt_want[i]);
    free(ti); free(wt); free(pm);
    double g[3] = {0.0, 1.0, -1.0};
    EXPECT(jvo_gelu(g, 3) == 0 && g[0] == 0.0 && fabs(g[1] - 0.8413447460685429) < 1e-12);
}

static void ragged_shapes(void) {
    const int shapes[][6] = {/* B, heads, H, W, wh, ww */
        {1, 1, 1, 1, 1, 1}, {2, 3, 5, 7, 4, 2}, {1, 2, 7, 7, 9, 3}, {1, 1, 9, 4, 3, 3}, {2, 1, 3, 11, 2, 16}};
    const int dims[] = {1, 3, 8};
    for (size_t si = 0; si < sizeof(shapes) / sizeof(shapes[0]); ++si)
        for (size_t di = 0; di < 3; ++di) {
            const int B = shapes[si][0], h = shapes[si][1], H = shapes[si][2], W = shapes[si][3];
            const int wh = shapes[si][4], ww = shapes[si][5], d = dims[di], N = H * W;
            const size_t n = (size_t)B * h * N * d;
            float *q = rnd(n, 1 + (unsigned)si), *k = rnd(n, 2 + (unsigned)si), *v = rnd(n, 3 + (unsigned)si);
            double *o = out(n), *o2 = out(n);
            EXPECT(jvo_full_attn(q, k, v, o, B, h, N, d, 0.5) == 0 && all_finite(o, n));
            EXPECT(jvo_window_attn(q, k, v, o2, B, h, H, W, d, wh, ww, 0.5) == 0 && all_finite(o2, n));
            /* window attention = full attention under the window mask built from the maps */
            int Hp, Wp, nw;
            EXPECT(jvo_window_geometry(H, W, wh, ww, &Hp, &Wp, &nw) == 0);
            int32_t *ti = (int32_t *)malloc((size_t)nw * wh * ww * sizeof(int32_t));
            uint8_t *pm = (uint8_t *)malloc((size_t)nw * wh * ww);
            int32_t *wt = (int32_t *)malloc((size_t)N * sizeof(int32_t));
            EXPECT(jvo_window_maps(H, W, wh, ww, ti, pm, wt) == 0);
            uint8_t *allow = (uint8_t *)malloc((size_t)N * N);
            for (int i = 0; i < N; ++i)
                for (int j = 0; j < N; ++j) allow[(size_t)i * N + j] = wt[i] == wt[j];
            double *o3 = out(n);
            EXPECT(jvo_masked_attn(q, k, v, o3, B, h, N, d, 0.5, allow) == 0);
            for (size_t i = 0; i < n; ++i) EXPECT(near(o3[i], o2[i]));
            /* sampled rows: first and last */
            int64_t rows[6] = {0, 0, 0, B - 1, h - 1, N - 1};
            double *orow = out(2 * (size_t)d);
            EXPECT(jvo_full_attn_rows(q, k, v, orow, B, h, N, d, 0.5, rows, 2) == 0);
            for (int c = 0; c < d; ++c) EXPECT(near(orow[c], o[c]) && near(orow[d + c], o[n - d + c]));
            EXPECT(jvo_window_attn_rows(q, k, v, orow, B, h, H, W, d, wh, ww, 0.5, rows, 2) == 0);
            for (int c = 0; c < d; ++c) EXPECT(near(orow[c], o2[c]) && near(orow[d + c], o2[n - d + c]));
            /* linear attention: state form = quadratic form */
            double *S = out((size_t)B * h * d * d), *z = out((size_t)B * h * d);
            EXPECT(jvo_linear_attn_state(q, k, v, o, S, z, B, h, N, d, 1e-6) == 0 && all_finite(o, n));
            EXPECT(jvo_linear_attn_quadratic(q, k, v, o2, B, h, N, d, 1e-6) == 0);
            for (size_t i = 0; i < n; ++i) EXPECT(fabs(o[i] - o2[i]) <= 1e-9 * (1.0 + fabs(o2[i])));
            EXPECT(jvo_linear_attn_rows(q, k, v, orow, B, h, N, d, 1e-6, rows, 2) == 0);
            for (int c = 0; c < d; ++c) EXPECT(near(orow[c], o2[c]) && near(orow[d + c], o2[n - d + c]));
            /* convolution branch: static bank and generated bank, 3 x 3 and 5 x 5 */
            for (int ks = 3; ks <= 5; ks += 2) {
                const int C = h * d, hidden = 3;
                float *w1 = rnd((size_t)hidden * C, 7), *b1 = rnd(hidden, 8);
                float *w2 = rnd((size_t)C * ks * ks * hidden, 9), *b2 = rnd((size_t)C * ks * ks, 10);
                double *kap = out((size_t)B * C * ks * ks);
                EXPECT(jvo_squeeze_kernel(v, w1, b1, w2, b2, kap, B, h, N, d, ks, hidden) == 0);
                EXPECT(all_finite(kap, (size_t)B * C * ks * ks));
                EXPECT(jvo_dwc(v, kap, o, B, h, H, W, d, ks, B) == 0 && all_finite(o, n));
                EXPECT(jvo_dwc(v, kap, o2, B, h, H, W, d, ks, 1) == 0 && all_finite(o2, n));
                free(w1); free(b1); free(w2); free(b2); free(kap);
            }
            /* encoder pieces on [T, C] with T = B * N, C = h * d */
            {
                const int64_t T = (int64_t)B * N;
                const int C = h * d, Nout = 5;
                double *x = out((size_t)T * C), *y = out((size_t)T * C), *yl = out((size_t)T * Nout);
                for (size_t i = 0; i < (size_t)T * C; ++i) x[i] = q[i];
                float *gam = rnd(C, 11), *bet = rnd(C, 12), *w = rnd((size_t)Nout * C, 13), *bb = rnd(Nout, 14);
                EXPECT(jvo_layernorm(x, gam, bet, y, T, C, 1e-6) == 0 && all_finite(y, (size_t)T * C));
                EXPECT(jvo_linear(x, w, bb, yl, T, Nout, C) == 0 && all_finite(yl, (size_t)T * Nout));
                EXPECT(jvo_linear(x, w, NULL, yl, T, Nout, C) == 0);
                EXPECT(jvo_gelu(yl, T * Nout) == 0 && all_finite(yl, (size_t)T * Nout));
                free(x); free(y); free(yl); free(gam); free(bet); free(w); free(bb);
            }
            free(q); free(k); free(v); free(o); free(o2); free(o3); free(ti); free(pm); free(wt);
            free(allow); free(orow); free(S); free(z);
        }
}

static void invalid_arguments(void) {
    float x[4] = {0};
    double o[4];
    EXPECT(jvo_full_attn(NULL, x, x, o, 1, 1, 1, 1, 1.0) == 1);
    EXPECT(jvo_full_attn(x, x, x, o, 1, 1, 0, 1, 1.0) == 1);
    EXPECT(jvo_window_attn(x, x, x, o, 1, 1, 2, 2, 1, 0, 1, 1.0) == 1);
    int a, b, c;
    EXPECT(jvo_window_geometry(0, 3, 1, 1, &a, &b, &c) == 1);
    uint8_t none[1] = {0};
    EXPECT(jvo_masked_attn(x, x, x, o, 1, 1, 1, 1, 1.0, none) == 1);   /* a row with no allowed key */
}

int main(void) {
    hand_cases();
    ragged_shapes();
    invalid_arguments();
    if (failures) {
        printf("%d check(s) failed\n", failures);
        return 1;
    }
    printf("oracle sanitize run: ok\n");
    return 0;
}
