// The depth-wise convolution branch of the paper's linear-attention block (Sec. 3.2.1, Eq. 4:
// O = LA(Q, K, V) + DWC(V)) -- the parts that are not fused into the bf16 apply pass:
//   squeeze_hidden / squeeze_kappa   the generator of the dynamic filters ("Squeeze Dynamic
//                                    Convolution": token mean of V -> Linear -> SiLU -> Linear)
//   v_sum_f32, dwc_add_f32           plain fp32 kernels for fp32 tensors
//   cast_to_bf16, reorder_w2,        the token-wise dynamic variant the paper rejects for its cost
//   pack_v_rows, dwc_token_add       (Tab. 1): the generator as two matrix products over all
//                                    tokens, then every token's own filters on its neighbourhood
//   token_hidden_f32, token_dwc_f32  the same variant for fp32 tensors, plain fp32 arithmetic
#include "jv_linear.h"
#include "jv_mfma.h"

namespace jv {

static size_t align64f(size_t floats) { return (floats + 63) & ~(size_t)63; }  // 256 bytes

jv_status plan_dwc(const jv_dwc_params *dwc, const LinearPlan &lp, int B, int heads, int N, DwcPlan *out) {
    DwcPlan p;
    const size_t base = align64f(linear_workspace_floats(lp, B, heads));
    p.total_floats = base;
    if (!dwc || dwc->mode == JV_DWC_NONE) {
        *out = p;
        return JV_OK;
    }
    if (dwc->mode != JV_DWC_STATIC && dwc->mode != JV_DWC_SQUEEZE_DYNAMIC && dwc->mode != JV_DWC_TOKEN_DYNAMIC)
        return fail(JV_ERR_INVALID_ARG, "unknown convolution mode");
    if (dwc->ksize != 3 && dwc->ksize != 5) return fail(JV_ERR_UNSUPPORTED, "ksize must be 3 or 5");
    const long long C = (long long)heads * kHeadDim;
    if (C > 8192) return fail(JV_ERR_UNSUPPORTED, "convolution branch: more than 8192 channels");
    p.mode = dwc->mode;
    p.ksize = dwc->ksize;
    if (dwc->mode == JV_DWC_STATIC) {
        if (!dwc->static_kernel || ((uintptr_t)dwc->static_kernel & 15))
            return fail(JV_ERR_INVALID_ARG, "static_kernel is null or not 16-byte aligned");
        p.static_kernel = dwc->static_kernel;
    } else {
        if (dwc->hidden <= 0) return fail(JV_ERR_INVALID_ARG, "hidden must be positive");
        if (dwc->hidden > 1024 || dwc->hidden % 4)
            return fail(JV_ERR_UNSUPPORTED, "hidden must be a multiple of 4, at most 1024");
        const void *ptrs[] = {dwc->w1, dwc->b1, dwc->w2, dwc->b2};
        for (const void *q : ptrs)
            if (!q || ((uintptr_t)q & 15))
                return fail(JV_ERR_INVALID_ARG, "generator weight is null or not 16-byte aligned");
        p.hidden = dwc->hidden;
        p.w1 = dwc->w1; p.b1 = dwc->b1; p.w2 = dwc->w2; p.b2 = dwc->b2;
        if (dwc->mode == JV_DWC_TOKEN_DYNAMIC) {
            if (dwc->hidden % 64) return fail(JV_ERR_UNSUPPORTED, "token-wise filters: hidden must be a multiple of 64");
            if (N <= 0) return fail(JV_ERR_INVALID_ARG, "token-wise filters: token count must be positive");
            const size_t M = (size_t)B * N, kk = (size_t)dwc->ksize * dwc->ksize;
            p.w1b_off = base;  // two bf16 per float of offset
            p.w2b_off = p.w1b_off + align64f((size_t)dwc->hidden * C / 2);
            p.b2p_off = p.w2b_off + align64f((size_t)C * kk * dwc->hidden / 2);
            p.vt_off = p.b2p_off + align64f((size_t)C * kk);
            p.u_off = p.vt_off + align64f(M * C / 2);
            p.tok_kappa_off = p.u_off + align64f(M * dwc->hidden / 2);
            p.la_off = p.tok_kappa_off + align64f(M * C * kk);  // the filters stay fp32
            p.total_floats = p.la_off + align64f(M * C);
            *out = p;
            return JV_OK;
        }
        p.vsum_off = base;
        p.hidden_off = p.vsum_off + align64f((size_t)lp.n_split * B * heads * kHeadDim);
        p.kappa_off = p.hidden_off + align64f((size_t)B * dwc->hidden);
        p.total_floats = p.kappa_off + align64f((size_t)B * C * dwc->ksize * dwc->ksize);
    }
    *out = p;
    return JV_OK;
}

// ---------------------------------------------------------------------------------------
// Generator, first layer: u[b][j] = silu(b1[j] + sum_c w1[j][c] g[c]),  g = (token sum of V) / N.
// grid (B, ceil(hidden / 4)), 256 threads, C floats of dynamic LDS; one wavefront per unit j.
// vsum holds n_part partial sums per (batch, head): [n_part][B*heads][64].
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
squeeze_hidden(const float *__restrict__ vsum, int n_part, const float *__restrict__ w1,
               const float *__restrict__ b1, float *__restrict__ u, int heads, int hidden,
               float inv_n) {
    extern __shared__ __align__(16) float gmean[];
    const int b = blockIdx.x, BH = gridDim.x * heads, C = heads * kHeadDim;
    for (int c = threadIdx.x; c < C; c += 256) {
        const float *src = vsum + (size_t)b * heads * kHeadDim + c;
        const size_t stride = (size_t)BH * kHeadDim;
        float s = 0.f;
        for (int p0 = 0; p0 < n_part; p0 += 8) {  // eight partials in flight at a time
            float part[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) part[i] = p0 + i < n_part ? src[(size_t)(p0 + i) * stride] : 0.f;
#pragma unroll
            for (int i = 0; i < 8; ++i) s += part[i];
        }
        gmean[c] = s * inv_n;
    }
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int j = blockIdx.y * 4 + wave;
    if (j >= hidden) return;
    const float *row = w1 + (size_t)j * C;
    float acc = 0.f;
    if ((C & 255) == 0) {  // 16-byte loads, lane-strided
        for (int c = 4 * lane; c < C; c += 256) {
            const f32x4 wv = *(const f32x4 *)(row + c), gv = *(const f32x4 *)(gmean + c);
            acc = fmaf(wv[0], gv[0], acc);
            acc = fmaf(wv[1], gv[1], acc);
            acc = fmaf(wv[2], gv[2], acc);
            acc = fmaf(wv[3], gv[3], acc);
        }
    } else {
        for (int c = lane; c < C; c += 64) acc = fmaf(row[c], gmean[c], acc);
    }
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) acc += __shfl_xor(acc, off, 64);
    if (lane == 0) {
        const float x = acc + b1[j];
        u[(size_t)b * hidden + j] = x / (1.0f + __expf(-x));
    }
}

// Second layer: kappa[b][row] = b2[row] + sum_j w2[row][j] u[b][j], row = channel * k*k + tap.
// grid (B, ceil(rows / 256)), 256 threads, hidden floats of dynamic LDS; one thread per row.
__global__ void __launch_bounds__(256)
squeeze_kappa(const float *__restrict__ u, const float *__restrict__ w2,
              const float *__restrict__ b2, float *__restrict__ kappa, int hidden, int rows) {
    extern __shared__ __align__(16) float us[];
    const int b = blockIdx.x;
    for (int j = threadIdx.x; j < hidden; j += 256) us[j] = u[(size_t)b * hidden + j];
    __syncthreads();
    const int row = blockIdx.y * 256 + threadIdx.x;
    if (row >= rows) return;
    const f32x4 *wrow = (const f32x4 *)(w2 + (size_t)row * hidden);
    float acc = 0.f;
    for (int j4 = 0; j4 < hidden / 4; ++j4) {
        const f32x4 w = wrow[j4];
        const f32x4 x = *(const f32x4 *)(us + 4 * j4);
        acc = fmaf(w[0], x[0], acc);
        acc = fmaf(w[1], x[1], acc);
        acc = fmaf(w[2], x[2], acc);
        acc = fmaf(w[3], x[3], acc);
    }
    kappa[(size_t)b * rows + row] = acc + b2[row];
}

jv_status squeeze_generate(const DwcPlan &dwc, float *ws, int n_part, int B, int heads, int N,
                           hipStream_t stream) {
    const int C = heads * kHeadDim, rows = C * dwc.ksize * dwc.ksize;
    jv_status st;
    hipLaunchKernelGGL(squeeze_hidden, dim3(B, (dwc.hidden + 3) / 4), dim3(256), C * sizeof(float),
                       stream, ws + dwc.vsum_off, n_part, dwc.w1, dwc.b1, ws + dwc.hidden_off, heads,
                       dwc.hidden, 1.0f / (float)N);
    if ((st = launch_status("squeeze_hidden")) != JV_OK) return st;
    hipLaunchKernelGGL(squeeze_kappa, dim3(B, (rows + 255) / 256), dim3(256),
                       dwc.hidden * sizeof(float), stream, ws + dwc.hidden_off, dwc.w2, dwc.b2,
                       ws + dwc.kappa_off, dwc.hidden, rows);
    return launch_status("squeeze_kappa");
}

// ---------------------------------------------------------------------------------------
// fp32 tensors: token sum of V and the convolution as plain kernels.
// ---------------------------------------------------------------------------------------

// grid (n_split, B*heads), 256 threads: vsum[part][bh][c] = sum over the chunk's tokens.
__global__ void __launch_bounds__(256)
v_sum_f32(TensorArg vt, float *__restrict__ vsum, int heads, int N, int chunk) {
    __shared__ float red[4][kHeadDim];
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads, part = blockIdx.x, BH = gridDim.y;
    const float *vp = (const float *)vt.ptr + b * vt.sb + h * vt.sh;
    const int c = threadIdx.x & 63, tg = threadIdx.x >> 6;
    const int n0 = part * chunk, n1 = min(N, n0 + chunk);
    float s = 0.f;
    for (int n = n0 + tg; n < n1; n += 4) s += vp[(long long)n * vt.sn + c];
    red[tg][c] = s;
    __syncthreads();
    if (tg == 0)
        vsum[((size_t)part * BH + bh) * kHeadDim + c] = (red[0][c] + red[1][c]) + (red[2][c] + red[3][c]);
}

// grid (ceil(N / 64), B*heads), 256 threads: o[n][c] += sum_taps kappa[c][tap] v[n + tap][c];
// a thread owns 4 channels of 4 tokens.
__global__ void __launch_bounds__(256)
dwc_add_f32(TensorArg vt, TensorArg ot, DwcArg cv, int ksize, int heads, int N) {
    __shared__ float kap[25][kHeadDim];
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
    const int kk = ksize * ksize, pad = ksize / 2;
    const float *kbase = cv.kappa + b * cv.kappa_sb + (size_t)h * kHeadDim * kk;
    for (int e = threadIdx.x; e < kHeadDim * kk; e += 256) kap[e % kk][e / kk] = kbase[e];
    __syncthreads();
    const float *vp = (const float *)vt.ptr + b * vt.sb + h * vt.sh;
    float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh;
    const int c4 = (threadIdx.x & 15) * 4, tr = threadIdx.x >> 4;
    for (int i = 0; i < 4; ++i) {
        const int n = blockIdx.x * 64 + i * 16 + tr;
        if (n >= N) break;
        if (n < cv.P) continue;  // prefix tokens get no convolution term
        const int r = (n - cv.P) / cv.W, c = (n - cv.P) - r * cv.W;
        f32x4 acc = *(const f32x4 *)(op + (long long)n * ot.sn + c4);
        for (int di = -pad; di <= pad; ++di)
            for (int dj = -pad; dj <= pad; ++dj) {
                const int r2 = r + di, c2 = c + dj;
                if (r2 < 0 || r2 >= cv.H || c2 < 0 || c2 >= cv.W) continue;
                const f32x4 vv = *(const f32x4 *)(vp + (long long)(cv.P + r2 * cv.W + c2) * vt.sn + c4);
                const f32x4 kv = *(const f32x4 *)&kap[(di + pad) * ksize + dj + pad][c4];
                acc[0] = fmaf(kv[0], vv[0], acc[0]);
                acc[1] = fmaf(kv[1], vv[1], acc[1]);
                acc[2] = fmaf(kv[2], vv[2], acc[2]);
                acc[3] = fmaf(kv[3], vv[3], acc[3]);
            }
        *(f32x4 *)(op + (long long)n * ot.sn + c4) = acc;
    }
}

// ---------------------------------------------------------------------------------------
// Token-wise dynamic filters.
// ---------------------------------------------------------------------------------------

// dst[i] = bf16(src[i]), eight elements per thread; n8 = element count / 8.
__global__ void __launch_bounds__(256)
cast_to_bf16(const float *__restrict__ src, unsigned short *__restrict__ dst, long long n8) {
    const long long i = blockIdx.x * 256ll + threadIdx.x;
    if (i >= n8) return;
    const f32x4 a = *(const f32x4 *)(src + 8 * i), b = *(const f32x4 *)(src + 8 * i + 4);
    u32x4 r = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])};
    *(u32x4 *)(dst + 8 * i) = r;
}

// Second generator layer, reordered so that the filters come out tap-major: row c*kk + tap of
// w2 [C*kk][hidden] becomes row tap*C + c of dst (bf16), and b2 likewise (fp32).  One thread per
// 8 elements of a row; n8 = C*kk*hidden / 8.
__global__ void __launch_bounds__(256)
reorder_w2(const float *__restrict__ w2, const float *__restrict__ b2, unsigned short *__restrict__ dst,
           float *__restrict__ b2p, int C, int kk, int hidden, long long n8) {
    const long long i = blockIdx.x * 256ll + threadIdx.x;
    if (i >= n8) return;
    const int per_row = hidden / 8, j8 = (int)(i % per_row);
    const int row = (int)(i / per_row), c = row / kk, tap = row % kk, to = tap * C + c;
    const float *src = w2 + (size_t)row * hidden + 8 * j8;
    const f32x4 a = *(const f32x4 *)src, b = *(const f32x4 *)(src + 4);
    u32x4 r = {pack_bf16x2(a[0], a[1]), pack_bf16x2(a[2], a[3]), pack_bf16x2(b[0], b[1]), pack_bf16x2(b[2], b[3])};
    *(u32x4 *)(dst + (size_t)to * hidden + 8 * j8) = r;
    if (j8 == 0) b2p[to] = b2[row];
}

// V in any strided layout -> rows [B*N][C] (channel = head*64 + c), 16 bytes per thread.
__global__ void __launch_bounds__(256)
pack_v_rows(TensorArg vt, unsigned short *__restrict__ rows, int heads, int N, long long total) {
    const long long idx = blockIdx.x * 256ll + threadIdx.x;
    if (idx >= total) return;
    const int groups = heads * 8, cg = (int)(idx % groups), h = cg >> 3, c8 = (cg & 7) * 8;
    const long long m = idx / groups;
    const int b = (int)(m / N), n = (int)(m % N);
    const unsigned short *src = (const unsigned short *)vt.ptr + b * vt.sb + h * vt.sh + (long long)n * vt.sn + c8;
    *(u32x4 *)(rows + idx * 8) = *(const u32x4 *)src;
}

__device__ inline float bf16_elem(const u32x4 &x, int e) {  // e = 0..7, compile-time after unrolling
    return (e & 1) ? bf16_hi(x[e >> 1]) : bf16_lo(x[e >> 1]);
}

// o[b, n, c] = la[b, n, c] + sum_taps kappa[b*N + n][tap][c] * v[b, n + tap, c] on the H x W
// grid behind P prefix tokens (prefix rows: o = la); kappa fp32, tap-major.  One thread per
// token and 8 channels; total = B*N*C/8 threads.  la and o may be the same fp32 tensor (each
// element is read and written by one thread).
template <int KS, bool O_BF16>
__global__ void __launch_bounds__(256)
dwc_token_add(TensorArg vt, TensorArg la, TensorArg ot, const float *__restrict__ kappa,
              int heads, int N, int P, int H, int W, long long total) {
    constexpr int KK = KS * KS, PAD = KS / 2;
    const long long idx = blockIdx.x * 256ll + threadIdx.x;
    if (idx >= total) return;
    const int groups = heads * 8, cg = (int)(idx % groups), h = cg >> 3, c8 = (cg & 7) * 8;
    const long long m = idx / groups;
    const int b = (int)(m / N), n = (int)(m % N);
    const float *lp = (const float *)la.ptr + b * la.sb + h * la.sh + (long long)n * la.sn + c8;
    const f32x4 l0 = *(const f32x4 *)lp, l1 = *(const f32x4 *)(lp + 4);
    float acc[8] = {l0[0], l0[1], l0[2], l0[3], l1[0], l1[1], l1[2], l1[3]};
    if (n >= P) {
        const int g = n - P, r = g / W, col = g - r * W;
        const int C = heads * kHeadDim;
        const float *kp = kappa + (size_t)m * C * KK + cg * 8;  // this thread's 8 channels, tap 0
        const unsigned short *vp = (const unsigned short *)vt.ptr + b * vt.sb + h * vt.sh + c8;
#pragma unroll
        for (int di = -PAD; di <= PAD; ++di)
#pragma unroll
            for (int dj = -PAD; dj <= PAD; ++dj) {
                const int tap = (di + PAD) * KS + dj + PAD;
                const int r2 = r + di, c2 = col + dj;
                const bool inside = r2 >= 0 && r2 < H && c2 >= 0 && c2 < W;
                const int nb = inside ? P + r2 * W + c2 : n;
                u32x4 vv = *(const u32x4 *)(vp + (long long)nb * vt.sn);
                if (!inside) vv = u32x4{0u, 0u, 0u, 0u};
                const f32x4 k0 = *(const f32x4 *)(kp + (size_t)tap * C), k1 = *(const f32x4 *)(kp + (size_t)tap * C + 4);
#pragma unroll
                for (int c = 0; c < 4; ++c) {
                    acc[c] = fmaf(k0[c], bf16_elem(vv, c), acc[c]);
                    acc[c + 4] = fmaf(k1[c], bf16_elem(vv, c + 4), acc[c + 4]);
                }
            }
    }
    if (O_BF16) {
        unsigned short *op = (unsigned short *)ot.ptr + b * ot.sb + h * ot.sh + (long long)n * ot.sn + c8;
        u32x4 out = {pack_bf16x2(acc[0], acc[1]), pack_bf16x2(acc[2], acc[3]),
                     pack_bf16x2(acc[4], acc[5]), pack_bf16x2(acc[6], acc[7])};
        *(u32x4 *)op = out;
    } else {
        float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh + (long long)n * ot.sn + c8;
        *(f32x4 *)op = f32x4{acc[0], acc[1], acc[2], acc[3]};
        *(f32x4 *)(op + 4) = f32x4{acc[4], acc[5], acc[6], acc[7]};
    }
}

template <int KS, bool O_BF16>
static void launch_token_add(hipStream_t stream, const Problem &pr, const TensorArg &la,
                             const float *kappa, long long total) {
    hipLaunchKernelGGL((dwc_token_add<KS, O_BF16>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                       stream, pr.v, la, pr.o, kappa, pr.heads, pr.N, pr.P, pr.H, pr.W, total);
}

jv_status token_dwc_forward(const Problem &pr, const TensorArg &la, const DwcPlan &dwc, float *ws,
                            hipStream_t stream) {
    const int C = pr.heads * kHeadDim, kk = dwc.ksize * dwc.ksize;
    const long long M = (long long)pr.B * pr.N;
    if (M * (C / 8) / 256 >= (1ll << 31) - 1) return fail(JV_ERR_UNSUPPORTED, "token-wise filters: too many tokens");
    unsigned short *w1b = (unsigned short *)(ws + dwc.w1b_off), *w2b = (unsigned short *)(ws + dwc.w2b_off);
    unsigned short *rows = (unsigned short *)(ws + dwc.vt_off), *u = (unsigned short *)(ws + dwc.u_off);
    float *kappa = ws + dwc.tok_kappa_off, *b2p = ws + dwc.b2p_off;
    jv_status st;
    long long n8 = (long long)dwc.hidden * C / 8;
    hipLaunchKernelGGL(cast_to_bf16, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream, dwc.w1, w1b, n8);
    if ((st = launch_status("cast_to_bf16")) != JV_OK) return st;
    n8 = (long long)C * kk * dwc.hidden / 8;
    hipLaunchKernelGGL(reorder_w2, dim3((unsigned)((n8 + 255) / 256)), dim3(256), 0, stream, dwc.w2, dwc.b2, w2b,
                       b2p, C, kk, dwc.hidden, n8);
    if ((st = launch_status("reorder_w2")) != JV_OK) return st;
    // V as the matrix [B*N][C]: in place when its layout already is one, else a packed copy.
    const void *a = pr.v.ptr;
    long long lda = pr.v.sn;
    const bool in_place = pr.v.sh == kHeadDim && pr.v.sn >= C && pr.v.sn % 8 == 0 &&
                          pr.v.sb == (long long)pr.N * pr.v.sn && pr.v.sn <= (1 << 21);
    const long long total = M * (C / 8);
    if (!in_place) {
        hipLaunchKernelGGL(pack_v_rows, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, pr.v, rows,
                           pr.heads, pr.N, total);
        if ((st = launch_status("pack_v_rows")) != JV_OK) return st;
        a = rows;
        lda = C;
    }
    if ((st = gemm_forward(a, w1b, dwc.b1, nullptr, u, M, dwc.hidden, C, JV_EPI_SILU, true, stream, lda)) != JV_OK)
        return st;
    if ((st = gemm_forward(u, w2b, b2p, nullptr, kappa, M, C * kk, dwc.hidden, JV_EPI_NONE, false, stream)) != JV_OK)
        return st;
    if (dwc.ksize == 3) {
        if (pr.o_bf16) launch_token_add<3, true>(stream, pr, la, kappa, total);
        else launch_token_add<3, false>(stream, pr, la, kappa, total);
    } else {
        if (pr.o_bf16) launch_token_add<5, true>(stream, pr, la, kappa, total);
        else launch_token_add<5, false>(stream, pr, la, kappa, total);
    }
    return launch_status("dwc_token_add");
}

// ---------------------------------------------------------------------------------------
// Token-wise dynamic filters on fp32 tensors: plain fp32 arithmetic, nothing materialised but
// the hidden layer.  One workgroup per grid token.
// ---------------------------------------------------------------------------------------

// u[m][j] = silu(b1[j] + sum_c w1[j][c] v[m][c]) for grid token m = b*N + n (n >= P); channel
// c = head*64 + c'.  grid (B*N), 256 threads, C floats of dynamic LDS (the token's V row); one
// wavefront per hidden unit at a time.
__global__ void __launch_bounds__(256)
token_hidden_f32(TensorArg vt, const float *__restrict__ w1, const float *__restrict__ b1,
                 float *__restrict__ u, int heads, int N, int P, int hidden) {
    extern __shared__ float vrow[];
    const int m = blockIdx.x, b = m / N, n = m - b * N;
    if (n < P) return;  // whole workgroup: prefix tokens have no filters
    const int C = heads * kHeadDim;
    const float *vp = (const float *)vt.ptr + b * vt.sb + (long long)n * vt.sn;
    for (int c = threadIdx.x; c < C; c += 256) vrow[c] = vp[(c >> 6) * vt.sh + (c & 63)];
    __syncthreads();
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    for (int j = wave; j < hidden; j += 4) {
        const float *wr = w1 + (size_t)j * C;
        float s = 0.f;
        for (int c = lane; c < C; c += 64) s = fmaf(wr[c], vrow[c], s);
#pragma unroll
        for (int off = 32; off > 0; off >>= 1) s += __shfl_xor(s, off, 64);
        if (lane == 0) {
            const float pre = s + b1[j];
            u[(size_t)m * hidden + j] = pre / (1.0f + expf(-pre));
        }
    }
}

// o[m][c] += sum_taps kappa[m][c][tap] v[m + tap][c],  kappa[m][c][tap] = b2[c k^2 + tap] +
// sum_j w2[c k^2 + tap][j] u[m][j]  (zero outside the H x W grid that follows P prefix tokens).
// grid (B*N), 256 threads (one channel each, strided), hidden floats of dynamic LDS.
__global__ void __launch_bounds__(256)
token_dwc_f32(TensorArg vt, TensorArg ot, const float *__restrict__ u, const float *__restrict__ w2,
              const float *__restrict__ b2, int heads, int N, int P, int H, int W, int hidden, int ksize) {
    extern __shared__ float urow[];
    const int m = blockIdx.x, b = m / N, n = m - b * N;
    if (n < P) return;  // whole workgroup
    for (int j = threadIdx.x; j < hidden; j += 256) urow[j] = u[(size_t)m * hidden + j];
    __syncthreads();
    const int C = heads * kHeadDim, kk = ksize * ksize, pad = ksize / 2;
    const int g = n - P, r = g / W, col = g - r * W;
    for (int c = threadIdx.x; c < C; c += 256) {
        const int h = c >> 6, c1 = c & 63;
        const float *vp = (const float *)vt.ptr + b * vt.sb + h * vt.sh + c1;
        float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh + (long long)n * ot.sn + c1;
        float acc = *op;
        for (int di = -pad; di <= pad; ++di)
            for (int dj = -pad; dj <= pad; ++dj) {
                const int r2 = r + di, c2 = col + dj;
                if (r2 < 0 || r2 >= H || c2 < 0 || c2 >= W) continue;
                const int row = c * kk + (di + pad) * ksize + dj + pad;
                const float *wr = w2 + (size_t)row * hidden;
                float kap = b2[row];
                for (int j = 0; j < hidden; j += 4) {
                    const f32x4 w4 = *(const f32x4 *)(wr + j);
                    kap = fmaf(w4[0], urow[j], fmaf(w4[1], urow[j + 1], fmaf(w4[2], urow[j + 2], fmaf(w4[3], urow[j + 3], kap))));
                }
                acc = fmaf(kap, vp[(long long)(P + r2 * W + c2) * vt.sn], acc);
            }
        *op = acc;
    }
}

jv_status token_dwc_forward_f32(const Problem &pr, const DwcPlan &dwc, float *ws, hipStream_t stream) {
    const int C = pr.heads * kHeadDim;
    const long long M = (long long)pr.B * pr.N;
    if (M >= (1ll << 31) - 1) return fail(JV_ERR_UNSUPPORTED, "token-wise filters: too many tokens");
    float *u = ws + dwc.tok_kappa_off;  // [B*N][hidden]; the region sized for the bf16 path's filters
    hipLaunchKernelGGL(token_hidden_f32, dim3((unsigned)M), dim3(256), C * sizeof(float), stream, pr.v,
                       dwc.w1, dwc.b1, u, pr.heads, pr.N, pr.P, dwc.hidden);
    jv_status st = launch_status("token_hidden_f32");
    if (st != JV_OK) return st;
    hipLaunchKernelGGL(token_dwc_f32, dim3((unsigned)M), dim3(256), dwc.hidden * sizeof(float), stream, pr.v,
                       pr.o, u, dwc.w2, dwc.b2, pr.heads, pr.N, pr.P, pr.H, pr.W, dwc.hidden, dwc.ksize);
    return launch_status("token_dwc_f32");
}

// ---------------------------------------------------------------------------------------
// The convolution branch for heads of 128 channels (bf16 tensors).  The apply pass of linear
// attention adds the convolution itself (la_apply_wide_bf16) and the state pass leaves the
// token sums of V; what is left here is the workspace plan and the generator's launch.
// ---------------------------------------------------------------------------------------

// Workspace of the wide-head block beyond the linear-attention states (float offsets from
// `base`): the partial token sums of V, the generator's hidden layer, the generated filters.
jv_status plan_dwc_wide(const jv_dwc_params *dwc, size_t base, int B, int heads, int N, DwcPlan *out) {
    DwcPlan p;
    // parameter validation as for 64-channel heads (C = 2 * heads * 64 channels)
    jv_status st = plan_dwc(dwc, plan_linear(1, 2 * heads, 256), 1, 2 * heads, 256, &p);
    if (st != JV_OK) return st;
    if (p.mode == JV_DWC_TOKEN_DYNAMIC)
        return fail(JV_ERR_UNSUPPORTED, "head_dim 128: token-wise filters are built for 64-channel heads");
    base = align64f(base);
    p.total_floats = base;
    if (p.mode == JV_DWC_SQUEEZE_DYNAMIC) {
        const size_t C = (size_t)heads * kHeadDimWide, kk = (size_t)p.ksize * p.ksize;
        p.vsum_off = base;
        p.hidden_off = p.vsum_off + align64f((size_t)plan_linear_wide(B, heads, N).n_split * B * C);
        p.kappa_off = p.hidden_off + align64f((size_t)B * (p.hidden > 0 ? p.hidden : 1));
        p.total_floats = p.kappa_off + align64f((size_t)B * C * kk);
    }
    *out = p;
    return JV_OK;
}

// The filters the apply pass adds for heads of 128 channels: the static bank as it is, or the
// bank generated per image from the token mean of V.
jv_status dwc_wide_filters(const Problem &pr, const DwcPlan &dwc, float *ws, hipStream_t stream, DwcArg *out) {
    DwcArg arg = {dwc.static_kernel, 0, pr.H, pr.W, pr.P};
    if (dwc.mode == JV_DWC_SQUEEZE_DYNAMIC) {
        const int n_part = plan_linear_wide(pr.B, pr.heads, pr.N).n_split;  // the state pass's chunks
        jv_status st;
        if ((st = squeeze_generate(dwc, ws, n_part, pr.B, 2 * pr.heads, pr.N, stream)) != JV_OK) return st;
        arg.kappa = ws + dwc.kappa_off;
        arg.kappa_sb = (long long)pr.heads * kHeadDimWide * dwc.ksize * dwc.ksize;
    }
    *out = arg;
    return JV_OK;
}

jv_status vsum_f32_launch(const Problem &pr, const LinearPlan &plan, float *vsum, hipStream_t stream) {
    hipLaunchKernelGGL(v_sum_f32, dim3(plan.n_split, pr.B * pr.heads), dim3(256), 0, stream, pr.v,
                       vsum, pr.heads, pr.N, plan.chunk);
    return launch_status("v_sum_f32");
}

jv_status dwc_add_f32_launch(const Problem &pr, const DwcArg &cv, int ksize, hipStream_t stream) {
    hipLaunchKernelGGL(dwc_add_f32, dim3((pr.N + 63) / 64, pr.B * pr.heads), dim3(256), 0, stream,
                       pr.v, pr.o, cv, ksize, pr.heads, pr.N);
    return launch_status("dwc_add_f32");
}

}  // namespace jv
