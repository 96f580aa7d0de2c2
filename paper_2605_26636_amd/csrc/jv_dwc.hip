// The depth-wise convolution branch of the paper's linear-attention block (Sec. 3.2.1, Eq. 4:
// O = LA(Q, K, V) + DWC(V)) -- the parts that are not fused into the bf16 apply pass:
//   squeeze_hidden / squeeze_kappa   the generator of the dynamic filters ("Squeeze Dynamic
//                                    Convolution": token mean of V -> Linear -> SiLU -> Linear)
//   v_sum_f32, dwc_add_f32           plain fp32 kernels for fp32 tensors
#include "jv_linear.h"
#include "jv_mfma.h"

namespace jv {

static size_t align64f(size_t floats) { return (floats + 63) & ~(size_t)63; }  // 256 bytes

jv_status plan_dwc(const jv_dwc_params *dwc, const LinearPlan &lp, int B, int heads, DwcPlan *out) {
    DwcPlan p;
    const size_t base = align64f(linear_workspace_floats(lp, B, heads));
    p.total_floats = base;
    if (!dwc || dwc->mode == JV_DWC_NONE) {
        *out = p;
        return JV_OK;
    }
    if (dwc->mode != JV_DWC_STATIC && dwc->mode != JV_DWC_SQUEEZE_DYNAMIC)
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
