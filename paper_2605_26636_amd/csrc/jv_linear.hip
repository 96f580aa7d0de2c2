// Linear attention (Eq. 2 of the paper, key-sum normaliser; phi = ReLU unless the focused map
// of Eq. 3 is asked for):
//   pass 1  la_state_*  : S_p = sum_j relu(k_j)^T v_j, z_p = sum_j relu(k_j) over one token chunk
//   pass 2  la_apply_*  : S = sum_p S_p, z = sum_p z_p;  o_i = relu(q_i) S / (relu(q_i).z + eps)
//
// Workspace layout (fp32): partial p of (batch b, head h) starts at
//   ((p * B*heads) + b*heads + h) * kStateFloats
// and holds S transposed, St[c2][c1] (c2 = value channel, c1 = key channel), then z[c1].
#include "jv_linear.h"

namespace jv {

LinearPlan plan_linear(int B, int heads, int N) {
    LinearPlan p;
    const long long bh = (long long)B * heads;
    // Aim for about two workgroups per compute unit, chunks of at least 256 tokens.
    long long want = (512 + bh - 1) / bh;
    long long max_split = (N + 255) / 256;
    if (want > max_split) want = max_split;
    if (want < 1) want = 1;
    if (want > 64) want = 64;
    long long chunk = (N + want - 1) / want;
    chunk = ((chunk + 255) / 256) * 256;
    p.chunk = (int)chunk;
    p.n_split = (int)((N + chunk - 1) / chunk);
    // token chunks of the apply pass: 1024 tokens, halved (down to 256) while that leaves less
    // than two workgroups per compute unit
    p.apply_tokens = 1024;
    while (p.apply_tokens > 256 && bh * ((N + p.apply_tokens - 1) / p.apply_tokens) < 512) p.apply_tokens /= 2;
    p.combine = p.n_split > 4;
    return p;
}

size_t linear_workspace_floats(const LinearPlan &p, int B, int heads) {
    return (size_t)(p.n_split + (p.combine ? 1 : 0)) * B * heads * kStateFloats;
}

// ---------------------------------------------------------------------------------------
// fp32 path: plain FMA arithmetic, used for fp32 tensors.
// ---------------------------------------------------------------------------------------

// Focused feature map (Eq. 3; see focus_bf16x8 in the bf16 path) applied in place to `rows`
// token rows of 64 already-rectified channels in shared memory; one thread per row.
__device__ inline void focus_rows_f32(float (*rows)[kHeadDim], int n_rows, int p, int t) {
    if (t < n_rows) {
        float *r = rows[t];
        float top = 0.f;
#pragma unroll 4
        for (int c = 0; c < kHeadDim; ++c) top = fmaxf(top, r[c]);
        if (top > 0.f) {
            const float inv_top = 1.0f / top;
            float ss = 0.f, sy = 0.f;
#pragma unroll 2
            for (int c = 0; c < kHeadDim; ++c) {
                const float x = r[c] * inv_top;
                float y = x;
                for (int i = 1; i < p; ++i) y *= x;
                ss = fmaf(x, x, ss);
                sy = fmaf(y, y, sy);
                r[c] = y;
            }
            const float scale = top * sqrtf(ss / sy);
#pragma unroll 4
            for (int c = 0; c < kHeadDim; ++c) r[c] *= scale;
        }
    }
}

// grid (n_split, B*heads), 256 threads.  Thread t owns S[16*(t/64) .. +15][t%64].
__global__ void __launch_bounds__(256)
la_state_f32(TensorArg kt, TensorArg vt, float *__restrict__ ws, int heads, int N, int chunk,
             int focus_p) {
    __shared__ float Ks[32][kHeadDim];
    __shared__ float Vs[32][kHeadDim];
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads, p = blockIdx.x;
    const int BH = gridDim.y;
    const float *kp = (const float *)kt.ptr + b * kt.sb + h * kt.sh;
    const float *vp = (const float *)vt.ptr + b * vt.sb + h * vt.sh;
    const int t = threadIdx.x, c2 = t & 63, rb = t >> 6;
    float acc[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) acc[r] = 0.f;
    float zacc = 0.f;
    const int n0 = p * chunk, n1 = min(N, n0 + chunk);
    for (int base = n0; base < n1; base += 32) {
        // 32 tokens x 64 channels = 512 float4; two per thread per tensor
        for (int e = t; e < 512; e += 256) {
            int j = e >> 4, c4 = (e & 15) * 4, n = base + j;
            float4 kk = make_float4(0.f, 0.f, 0.f, 0.f), vv = kk;
            if (n < n1) {
                kk = *(const float4 *)(kp + (long long)n * kt.sn + c4);
                vv = *(const float4 *)(vp + (long long)n * vt.sn + c4);
            }
            Ks[j][c4 + 0] = fmaxf(kk.x, 0.f);
            Ks[j][c4 + 1] = fmaxf(kk.y, 0.f);
            Ks[j][c4 + 2] = fmaxf(kk.z, 0.f);
            Ks[j][c4 + 3] = fmaxf(kk.w, 0.f);
            *(float4 *)&Vs[j][c4] = vv;
        }
        __syncthreads();
        if (focus_p > 1) {  // uniform
            focus_rows_f32(Ks, 32, focus_p, t);
            __syncthreads();
        }
#pragma unroll 4
        for (int j = 0; j < 32; ++j) {
            float vj = Vs[j][c2];
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[r] = fmaf(Ks[j][rb * 16 + r], vj, acc[r]);
            if (rb == 0) zacc += Ks[j][c2];
        }
        __syncthreads();
    }
    float *out = ws + ((size_t)p * BH + bh) * kStateFloats;
#pragma unroll
    for (int r = 0; r < 16; ++r) out[c2 * kHeadDim + rb * 16 + r] = acc[r];
    if (rb == 0) out[kHeadDim * kHeadDim + c2] = zacc;
}

// grid (ceil(N/256), B*heads), 256 threads.
__global__ void __launch_bounds__(256)
la_apply_f32(TensorArg qt, TensorArg ot, const float *__restrict__ ws, int heads, int N,
             int n_split, float eps, int focus_p) {
    __shared__ float S[kHeadDim][kHeadDim + 1];  // S[c1][c2]
    __shared__ float z[kHeadDim];
    __shared__ float Qs[64][kHeadDim];
    const int bh = blockIdx.y, b = bh / heads, h = bh % heads;
    const int BH = gridDim.y;
    const float *qp = (const float *)qt.ptr + b * qt.sb + h * qt.sh;
    float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh;
    const int t = threadIdx.x;
    for (int e = t; e < kStateFloats; e += 256) {
        float s = 0.f;
        for (int p = 0; p < n_split; ++p) s += ws[((size_t)p * BH + bh) * kStateFloats + e];
        if (e < kHeadDim * kHeadDim) S[e & 63][e >> 6] = s;  // stored transposed in the workspace
        else z[e - kHeadDim * kHeadDim] = s;
    }
    const int c2 = t & 63, tg = t >> 6;
    const int n0 = blockIdx.x * 256, n1 = min(N, n0 + 256);
    for (int base = n0; base < n1; base += 64) {
        __syncthreads();
        for (int e = t; e < 1024; e += 256) {
            int j = e >> 4, c4 = (e & 15) * 4, n = base + j;
            float4 qq = make_float4(0.f, 0.f, 0.f, 0.f);
            if (n < n1) qq = *(const float4 *)(qp + (long long)n * qt.sn + c4);
            Qs[j][c4 + 0] = fmaxf(qq.x, 0.f);
            Qs[j][c4 + 1] = fmaxf(qq.y, 0.f);
            Qs[j][c4 + 2] = fmaxf(qq.z, 0.f);
            Qs[j][c4 + 3] = fmaxf(qq.w, 0.f);
        }
        __syncthreads();
        if (focus_p > 1) {  // uniform
            focus_rows_f32(Qs, 64, focus_p, t);
            __syncthreads();
        }
        for (int jj = 0; jj < 16; ++jj) {
            int j = tg * 16 + jj, n = base + j;
            if (n >= n1) break;
            float num = 0.f, den = 0.f;
#pragma unroll 8
            for (int c1 = 0; c1 < kHeadDim; ++c1) {
                float qv = Qs[j][c1];
                num = fmaf(qv, S[c1][c2], num);
                den = fmaf(qv, z[c1], den);
            }
            op[(long long)n * ot.sn + c2] = num / (den + eps);
        }
    }
}

size_t linear_workspace_bytes(int B, int heads, int N) {
    return linear_workspace_floats(plan_linear(B, heads, N), B, heads) * sizeof(float);
}

// The block of Eq. 4.  Order of launches: state pass (which also sums V over the tokens when
// the filters are generated from it), optional combine, filter generator, apply pass (bf16:
// the convolution is fused into it; fp32: a pass of its own adds it).
jv_status linear_block_forward(const Problem &pr, float eps, const jv_dwc_params *dwc,
                               void *workspace, size_t workspace_bytes, hipStream_t stream,
                               int focus_p) {
    if (focus_p < 1 || focus_p > 16) return fail(JV_ERR_INVALID_ARG, "focusing power must be 1 .. 16");
    if (pr.D == kHeadDimWide) {
        if (focus_p != 1) return fail(JV_ERR_UNSUPPORTED, "head_dim 128: the focused map is built for 64-channel heads");
        DwcPlan cv;
        jv_status st = plan_dwc_wide(dwc, linear_wide_workspace_floats(pr.B, pr.heads, pr.N), pr.B, pr.heads, pr.N, &cv);
        if (st != JV_OK) return st;
        const size_t need = cv.total_floats * sizeof(float);
        if (workspace_bytes < need)
            return fail(JV_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes, need);
        float *ws = (float *)workspace;
        if (cv.mode == JV_DWC_NONE) return linear_wide_bf16(pr, eps, ws, stream);
        float *vsum = cv.mode == JV_DWC_SQUEEZE_DYNAMIC ? ws + cv.vsum_off : nullptr;
        if ((st = linear_wide_state(pr, ws, vsum, stream)) != JV_OK) return st;
        DwcArg arg;
        if ((st = dwc_wide_filters(pr, cv, ws, stream, &arg)) != JV_OK) return st;
        return linear_wide_apply(pr, eps, ws, stream, cv.ksize, &arg);
    }
    const LinearPlan plan = plan_linear(pr.B, pr.heads, pr.N);
    DwcPlan cv;
    jv_status st = plan_dwc(dwc, plan, pr.B, pr.heads, pr.N, &cv);
    if (st != JV_OK) return st;
    if (workspace_bytes < cv.total_floats * sizeof(float))
        return fail(JV_ERR_WORKSPACE_TOO_SMALL, "workspace has %zu bytes, %zu needed", workspace_bytes,
                    cv.total_floats * sizeof(float));
    float *ws = (float *)workspace;
    if (cv.mode == JV_DWC_TOKEN_DYNAMIC) {
        // Plain linear attention into an fp32 tensor (O itself when it is fp32), then one pass
        // that adds every token's own convolution term and rounds once.
        if (!pr.bf16) {  // fp32 tensors: the plain two-pass attention, then the convolution added in place
            const int BH = pr.B * pr.heads;
            hipLaunchKernelGGL(la_state_f32, dim3(plan.n_split, BH), dim3(256), 0, stream, pr.k, pr.v, ws,
                               pr.heads, pr.N, plan.chunk, focus_p);
            if ((st = launch_status("la_state_f32")) != JV_OK) return st;
            hipLaunchKernelGGL(la_apply_f32, dim3((pr.N + 255) / 256, BH), dim3(256), 0, stream, pr.q, pr.o,
                               ws, pr.heads, pr.N, plan.n_split, eps, focus_p);
            if ((st = launch_status("la_apply_f32")) != JV_OK) return st;
            return token_dwc_forward_f32(pr, cv, ws, stream);
        }
        Problem la = pr;
        if (pr.o_bf16) {
            const long long C = (long long)pr.heads * kHeadDim;
            la.o = {ws + cv.la_off, (long long)pr.N * C, kHeadDim, C};
            la.o_bf16 = false;
        }
        DwcPlan none = cv;
        none.mode = JV_DWC_NONE;
        if ((st = linear_bf16(la, plan, eps, ws, none, focus_p, stream)) != JV_OK) return st;
        return token_dwc_forward(pr, la.o, cv, ws, stream);
    }
    if (pr.bf16) return linear_bf16(pr, plan, eps, ws, cv, focus_p, stream);
    const int BH = pr.B * pr.heads;
    hipLaunchKernelGGL(la_state_f32, dim3(plan.n_split, BH), dim3(256), 0, stream, pr.k, pr.v, ws,
                       pr.heads, pr.N, plan.chunk, focus_p);
    if ((st = launch_status("la_state_f32")) != JV_OK) return st;
    hipLaunchKernelGGL(la_apply_f32, dim3((pr.N + 255) / 256, BH), dim3(256), 0, stream, pr.q, pr.o,
                       ws, pr.heads, pr.N, plan.n_split, eps, focus_p);
    if ((st = launch_status("la_apply_f32")) != JV_OK) return st;
    if (cv.mode == JV_DWC_NONE) return JV_OK;
    DwcArg arg = {cv.static_kernel, 0, pr.H, pr.W, pr.P};
    if (cv.mode == JV_DWC_SQUEEZE_DYNAMIC) {
        if ((st = vsum_f32_launch(pr, plan, ws + cv.vsum_off, stream)) != JV_OK) return st;
        if ((st = squeeze_generate(cv, ws, plan.n_split, pr.B, pr.heads, pr.N, stream)) != JV_OK) return st;
        arg.kappa = ws + cv.kappa_off;
        arg.kappa_sb = (long long)pr.heads * kHeadDim * cv.ksize * cv.ksize;
    }
    return dwc_add_f32_launch(pr, arg, cv.ksize, stream);
}

jv_status linear_forward(const Problem &pr, float eps, void *workspace, hipStream_t stream) {
    const size_t bytes = pr.D == kHeadDimWide ? linear_wide_workspace_floats(pr.B, pr.heads, pr.N) * sizeof(float)
                                              : linear_workspace_bytes(pr.B, pr.heads, pr.N);
    return linear_block_forward(pr, eps, nullptr, workspace, bytes, stream);
}

}  // namespace jv

// ---------------------------------------------------------------------------------------
// Scratch of the allocation-free entry point (jv_linear_attn_fwd_static): the partial and
// combined linear-attention states live in a fixed array in device memory that belongs to the
// library's code object -- one copy per GPU, at its own address on each, held until the
// process ends.  In host code the array's name is only a handle for the symbol lookup below;
// what the kernels get is the device address that lookup returns.
// ---------------------------------------------------------------------------------------
static __device__ __align__(256) unsigned char jv_static_scratch[JV_STATIC_SCRATCH_BYTES];

namespace jv {
// Device address of jv_static_scratch on the current device, looked up once per device.
static jv_status static_scratch_address(void **out) {
    constexpr int kMaxDevices = 64;
    static std::atomic<void *> address[kMaxDevices];  // zero-initialised
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(JV_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    if (dev < 0 || dev >= kMaxDevices) return fail(JV_ERR_UNSUPPORTED, "device ordinal %d above %d", dev, kMaxDevices - 1);
    void *p = address[dev].load(std::memory_order_acquire);
    if (!p) {
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(jv_static_scratch));
        if (e != hipSuccess || !p)
            return fail(JV_ERR_HIP, "hipGetSymbolAddress(static scratch): %s", hipGetErrorString(e));
        address[dev].store(p, std::memory_order_release);  // (two threads may both look it up: same value)
    }
    *out = p;
    return JV_OK;
}
}  // namespace jv

static jv_status check_linear_args(float eps, const void *workspace) {
    if (!(eps >= 0.0f)) return jv::fail(JV_ERR_INVALID_ARG, "eps must be >= 0");
    if (!workspace) return jv::fail(JV_ERR_INVALID_ARG, "workspace is null");
    if ((uintptr_t)workspace & 255)
        return jv::fail(JV_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    return JV_OK;
}

extern "C" {

size_t jv_linear_attn_workspace_bytes(const jv_attn_desc *desc) {
    return jv_linear_block_workspace_bytes(desc, nullptr);
}

size_t jv_linear_block_workspace_bytes(const jv_attn_desc *desc, const jv_dwc_params *dwc) {
    jv::clear_error();
    if (jv::check_desc(desc) != JV_OK) return 0;
    jv::DwcPlan cv;
    const int N = desc->n_prefix + desc->grid_h * desc->grid_w;
    if (desc->head_dim == jv::kHeadDimWide) {
        if (jv::plan_dwc_wide(dwc, jv::linear_wide_workspace_floats(desc->batch, desc->heads, N), desc->batch,
                              desc->heads, N, &cv) != JV_OK)
            return 0;
        return cv.total_floats * sizeof(float);
    }
    const jv::LinearPlan plan = jv::plan_linear(desc->batch, desc->heads, N);
    if (jv::plan_dwc(dwc, plan, desc->batch, desc->heads, N, &cv) != JV_OK) return 0;
    return cv.total_floats * sizeof(float);
}

jv_status jv_linear_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                             const void *v, void *o, float eps, void *workspace,
                             size_t workspace_bytes, void *hip_stream) {
    return jv_linear_block_fwd(desc, q, k, v, o, eps, nullptr, workspace, workspace_bytes, hip_stream);
}

jv_status jv_linear_block_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                              const void *v, void *o, float eps, const jv_dwc_params *dwc,
                              void *workspace, size_t workspace_bytes, void *hip_stream) {
    jv::clear_error();
    jv::Problem pr;
    jv_status st = jv::make_problem(desc, q, k, v, o, &pr);
    if (st != JV_OK) return st;
    if ((st = check_linear_args(eps, workspace)) != JV_OK) return st;
    return jv::linear_block_forward(pr, eps, dwc, workspace, workspace_bytes, (hipStream_t)hip_stream);
}

jv_status jv_linear_attn_fwd_static(const jv_attn_desc *desc, const void *q, const void *k,
                                    const void *v, void *o, float eps, void *hip_stream) {
    jv::clear_error();
    jv::Problem pr;
    jv_status st = jv::make_problem(desc, q, k, v, o, &pr);
    if (st != JV_OK) return st;
    if (!(eps >= 0.0f)) return jv::fail(JV_ERR_INVALID_ARG, "eps must be >= 0");
    jv::DwcPlan plain;
    if ((st = jv::plan_dwc(nullptr, jv::plan_linear(pr.B, pr.heads, pr.N), pr.B, pr.heads, pr.N, &plain)) != JV_OK)
        return st;
    // what jv_linear_attn_workspace_bytes answers
    const size_t need = (pr.D == jv::kHeadDimWide ? jv::linear_wide_workspace_floats(pr.B, pr.heads, pr.N)
                                                  : plain.total_floats) * sizeof(float);
    if (need > (size_t)JV_STATIC_SCRATCH_BYTES)
        return jv::fail(JV_ERR_UNSUPPORTED, "this problem needs %zu bytes of scratch, the static scratch holds %zu",
                        need, (size_t)JV_STATIC_SCRATCH_BYTES);
    void *scratch = nullptr;
    if ((st = jv::static_scratch_address(&scratch)) != JV_OK) return st;
    // Nothing in the scratch has to start at zero: the state pass writes every partial state it
    // later reads in full.
    return jv::linear_block_forward(pr, eps, nullptr, scratch, need, (hipStream_t)hip_stream);
}

jv_status jv_linear_block_focused_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                                      const void *v, void *o, float eps, int32_t focus_p,
                                      const jv_dwc_params *dwc, void *workspace,
                                      size_t workspace_bytes, void *hip_stream) {
    jv::clear_error();
    jv::Problem pr;
    jv_status st = jv::make_problem(desc, q, k, v, o, &pr);
    if (st != JV_OK) return st;
    if ((st = check_linear_args(eps, workspace)) != JV_OK) return st;
    return jv::linear_block_forward(pr, eps, dwc, workspace, workspace_bytes, (hipStream_t)hip_stream, focus_p);
}

}  // extern "C"
