// Softmax attention over windows of the token grid (Sec. 3.2.2 of the paper) and over the whole
// grid (Eq. 1).  Full attention is the one-window case of the same kernels: a window that
// spans the grid.  Queries and keys are addressed by (window, slot); slot -> token is the
// row-major position inside the window, and slots that fall outside the H x W grid are
// padding: excluded as keys, skipped as queries.
#include <math.h>

#include "jv_common.h"

namespace jv {

// slot of window (wy, wx) -> token index, or -1 for padding / past the window.
__device__ inline int slot_token(const WindowGeom &g, int wy, int wx, int slot) {
    if (slot >= g.slots) return -1;
    int r = wy * g.wh + slot / g.ww, c = wx * g.ww + slot % g.ww;
    return (r < g.H && c < g.W) ? r * g.W + c : -1;
}

__device__ inline float wave_max(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
    return x;
}
__device__ inline float wave_sum(float x) {
#pragma unroll
    for (int off = 32; off > 0; off >>= 1) x += __shfl_xor(x, off, 64);
    return x;
}

// ---------------------------------------------------------------------------------------
// fp32 path.  One wavefront per query slot; a workgroup holds four consecutive slots of one
// window.  Key tiles of 64 slots: lane j scores key j (dot product over 64 channels), the
// tile joins the running softmax, then lane c accumulates channel c of the output.
// Only the first q_slots query slots of every window are computed.
// grid (ceil(q_slots/4), n_win, B*heads), 256 threads.
// ---------------------------------------------------------------------------------------
__global__ void __launch_bounds__(256)
attn_f32(TensorArg qt, TensorArg kt, TensorArg vt, TensorArg ot, WindowGeom g, int heads,
         float scale, int q_slots) {
    __shared__ float qs[4][kHeadDim];
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int bh = blockIdx.z, b = bh / heads, h = bh % heads;
    const int win = blockIdx.y, wy = win / g.wins_x, wx = win % g.wins_x;
    const int qslot = blockIdx.x * 4 + wave;
    const int qtok = qslot < q_slots ? slot_token(g, wy, wx, qslot) : -1;
    if (qtok < 0) return;  // wave-uniform: padded query slots produce nothing
    const float *qp = (const float *)qt.ptr + b * qt.sb + h * qt.sh + (long long)qtok * qt.sn;
    const float *kp = (const float *)kt.ptr + b * kt.sb + h * kt.sh;
    const float *vp = (const float *)vt.ptr + b * vt.sb + h * vt.sh;
    float *op = (float *)ot.ptr + b * ot.sb + h * ot.sh + (long long)qtok * ot.sn;
    qs[wave][lane] = qp[lane];  // read back by the same wave only
    float m = -INFINITY, l = 0.f, acc = 0.f;
    for (int s0 = 0; s0 < g.slots; s0 += 64) {
        const int tok = slot_token(g, wy, wx, s0 + lane);
        float s = -INFINITY;
        if (tok >= 0) {
            const float4 *krow = (const float4 *)(kp + (long long)tok * kt.sn);
            float dot = 0.f;
#pragma unroll
            for (int c4 = 0; c4 < 16; ++c4) {
                float4 kk = krow[c4];
                dot = fmaf(qs[wave][4 * c4 + 0], kk.x, dot);
                dot = fmaf(qs[wave][4 * c4 + 1], kk.y, dot);
                dot = fmaf(qs[wave][4 * c4 + 2], kk.z, dot);
                dot = fmaf(qs[wave][4 * c4 + 3], kk.w, dot);
            }
            s = dot * scale;
        }
        const float tile_max = wave_max(s);
        if (tile_max == -INFINITY) continue;  // a tile of padding only
        const float m_new = fmaxf(m, tile_max);
        const float alpha = expf(m - m_new);  // exp(-inf) = 0 on the first live tile
        const float p = (tok >= 0) ? expf(s - m_new) : 0.f;
        l = l * alpha + wave_sum(p);
        acc *= alpha;
        for (int j = 0; j < 64; ++j) {
            const int tj = __shfl(tok, j, 64);
            if (tj < 0) continue;  // wave-uniform
            const float pj = __shfl(p, j, 64);
            acc = fmaf(pj, vp[(long long)tj * vt.sn + lane], acc);
        }
        m = m_new;
    }
    op[lane] = acc / l;
}

// q_slots: number of leading query slots of each window to compute (all keys always take part).
jv_status attn_bf16(const Problem &pr, const WindowGeom &g, float scale, int q_slots, hipStream_t stream);

static jv_status attn_dispatch(const Problem &pr, const WindowGeom &g, float scale, int q_slots,
                               hipStream_t stream) {
    if (pr.bf16) return attn_bf16(pr, g, scale, q_slots, stream);
    const long long qblocks = (q_slots + 3) / 4;
    if (g.n_win > 65535) return fail(JV_ERR_UNSUPPORTED, "more than 65535 windows");
    hipLaunchKernelGGL(attn_f32, dim3((unsigned)qblocks, g.n_win, pr.B * pr.heads), dim3(256), 0,
                       stream, pr.q, pr.k, pr.v, pr.o, g, pr.heads, scale, q_slots);
    return launch_status("attn_f32");
}

// All tokens of the sequence as one window of 1 x N slots (token = slot).
static WindowGeom sequence_geom(int N) {
    WindowGeom g;
    g.H = 1; g.W = N; g.wh = 1; g.ww = N;
    g.Hp = 1; g.Wp = N; g.wins_x = 1; g.wins_y = 1; g.n_win = 1; g.slots = N;
    return g;
}

// The same tensors from token `first` on.
static TensorArg from_token(const TensorArg &t, int first, bool bf16) {
    TensorArg r = t;
    r.ptr = (const char *)t.ptr + (long long)first * t.sn * (bf16 ? 2 : 4);
    return r;
}

jv_status window_check(const Problem &pr, int wh, int ww) {
    WindowGeom g;
    jv_status st = make_window_geom(pr.H, pr.W, wh, ww, &g);
    if (st != JV_OK) return st;
    if (g.n_win > 65535) return fail(JV_ERR_UNSUPPORTED, "more than 65535 windows");
    return JV_OK;
}

jv_status window_forward(const Problem &pr, int wh, int ww, float scale, hipStream_t stream) {
    WindowGeom g;
    jv_status st = window_check(pr, wh, ww);
    if (st != JV_OK) return st;
    make_window_geom(pr.H, pr.W, wh, ww, &g);
    if (pr.P == 0) return attn_dispatch(pr, g, resolve_scale(scale, pr.D), g.slots, stream);
    // Prefix tokens: the grid tokens run window attention among themselves; the prefix
    // tokens (the first P query slots of the whole sequence) attend to every token.
    Problem grid = pr;
    grid.P = 0;
    grid.N = pr.H * pr.W;
    grid.q = from_token(pr.q, pr.P, pr.bf16);
    grid.k = from_token(pr.k, pr.P, pr.bf16);
    grid.v = from_token(pr.v, pr.P, pr.bf16);
    grid.o = from_token(pr.o, pr.P, pr.o_bf16);
    if ((st = attn_dispatch(grid, g, resolve_scale(scale, pr.D), g.slots, stream)) != JV_OK) return st;
    return attn_dispatch(pr, sequence_geom(pr.N), resolve_scale(scale, pr.D), pr.P, stream);
}

jv_status full_forward(const Problem &pr, float scale, hipStream_t stream) {
    if (pr.P > 0) return attn_dispatch(pr, sequence_geom(pr.N), resolve_scale(scale, pr.D), pr.N, stream);
    // One window that spans the grid; the token order inside it is the raster order.
    WindowGeom g;
    g.H = pr.H; g.W = pr.W; g.wh = pr.H; g.ww = pr.W;
    g.Hp = pr.H; g.Wp = pr.W; g.wins_x = 1; g.wins_y = 1; g.n_win = 1; g.slots = pr.N;
    return attn_dispatch(pr, g, resolve_scale(scale, pr.D), g.slots, stream);
}

}  // namespace jv

extern "C" {

jv_status jv_window_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                             const void *v, void *o, int32_t win_h, int32_t win_w, float scale,
                             void *hip_stream) {
    jv::clear_error();
    jv::Problem pr;
    jv_status st = jv::make_problem(desc, q, k, v, o, &pr);
    if (st != JV_OK) return st;
    return jv::window_forward(pr, win_h, win_w, scale, (hipStream_t)hip_stream);
}

jv_status jv_full_attn_fwd(const jv_attn_desc *desc, const void *q, const void *k,
                           const void *v, void *o, float scale, void *hip_stream) {
    jv::clear_error();
    jv::Problem pr;
    jv_status st = jv::make_problem(desc, q, k, v, o, &pr);
    if (st != JV_OK) return st;
    return jv::full_forward(pr, scale, (hipStream_t)hip_stream);
}

}  // extern "C"
