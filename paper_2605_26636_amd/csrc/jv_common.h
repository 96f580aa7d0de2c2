// Shared host-side plumbing of the JetViT mixer library: error reporting,
// descriptor validation, kernel-argument structs.  No kernel code lives here.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "jetvit.h"

namespace jv {

constexpr int kHeadDim = 64;       // the head width every kernel family is built for ...
constexpr int kHeadDimWide = 128;  // ... and the wide heads of the paper's largest backbones (bf16 tensors only)

// Thread-local description of the last failure; returns `st` for tail calls.
jv_status fail(jv_status st, const char *fmt, ...);
void clear_error();

// One [batch, heads, N, 64] tensor as a kernel sees it (element strides).
struct TensorArg {
    const void *ptr;
    long long sb, sh, sn;
};

// Everything a mixer kernel needs to know about the problem.
struct Problem {
    int B, heads, H, W, N;  // N = P + H * W tokens
    int P;                  // prefix tokens in front of the grid
    int D;                  // head_dim: kHeadDim or kHeadDimWide
    bool bf16;      // element type of Q, K, V
    bool o_bf16;    // element type of O
    TensorArg q, k, v, o;
};

// Validates the descriptor and the four base pointers; fills `out`.
jv_status make_problem(const jv_attn_desc *desc, const void *q, const void *k, const void *v,
                       void *o, Problem *out);
// Descriptor-only part of the validation (no pointers).
jv_status check_desc(const jv_attn_desc *desc);

inline jv_status launch_status(const char *what) {
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(JV_ERR_HIP, "%s: %s", what, hipGetErrorString(e));
    return JV_OK;
}

// Kernels that use more than 64 KB of dynamic LDS need their limit raised, once per device (the
// attribute belongs to the device's copy of the kernel).  One LdsLimit object per kernel, with
// static storage: it remembers the devices (by ordinal, the first 64) that have been set.
struct LdsLimit {
    std::atomic<unsigned long long> devices_done{0};
};
inline jv_status ensure_lds_limit(LdsLimit &state, const void *kernel, int bytes) {
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(JV_ERR_HIP, "hipGetDevice: %s", hipGetErrorString(e));
    const unsigned long long bit = dev >= 0 && dev < 64 ? 1ull << dev : 0ull;
    if (bit && (state.devices_done.load(std::memory_order_acquire) & bit)) return JV_OK;
    e = hipFuncSetAttribute(kernel, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e != hipSuccess) return fail(JV_ERR_HIP, "hipFuncSetAttribute: %s", hipGetErrorString(e));
    if (bit) state.devices_done.fetch_or(bit, std::memory_order_release);
    return JV_OK;
}

inline float resolve_scale(float scale, int head_dim) {  // default 1/sqrt(head_dim); NaN fails the comparison too
    return (scale > 0.0f) ? scale : (head_dim == kHeadDimWide ? 0.08838834764831845f : 0.125f);
}

// Window partition of an H x W grid (bottom/right padding, windows anchored at (0,0)).
struct WindowGeom {
    int H, W, wh, ww;
    int Hp, Wp, wins_x, wins_y, n_win, slots;  // slots = wh*ww
};
jv_status make_window_geom(int H, int W, int wh, int ww, WindowGeom *g);

// Mixer launchers on a validated problem (used by the C entry points and by the encoder).
size_t linear_workspace_bytes(int B, int heads, int N);
jv_status linear_forward(const Problem &pr, float eps, void *workspace, hipStream_t stream);
jv_status window_forward(const Problem &pr, int wh, int ww, float scale, hipStream_t stream);
jv_status full_forward(const Problem &pr, float scale, hipStream_t stream);

// Host-only checks of what the launchers above would refuse, so that a caller with several
// launches ahead (the encoder) can refuse before the first one.
jv_status window_check(const Problem &pr, int wh, int ww);
jv_status gemm_check_shape(long long M, int N, int K, long long lda = 0);

// y = epilogue(a w^T + bias) on the matrix cores (see jv_gemm_bias_act); lda: elements between
// rows of a (0 = K, i.e. contiguous rows), a multiple of 8.
jv_status gemm_forward(const void *a, const void *w, const float *bias, const void *residual,
                       void *y, long long M, int N, int K, int epi, bool out_bf16,
                       hipStream_t stream, long long lda = 0);

}  // namespace jv
