// Internal: launch plan of the two-pass linear attention and of the block's convolution branch,
// shared by the fp32 and bf16 paths.
#pragma once
#include "jv_common.h"

namespace jv {

constexpr int kStateFloats = kHeadDim * kHeadDim + kHeadDim;  // St[c2][c1] then z[c1]

struct LinearPlan {
    int n_split;       // token chunks per (batch, head) in the state pass
    int chunk;         // tokens per chunk (multiple of 256 unless it covers all of N)
    int apply_tokens;  // tokens per workgroup in the apply pass
    bool combine;      // sum the partial states in a pass of their own (many chunks)
};

LinearPlan plan_linear(int B, int heads, int N);
size_t linear_workspace_floats(const LinearPlan &p, int B, int heads);

// The depth-wise convolution branch of the block (Eq. 4) as the launchers see it.  Workspace
// regions (float offsets from the workspace base) follow the linear-attention states.
struct DwcPlan {
    int mode = JV_DWC_NONE;  // jv_dwc_mode
    int ksize = 3, hidden = 0;
    const float *static_kernel = nullptr, *w1 = nullptr, *b1 = nullptr, *w2 = nullptr, *b2 = nullptr;
    size_t vsum_off = 0;    // [n_split][B*heads][64] partial token sums of V (dynamic mode)
    size_t hidden_off = 0;  // [B][hidden] generator hidden layer (dynamic mode)
    size_t kappa_off = 0;   // [B][C][k*k] generated filters (dynamic mode)
    // Token-wise dynamic mode (regions of bf16 elements unless noted, offsets still in floats):
    size_t w1b_off = 0;     // [hidden][C] generator weights rounded to bf16
    size_t w2b_off = 0;     // [k*k][C][hidden]: rows reordered tap-major
    size_t b2p_off = 0;     // fp32 [k*k][C]: the second bias in the same order
    size_t vt_off = 0;      // [B*N][C] V as token rows, when its own layout is not such a matrix
    size_t u_off = 0;       // [B*N][hidden] hidden layer of every token
    size_t tok_kappa_off = 0;  // fp32 [B*N][k*k][C] filters of every token, tap-major
    size_t la_off = 0;      // fp32 [B*N][C] linear-attention term before the convolution is added
    size_t total_floats = 0;
};
// Fills the offsets for a validated parameter block; dwc may be null (mode none).  N = tokens
// per image (prefix included); only the token-wise mode sizes anything by it.
jv_status plan_dwc(const jv_dwc_params *dwc, const LinearPlan &lp, int B, int heads, int N, DwcPlan *out);

// What the apply kernels need of the convolution: filters [.., C, k*k] with a batch stride
// (0 for a static bank) on the H x W grid that follows P prefix tokens.
struct DwcArg {
    const float *kappa;
    long long kappa_sb;
    int H, W;
    int P;  // prefix tokens in front of the grid: token n is grid cell n - P; they take no part
};

// focus_p: 1 = ReLU feature map; >= 2 = focused map of Eq. 3 with that integer power.
jv_status linear_bf16(const Problem &pr, const LinearPlan &plan, float eps, float *ws,
                      const DwcPlan &dwc, int focus_p, hipStream_t stream);

// head_dim 128 (bf16 tensors): launch plan and workspace floats of the states; the state pass
// (with `vsum`, [n_split][B][C] floats, it also leaves the partial token sums of V), the apply
// pass (with `cv` it adds the block's convolution, filters of ksize x ksize taps), and both.
// Operands of a linear-attention block's output projection with the apply pass folded in
// (jv_encoder_fuse_linear_projection): states [B*heads][kStateFloats] fp32, w_fold [B][C][C] bf16,
// a_out [B*N][C] bf16; ws as for linear_bf16.
jv_status linear_fused_projection_operands(const Problem &pr, float eps, float *ws, float *states,
                                           const void *w_o, void *w_fold, void *a_out, hipStream_t stream);
LinearPlan plan_linear_wide(int B, int heads, int N);
size_t linear_wide_workspace_floats(int B, int heads, int N);
jv_status linear_wide_state(const Problem &pr, float *ws, float *vsum, hipStream_t stream);
jv_status linear_wide_apply(const Problem &pr, float eps, float *ws, hipStream_t stream, int ksize, const DwcArg *cv);
jv_status linear_wide_bf16(const Problem &pr, float eps, float *ws, hipStream_t stream);

// head_dim 128: the block's convolution branch (static or squeeze-dynamic filters); `base` =
// floats the linear-attention states take (linear_wide_workspace_floats).  dwc_wide_filters
// runs the generator on the token sums the state pass left (squeeze-dynamic mode) and fills the
// argument of the apply pass.
jv_status plan_dwc_wide(const jv_dwc_params *dwc, size_t base, int B, int heads, int N, DwcPlan *out);
jv_status dwc_wide_filters(const Problem &pr, const DwcPlan &dwc, float *ws, hipStream_t stream, DwcArg *out);

// Generator of the dynamic filters: partial token sums of V -> hidden layer -> filters.
jv_status squeeze_generate(const DwcPlan &dwc, float *ws, int n_part, int B, int heads, int N,
                           hipStream_t stream);

// fp32 tensors: partial token sums of V, and o += DWC(v) as a pass of its own.
jv_status vsum_f32_launch(const Problem &pr, const LinearPlan &plan, float *vsum, hipStream_t stream);
jv_status dwc_add_f32_launch(const Problem &pr, const DwcArg &cv, int ksize, hipStream_t stream);

// Token-wise dynamic filters (bf16 tensors): generator as two matrix products over all tokens,
// then o = la + DWC(v) with each token's own filters; la is the fp32 linear-attention term
// (pr.o itself when O is fp32).
jv_status token_dwc_forward(const Problem &pr, const TensorArg &la, const DwcPlan &dwc, float *ws,
                            hipStream_t stream);

// The same for fp32 tensors: pr.o already holds the linear-attention term; adds the convolution.
jv_status token_dwc_forward_f32(const Problem &pr, const DwcPlan &dwc, float *ws, hipStream_t stream);

jv_status linear_block_forward(const Problem &pr, float eps, const jv_dwc_params *dwc,
                               void *workspace, size_t workspace_bytes, hipStream_t stream,
                               int focus_p = 1);

}  // namespace jv
