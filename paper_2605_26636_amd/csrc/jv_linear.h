// Internal: launch plan of the two-pass linear attention, shared by the fp32 and bf16 paths.
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

jv_status linear_bf16(const Problem &pr, const LinearPlan &plan, float eps, float *ws,
                      hipStream_t stream);

}  // namespace jv
