#include "jv_common.h"
namespace jv {
struct LinearPlan { int n_split, chunk, apply_tokens; };
jv_status linear_bf16(const Problem &, const LinearPlan &, float, float *, hipStream_t) {
    return fail(JV_ERR_UNSUPPORTED, "bf16 linear attention is not built yet");
}
}
