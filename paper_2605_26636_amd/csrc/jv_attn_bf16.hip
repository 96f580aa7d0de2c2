#include "jv_common.h"
namespace jv {
jv_status attn_bf16(const Problem &, const WindowGeom &, float, hipStream_t) {
    return fail(JV_ERR_UNSUPPORTED, "bf16 attention is not built yet");
}
}
