// Host-side entry points that launch nothing: version, status strings, error
// text, descriptor validation, window geometry.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>

#include "jv_common.h"

namespace jv {

static thread_local char g_err[512] = "";

jv_status fail(jv_status st, const char *fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

void clear_error() { g_err[0] = '\0'; }

static bool dtype_ok(jv_dtype t) { return t == JV_F32 || t == JV_BF16; }

static jv_status check_strides(const char *name, const jv_strides &s, int64_t align_elems, int head_dim) {
    if (s.stride_n < head_dim) return fail(JV_ERR_INVALID_ARG, "%s: stride_n < head_dim", name);
    if (s.stride_b < 0 || s.stride_h < 0)
        return fail(JV_ERR_INVALID_ARG, "%s: negative stride", name);
    if (s.stride_b % align_elems || s.stride_h % align_elems || s.stride_n % align_elems)
        return fail(JV_ERR_INVALID_ARG, "%s: strides must keep rows 16-byte aligned", name);
    return JV_OK;
}

jv_status check_desc(const jv_attn_desc *d) {
    if (!d) return fail(JV_ERR_INVALID_ARG, "descriptor is null");
    if (d->batch <= 0 || d->heads <= 0 || d->grid_h <= 0 || d->grid_w <= 0)
        return fail(JV_ERR_INVALID_ARG, "batch, heads, grid_h, grid_w must be positive");
    if ((int64_t)d->grid_h * d->grid_w > (1 << 24))
        return fail(JV_ERR_UNSUPPORTED, "more than 2^24 tokens per image");
    if (d->n_prefix < 0 || d->n_prefix > 64)
        return fail(JV_ERR_INVALID_ARG, "n_prefix must be 0 .. 64");
    if ((int64_t)d->batch * d->heads > 65535)
        return fail(JV_ERR_UNSUPPORTED, "batch * heads above 65535");
    if (d->head_dim <= 0) return fail(JV_ERR_INVALID_ARG, "head_dim must be positive");
    if (d->head_dim != kHeadDim && d->head_dim != kHeadDimWide)
        return fail(JV_ERR_UNSUPPORTED, "head_dim must be 64 or 128");
    if (!dtype_ok(d->dtype) || !dtype_ok(d->o_dtype))
        return fail(JV_ERR_INVALID_ARG, "unknown dtype");
    if (d->head_dim == kHeadDimWide && d->dtype != JV_BF16)
        return fail(JV_ERR_UNSUPPORTED, "head_dim 128 is built for bf16 tensors only");
    if (d->dtype == JV_F32 && d->o_dtype != JV_F32)
        return fail(JV_ERR_UNSUPPORTED, "fp32 inputs need an fp32 output");
    const int64_t in_align = d->dtype == JV_BF16 ? 8 : 4;
    const int64_t out_align = d->o_dtype == JV_BF16 ? 8 : 4;
    jv_status st;
    if ((st = check_strides("q", d->q, in_align, d->head_dim)) != JV_OK) return st;
    if ((st = check_strides("k", d->k, in_align, d->head_dim)) != JV_OK) return st;
    if ((st = check_strides("v", d->v, in_align, d->head_dim)) != JV_OK) return st;
    if ((st = check_strides("o", d->o, out_align, d->head_dim)) != JV_OK) return st;
    return JV_OK;
}

jv_status make_problem(const jv_attn_desc *d, const void *q, const void *k, const void *v,
                       void *o, Problem *p) {
    jv_status st = check_desc(d);
    if (st != JV_OK) return st;
    if (!q || !k || !v || !o) return fail(JV_ERR_INVALID_ARG, "q, k, v, o must be non-null");
    if (((uintptr_t)q | (uintptr_t)k | (uintptr_t)v | (uintptr_t)o) & 15)
        return fail(JV_ERR_INVALID_ARG, "q, k, v, o must be 16-byte aligned");
    // O may not overlap an input: compare the byte ranges the four tensors span.
    const int64_t N = d->n_prefix + (int64_t)d->grid_h * d->grid_w;
    auto span = [&](const jv_strides &t, int64_t esz) {
        return ((d->batch - 1) * t.stride_b + (d->heads - 1) * t.stride_h + (N - 1) * t.stride_n + d->head_dim) * esz;
    };
    const int64_t in_esz = d->dtype == JV_BF16 ? 2 : 4, out_esz = d->o_dtype == JV_BF16 ? 2 : 4;
    const uintptr_t o0 = (uintptr_t)o, o1 = o0 + (uintptr_t)span(d->o, out_esz);
    const void *ins[3] = {q, k, v};
    const jv_strides *in_strides[3] = {&d->q, &d->k, &d->v};
    for (int i = 0; i < 3; ++i) {
        const uintptr_t i0 = (uintptr_t)ins[i], i1 = i0 + (uintptr_t)span(*in_strides[i], in_esz);
        if (o0 < i1 && i0 < o1) return fail(JV_ERR_INVALID_ARG, "o must not overlap an input");
    }
    p->B = d->batch;
    p->heads = d->heads;
    p->H = d->grid_h;
    p->W = d->grid_w;
    p->P = d->n_prefix;
    p->N = d->n_prefix + d->grid_h * d->grid_w;
    p->D = d->head_dim;
    p->bf16 = d->dtype == JV_BF16;
    p->o_bf16 = d->o_dtype == JV_BF16;
    p->q = {q, d->q.stride_b, d->q.stride_h, d->q.stride_n};
    p->k = {k, d->k.stride_b, d->k.stride_h, d->k.stride_n};
    p->v = {v, d->v.stride_b, d->v.stride_h, d->v.stride_n};
    p->o = {o, d->o.stride_b, d->o.stride_h, d->o.stride_n};
    return JV_OK;
}

jv_status make_window_geom(int H, int W, int wh, int ww, WindowGeom *g) {
    if (H <= 0 || W <= 0) return fail(JV_ERR_INVALID_ARG, "grid must be positive");
    if (wh <= 0 || ww <= 0) return fail(JV_ERR_INVALID_ARG, "window must be positive");
    if ((int64_t)H * W > (1 << 24)) return fail(JV_ERR_UNSUPPORTED, "more than 2^24 tokens");
    if (wh > (1 << 14) || ww > (1 << 14))
        return fail(JV_ERR_UNSUPPORTED, "window side above 16384");
    g->H = H; g->W = W; g->wh = wh; g->ww = ww;
    g->wins_y = (H + wh - 1) / wh;
    g->wins_x = (W + ww - 1) / ww;
    g->Hp = g->wins_y * wh;
    g->Wp = g->wins_x * ww;
    if ((int64_t)g->Hp * g->Wp > 0x7fffffffll)
        return fail(JV_ERR_UNSUPPORTED, "padded grid above 2^31 - 1 cells");
    g->n_win = g->wins_x * g->wins_y;
    g->slots = wh * ww;  // at most 2^28
    return JV_OK;
}

}  // namespace jv

extern "C" {

const char *jv_version(void) { return "jetvit-mi355x 0.1 (gfx950)"; }

const char *jv_status_string(jv_status s) {
    switch (s) {
        case JV_OK: return "ok";
        case JV_ERR_INVALID_ARG: return "invalid argument";
        case JV_ERR_UNSUPPORTED: return "unsupported";
        case JV_ERR_WORKSPACE_TOO_SMALL: return "workspace too small";
        case JV_ERR_HIP: return "HIP runtime error";
    }
    return "unknown status";
}

const char *jv_last_error(void) { return jv::g_err; }

jv_status jv_window_geometry(int32_t grid_h, int32_t grid_w, int32_t win_h, int32_t win_w,
                             int32_t *padded_h, int32_t *padded_w, int32_t *n_windows) {
    jv::clear_error();
    jv::WindowGeom g;
    jv_status st = jv::make_window_geom(grid_h, grid_w, win_h, win_w, &g);
    if (st != JV_OK) return st;
    if (!padded_h || !padded_w || !n_windows)
        return jv::fail(JV_ERR_INVALID_ARG, "output pointers must be non-null");
    *padded_h = g.Hp;
    *padded_w = g.Wp;
    *n_windows = g.n_win;
    return JV_OK;
}

}  // extern "C"
