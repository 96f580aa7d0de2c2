"""ctypes front end of the CPU oracle (oracle/jvoracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's CPU-baseline leg.  Nothing in the product package imports it, and
it imports nothing from the product package.

Inputs are numpy float32 arrays (bf16 test data widened exactly beforehand),
contiguous [B, heads, N, d]; results are float64.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        _lib = ctypes.CDLL(path)
    return _lib


def _f32(a):
    a = np.ascontiguousarray(a, dtype=np.float32)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def _rows(rows):
    r = np.ascontiguousarray(rows, dtype=np.int64).reshape(-1, 3)
    return r, r.ctypes.data_as(ctypes.c_void_p)


def _check(rc, name):
    if rc != 0:
        raise ValueError(f"oracle {name}: invalid argument")


def _shape4(q, k, v):
    if q.ndim != 4 or q.shape != k.shape or q.shape != v.shape:
        raise ValueError("q, k, v must share one [B, heads, N, d] shape")
    return q.shape


def full_attn(q, k, v, scale=None):
    """Eq. 1: softmax(q k^T * scale) v per (batch, head); scale defaults to 1/sqrt(d)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    o = np.empty(q.shape, dtype=np.float64)
    _check(lib().jvo_full_attn(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p),
                               B, h, N, d, ctypes.c_double(scale)), "full_attn")
    return o


def full_attn_rows(q, k, v, rows, scale=None):
    """Rows (b, head, i) of full attention -> [n_rows, d]."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    rows, rp = _rows(rows)
    o = np.empty((rows.shape[0], d), dtype=np.float64)
    _check(lib().jvo_full_attn_rows(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h, N, d,
                                    ctypes.c_double(scale), rp, rows.shape[0]), "full_attn_rows")
    return o


def full_attn_probs(q, k, scale=None):
    """Normalised probabilities [N, N] of one head (q, k are [N, d])."""
    q, qp = _f32(q); k, kp = _f32(k)
    N, d = q.shape
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    p = np.empty((N, N), dtype=np.float64)
    _check(lib().jvo_full_attn_probs(qp, kp, p.ctypes.data_as(ctypes.c_void_p), N, d,
                                     ctypes.c_double(scale)), "full_attn_probs")
    return p


def masked_attn(q, k, v, allow, scale=None):
    """Full attention restricted by a 0/1 mask allow[i, j] shared by all heads."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    allow = np.ascontiguousarray(allow, dtype=np.uint8)
    if allow.shape != (N, N):
        raise ValueError("allow must be [N, N]")
    o = np.empty(q.shape, dtype=np.float64)
    _check(lib().jvo_masked_attn(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h, N, d,
                                 ctypes.c_double(scale), allow.ctypes.data_as(ctypes.c_void_p)),
           "masked_attn")
    return o


def window_geometry(H, W, wh, ww):
    """(padded_h, padded_w, n_windows) of the bottom/right-padded grid."""
    Hp = ctypes.c_int(); Wp = ctypes.c_int(); nw = ctypes.c_int()
    _check(lib().jvo_window_geometry(H, W, wh, ww, ctypes.byref(Hp), ctypes.byref(Wp),
                                     ctypes.byref(nw)), "window_geometry")
    return Hp.value, Wp.value, nw.value


def window_maps(H, W, wh, ww):
    """(token_index int32 [n_win, wh*ww], pad_mask uint8 same, window_of_token int32 [H*W])."""
    _, _, nw = window_geometry(H, W, wh, ww)
    ti = np.empty((nw, wh * ww), dtype=np.int32)
    pm = np.empty((nw, wh * ww), dtype=np.uint8)
    wt = np.empty(H * W, dtype=np.int32)
    _check(lib().jvo_window_maps(H, W, wh, ww, ti.ctypes.data_as(ctypes.c_void_p),
                                 pm.ctypes.data_as(ctypes.c_void_p),
                                 wt.ctypes.data_as(ctypes.c_void_p)), "window_maps")
    return ti, pm, wt


def window_attn(q, k, v, H, W, wh, ww, scale=None):
    """Window attention on the H x W grid (N = H*W) with wh x ww windows."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    if N != H * W:
        raise ValueError("N != H*W")
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    o = np.empty(q.shape, dtype=np.float64)
    _check(lib().jvo_window_attn(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h, H, W, d,
                                 wh, ww, ctypes.c_double(scale)), "window_attn")
    return o


def window_attn_rows(q, k, v, H, W, wh, ww, rows, scale=None):
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    if N != H * W:
        raise ValueError("N != H*W")
    scale = 1.0 / np.sqrt(d) if scale is None else scale
    rows, rp = _rows(rows)
    o = np.empty((rows.shape[0], d), dtype=np.float64)
    _check(lib().jvo_window_attn_rows(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h, H, W,
                                      d, wh, ww, ctypes.c_double(scale), rp, rows.shape[0]),
           "window_attn_rows")
    return o


def prefix_window_allow(P, H, W, wh, ww):
    """0/1 matrix allow[i, j] of window attention on a sequence of P prefix tokens followed by the
    H x W grid (the library's stated rule; the paper gives none): a grid token sees the grid
    tokens of its own window and no prefix token; a prefix token sees every token."""
    _, _, wt = window_maps(H, W, wh, ww)
    N = P + H * W
    allow = np.zeros((N, N), dtype=np.uint8)
    allow[:P, :] = 1
    allow[P:, P:] = (wt[:, None] == wt[None, :]).astype(np.uint8)
    return allow


def window_attn_prefix(q, k, v, P, H, W, wh, ww, scale=None):
    """Window attention with P prefix tokens in front of the grid: masked full attention under
    prefix_window_allow."""
    return masked_attn(q, k, v, prefix_window_allow(P, H, W, wh, ww), scale)


def linear_attn_quadratic(q, k, v, eps=1e-6):
    """ReLU linear attention in its explicit N x N form (the reference form)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    o = np.empty(q.shape, dtype=np.float64)
    _check(lib().jvo_linear_attn_quadratic(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h,
                                           N, d, ctypes.c_double(eps)), "linear_attn_quadratic")
    return o


def linear_attn_rows(q, k, v, rows, eps=1e-6):
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    rows, rp = _rows(rows)
    o = np.empty((rows.shape[0], d), dtype=np.float64)
    _check(lib().jvo_linear_attn_rows(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p), B, h, N, d,
                                      ctypes.c_double(eps), rp, rows.shape[0]), "linear_attn_rows")
    return o


def linear_attn_state(q, k, v, eps=1e-6):
    """ReLU linear attention through the d x d state; returns (o, S, z)."""
    q, qp = _f32(q); k, kp = _f32(k); v, vp = _f32(v)
    B, h, N, d = _shape4(q, k, v)
    o = np.empty(q.shape, dtype=np.float64)
    S = np.empty((B, h, d, d), dtype=np.float64)
    z = np.empty((B, h, d), dtype=np.float64)
    _check(lib().jvo_linear_attn_state(qp, kp, vp, o.ctypes.data_as(ctypes.c_void_p),
                                       S.ctypes.data_as(ctypes.c_void_p),
                                       z.ctypes.data_as(ctypes.c_void_p), B, h, N, d,
                                       ctypes.c_double(eps)), "linear_attn_state")
    return o, S, z


# ---------------------------------------------------------------------------
# Encoder pieces and the depth-wise-convolution branch of the linear block
# ---------------------------------------------------------------------------
def _f64(a):
    a = np.ascontiguousarray(a, dtype=np.float64)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def layernorm(x, gamma, beta, eps=1e-6):
    """LayerNorm over the last axis (population variance); x float64 [..., C]."""
    x, xp = _f64(x)
    C = x.shape[-1]
    gamma, gp = _f32(gamma); beta, bp = _f32(beta)
    y = np.empty_like(x)
    _check(lib().jvo_layernorm(xp, gp, bp, y.ctypes.data_as(ctypes.c_void_p),
                               ctypes.c_int64(x.size // C), C, ctypes.c_double(eps)), "layernorm")
    return y


def linear(a, w, b=None):
    """y = a W^T + b with a float64 [..., K], W float32 [N, K], b float32 [N] or None."""
    a, ap = _f64(a)
    w, wp = _f32(w)
    N, K = w.shape
    if a.shape[-1] != K:
        raise ValueError("inner dimensions differ")
    bp = None
    if b is not None:
        b, bp = _f32(b)
    y = np.empty(a.shape[:-1] + (N,), dtype=np.float64)
    _check(lib().jvo_linear(ap, wp, bp, y.ctypes.data_as(ctypes.c_void_p),
                            ctypes.c_int64(a.size // K), N, K), "linear")
    return y


def gelu(x):
    """Exact (erf) GELU; returns a new float64 array."""
    y = np.array(x, dtype=np.float64, order="C", copy=True)
    _check(lib().jvo_gelu(y.ctypes.data_as(ctypes.c_void_p), ctypes.c_int64(y.size)), "gelu")
    return y


def dwc(v, kernel, H, W):
    """Depth-wise k x k cross-correlation of V [B, heads, H*W, d] with kernel [1 or B, C, k, k]."""
    v, vp = _f32(v)
    B, h, N, d = v.shape
    kernel, kp = _f64(kernel)
    kb, C, k, k2 = kernel.shape
    if N != H * W or C != h * d or k != k2:
        raise ValueError("shape mismatch")
    out = np.empty(v.shape, dtype=np.float64)
    _check(lib().jvo_dwc(vp, kp, out.ctypes.data_as(ctypes.c_void_p), B, h, H, W, d, k, kb), "dwc")
    return out


def squeeze_kernel(v, w1, b1, w2, b2, k):
    """Per-image depth-wise kernels [B, C, k, k] generated from mean_n V by Linear-SiLU-Linear."""
    v, vp = _f32(v)
    B, h, N, d = v.shape
    w1, w1p = _f32(w1); b1, b1p = _f32(b1); w2, w2p = _f32(w2); b2, b2p = _f32(b2)
    hidden, C = w1.shape
    if C != h * d or w2.shape != (C * k * k, hidden):
        raise ValueError("shape mismatch")
    kappa = np.empty((B, C, k, k), dtype=np.float64)
    _check(lib().jvo_squeeze_kernel(vp, w1p, b1p, w2p, b2p, kappa.ctypes.data_as(ctypes.c_void_p),
                                    B, h, N, d, k, hidden), "squeeze_kernel")
    return kappa


def tokenwise_kernels(v, w1, b1, w2, b2, k):
    """Filters of every token, [B, N, C, k, k]: the Linear-SiLU-Linear generator of the dynamic
    convolution applied to each token's own V row (channel = head * d + c) instead of the token
    average -- the per-token kernel generation the paper tried first (Sec. 3.2.1; Tab. 1,
    "Token-wise Dynamic DWC").  float64."""
    v = np.asarray(v, dtype=np.float64)
    B, h, N, d = v.shape
    w1 = np.asarray(w1, dtype=np.float64); b1 = np.asarray(b1, dtype=np.float64)
    w2 = np.asarray(w2, dtype=np.float64); b2 = np.asarray(b2, dtype=np.float64)
    C = h * d
    if w1.shape[1] != C or w2.shape != (C * k * k, w1.shape[0]):
        raise ValueError("shape mismatch")
    rows = v.transpose(0, 2, 1, 3).reshape(B, N, C)
    pre = rows @ w1.T + b1
    u = pre / (1.0 + np.exp(-pre))
    return (u @ w2.T + b2).reshape(B, N, C, k, k)


def dwc_tokenwise(v, kappa, H, W):
    """out[b, h, n, c] = sum_{di, dj} kappa[b, n, h*d + c, di, dj] * V[b, h, (r + di - k/2,
    s + dj - k/2), c] for grid token n = (r, s), zero outside the grid: a depth-wise
    cross-correlation in which the output token brings its own filters.  V [B, h, H*W, d],
    kappa [B, H*W, C, k, k]; float64."""
    v = np.asarray(v, dtype=np.float64)
    B, h, N, d = v.shape
    k = kappa.shape[-1]
    if N != H * W or kappa.shape != (B, N, h * d, k, k):
        raise ValueError("shape mismatch")
    pad = k // 2
    grid = np.zeros((B, h, H + 2 * pad, W + 2 * pad, d))
    grid[:, :, pad:pad + H, pad:pad + W] = v.reshape(B, h, H, W, d)
    kap = kappa.reshape(B, H, W, h, d, k, k).transpose(0, 3, 1, 2, 4, 5, 6)  # [B, h, H, W, d, k, k]
    out = np.zeros((B, h, H, W, d))
    for di in range(k):
        for dj in range(k):
            out += kap[..., di, dj] * grid[:, :, di:di + H, dj:dj + W]
    return out.reshape(B, h, N, d)


def focused_map(x, p):
    """Focused feature map, Eq. 3: phi_p(x) = |r| / |r^p| * r^p with r = max(x, 0), the power
    element-wise and the Euclidean norms over the last axis (the channels of one token's head).
    The printed denominator is read as the norm of the powered vector, which makes the map
    norm-preserving; rows with r = 0 map to 0.  float64."""
    r = np.maximum(np.asarray(x, dtype=np.float64), 0.0)
    y = r ** p
    nr = np.sqrt((r * r).sum(axis=-1, keepdims=True))
    ny = np.sqrt((y * y).sum(axis=-1, keepdims=True))
    return np.where(ny > 0, y * (nr / np.where(ny > 0, ny, 1.0)), 0.0)


def focused_linear_attn(q, k, v, p, eps=1e-6):
    """Linear attention in its quadratic form (Eq. 2, key-sum normaliser) with the focused map
    of Eq. 3 on queries and keys:  a_ij = phi_p(q_i) . phi_p(k_j);  o_i = sum_j a_ij v_j /
    (sum_j a_ij + eps).  [B, h, N, d] arrays, float64 arithmetic."""
    fq, fk = focused_map(q, p), focused_map(k, p)
    a = np.einsum("bhic,bhjc->bhij", fq, fk)
    num = np.einsum("bhij,bhjc->bhic", a, np.asarray(v, dtype=np.float64))
    return num / (a.sum(axis=-1, keepdims=True) + eps)


def linear_block(q, k, v, H, W, eps=1e-6, static_kernel=None, squeeze=None, ksize=3, focus_p=1,
                 token=None):
    """The paper's linear-attention block output, Eq. 4: normalised ReLU linear attention plus
    DWC(V).  static_kernel: [C, k, k]; squeeze: (w1, b1, w2, b2) for the dynamic kernel; token:
    the same four for the per-token variant (generator and convolution on the grid tokens);
    focus_p > 1: the focused map of Eq. 3 instead of ReLU (the variant Table 1 lists).
    Tokens beyond H * W are prefix tokens in front of the grid (the library's stated rule): they
    are ordinary tokens of the linear attention and of the token average that generates the
    dynamic filters, but the convolution runs over the grid tokens only."""
    P = q.shape[2] - H * W
    if P < 0:
        raise ValueError("fewer tokens than grid cells")
    o = linear_attn_quadratic(q, k, v, eps) if focus_p == 1 else focused_linear_attn(q, k, v, focus_p, eps)
    vg = np.ascontiguousarray(np.asarray(v)[:, :, P:])
    if static_kernel is not None:
        o[:, :, P:] += dwc(vg, np.asarray(static_kernel, dtype=np.float64)[None], H, W)
    if squeeze is not None:
        o[:, :, P:] += dwc(vg, squeeze_kernel(v, *squeeze, ksize), H, W)
    if token is not None:
        o[:, :, P:] += dwc_tokenwise(vg, tokenwise_kernels(vg, *token, ksize), H, W)
    return o


MIX_LINEAR, MIX_WINDOW, MIX_FULL = 0, 1, 2


def encoder_block(x, wts, mixer, H, W, heads, window=(16, 16), ln_eps=1e-6, la_eps=1e-6, la_focus_p=1,
                  n_prefix=0):
    """One pre-LN block:  x += W_O mix(split_heads(W_qkv LN(x))) + b_O;  x += MLP(LN(x)).
    x float64 [B, N, C]; wts: dict of float32 arrays (ln1_g, ln1_b, w_qkv [3C, C], b_qkv, w_o,
    b_o, ln2_g, ln2_b, w_fc1, b_fc1, w_fc2, b_fc2; optionally "dwc": dict with static_kernel or
    squeeze = (w1, b1, w2, b2), and ksize, for a linear-attention block).  Q, K, V reach the mixer routines as
    float32 (their input type): a 2^-24 rounding, far below every tolerance used."""
    B, N, C = x.shape
    d = C // heads
    a = layernorm(x, wts["ln1_g"], wts["ln1_b"], ln_eps)
    qkv = linear(a, wts["w_qkv"], wts["b_qkv"]).reshape(B, N, 3, heads, d)
    q, k, v = (np.ascontiguousarray(qkv[:, :, i].transpose(0, 2, 1, 3)).astype(np.float32)
               for i in range(3))
    if mixer == MIX_LINEAR:
        dwc_cfg = wts.get("dwc") or {}   # the block's convolution branch (Eq. 4), if it has one
        if dwc_cfg or la_focus_p > 1 or n_prefix > 0:
            o = linear_block(q, k, v, H, W, la_eps, static_kernel=dwc_cfg.get("static_kernel"),
                             squeeze=dwc_cfg.get("squeeze"), ksize=dwc_cfg.get("ksize", 3),
                             focus_p=la_focus_p, token=dwc_cfg.get("token"))
        else:
            o = linear_attn_quadratic(q, k, v, la_eps)
    elif mixer == MIX_WINDOW:
        o = (window_attn(q, k, v, H, W, window[0], window[1]) if n_prefix == 0
             else window_attn_prefix(q, k, v, n_prefix, H, W, window[0], window[1]))
    else:
        o = full_attn(q, k, v)
    o = o.transpose(0, 2, 1, 3).reshape(B, N, C)
    x = x + linear(o, wts["w_o"], wts["b_o"])
    m = layernorm(x, wts["ln2_g"], wts["ln2_b"], ln_eps)
    hmid = gelu(linear(m, wts["w_fc1"], wts["b_fc1"]))
    return x + linear(hmid, wts["w_fc2"], wts["b_fc2"])


def encoder_forward(x, blocks, pattern, H, W, heads, window=(16, 16), ln_eps=1e-6, la_eps=1e-6,
                    taps=None, la_focus_p=1, n_prefix=0):
    """Hybrid encoder: blocks[l] run with mixer pattern[l]; returns the residual stream.  With
    taps (an iterable of block indices) returns (stream, {l: stream after block l}): the
    intermediate features a dense-prediction head reads (Sec. 4.1, 4.2)."""
    x = np.asarray(x, dtype=np.float64)
    kept = {}
    for l, (wts, mixer) in enumerate(zip(blocks, pattern)):
        x = encoder_block(x, wts, mixer, H, W, heads, window, ln_eps, la_eps, la_focus_p, n_prefix)
        if taps is not None and l in taps:
            kept[l] = x.copy()
    return x if taps is None else (x, kept)
