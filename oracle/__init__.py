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
