"""Thin ctypes binding of libjetvit.so (include/jetvit.h).

Argument marshalling only: every computation runs inside the library's HIP
kernels.  Tensors are torch tensors on the GPU (torch is used for device memory
and streams); the functions carry the names of the C entry points.  There is no
CPU fallback: a missing library or a non-OK status raises.
"""
import ctypes
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libjetvit.so")

JV_OK, JV_ERR_INVALID_ARG, JV_ERR_UNSUPPORTED, JV_ERR_WORKSPACE_TOO_SMALL, JV_ERR_HIP = range(5)
JV_F32, JV_BF16 = 0, 1

EXPORTS = [
    "jv_version", "jv_status_string", "jv_last_error",
    "jv_linear_attn_workspace_bytes", "jv_linear_attn_fwd", "jv_linear_attn_fwd_static",
    "jv_linear_block_workspace_bytes", "jv_linear_block_fwd", "jv_linear_block_focused_fwd",
    "jv_window_geometry", "jv_window_maps_host", "jv_window_maps_device",
    "jv_window_attn_fwd", "jv_full_attn_fwd",
    "jv_layernorm_fwd", "jv_gemm_bias_act",
    "jv_encoder_create", "jv_encoder_workspace_bytes", "jv_encoder_forward", "jv_encoder_forward_taps", "jv_encoder_destroy",
    "jv_encoder_fold_bytes", "jv_encoder_fold_layernorm", "jv_encoder_fuse_linear_projection",
]
JV_EPI_NONE, JV_EPI_GELU, JV_EPI_RESIDUAL, JV_EPI_SILU = 0, 1, 2, 3
JV_DWC_NONE, JV_DWC_STATIC, JV_DWC_SQUEEZE_DYNAMIC, JV_DWC_TOKEN_DYNAMIC = 0, 1, 2, 3


class JvStrides(ctypes.Structure):
    _fields_ = [("stride_b", ctypes.c_int64), ("stride_h", ctypes.c_int64),
                ("stride_n", ctypes.c_int64)]


class JvAttnDesc(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("grid_h", ctypes.c_int32), ("grid_w", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("dtype", ctypes.c_int), ("o_dtype", ctypes.c_int),
                ("q", JvStrides), ("k", JvStrides), ("v", JvStrides), ("o", JvStrides),
                ("n_prefix", ctypes.c_int32)]


class JvDwcParams(ctypes.Structure):
    _fields_ = [("mode", ctypes.c_int), ("ksize", ctypes.c_int32), ("hidden", ctypes.c_int32),
                ("static_kernel", ctypes.c_void_p), ("w1", ctypes.c_void_p), ("b1", ctypes.c_void_p),
                ("w2", ctypes.c_void_p), ("b2", ctypes.c_void_p)]


class JvEncoderConfig(ctypes.Structure):
    _fields_ = [("n_blocks", ctypes.c_int32), ("width", ctypes.c_int32), ("heads", ctypes.c_int32),
                ("mlp_hidden", ctypes.c_int32), ("win_h", ctypes.c_int32), ("win_w", ctypes.c_int32),
                ("ln_eps", ctypes.c_float), ("la_eps", ctypes.c_float),
                ("pattern", ctypes.POINTER(ctypes.c_uint8)), ("la_focus_p", ctypes.c_int32),
                ("n_prefix", ctypes.c_int32), ("stream_dtype", ctypes.c_int32)]


BLOCK_FIELDS = ["ln1_g", "ln1_b", "w_qkv", "b_qkv", "w_o", "b_o", "ln2_g", "ln2_b", "w_fc1", "b_fc1",
                "w_fc2", "b_fc2"]


class JvBlockWeights(ctypes.Structure):
    _fields_ = [(name, ctypes.c_void_p) for name in BLOCK_FIELDS] + [("dwc", ctypes.POINTER(JvDwcParams))]


class JvError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"jetvit status {status}: {text}")
        self.status = status


_lib = None


def lib():
    """Load libjetvit.so (built in-tree by build.py); fails loudly when it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2605_26636_amd.build` "
                               "(there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        L.jv_version.restype = ctypes.c_char_p
        L.jv_status_string.restype = ctypes.c_char_p
        L.jv_last_error.restype = ctypes.c_char_p
        L.jv_linear_attn_workspace_bytes.restype = ctypes.c_size_t
        L.jv_linear_attn_workspace_bytes.argtypes = [ctypes.POINTER(JvAttnDesc)]
        vp = ctypes.c_void_p
        L.jv_linear_attn_fwd.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp,
                                         ctypes.c_float, vp, ctypes.c_size_t, vp]
        L.jv_linear_attn_fwd_static.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp, ctypes.c_float, vp]
        L.jv_linear_block_workspace_bytes.restype = ctypes.c_size_t
        L.jv_linear_block_workspace_bytes.argtypes = [ctypes.POINTER(JvAttnDesc),
                                                      ctypes.POINTER(JvDwcParams)]
        L.jv_linear_block_fwd.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp, ctypes.c_float,
                                          ctypes.POINTER(JvDwcParams), vp, ctypes.c_size_t, vp]
        L.jv_linear_block_focused_fwd.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp, ctypes.c_float,
                                                  ctypes.c_int32, ctypes.POINTER(JvDwcParams), vp, ctypes.c_size_t, vp]
        L.jv_window_attn_fwd.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp,
                                         ctypes.c_int32, ctypes.c_int32, ctypes.c_float, vp]
        L.jv_full_attn_fwd.argtypes = [ctypes.POINTER(JvAttnDesc), vp, vp, vp, vp,
                                       ctypes.c_float, vp]
        i32 = ctypes.c_int32
        L.jv_window_geometry.argtypes = [i32, i32, i32, i32, vp, vp, vp]
        L.jv_window_maps_host.argtypes = [i32, i32, i32, i32, vp, vp, vp]
        L.jv_window_maps_device.argtypes = [i32, i32, i32, i32, vp, vp, vp, vp]
        i64 = ctypes.c_int64
        L.jv_layernorm_fwd.argtypes = [vp, vp, vp, vp, i64, i32, ctypes.c_float, ctypes.c_int,
                                       ctypes.c_int, vp]
        L.jv_gemm_bias_act.argtypes = [vp, vp, vp, vp, vp, i64, i32, i32, ctypes.c_int,
                                       ctypes.c_int, vp]
        L.jv_encoder_create.argtypes = [ctypes.POINTER(JvEncoderConfig),
                                        ctypes.POINTER(JvBlockWeights), ctypes.POINTER(vp)]
        L.jv_encoder_workspace_bytes.restype = ctypes.c_size_t
        L.jv_encoder_workspace_bytes.argtypes = [vp, i32, i32, i32]
        L.jv_encoder_forward.argtypes = [vp, vp, vp, i32, i32, i32, vp, ctypes.c_size_t, vp]
        L.jv_encoder_forward_taps.argtypes = [vp, vp, vp, i32, i32, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
        L.jv_encoder_fold_bytes.restype = ctypes.c_size_t
        L.jv_encoder_fold_bytes.argtypes = [vp]
        L.jv_encoder_fold_layernorm.argtypes = [vp, vp, ctypes.c_size_t, vp]
        L.jv_encoder_fuse_linear_projection.argtypes = [vp, i32]
        L.jv_encoder_destroy.restype = None
        L.jv_encoder_destroy.argtypes = [vp]
        _lib = L
    return _lib


def _check(status):
    if status != JV_OK:
        raise JvError(status, lib().jv_last_error().decode() or
                      lib().jv_status_string(status).decode())


def _dtype_code(t):
    if t.dtype == torch.float32:
        return JV_F32
    if t.dtype == torch.bfloat16:
        return JV_BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _strides(t):
    if t.dim() != 4 or t.stride(3) != 1:
        raise ValueError("tensors must be [batch, heads, N, head_dim] views with a contiguous last axis")
    return JvStrides(t.stride(0), t.stride(1), t.stride(2))


def make_desc(q, k, v, o, grid):
    """Descriptor for [B, heads, N, d] tensor views q, k, v, o on an H x W grid; tokens beyond
    H * W are prefix tokens in front of the grid (N = n_prefix + H * W)."""
    B, heads, N, d = q.shape
    H, W = grid
    if N < H * W:
        raise ValueError("fewer tokens than grid cells")
    for t in (k, v, o):
        if tuple(t.shape) != (B, heads, N, d):
            raise ValueError("q, k, v, o must share one shape")
    if not (q.dtype == k.dtype == v.dtype):
        raise TypeError("q, k, v must share one dtype")
    for t in (q, k, v, o):
        if not t.is_cuda:
            raise ValueError("tensors must live on the GPU")
    return JvAttnDesc(B, heads, H, W, d, _dtype_code(q), _dtype_code(o),
                      _strides(q), _strides(k), _strides(v), _strides(o), N - H * W)


def _stream(stream):
    s = torch.cuda.current_stream() if stream is None else stream
    return ctypes.c_void_p(s.cuda_stream)


def jv_version():
    return lib().jv_version().decode()


def jv_linear_attn_workspace_bytes(desc):
    return int(lib().jv_linear_attn_workspace_bytes(ctypes.byref(desc)))


def jv_linear_attn_fwd(q, k, v, o, grid, eps=1e-6, workspace=None, stream=None):
    """o <- ReLU linear attention of (q, k, v); returns the workspace tensor used."""
    desc = make_desc(q, k, v, o, grid)
    need = jv_linear_attn_workspace_bytes(desc)
    if workspace is None:
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().jv_linear_attn_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                    o.data_ptr(), eps, workspace.data_ptr(),
                                    workspace.numel() * workspace.element_size(), _stream(stream)))
    return workspace


JV_STATIC_SCRATCH_BYTES = 32 << 20


def jv_linear_attn_fwd_static(q, k, v, o, grid, eps=1e-6, stream=None):
    """o <- ReLU linear attention of (q, k, v) through the entry point that takes its scratch from
    the library's fixed device array (allocates nothing)."""
    desc = make_desc(q, k, v, o, grid)
    _check(lib().jv_linear_attn_fwd_static(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                           o.data_ptr(), eps, _stream(stream)))


def make_dwc_params(static_kernel=None, squeeze=None, ksize=3, token=None):
    """jv_dwc_params from device fp32 tensors: static_kernel [C, k, k], or squeeze =
    (w1 [hidden, C], b1 [hidden], w2 [C*k*k, hidden], b2 [C*k*k]) for per-image filters, or
    token = the same four tensors for per-token filters; none of them = no convolution."""
    if (static_kernel is not None) + (squeeze is not None) + (token is not None) > 1:
        raise ValueError("give a static kernel or one set of generator weights, not several")
    for t in ([static_kernel] if static_kernel is not None else []) + list(squeeze or []) + list(token or []):
        if t.dtype != torch.float32 or not t.is_cuda or not t.is_contiguous():
            raise ValueError("convolution parameters must be contiguous fp32 device tensors")
    if static_kernel is not None:
        return JvDwcParams(JV_DWC_STATIC, ksize, 0, static_kernel.data_ptr(), None, None, None, None)
    if squeeze is not None:
        w1, b1, w2, b2 = squeeze
        return JvDwcParams(JV_DWC_SQUEEZE_DYNAMIC, ksize, w1.shape[0], None, w1.data_ptr(),
                           b1.data_ptr(), w2.data_ptr(), b2.data_ptr())
    if token is not None:
        w1, b1, w2, b2 = token
        return JvDwcParams(JV_DWC_TOKEN_DYNAMIC, ksize, w1.shape[0], None, w1.data_ptr(),
                           b1.data_ptr(), w2.data_ptr(), b2.data_ptr())
    return JvDwcParams(JV_DWC_NONE, ksize, 0, None, None, None, None, None)


def jv_linear_block_workspace_bytes(desc, dwc):
    return int(lib().jv_linear_block_workspace_bytes(ctypes.byref(desc), ctypes.byref(dwc)))


def jv_linear_block_fwd(q, k, v, o, grid, eps=1e-6, static_kernel=None, squeeze=None, ksize=3,
                        workspace=None, stream=None, token=None):
    """o <- linear attention + depth-wise convolution of v (the paper's linear-attention block);
    returns the workspace tensor used."""
    desc = make_desc(q, k, v, o, grid)
    dwc = make_dwc_params(static_kernel, squeeze, ksize, token)
    if workspace is None:
        need = jv_linear_block_workspace_bytes(desc, dwc)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().jv_linear_block_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                     o.data_ptr(), eps, ctypes.byref(dwc), workspace.data_ptr(),
                                     workspace.numel() * workspace.element_size(), _stream(stream)))
    return workspace


def jv_linear_block_focused_fwd(q, k, v, o, grid, focus_p, eps=1e-6, static_kernel=None, squeeze=None,
                                ksize=3, workspace=None, stream=None, token=None):
    """The linear-attention block with the focused feature map of power focus_p in place of
    ReLU; returns the workspace tensor used."""
    desc = make_desc(q, k, v, o, grid)
    dwc = make_dwc_params(static_kernel, squeeze, ksize, token)
    if workspace is None:
        need = jv_linear_block_workspace_bytes(desc, dwc)
        workspace = torch.empty(max(need, 256), dtype=torch.uint8, device=q.device)
    _check(lib().jv_linear_block_focused_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                             o.data_ptr(), eps, focus_p, ctypes.byref(dwc),
                                             workspace.data_ptr(),
                                             workspace.numel() * workspace.element_size(), _stream(stream)))
    return workspace


def jv_window_attn_fwd(q, k, v, o, grid, window, scale=0.0, stream=None):
    desc = make_desc(q, k, v, o, grid)
    _check(lib().jv_window_attn_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                    o.data_ptr(), window[0], window[1], scale, _stream(stream)))


def jv_full_attn_fwd(q, k, v, o, grid, scale=0.0, stream=None):
    desc = make_desc(q, k, v, o, grid)
    _check(lib().jv_full_attn_fwd(ctypes.byref(desc), q.data_ptr(), k.data_ptr(), v.data_ptr(),
                                  o.data_ptr(), scale, _stream(stream)))


def jv_window_geometry(grid_h, grid_w, win_h, win_w):
    """(padded_h, padded_w, n_windows); host computation."""
    out = (ctypes.c_int32 * 3)()
    base = ctypes.addressof(out)
    _check(lib().jv_window_geometry(grid_h, grid_w, win_h, win_w, base, base + 4, base + 8))
    return out[0], out[1], out[2]


def jv_window_maps_host(grid_h, grid_w, win_h, win_w):
    """(token_index, pad_mask, window_of_token) as numpy arrays, computed on the host."""
    import numpy as np
    _, _, nw = jv_window_geometry(grid_h, grid_w, win_h, win_w)
    ti = np.empty((nw, win_h * win_w), dtype=np.int32)
    pm = np.empty((nw, win_h * win_w), dtype=np.uint8)
    wt = np.empty(grid_h * grid_w, dtype=np.int32)
    _check(lib().jv_window_maps_host(grid_h, grid_w, win_h, win_w, ti.ctypes.data, pm.ctypes.data,
                                     wt.ctypes.data))
    return ti, pm, wt


def jv_window_maps_device(grid_h, grid_w, win_h, win_w, device="cuda", stream=None):
    """(token_index, pad_mask, window_of_token) as device tensors, computed by a kernel."""
    _, _, nw = jv_window_geometry(grid_h, grid_w, win_h, win_w)
    ti = torch.empty((nw, win_h * win_w), dtype=torch.int32, device=device)
    pm = torch.empty((nw, win_h * win_w), dtype=torch.uint8, device=device)
    wt = torch.empty(grid_h * grid_w, dtype=torch.int32, device=device)
    _check(lib().jv_window_maps_device(grid_h, grid_w, win_h, win_w, ti.data_ptr(), pm.data_ptr(),
                                       wt.data_ptr(), _stream(stream)))
    return ti, pm, wt


def jv_layernorm_fwd(x, gamma, beta, y, eps=1e-6, stream=None):
    """y <- LayerNorm(x) over the last axis; x fp32/bf16 [rows, cols], y bf16/fp32, gamma/beta fp32."""
    rows, cols = x.shape
    if not (x.is_contiguous() and y.is_contiguous() and tuple(y.shape) == (rows, cols)):
        raise ValueError("x and y must be contiguous [rows, cols]")
    _check(lib().jv_layernorm_fwd(x.data_ptr(), gamma.data_ptr(), beta.data_ptr(), y.data_ptr(),
                                  rows, cols, eps, _dtype_code(x), _dtype_code(y), _stream(stream)))


def jv_gemm_bias_act(a, w, bias, residual, y, epilogue=JV_EPI_NONE, stream=None):
    """y <- epilogue(a w^T + bias); a bf16 [M, K], w bf16 [N, K], bias fp32 [N] or None,
    y bf16 or fp32 [M, N], residual None or [M, N] of y's element type."""
    M, K = a.shape
    N = w.shape[0]
    if w.shape[1] != K or tuple(y.shape) != (M, N):
        raise ValueError("shape mismatch")
    for t in (a, w, y):
        if not t.is_contiguous():
            raise ValueError("operands must be contiguous")
    if a.dtype != torch.bfloat16 or w.dtype != torch.bfloat16:
        raise TypeError("a and w must be bf16")
    if residual is not None and (residual.dtype != y.dtype or tuple(residual.shape) != (M, N)
                                 or not residual.is_contiguous()):
        raise TypeError("residual must be a contiguous [M, N] tensor of y's element type")
    _check(lib().jv_gemm_bias_act(a.data_ptr(), w.data_ptr(),
                                  None if bias is None else bias.data_ptr(),
                                  None if residual is None else residual.data_ptr(), y.data_ptr(),
                                  M, N, K, epilogue, _dtype_code(y), _stream(stream)))


class Encoder:
    """Handle of a jv_encoder.  `blocks` is a list of dicts of device tensors (BLOCK_FIELDS:
    weights bf16, biases and LayerNorm parameters fp32); the tensors are kept alive here."""

    def __init__(self, blocks, pattern, heads, mlp_hidden, window=(16, 16), ln_eps=1e-6, la_eps=1e-6,
                 la_focus_p=1, n_prefix=0, stream_dtype=torch.float32, fold_layernorm=False):
        self.blocks = blocks
        self.width = blocks[0]["w_o"].shape[0]
        n = len(blocks)
        self._pattern = (ctypes.c_uint8 * n)(*pattern)
        cfg = JvEncoderConfig(n, self.width, heads, mlp_hidden, window[0], window[1], ln_eps, la_eps,
                              ctypes.cast(self._pattern, ctypes.POINTER(ctypes.c_uint8)), la_focus_p, n_prefix,
                              JV_BF16 if stream_dtype == torch.bfloat16 else JV_F32)
        if stream_dtype not in (torch.float32, torch.bfloat16):
            raise TypeError("the residual stream is fp32 or bf16")
        self.stream_dtype = stream_dtype
        table = (JvBlockWeights * n)()
        self._dwc = []   # parameter structs stay alive until the encoder has copied them
        for i, b in enumerate(blocks):
            for name in BLOCK_FIELDS:
                setattr(table[i], name, b[name].data_ptr())
            # optional convolution branch of a linear-attention block: b["dwc"] is a dict with
            # "static_kernel", "squeeze" or "token" (tuple of device tensors) and "ksize"
            if b.get("dwc") is not None:
                d = b["dwc"]
                params = make_dwc_params(d.get("static_kernel"), d.get("squeeze"), d.get("ksize", 3), d.get("token"))
                self._dwc.append(params)
                table[i].dwc = ctypes.pointer(params)
        self._handle = ctypes.c_void_p()
        _check(lib().jv_encoder_create(ctypes.byref(cfg), table, ctypes.byref(self._handle)))
        self._folded = None
        if fold_layernorm:
            self.fold_layernorm()

    def fold_layernorm(self, enable=True, stream=None):
        """Fold the LayerNorms into the products behind them (jv_encoder_fold_layernorm): the
        folded weights live in a device tensor kept alive here."""
        if not enable:
            _check(lib().jv_encoder_fold_layernorm(self._handle, None, 0, _stream(stream)))
            self._folded = None
            return
        need = int(lib().jv_encoder_fold_bytes(self._handle))
        buf = torch.empty(max(need, 256), dtype=torch.uint8, device=self.blocks[0]["w_o"].device)
        _check(lib().jv_encoder_fold_layernorm(self._handle, buf.data_ptr(), buf.numel(), _stream(stream)))
        self._folded = buf

    def fuse_linear_projection(self, enable=True):
        """Fold the apply pass of the linear-attention blocks into their output projection
        (jv_encoder_fuse_linear_projection)."""
        _check(lib().jv_encoder_fuse_linear_projection(self._handle, 1 if enable else 0))

    def workspace_bytes(self, batch, grid):
        return int(lib().jv_encoder_workspace_bytes(self._handle, batch, grid[0], grid[1]))

    def forward(self, x, y, grid, workspace=None, stream=None, taps=None):
        """y <- encoder(x); x, y [batch, N, width] of the stream's element type on the GPU; returns
        the workspace used.  taps: optional dict {block index: tensor like y} that receives the
        residual stream after those blocks (jv_encoder_forward_taps)."""
        batch = x.shape[0]
        sd = self.stream_dtype
        if x.dtype != sd or y.dtype != sd or not x.is_contiguous() or not y.is_contiguous():
            raise ValueError("x and y must be contiguous tensors of the stream's element type")
        if workspace is None:
            workspace = torch.empty(self.workspace_bytes(batch, grid), dtype=torch.uint8, device=x.device)
        if not taps:
            _check(lib().jv_encoder_forward(self._handle, x.data_ptr(), y.data_ptr(), batch, grid[0],
                                            grid[1], workspace.data_ptr(), workspace.numel(),
                                            _stream(stream)))
            return workspace
        order = sorted(taps)
        for l in order:
            t = taps[l]
            if t.dtype != sd or not t.is_contiguous() or t.shape != y.shape:
                raise ValueError("tap tensors must be contiguous, of the type and shape of y")
        blocks = (ctypes.c_int32 * len(order))(*order)
        outs = (ctypes.c_void_p * len(order))(*[taps[l].data_ptr() for l in order])
        _check(lib().jv_encoder_forward_taps(self._handle, x.data_ptr(), y.data_ptr(), batch, grid[0],
                                             grid[1], len(order), blocks, outs, workspace.data_ptr(),
                                             workspace.numel(), _stream(stream)))
        return workspace

    def close(self):
        if self._handle:
            lib().jv_encoder_destroy(self._handle)
            self._handle = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass
