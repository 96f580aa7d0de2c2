"""Host-side checks of the C ABI: the library loads, exports every declared symbol, and its
host-only entry points (geometry, host maps, argument validation) behave as documented."""
import ctypes
import os
import re

import numpy as np
import pytest

import oracle
from paper_2605_26636_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    names = set()
    for fn in os.listdir(os.path.join(ROOT, "include")):
        text = open(os.path.join(ROOT, "include", fn)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(jv_[a-z0-9_]+)\s*\(", text))
    return names


def test_library_exports_every_declared_symbol():
    L = binding.lib()
    declared = _declared_symbols()
    assert declared, "no declarations found"
    for name in declared:
        assert hasattr(L, name), f"{name} is declared but not exported"
    assert set(binding.EXPORTS) == declared
    assert b"gfx950" in L.jv_version()


def test_geometry_and_host_maps_match_the_oracle_bit_for_bit():
    cases = [(3, 3, 2, 2), (37, 37, 8, 8), (64, 64, 16, 16), (16, 16, 8, 8), (5, 9, 4, 2),
             (7, 7, 7, 7), (7, 7, 9, 3), (1, 1, 1, 1), (128, 128, 16, 16)]
    for H, W, wh, ww in cases:
        assert binding.jv_window_geometry(H, W, wh, ww) == oracle.window_geometry(H, W, wh, ww)
        got = binding.jv_window_maps_host(H, W, wh, ww)
        want = oracle.window_maps(H, W, wh, ww)
        for g, w in zip(got, want):
            assert g.dtype == w.dtype and g.shape == w.shape
            assert g.tobytes() == w.tobytes()


def test_argument_validation_launches_nothing():
    L = binding.lib()
    d = binding.JvAttnDesc(1, 2, 4, 4, 64, binding.JV_F32, binding.JV_F32,
                           binding.JvStrides(2 * 16 * 64, 16 * 64, 64),
                           binding.JvStrides(2 * 16 * 64, 16 * 64, 64),
                           binding.JvStrides(2 * 16 * 64, 16 * 64, 64),
                           binding.JvStrides(2 * 16 * 64, 16 * 64, 64))
    assert binding.jv_linear_attn_workspace_bytes(d) > 0
    Q, K, V, O = 0x10000, 0x20000, 0x30000, 0x40000   # never dereferenced: every call below is refused
    # null tensors
    assert L.jv_full_attn_fwd(ctypes.byref(d), None, None, None, None, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert b"non-null" in L.jv_last_error()
    # head_dim other than 64 or 128; 128 with fp32 tensors
    d2 = binding.JvAttnDesc.from_buffer_copy(d)
    for width in (32, 96, 256):
        d2.head_dim = width
        for t in (d2.q, d2.k, d2.v, d2.o):
            t.stride_n, t.stride_h, t.stride_b = 256, 16 * 256, 2 * 16 * 256
        assert L.jv_full_attn_fwd(ctypes.byref(d2), Q, K, V, O, 0.0, None) == binding.JV_ERR_UNSUPPORTED
        assert b"head_dim" in L.jv_last_error()
        assert binding.jv_linear_attn_workspace_bytes(d2) == 0
    d2.head_dim = 128
    assert L.jv_full_attn_fwd(ctypes.byref(d2), Q, K, V, O, 0.0, None) == binding.JV_ERR_UNSUPPORTED
    assert b"bf16" in L.jv_last_error()
    d2.dtype = d2.o_dtype = binding.JV_BF16
    d2.q.stride_n = 64                                     # a row stride below the head width
    assert L.jv_full_attn_fwd(ctypes.byref(d2), Q, K, V, O, 0.0, None) == binding.JV_ERR_INVALID_ARG
    # misaligned pointer, aliasing output, bad window, bad eps, small workspace
    assert L.jv_full_attn_fwd(ctypes.byref(d), Q, K, V, O + 4, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert L.jv_full_attn_fwd(ctypes.byref(d), Q, K, V, Q, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert b"overlap" in L.jv_last_error()
    # ... also when O only overlaps the tail of an input (each tensor spans 8192 bytes here)
    assert L.jv_full_attn_fwd(ctypes.byref(d), Q, K, V, V + 8192 - 256, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert b"overlap" in L.jv_last_error()
    assert L.jv_full_attn_fwd(ctypes.byref(d), Q, K, V, K - 8192 + 16, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert L.jv_window_attn_fwd(ctypes.byref(d), Q, K, V, O, 0, 4, 0.0, None) == binding.JV_ERR_INVALID_ARG
    assert b"window" in L.jv_last_error()
    assert L.jv_linear_attn_fwd(ctypes.byref(d), Q, K, V, O, -1.0, 256, 1 << 30, None) == binding.JV_ERR_INVALID_ARG
    assert L.jv_linear_attn_fwd(ctypes.byref(d), Q, K, V, O, 1e-6, 256, 16, None) == binding.JV_ERR_WORKSPACE_TOO_SMALL
    assert L.jv_linear_attn_fwd(ctypes.byref(d), Q, K, V, O, 1e-6, None, 1 << 30, None) == binding.JV_ERR_INVALID_ARG
    # stride that breaks row alignment
    d3 = binding.JvAttnDesc.from_buffer_copy(d)
    d3.q.stride_n = 66
    assert L.jv_full_attn_fwd(ctypes.byref(d3), Q, K, V, O, 0.0, None) == binding.JV_ERR_INVALID_ARG
    # a padded grid whose cell count does not fit 32 bits
    with pytest.raises(binding.JvError):
        binding.jv_window_geometry(1 << 24, 1, 1, 1 << 14)
    with pytest.raises(binding.JvError):
        binding.jv_window_geometry(4, 4, 0, 2)
    assert L.jv_status_string(3) == b"workspace too small"


def test_block_workspace_query_by_convolution_mode():
    """jv_linear_block_workspace_bytes (host only): grows with the mode's buffers; the token-wise
    mode holds the fp32 filters of every token; parameter blocks the library does not support
    answer 0."""
    B, heads, H, W, P = 2, 3, 10, 12, 4
    C, N, hidden, k = heads * 64, P + H * W, 64, 3
    s = binding.JvStrides(heads * N * 64, N * 64, 64)
    d = binding.JvAttnDesc(B, heads, H, W, 64, binding.JV_BF16, binding.JV_BF16, s, s, s, s, P)
    fake = ctypes.c_void_p(4096)   # 16-byte aligned, never dereferenced by the query

    def params(mode, ksize=k, hid=hidden):
        return binding.JvDwcParams(mode, ksize, hid, fake, fake, fake, fake, fake)

    plain = binding.jv_linear_attn_workspace_bytes(d)
    assert plain > 0 and plain % 256 == 0
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_NONE)) == plain
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_STATIC)) == plain
    squeeze = binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_SQUEEZE_DYNAMIC))
    assert plain + 4 * (B * C * k * k + B * hidden) <= squeeze < plain + (1 << 20)
    token = binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_TOKEN_DYNAMIC))
    M = B * N
    exact = (2 * hidden * C + 2 * C * k * k * hidden      # bf16 generator weights
             + 4 * C * k * k                              # reordered second bias
             + 2 * M * C + 2 * M * hidden                 # V rows, hidden layer
             + 4 * M * C * k * k + 4 * M * C)             # fp32 filters of every token, fp32 attention term
    assert plain + exact <= token <= plain + exact + 7 * 256
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_TOKEN_DYNAMIC, hid=40)) == 0
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_STATIC, ksize=4)) == 0
    assert binding.jv_linear_block_workspace_bytes(d, params(4)) == 0


def test_block_workspace_query_for_wide_heads():
    """The same query for heads of 128 channels (host only): four 64 x 64 quadrant states per head
    and chunk plus their sums; static filters need nothing more, squeeze-dynamic filters the
    partial token sums of V, the hidden layer and one filter bank per image; the token-wise
    variant is not built for wide heads."""
    B, heads, H, W = 2, 3, 40, 48
    C, N, hidden, k = heads * 128, H * W, 32, 3
    s = binding.JvStrides(heads * N * 128, N * 128, 128)
    d = binding.JvAttnDesc(B, heads, H, W, 128, binding.JV_BF16, binding.JV_BF16, s, s, s, s, 0)
    fake = ctypes.c_void_p(4096)

    def params(mode, hid=hidden):
        return binding.JvDwcParams(mode, k, hid, fake, fake, fake, fake, fake)

    plain = binding.jv_linear_attn_workspace_bytes(d)
    state = 4 * (64 * 64 + 64)                      # one quadrant state, bytes
    assert plain >= 2 * 4 * B * heads * state        # at least one partial and the sum, four quadrants each
    assert plain % (4 * B * heads * state) == 0      # (n_split + 1) of them
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_NONE)) == plain
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_STATIC)) == plain
    squeeze = binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_SQUEEZE_DYNAMIC))
    n_split = plain // (4 * B * heads * state) - 1
    need = 4 * (n_split * B * C + B * hidden + B * C * k * k)
    assert plain + need <= squeeze <= plain + need + 4 * 256
    assert binding.jv_linear_block_workspace_bytes(d, params(binding.JV_DWC_TOKEN_DYNAMIC, hid=64)) == 0
    d.dtype = d.o_dtype = binding.JV_F32             # wide heads are built for bf16 tensors
    assert binding.jv_linear_attn_workspace_bytes(d) == 0


def test_gemm_shape_limits_are_checked_on_the_host():
    """jv_gemm_bias_act refuses on the host what its kernel cannot address; large token counts
    (a 256 x 256 grid at batch 4 against a 4096-wide hidden layer) are inside the limits."""
    L = binding.lib()
    A, W, Y = 0x100000, 0x200000, 0x300000   # never dereferenced
    call = lambda M, N, K: L.jv_gemm_bias_act(A, W, None, None, Y, M, N, K, binding.JV_EPI_NONE, binding.JV_BF16, None)
    assert call(16, 64, 96) == binding.JV_ERR_UNSUPPORTED       # K % 64
    assert call(16, 60, 64) == binding.JV_ERR_UNSUPPORTED       # N % 8
    assert call(0, 64, 64) == binding.JV_ERR_INVALID_ARG
    assert call(16, 64, 1 << 22) == binding.JV_ERR_UNSUPPORTED  # rows above 2^21 elements
    assert call((1 << 30) + 1, 64, 64) == binding.JV_ERR_UNSUPPORTED


def test_encoder_options_refuse_a_null_encoder():
    """Host-only entry points of the encoder object: a null handle is an argument error."""
    L = binding.lib()
    assert L.jv_encoder_fuse_linear_projection(None, 1) == binding.JV_ERR_INVALID_ARG
    assert L.jv_encoder_fold_layernorm(None, None, 0, None) == binding.JV_ERR_INVALID_ARG
    assert L.jv_encoder_fold_bytes(None) == 0


def test_encoder_workspace_query_follows_the_options():
    """jv_encoder_workspace_bytes is host arithmetic: the base buffers, plus the partial results
    of fc2's K split when its output has fewer than 128 tiles (few tokens), plus the states and
    per-image weights of the fused linear-attention projection when that option is on."""
    import torch
    heads, hidden, C = 16, 4096, 1024

    def weights():   # host tensors: creating an encoder only records the pointers
        z = lambda *s: torch.zeros(*s, dtype=torch.float32)
        w = lambda *s: torch.zeros(*s, dtype=torch.bfloat16)
        return {"ln1_g": z(C), "ln1_b": z(C), "w_qkv": w(3 * C, C), "b_qkv": z(3 * C), "w_o": w(C, C), "b_o": z(C),
                "ln2_g": z(C), "ln2_b": z(C), "w_fc1": w(hidden, C), "b_fc1": z(hidden), "w_fc2": w(C, hidden), "b_fc2": z(C)}

    a256 = lambda n: (n + 255) // 256 * 256
    enc = binding.Encoder([weights(), weights()], [0, 2], heads, hidden)
    base = lambda B, N: a256(B * N * C * 2) + a256(B * N * 3 * C * 2 if 3 * C > hidden else B * N * hidden * 2)
    # 4 x 4096 tokens: 256 output tiles, no split; 1 x 8192: 128 tiles, two parts; 1 x 4096: 64 tiles, four parts
    w_big, w_two, w_four = enc.workspace_bytes(4, (64, 64)), enc.workspace_bytes(1, (64, 128)), enc.workspace_bytes(1, (64, 64))
    la = lambda B, N, total: total - base(B, N)     # what is left: linear-attention states (+ options)
    la_big = la(4, 4096, w_big)
    assert 0 < la_big < 64 << 20
    assert la(1, 8192, w_two) - 2 * 8192 * C * 4 < 64 << 20 and la(1, 8192, w_two) > 2 * 8192 * C * 4
    assert la(1, 4096, w_four) - 4 * 4096 * C * 4 < 64 << 20 and la(1, 4096, w_four) > 4 * 4096 * C * 4
    enc.fuse_linear_projection(True)
    extra = enc.workspace_bytes(4, (64, 64)) - w_big
    assert extra == a256(4 * heads * (64 * 64 + 64) * 4) + a256(4 * C * C * 2)
    with_option = enc.workspace_bytes(4, (18, 18))       # 324 tokens per image: no block fuses
    enc.fuse_linear_projection(False)
    assert enc.workspace_bytes(4, (18, 18)) == with_option
    enc.close()
