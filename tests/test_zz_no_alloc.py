"""The allocation-free entry point of linear attention (jv_linear_attn_fwd_static: scratch in a
fixed device array of the library) against the ordinary entry point, through the C ABI: same
kernels, so the same bits; two calls in a row, the second on a smaller problem (the array keeps
the first call's contents)."""
import ctypes

import pytest
import torch

from paper_2605_26636_amd import binding, synth
from parity import to_device

pytestmark = pytest.mark.gpu


def _pair(cfg, B, heads, H, W, bf16, out_dtype):
    q, k, v = synth.qkv(cfg, B, heads, H * W, 64, 0.5, bf16)
    dq, dk, dv = (to_device(x, bf16) for x in (q, k, v))
    want = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_linear_attn_fwd(dq, dk, dv, want, (H, W))
    got = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_linear_attn_fwd_static(dq, dk, dv, got, (H, W))
    torch.cuda.synchronize()
    return got, want


def test_static_scratch_entry_point_matches_the_workspace_entry_point():
    # several chunks per head and a ragged tail, then a smaller problem on the used array
    for shape in ((2, 3, 48, 40, True, torch.bfloat16), (1, 2, 9, 7, True, torch.float32)):
        got, want = _pair(41, *shape)
        assert torch.isfinite(got.float()).all()
        assert torch.equal(got, want)
    # fp32 tensors, again larger then smaller
    for shape in ((1, 2, 20, 33, False, torch.float32), (1, 1, 3, 3, False, torch.float32)):
        got, want = _pair(42, *shape)
        assert torch.equal(got, want)
    # the benchmark layer (17 MB of partial states) fits the array
    c = synth.CONFIGS[2]
    got, want = _pair(43, c["B"], c["heads"], c["H"], c["W"], True, torch.bfloat16)
    assert torch.equal(got, want)


def test_static_scratch_entry_point_refuses_what_does_not_fit():
    # a problem whose states exceed the array is refused before anything is launched
    B, heads, H, W = 64, 64, 64, 64
    s = binding.JvStrides(heads * H * W * 64, H * W * 64, 64)
    d = binding.JvAttnDesc(B, heads, H, W, 64, binding.JV_BF16, binding.JV_BF16, s, s, s, s)
    assert binding.jv_linear_attn_workspace_bytes(d) > binding.JV_STATIC_SCRATCH_BYTES
    span = 2 * B * heads * H * W * 64
    base = 1 << 40   # never dereferenced
    L = binding.lib()
    st = L.jv_linear_attn_fwd_static(ctypes.byref(d), base, base + span, base + 2 * span, base + 3 * span, 1e-6, None)
    assert st == binding.JV_ERR_UNSUPPORTED
    assert b"static scratch" in L.jv_last_error()
