"""GPU parity, bf16 linear attention (matrix-core path) against the CPU oracle.

Tolerance: max |g - r| / RMS(r) <= 2e-2 with bf16 inputs and fp32 accumulation, checked on the
fp32-output run; the bf16-output run must be the nearest-even rounding of it, bit for bit
(parity.check_bf16_pair)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import (BF16_TOL, check, check_bf16_pair, err_bf16, err_bf16_stored, to_device,
                    to_host)

pytestmark = pytest.mark.gpu


def _run(q, k, v, H, W, eps=1e-6, out_dtype=torch.bfloat16):
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W), eps)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("B,heads,H,W", [
    (2, 3, 37, 37),    # N = 1369: several 64-token tiles and a ragged tail
    (1, 2, 5, 7),      # N = 35: less than one tile
    (1, 1, 1, 1),      # a single token
    (1, 2, 64, 65),    # N = 4160: several chunks per head, ragged
    (3, 2, 16, 16),    # N = 256: exactly one workgroup tile set
])
def test_small_shapes_elementwise(B, heads, H, W):
    N = H * W
    q, k, v = synth.qkv(20, B, heads, N, 64, 0.5, True)
    ref = oracle.linear_attn_quadratic(q, k, v, 1e-6)
    o32, o16 = _run(q, k, v, H, W, out_dtype=torch.float32), _run(q, k, v, H, W)
    check(err_bf16(to_host(o32), ref), 1e-3)   # exact bf16 products, fp32 accumulate, hi/lo state
    check_bf16_pair(o32, o16, ref)


def test_config2_full_size_elementwise():
    c = synth.CONFIGS[2]
    q, k, v = synth.config_qkv(2)
    ref, _, _ = oracle.linear_attn_state(q, k, v, 1e-6)   # O(N) form; equality with the
    o = _run(q, k, v, c["H"], c["W"])                     # quadratic form is pinned on the CPU
    check_bf16_pair(_run(q, k, v, c["H"], c["W"], out_dtype=torch.float32), o, ref)
    rows = synth.sample_rows(c["B"], c["heads"], c["H"] * c["W"], 64, seed=2)
    quad = oracle.linear_attn_rows(q, k, v, rows, 1e-6)
    rms = np.sqrt(np.mean(ref * ref))
    got = to_host(o)
    check(err_bf16_stored(np.stack([got[b, h, i] for b, h, i in rows]), quad, rms), BF16_TOL)


def test_long_grid_many_chunks_sampled_rows():
    # 256 x 256 grid, one image: 65 536 tokens, 16 heads -> many partial states per head
    B, heads, H, W = 1, 16, 256, 256
    q, k, v = synth.qkv(3, B, heads, H * W, 64, 0.125, True)
    o = _run(q, k, v, H, W)
    rows = synth.sample_rows(B, heads, H * W, 96, seed=4)
    ref = oracle.linear_attn_rows(q, k, v, rows, 1e-6)
    check_bf16_pair(_run(q, k, v, H, W, out_dtype=torch.float32), o, ref, rows)
    assert torch.isfinite(o.float()).all()


def test_strided_qkv_views_and_rerun_is_bitwise_stable():
    B, heads, H, W = 2, 4, 20, 24
    N = H * W
    q, k, v = synth.qkv(21, B, heads, N, 64, 0.5, True)
    fused = torch.empty(B, N, 3, heads, 64, device="cuda", dtype=torch.bfloat16)
    for i, x in enumerate((q, k, v)):
        fused[:, :, i] = to_device(x, True).permute(0, 2, 1, 3)
    dq, dk, dv = (fused[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    o1 = torch.empty(B, N, heads, 64, device="cuda", dtype=torch.bfloat16).permute(0, 2, 1, 3)
    o2 = torch.empty(B, N, heads, 64, device="cuda", dtype=torch.bfloat16).permute(0, 2, 1, 3)
    binding.jv_linear_attn_fwd(dq, dk, dv, o1, (H, W))
    binding.jv_linear_attn_fwd(dq, dk, dv, o2, (H, W))
    assert torch.equal(o1, o2)
    check(err_bf16_stored(to_host(o1), oracle.linear_attn_quadratic(q, k, v, 1e-6)), BF16_TOL)


def test_all_negative_queries_give_exact_zero_bf16():
    B, heads, H, W = 1, 2, 9, 9
    q, k, v = synth.qkv(22, B, heads, H * W, 64, 1.0, True)
    o = _run(-np.abs(q), k, v, H, W)
    assert torch.count_nonzero(o.float()).item() == 0
