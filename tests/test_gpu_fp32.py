"""GPU parity, fp32: config 1 (B1, 16x16 grid, 6 heads x 64) and ragged/edge shapes, all three
mixers, element by element against the CPU oracle; window/padding maps bit-exact."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import check, FP32_TOL, err_fp32, to_device, to_host

pytestmark = pytest.mark.gpu


def _run_all(q, k, v, H, W, window, eps=1e-6):
    dq, dk, dv = (to_device(x, False) for x in (q, k, v))
    out = {}
    o = torch.empty_like(dq); binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W), eps); out["linear"] = to_host(o)
    o = torch.empty_like(dq); binding.jv_window_attn_fwd(dq, dk, dv, o, (H, W), window); out["window"] = to_host(o)
    o = torch.empty_like(dq); binding.jv_full_attn_fwd(dq, dk, dv, o, (H, W)); out["full"] = to_host(o)
    torch.cuda.synchronize()
    return out


def test_config1_all_three_mixers():
    c = synth.CONFIGS[1]
    q, k, v = synth.config_qkv(1)
    got = _run_all(q, k, v, c["H"], c["W"], c["window"])
    check(err_fp32(got["linear"], oracle.linear_attn_quadratic(q, k, v, 1e-6)), FP32_TOL)
    check(err_fp32(got["window"], oracle.window_attn(q, k, v, c["H"], c["W"], *c["window"])), FP32_TOL)
    check(err_fp32(got["full"], oracle.full_attn(q, k, v)), FP32_TOL)


@pytest.mark.parametrize("B,heads,H,W,window", [
    (2, 3, 7, 9, (4, 4)),      # ragged grid, padded windows, N = 63 (not a multiple of any tile)
    (1, 2, 37, 37, (8, 8)),    # the 518 px / patch 14 geometry
    (1, 1, 1, 1, (1, 1)),      # a single token
    (1, 2, 5, 67, (5, 67)),    # window = grid, N = 335 spans several key tiles with a tail
    (3, 1, 16, 24, (16, 3)),   # rectangular windows
    (1, 1, 20, 20, (32, 32)),  # window larger than the grid
])
def test_ragged_and_edge_shapes(B, heads, H, W, window):
    N = H * W
    q, k, v = synth.qkv(7, B, heads, N, 64, 1.0, False)
    got = _run_all(q, k, v, H, W, window)
    check(err_fp32(got["linear"], oracle.linear_attn_quadratic(q, k, v, 1e-6)), FP32_TOL)
    check(err_fp32(got["window"], oracle.window_attn(q, k, v, H, W, *window)), FP32_TOL)
    check(err_fp32(got["full"], oracle.full_attn(q, k, v)), FP32_TOL)


def test_long_sequence_split_reduction_fp32():
    # N large enough that the state reduction is split over several workgroups per head
    B, heads, H, W = 1, 2, 48, 50
    q, k, v = synth.qkv(8, B, heads, H * W, 64, 1.0, False)
    dq, dk, dv = (to_device(x, False) for x in (q, k, v))
    o = torch.empty_like(dq)
    binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W), 1e-6)
    ref, _, _ = oracle.linear_attn_state(q, k, v, 1e-6)
    check(err_fp32(to_host(o), ref), FP32_TOL)


def test_strided_views_of_a_fused_qkv_buffer():
    # [B, N, 3, heads, d] as a QKV projection writes it; the mixers read it in place
    B, heads, H, W = 2, 3, 6, 10
    N = H * W
    q, k, v = synth.qkv(9, B, heads, N, 64, 1.0, False)
    fused = torch.empty(B, N, 3, heads, 64, device="cuda")
    for i, x in enumerate((q, k, v)):
        fused[:, :, i] = torch.from_numpy(x).cuda().permute(0, 2, 1, 3)
    dq, dk, dv = (fused[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    obuf = torch.empty(B, N, heads, 64, device="cuda")
    o = obuf.permute(0, 2, 1, 3)
    binding.jv_full_attn_fwd(dq, dk, dv, o, (H, W))
    check(err_fp32(to_host(o), oracle.full_attn(q, k, v)), FP32_TOL)
    binding.jv_window_attn_fwd(dq, dk, dv, o, (H, W), (4, 4))
    check(err_fp32(to_host(o), oracle.window_attn(q, k, v, H, W, 4, 4)), FP32_TOL)
    binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W))
    check(err_fp32(to_host(o), oracle.linear_attn_quadratic(q, k, v, 1e-6)), FP32_TOL)


def test_non_default_scale_and_eps():
    B, heads, H, W = 1, 2, 8, 8
    q, k, v = synth.qkv(10, B, heads, H * W, 64, 1.0, False)
    dq, dk, dv = (to_device(x, False) for x in (q, k, v))
    o = torch.empty_like(dq)
    binding.jv_full_attn_fwd(dq, dk, dv, o, (H, W), scale=0.05)
    check(err_fp32(to_host(o), oracle.full_attn(q, k, v, scale=0.05)), FP32_TOL)
    binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W), eps=3.0)
    check(err_fp32(to_host(o), oracle.linear_attn_quadratic(q, k, v, 3.0)), FP32_TOL)


def test_all_negative_queries_give_exact_zero():
    B, heads, H, W = 1, 1, 4, 4
    q, k, v = synth.qkv(11, B, heads, H * W, 64, 1.0, False)
    dq, dk, dv = (to_device(x, False) for x in (-np.abs(q), k, v))
    o = torch.full_like(dq, 7.0)
    binding.jv_linear_attn_fwd(dq, dk, dv, o, (H, W))
    assert torch.count_nonzero(o).item() == 0


def test_device_maps_are_bit_exact():
    for H, W, wh, ww in [(3, 3, 2, 2), (37, 37, 8, 8), (64, 64, 16, 16), (16, 16, 8, 8),
                         (5, 9, 4, 2), (256, 256, 16, 16), (7, 7, 9, 3)]:
        ti, pm, wt = binding.jv_window_maps_device(H, W, wh, ww)
        want = oracle.window_maps(H, W, wh, ww)
        for g, w in zip((ti, pm, wt), want):
            g = g.cpu().numpy()
            assert g.dtype == w.dtype and g.shape == w.shape and g.tobytes() == w.tobytes()


def test_padding_never_reaches_the_output():
    # window attention on a ragged grid: poison everything around the tensors with NaN
    B, heads, H, W = 1, 2, 5, 7
    N = H * W
    q, k, v = synth.qkv(12, B, heads, N, 64, 1.0, False)
    big = torch.full((3, B, heads, N + 8, 64), float("nan"), device="cuda")
    views = []
    for i, x in enumerate((q, k, v)):
        big[i, :, :, 4:4 + N] = torch.from_numpy(x).cuda()
        views.append(big[i, :, :, 4:4 + N])
    o = torch.empty(B, heads, N, 64, device="cuda")
    binding.jv_window_attn_fwd(*views, o, (H, W), (4, 4))
    check(err_fp32(to_host(o), oracle.window_attn(q, k, v, H, W, 4, 4)), FP32_TOL)