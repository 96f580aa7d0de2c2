"""GPU parity on a seeded sweep of small random geometries: every mixer, with and without prefix
tokens, on grids and windows that hit the kernels' ragged paths (partial tiles and stages,
windows larger than the grid, one-row and one-column grids, row-spanning windows)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import BF16_TOL, FP32_TOL, check, check_bf16_pair, err_bf16, err_fp32, to_device, to_host

pytestmark = pytest.mark.gpu


def _cases(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for i in range(n):
        H, W = int(rng.integers(1, 41)), int(rng.integers(1, 41))
        kind = int(rng.integers(0, 4))
        if kind == 0:      # small square-ish windows
            wh, ww = int(rng.integers(1, 9)), int(rng.integers(1, 9))
        elif kind == 1:    # row-spanning windows
            wh, ww = int(rng.integers(1, H + 1)), W
        elif kind == 2:    # the 256-slot and 64-slot shapes
            wh, ww = [(16, 16), (8, 8), (8, 32), (4, 16)][int(rng.integers(0, 4))]
        else:              # anything, possibly larger than the grid
            wh, ww = int(rng.integers(1, 50)), int(rng.integers(1, 50))
        P = int(rng.choice([0, 0, 0, 1, 5, 33]))
        out.append((i, int(rng.integers(1, 3)), int(rng.integers(1, 4)), H, W, wh, ww, P))
    return out


def _run(fn, q, k, v, bf16, out_dtype, *args, **kw):
    dq, dk, dv = (to_device(x, bf16) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    fn(dq, dk, dv, o, *args, **kw)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("case", _cases(36, 2024), ids=lambda c: "case%d_%dx%d_w%dx%d_p%d" % (c[0], c[3], c[4], c[5], c[6], c[7]))
def test_bf16_random_geometry(case):
    i, B, heads, H, W, wh, ww, P = case
    N = P + H * W
    q, k, v = synth.qkv(7000 + i, B, heads, N, 64, 0.7, True)
    ref = oracle.full_attn(q, k, v)
    check_bf16_pair(_run(binding.jv_full_attn_fwd, q, k, v, True, torch.float32, (H, W)),
                    _run(binding.jv_full_attn_fwd, q, k, v, True, torch.bfloat16, (H, W)), ref)
    ref = oracle.window_attn_prefix(q, k, v, P, H, W, wh, ww)
    check_bf16_pair(_run(binding.jv_window_attn_fwd, q, k, v, True, torch.float32, (H, W), (wh, ww)),
                    _run(binding.jv_window_attn_fwd, q, k, v, True, torch.bfloat16, (H, W), (wh, ww)), ref)
    C = heads * 64
    ks = 3 if i % 2 == 0 else 5
    kern = synth.dwc_static_kernel(C, ks, 7100 + i)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, static_kernel=kern, ksize=ks, focus_p=1 + i % 3)
    dk = torch.from_numpy(kern).cuda()
    check_bf16_pair(
        _run(binding.jv_linear_block_focused_fwd, q, k, v, True, torch.float32, (H, W), 1 + i % 3, static_kernel=dk, ksize=ks),
        _run(binding.jv_linear_block_focused_fwd, q, k, v, True, torch.bfloat16, (H, W), 1 + i % 3, static_kernel=dk, ksize=ks),
        ref)


@pytest.mark.parametrize("case", _cases(12, 2025), ids=lambda c: "case%d_%dx%d_w%dx%d_p%d" % (c[0], c[3], c[4], c[5], c[6], c[7]))
def test_fp32_random_geometry(case):
    i, B, heads, H, W, wh, ww, P = case
    N = P + H * W
    q, k, v = synth.qkv(7500 + i, B, heads, N, 64, 1.0, False)
    check(err_fp32(to_host(_run(binding.jv_full_attn_fwd, q, k, v, False, torch.float32, (H, W))),
                   oracle.full_attn(q, k, v)), FP32_TOL)
    check(err_fp32(to_host(_run(binding.jv_window_attn_fwd, q, k, v, False, torch.float32, (H, W), (wh, ww))),
                   oracle.window_attn_prefix(q, k, v, P, H, W, wh, ww)), FP32_TOL)
    sq = synth.squeeze_weights(heads * 64, 8, 3, 7600 + i)
    got = _run(binding.jv_linear_block_fwd, q, k, v, False, torch.float32, (H, W),
               squeeze=tuple(torch.from_numpy(a).cuda() for a in sq))
    check(err_fp32(to_host(got), oracle.linear_block(q, k, v, H, W, 1e-6, squeeze=sq)), FP32_TOL)
