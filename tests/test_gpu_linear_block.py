"""GPU parity of the paper's linear-attention block (Eq. 4: linear attention + depth-wise
convolution of V, static or squeeze-dynamic filters) against the CPU oracle.

fp32 tensors: max |g - r| / max(|r|, RMS r) <= 1e-4.  bf16 tensors (fp32 accumulation):
max |g - r| / RMS r <= 2e-2 on the fp32-output run; the bf16-output run is its rounding."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import BF16_TOL, FP32_TOL, check, check_bf16_pair, err_bf16, err_fp32, to_device, to_host

pytestmark = pytest.mark.gpu


def _dev(*arrays):
    return tuple(torch.from_numpy(np.ascontiguousarray(a)).cuda() for a in arrays)


def _block(q, k, v, H, W, bf16, out_dtype, **kw):
    dq, dk, dv = (to_device(x, bf16) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_linear_block_fwd(dq, dk, dv, o, (H, W), 1e-6, **kw)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("ksize", [3, 5])
@pytest.mark.parametrize("B,heads,H,W", [(1, 6, 16, 16), (2, 2, 5, 7), (1, 1, 1, 1), (1, 2, 3, 40)])
def test_fp32_static_and_dynamic(B, heads, H, W, ksize):
    C, hidden = heads * 64, 8
    q, k, v = synth.qkv(30, B, heads, H * W, 64, 1.0, False)
    kern = synth.dwc_static_kernel(C, ksize, 3100 + ksize)
    sq = synth.squeeze_weights(C, hidden, ksize, 3200 + ksize)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, static_kernel=kern, ksize=ksize)
    got = _block(q, k, v, H, W, False, torch.float32, static_kernel=_dev(kern)[0], ksize=ksize)
    check(err_fp32(to_host(got), ref), FP32_TOL)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, squeeze=sq, ksize=ksize)
    got = _block(q, k, v, H, W, False, torch.float32, squeeze=_dev(*sq), ksize=ksize)
    check(err_fp32(to_host(got), ref), FP32_TOL)


@pytest.mark.parametrize("ksize", [3, 5])
@pytest.mark.parametrize("B,heads,H,W", [
    (2, 3, 37, 37),   # ragged tiles, rows shorter than a tile
    (1, 2, 5, 7),     # less than one tile
    (1, 1, 1, 1),     # a single token: only the centre tap is inside the grid
    (1, 2, 20, 130),  # rows longer than two tiles, several chunks
    (3, 2, 16, 16),
])
def test_bf16_static_and_dynamic(B, heads, H, W, ksize):
    C, hidden = heads * 64, 16
    q, k, v = synth.qkv(31, B, heads, H * W, 64, 0.5, True)
    kern = synth.dwc_static_kernel(C, ksize, 3300 + ksize)
    sq = synth.squeeze_weights(C, hidden, ksize, 3400 + ksize)
    for kw_ref, kw_gpu in (
            (dict(static_kernel=kern), dict(static_kernel=_dev(kern)[0])),
            (dict(squeeze=sq), dict(squeeze=_dev(*sq)))):
        ref = oracle.linear_block(q, k, v, H, W, 1e-6, ksize=ksize, **kw_ref)
        o32 = _block(q, k, v, H, W, True, torch.float32, ksize=ksize, **kw_gpu)
        o16 = _block(q, k, v, H, W, True, torch.bfloat16, ksize=ksize, **kw_gpu)
        check(err_bf16(to_host(o32), ref), 2e-3)   # fp32 stencil on exact bf16 values
        check_bf16_pair(o32, o16, ref)


def test_special_filters_bf16():
    """Zero filters give plain linear attention bit for bit; a centre-delta filter adds V."""
    B, heads, H, W = 1, 2, 12, 9
    C = heads * 64
    q, k, v = synth.qkv(32, B, heads, H * W, 64, 0.5, True)
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    plain = torch.empty_like(dq, dtype=torch.float32)
    binding.jv_linear_attn_fwd(dq, dk, dv, plain, (H, W))
    zero = torch.zeros(C, 3, 3, device="cuda")
    got = torch.empty_like(plain)
    binding.jv_linear_block_fwd(dq, dk, dv, got, (H, W), static_kernel=zero)
    assert torch.equal(got, plain)
    none = torch.empty_like(plain)
    binding.jv_linear_block_fwd(dq, dk, dv, none, (H, W))
    assert torch.equal(none, plain)
    delta = zero.clone()
    delta[:, 1, 1] = 1.0
    binding.jv_linear_block_fwd(dq, dk, dv, got, (H, W), static_kernel=delta)
    assert torch.equal(got, plain + dv.float())


def test_config2_block_sampled_rows():
    """The block at the benchmark workload's size (batch 8, 64 x 64 grid, 16 heads), squeeze-
    dynamic 3 x 3 filters with hidden width C / 16; sampled rows against the oracle."""
    c = synth.CONFIGS[2]
    B, heads, H, W = c["B"], c["heads"], c["H"], c["W"]
    C, hidden, N = heads * 64, heads * 4, H * W
    q, k, v = synth.config_qkv(2)
    sq = synth.squeeze_weights(C, hidden, 3, 3500)
    o32 = _block(q, k, v, H, W, True, torch.float32, squeeze=_dev(*sq))
    o16 = _block(q, k, v, H, W, True, torch.bfloat16, squeeze=_dev(*sq))
    rows = synth.sample_rows(B, heads, N, 96, seed=35)
    rows[1] = (0, 0, W - 1); rows[2] = (B - 1, 3, N - W); rows[3] = (1, 5, 17 * W)  # grid borders
    la = oracle.linear_attn_rows(q, k, v, rows, 1e-6)
    conv = oracle.dwc(v, oracle.squeeze_kernel(v, *sq, 3), H, W)
    ref = la + np.stack([conv[b, h, i] for b, h, i in rows])
    check_bf16_pair(o32, o16, ref, rows)


def test_block_rejects_bad_parameters():
    q = torch.zeros(1, 1, 16, 64, device="cuda")
    o = torch.empty_like(q)
    with pytest.raises(binding.JvError) as e:
        binding.jv_linear_block_fwd(q, q.clone(), q.clone(), o, (4, 4),
                                    static_kernel=torch.zeros(64, 4, 4, device="cuda"), ksize=4)
    assert e.value.status == binding.JV_ERR_UNSUPPORTED


# ---- the block with the focused feature map (Eq. 3) in place of ReLU ----------------------------

def _focused(q, k, v, H, W, p, bf16, out_dtype, **kw):
    dq, dk, dv = (to_device(x, bf16) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_linear_block_focused_fwd(dq, dk, dv, o, (H, W), p, 1e-6, **kw)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("p", [2, 3])
@pytest.mark.parametrize("B,heads,H,W", [(1, 6, 16, 16), (2, 2, 5, 7), (1, 1, 1, 1), (1, 2, 3, 40)])
def test_focused_fp32(B, heads, H, W, p):
    C = heads * 64
    q, k, v = synth.qkv(40, B, heads, H * W, 64, 1.0, False)
    ref = oracle.focused_linear_attn(q, k, v, p)
    check(err_fp32(to_host(_focused(q, k, v, H, W, p, False, torch.float32)), ref), FP32_TOL)
    kern = synth.dwc_static_kernel(C, 3, 4100)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, static_kernel=kern, focus_p=p)
    got = _focused(q, k, v, H, W, p, False, torch.float32, static_kernel=_dev(kern)[0])
    check(err_fp32(to_host(got), ref), FP32_TOL)


@pytest.mark.parametrize("p", [2, 3, 5])
@pytest.mark.parametrize("B,heads,H,W", [
    (2, 3, 37, 37),   # ragged tiles
    (1, 2, 5, 7),     # less than one tile
    (1, 1, 1, 1),
    (1, 2, 20, 130),  # several chunks
])
def test_focused_bf16(B, heads, H, W, p):
    C = heads * 64
    q, k, v = synth.qkv(41, B, heads, H * W, 64, 0.5, True)
    ref = oracle.focused_linear_attn(q, k, v, p)
    check_bf16_pair(_focused(q, k, v, H, W, p, True, torch.float32),
                    _focused(q, k, v, H, W, p, True, torch.bfloat16), ref)
    sq = synth.squeeze_weights(C, 16, 3, 4200)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, squeeze=sq, focus_p=p)
    check_bf16_pair(_focused(q, k, v, H, W, p, True, torch.float32, squeeze=_dev(*sq)),
                    _focused(q, k, v, H, W, p, True, torch.bfloat16, squeeze=_dev(*sq)), ref)


def test_focused_special_cases():
    """p = 1 is the ReLU block bit for bit; rows without a positive entry give zero weights;
    huge magnitudes do not overflow (the rows are normalised before the power)."""
    B, heads, H, W = 1, 2, 12, 9
    q, k, v = synth.qkv(42, B, heads, H * W, 64, 0.5, True)
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    a, b = torch.empty_like(dq, dtype=torch.float32), torch.empty_like(dq, dtype=torch.float32)
    binding.jv_linear_attn_fwd(dq, dk, dv, a, (H, W))
    binding.jv_linear_block_focused_fwd(dq, dk, dv, b, (H, W), 1)
    assert torch.equal(a, b)
    qn = -np.abs(q)
    o = _focused(qn, k, v, H, W, 3, True, torch.float32)
    assert torch.count_nonzero(o) == 0
    big = synth.round_to_bf16(q * 1e12)
    ref = oracle.focused_linear_attn(big, k, v, 3)
    check(err_bf16(to_host(_focused(big, k, v, H, W, 3, True, torch.float32)), ref), BF16_TOL)
    with pytest.raises(binding.JvError):
        binding.jv_linear_block_focused_fwd(dq, dk, dv, b, (H, W), 0)
