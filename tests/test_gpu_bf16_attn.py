"""GPU parity, bf16 window and full attention (matrix-core path) against the CPU oracle.

Tolerance: max |g - r| / RMS(r) <= 2e-2 with bf16 inputs and fp32 softmax/accumulation, checked
on the fp32-output run; the bf16-output run must be the nearest-even rounding of it, bit for bit
(parity.check_bf16_pair)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import BF16_TOL, check, check_bf16_pair, err_bf16, rows_of, to_device, to_host

pytestmark = pytest.mark.gpu


def _full(q, k, v, H, W, out_dtype=torch.bfloat16, scale=0.0):
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_full_attn_fwd(dq, dk, dv, o, (H, W), scale)
    torch.cuda.synchronize()
    return o


def _window(q, k, v, H, W, window, out_dtype=torch.bfloat16, scale=0.0):
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    binding.jv_window_attn_fwd(dq, dk, dv, o, (H, W), window, scale)
    torch.cuda.synchronize()
    return o


@pytest.mark.parametrize("B,heads,H,W,vscale", [
    (2, 3, 16, 16, 1.0),    # N = 256: one query block, four key stages; peaked softmax
    (1, 2, 37, 37, 0.125),  # N = 1369: ragged query block and ragged key stage
    (1, 2, 5, 7, 1.0),      # N = 35: less than one tile
    (1, 1, 1, 1, 1.0),      # a single token
    (2, 2, 24, 40, 0.5),    # N = 960
    (1, 2, 33, 33, 1.0),    # N = 1089 = 17 stages + 1 key: 512-slot workgroups, one-key tail
    (1, 2, 40, 27, 0.5),    # N = 1080 = 16 stages + 56 keys: tail longer than one tile
])
def test_full_attention_small_shapes(B, heads, H, W, vscale):
    q, k, v = synth.qkv(30, B, heads, H * W, 64, vscale, True)
    ref = oracle.full_attn(q, k, v)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32), _full(q, k, v, H, W), ref)


@pytest.mark.parametrize("B,heads,H,W,window,vscale", [
    (2, 2, 16, 16, (8, 8), 1.0),      # config-1 geometry in bf16
    (1, 2, 37, 37, (8, 8), 0.125),    # padded 40 x 40, windows of 64 / 40 / 25 real tokens
    (1, 2, 32, 48, (16, 16), 0.5),    # 256-slot windows
    (2, 1, 7, 9, (4, 4), 1.0),        # tiny ragged windows
    (1, 2, 20, 20, (32, 32), 1.0),    # window larger than the grid
    (1, 2, 18, 30, (6, 30), 1.0),     # windows spanning whole rows
    (1, 1, 40, 24, (24, 16), 0.5),    # 384-slot rectangular windows, ragged at the bottom
    (1, 1, 50, 64, (20, 64), 1.0),    # 1280-slot windows of whole rows; the last one holds 640 tokens
    (1, 2, 16, 64, (8, 32), 0.5),     # 256-slot windows, one window row = one key tile
    (1, 2, 8, 128, (4, 64), 0.5),     # 256-slot windows, a window row = two key tiles
    (1, 1, 4, 256, (2, 128), 0.5),    # 256-slot windows, a window row = four key tiles
    (2, 1, 3, 512, (1, 256), 0.5),    # 256-slot windows of one grid row each
    (1, 1, 256, 2, (128, 2), 0.5),    # 256-slot windows, sixteen window rows per key tile
    (1, 2, 64, 8, (64, 4), 0.5),      # 256-slot windows, eight window rows per key tile
])
def test_window_attention_small_shapes(B, heads, H, W, window, vscale):
    q, k, v = synth.qkv(31, B, heads, H * W, 64, vscale, True)
    ref = oracle.window_attn(q, k, v, H, W, *window)
    check_bf16_pair(_window(q, k, v, H, W, window, torch.float32), _window(q, k, v, H, W, window), ref)


def test_whole_grid_window_equals_full_attention_bitwise():
    B, heads, H, W = 1, 2, 12, 20
    q, k, v = synth.qkv(32, B, heads, H * W, 64, 1.0, True)
    assert torch.equal(_window(q, k, v, H, W, (H, W)), _full(q, k, v, H, W))


def test_non_default_scale():
    B, heads, H, W = 1, 2, 10, 10
    q, k, v = synth.qkv(33, B, heads, H * W, 64, 1.0, True)
    ref = oracle.full_attn(q, k, v, scale=0.3)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32, 0.3), _full(q, k, v, H, W, scale=0.3), ref)


def test_large_logits_need_the_running_maximum():
    # logits of magnitude ~ 60: without max subtraction exp overflows; with a stale reference the
    # deferred rescaling must still trigger.  Keys sorted by norm so the maximum keeps rising.
    B, heads, H, W = 1, 1, 16, 32
    q, k, v = synth.qkv(34, B, heads, H * W, 64, 1.0, True)
    ramp = np.linspace(0.2, 6.0, H * W, dtype=np.float32).reshape(1, 1, -1, 1)
    k = synth.round_to_bf16(k * ramp)
    ref = oracle.full_attn(q, k, v)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32), _full(q, k, v, H, W), ref)


def test_config2_window_and_full_elementwise():
    """The benchmark layer at full size, every element of both mixers against the oracle (every
    workgroup of the timed launches is covered)."""
    c = synth.CONFIGS[2]
    H, W = c["H"], c["W"]
    q, k, v = synth.config_qkv(2)
    o = _window(q, k, v, H, W, c["window"])
    ref = oracle.window_attn(q, k, v, H, W, *c["window"])
    check_bf16_pair(_window(q, k, v, H, W, c["window"], torch.float32), o, ref)
    assert torch.isfinite(o.float()).all()
    o = _full(q, k, v, H, W)
    ref = oracle.full_attn(q, k, v)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32), o, ref)
    assert torch.isfinite(o.float()).all()


@pytest.mark.parametrize("mixer,B,heads,H,W,window", [
    ("full", 2, 2, 40, 40, None),          # ring kernel: 25 key stages, ragged query block
    ("window", 4, 4, 64, 64, (16, 16)),    # persistent 256-slot kernel, several windows per workgroup
    ("window", 4, 4, 37, 37, (8, 8)),      # one wavefront per window, padded
    ("window", 1, 2, 40, 24, (24, 16)),    # streaming kernel
    ("window", 2, 2, 24, 24, (12, 12)),    # window-resident kernel, 144 slots
])
def test_rerun_is_bitwise_stable(mixer, B, heads, H, W, window):
    """The kernels order their LDS traffic with counted waits and barriers; a missing one shows
    as run-to-run differences.  Same inputs, several launches, same bits."""
    q, k, v = synth.qkv(36, B, heads, H * W, 64, 0.5, True)
    run = (lambda: _full(q, k, v, H, W)) if mixer == "full" else (lambda: _window(q, k, v, H, W, window))
    first = run()
    for _ in range(4):
        assert torch.equal(run(), first)


def test_config4_padded_windows_full_size_elementwise():
    c = synth.CONFIGS[4]
    H, W = c["H"], c["W"]
    q, k, v = synth.config_qkv(4)
    ti, pm, wt = binding.jv_window_maps_device(H, W, *c["window"])
    for got, want in zip((ti, pm, wt), oracle.window_maps(H, W, *c["window"])):
        assert got.cpu().numpy().tobytes() == want.tobytes()
    o = _window(q, k, v, H, W, c["window"])
    ref = oracle.window_attn(q, k, v, H, W, *c["window"])
    check_bf16_pair(_window(q, k, v, H, W, c["window"], torch.float32), o, ref)


def test_config3_full_attention_16k_tokens_sampled_rows():
    c = synth.CONFIGS[3]
    H, W, N = c["H"], c["W"], c["H"] * c["W"]
    q, k, v = synth.config_qkv(3)
    rows = synth.sample_rows(c["B"], c["heads"], N, 256, seed=6)
    o = _full(q, k, v, H, W)
    ref = oracle.full_attn_rows(q, k, v, rows)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32), o, ref, rows)


def test_full_attention_65536_tokens_sampled_rows():
    """The largest image of the token-count sweep (256 x 256 grid) through full attention: 2 048
    key tiles per query block, 256 query blocks per head; two heads, sampled rows."""
    B, heads, H, W = 1, 2, 256, 256
    N = H * W
    q, k, v = synth.qkv(3, B, heads, N, 64, 0.125, True)
    rows = synth.sample_rows(B, heads, N, 96, seed=9)
    o = _full(q, k, v, H, W)
    ref = oracle.full_attn_rows(q, k, v, rows)
    check_bf16_pair(_full(q, k, v, H, W, torch.float32), o, ref, rows)


def test_padding_is_masked_not_merely_zero():
    # NaN around the tensors: padded key slots must never be read into the result
    B, heads, H, W = 1, 2, 13, 11
    N = H * W
    q, k, v = synth.qkv(35, B, heads, N, 64, 1.0, True)
    big = torch.full((3, B, heads, N + 16, 64), float("nan"), device="cuda", dtype=torch.bfloat16)
    views = []
    for i, x in enumerate((q, k, v)):
        big[i, :, :, 8:8 + N] = to_device(x, True)
        views.append(big[i, :, :, 8:8 + N])
    o = torch.empty(B, heads, N, 64, device="cuda", dtype=torch.float32)
    binding.jv_window_attn_fwd(*views, o, (H, W), (8, 8))
    check(err_bf16(to_host(o), oracle.window_attn(q, k, v, H, W, 8, 8)), BF16_TOL)
    # constant positive shift of V: a zero-valued (unmasked) pad key would pull outputs towards 0
    v2 = synth.round_to_bf16(v + 4.0)
    o2 = _window(q, k, v2, H, W, (8, 8), torch.float32)
    check(err_bf16(to_host(o2), oracle.window_attn(q, k, v2, H, W, 8, 8)), BF16_TOL)

@pytest.mark.parametrize("B,H,W", [(32, 32, 32), (2, 128, 128), (1, 256, 256)])
def test_window_attention_token_sweep_sampled_rows(B, H, W):
    """16 x 16 windows over the token-count sweep (1 024, 16 384 and 65 536 tokens per image at a
    constant 32 768 or 65 536 tokens per batch), sampled rows against the oracle."""
    heads, N = 16, H * W
    q, k, v = synth.qkv(3, B, heads, N, 64, 0.125, True)
    rows = synth.sample_rows(B, heads, N, 256, seed=7 + H)
    o = _window(q, k, v, H, W, (16, 16))
    ref = oracle.window_attn_rows(q, k, v, H, W, 16, 16, rows)
    check_bf16_pair(_window(q, k, v, H, W, (16, 16), torch.float32), o, ref, rows)
    assert torch.isfinite(o.float()).all()
