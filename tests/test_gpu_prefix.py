"""GPU parity with prefix tokens (class / register tokens) in front of the grid, against the
oracle's statement of the library's rule: full and linear attention take all N tokens; window
attention gives grid tokens their window and prefix tokens the whole sequence; the block's
convolution runs over the grid only.  Tolerances as for the other mixers."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import BF16_TOL, FP32_TOL, check, check_bf16_pair, err_bf16, err_fp32, to_device, to_host

pytestmark = pytest.mark.gpu


def _run(fn, q, k, v, bf16, out_dtype, *args, **kw):
    dq, dk, dv = (to_device(x, bf16) for x in (q, k, v))
    o = torch.full(dq.shape, float("nan"), dtype=out_dtype, device="cuda")
    fn(dq, dk, dv, o, *args, **kw)
    torch.cuda.synchronize()
    return o


CASES = [  # P, B, heads, H, W, window
    (5, 2, 2, 16, 16, (8, 8)),     # class + 4 registers; 64-slot windows
    (1, 1, 2, 32, 32, (16, 16)),   # 256-slot windows on a divisible grid
    (4, 1, 2, 37, 37, (8, 8)),     # padded grid
    (7, 1, 1, 5, 7, (4, 4)),       # more prefix than a window row; tiny ragged windows
    (64, 1, 1, 18, 30, (6, 30)),   # the largest prefix; row-spanning windows
]


@pytest.mark.parametrize("P,B,heads,H,W,window", CASES)
def test_bf16_mixers_with_prefix(P, B, heads, H, W, window):
    N = P + H * W
    q, k, v = synth.qkv(60, B, heads, N, 64, 0.5, True)
    ref = oracle.full_attn(q, k, v)
    check_bf16_pair(_run(binding.jv_full_attn_fwd, q, k, v, True, torch.float32, (H, W)),
                    _run(binding.jv_full_attn_fwd, q, k, v, True, torch.bfloat16, (H, W)), ref)
    ref = oracle.window_attn_prefix(q, k, v, P, H, W, *window)
    check_bf16_pair(_run(binding.jv_window_attn_fwd, q, k, v, True, torch.float32, (H, W), window),
                    _run(binding.jv_window_attn_fwd, q, k, v, True, torch.bfloat16, (H, W), window), ref)
    ref = oracle.linear_attn_quadratic(q, k, v)
    check_bf16_pair(_run(binding.jv_linear_attn_fwd, q, k, v, True, torch.float32, (H, W)),
                    _run(binding.jv_linear_attn_fwd, q, k, v, True, torch.bfloat16, (H, W)), ref)
    C = heads * 64
    sq = synth.squeeze_weights(C, 8, 3, 6100)
    dsq = tuple(torch.from_numpy(a).cuda() for a in sq)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, squeeze=sq)
    check_bf16_pair(_run(binding.jv_linear_block_fwd, q, k, v, True, torch.float32, (H, W), squeeze=dsq),
                    _run(binding.jv_linear_block_fwd, q, k, v, True, torch.bfloat16, (H, W), squeeze=dsq), ref)
    kern = synth.dwc_static_kernel(C, 5, 6200)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, static_kernel=kern, ksize=5)
    got = _run(binding.jv_linear_block_fwd, q, k, v, True, torch.float32, (H, W),
               static_kernel=torch.from_numpy(kern).cuda(), ksize=5)
    check(err_bf16(to_host(got), ref), BF16_TOL)


@pytest.mark.parametrize("P,B,heads,H,W,window", CASES[:4])
def test_fp32_mixers_with_prefix(P, B, heads, H, W, window):
    N = P + H * W
    q, k, v = synth.qkv(61, B, heads, N, 64, 1.0, False)
    check(err_fp32(to_host(_run(binding.jv_full_attn_fwd, q, k, v, False, torch.float32, (H, W))),
                   oracle.full_attn(q, k, v)), FP32_TOL)
    check(err_fp32(to_host(_run(binding.jv_window_attn_fwd, q, k, v, False, torch.float32, (H, W), window)),
                   oracle.window_attn_prefix(q, k, v, P, H, W, *window)), FP32_TOL)
    C = heads * 64
    kern = synth.dwc_static_kernel(C, 3, 6300)
    got = _run(binding.jv_linear_block_fwd, q, k, v, False, torch.float32, (H, W),
               static_kernel=torch.from_numpy(kern).cuda())
    check(err_fp32(to_host(got), oracle.linear_block(q, k, v, H, W, 1e-6, static_kernel=kern)), FP32_TOL)


def test_prefix_rows_do_not_disturb_grid_rows_of_window_attention():
    """Grid rows with prefix tokens present are bit-identical to window attention on the grid
    tokens alone (the same kernels on the same rows); the prefix rows are full attention's (a
    kernel of their own that splits the keys, so equal to the oracle within the tolerance, not
    bit for bit to the full-attention kernel)."""
    P, B, heads, H, W, window = 5, 1, 2, 32, 32, (16, 16)
    N = P + H * W
    q, k, v = synth.qkv(62, B, heads, N, 64, 0.5, True)
    o = _run(binding.jv_window_attn_fwd, q, k, v, True, torch.bfloat16, (H, W), window)
    grid = _run(binding.jv_window_attn_fwd, *(np.ascontiguousarray(t[:, :, P:]) for t in (q, k, v)),
                True, torch.bfloat16, (H, W), window)
    assert torch.equal(o[:, :, P:], grid)
    o32 = _run(binding.jv_window_attn_fwd, q, k, v, True, torch.float32, (H, W), window)
    ref = oracle.full_attn(q, k, v)[:, :, :P]
    check(err_bf16(to_host(o32[:, :, :P]), ref), BF16_TOL)


def test_encoder_with_prefix_tokens():
    P, B, H, W, heads, hidden = 5, 2, 8, 8, 2, 256
    C, N = heads * 64, P + H * W
    x = synth.normal((B, N, C), 6400)
    blocks = [synth.block_weights(C, hidden, 6410 + i) for i in range(3)]
    blocks[0]["dwc"] = {"squeeze": synth.squeeze_weights(C, 8, 3, 6420), "ksize": 3}
    pattern = [0, 1, 2]
    dev = []
    for b in blocks:
        d = {}
        for key, val in b.items():
            if key == "dwc":
                d[key] = {"ksize": 3, "squeeze": tuple(torch.from_numpy(a).cuda() for a in val["squeeze"])}
            else:
                t = torch.from_numpy(val).cuda()
                d[key] = t.to(torch.bfloat16) if key.startswith("w_") else t
        dev.append(d)
    enc = binding.Encoder(dev, pattern, heads, hidden, window=(4, 4), n_prefix=P)
    dx = torch.from_numpy(x).cuda()
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 4), n_prefix=P)
    check(err_bf16(to_host(y), ref), BF16_TOL)
    enc.close()


def test_prefix_count_is_validated():
    q = torch.zeros(1, 1, 65 + 16, 64, device="cuda", dtype=torch.bfloat16)
    o = torch.empty_like(q)
    with pytest.raises(binding.JvError):
        binding.jv_full_attn_fwd(q, q.clone(), q.clone(), o, (4, 4))   # 65 prefix tokens


def test_config2_size_with_prefix_sampled_rows():
    """The benchmark layer (batch 8, 64x64 grid, 16 heads) with a class token and four register
    tokens in front, at full size, on sampled rows: the prefix rows and the first and last grid
    rows are always in the sample."""
    P, B, heads, H, W, window = 5, 8, 16, 64, 64, (16, 16)
    N = P + H * W
    q, k, v = synth.qkv(63, B, heads, N, 64, 0.125, True)
    rows = synth.sample_rows(B, heads, N, 384, seed=9)
    rows[1:6, 2] = np.arange(P)              # every prefix row of some (batch, head)
    rows[6, 2] = P                           # first grid token
    is_prefix = rows[:, 2] < P
    grid_rows = rows[~is_prefix].copy()
    grid_rows[:, 2] -= P
    qg, kg, vg = (np.ascontiguousarray(t[:, :, P:]) for t in (q, k, v))
    # full attention: all N tokens
    ref = oracle.full_attn_rows(q, k, v, rows)
    check_bf16_pair(_run(binding.jv_full_attn_fwd, q, k, v, True, torch.float32, (H, W)),
                    _run(binding.jv_full_attn_fwd, q, k, v, True, torch.bfloat16, (H, W)), ref, rows)
    # window attention: grid rows see their window of the grid, prefix rows everything
    ref = np.empty((rows.shape[0], 64))
    ref[is_prefix] = oracle.full_attn_rows(q, k, v, rows[is_prefix])
    ref[~is_prefix] = oracle.window_attn_rows(qg, kg, vg, H, W, *window, grid_rows)
    check_bf16_pair(_run(binding.jv_window_attn_fwd, q, k, v, True, torch.float32, (H, W), window),
                    _run(binding.jv_window_attn_fwd, q, k, v, True, torch.bfloat16, (H, W), window), ref, rows)
    # linear attention: all N tokens
    ref = oracle.linear_attn_rows(q, k, v, rows)
    check_bf16_pair(_run(binding.jv_linear_attn_fwd, q, k, v, True, torch.float32, (H, W)),
                    _run(binding.jv_linear_attn_fwd, q, k, v, True, torch.bfloat16, (H, W)), ref, rows)
