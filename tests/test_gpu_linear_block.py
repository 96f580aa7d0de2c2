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


@pytest.mark.parametrize("ksize", [3, 5])
@pytest.mark.parametrize("B,heads,H,W,P", [
    (2, 3, 37, 37, 0),   # ragged matrix tiles
    (1, 2, 5, 7, 0),
    (1, 1, 1, 1, 0),     # a single token: only the centre tap is inside the grid
    (1, 2, 20, 130, 0),
    (2, 2, 12, 9, 5),    # prefix tokens in front of the grid: no convolution term for them
])
def test_bf16_token_wise_dynamic(B, heads, H, W, P, ksize):
    """Per-token dynamic filters (Tab. 1, "Token-wise Dynamic DWC"): generator on every token's
    V row, each token's own filters on its neighbourhood.

    Inputs are bf16 values, the generator's matrices included (as for every bf16 workload: rounded
    once on the host, so the matrix cores multiply exactly what the oracle sees); the kernels
    round the hidden layer to bf16 and keep the filters in fp32.  The bar is the plain one for
    bf16 inputs with fp32 accumulation, 2e-2 RMS; the same run is also compared with the oracle
    evaluated with that one rounding, which it must reproduce far more closely."""
    C, hidden = heads * 64, 64
    q, k, v = synth.qkv(33, B, heads, P + H * W, 64, 0.5, True)
    w1, b1, w2, b2 = synth.squeeze_weights(C, hidden, ksize, 3500 + ksize)
    tok = (synth.round_to_bf16(w1), b1, synth.round_to_bf16(w2), b2)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, ksize=ksize, token=tok)
    o32 = _block(q, k, v, H, W, True, torch.float32, ksize=ksize, token=_dev(*tok))
    o16 = _block(q, k, v, H, W, True, torch.bfloat16, ksize=ksize, token=_dev(*tok))
    check_bf16_pair(o32, o16, ref)
    # the hidden layer's rounding applied to the oracle's own stages
    rb = lambda a: synth.round_to_bf16(np.asarray(a, dtype=np.float32)).astype(np.float64)
    w1, b1, w2, b2 = tok
    vg = np.ascontiguousarray(v[:, :, P:])
    rows = vg.transpose(0, 2, 1, 3).reshape(B, H * W, C).astype(np.float64)
    pre = rows @ w1.astype(np.float64).T + b1
    u = rb(pre / (1.0 + np.exp(-pre)))
    kap_r = (u @ w2.astype(np.float64).T + b2).reshape(B, H * W, C, ksize, ksize)
    la = oracle.linear_attn_quadratic(q, k, v, 1e-6)
    same = la.copy()
    same[:, :, P:] += oracle.dwc_tokenwise(vg, kap_r, H, W)
    # (fp32 against fp64 accumulation flips the bf16 rounding of a few hidden units by one ulp)
    g32, rms = to_host(o32), np.sqrt(np.mean(ref * ref))
    check(float(np.sqrt(np.mean((g32 - same) ** 2)) / rms), 3e-4)
    check(err_bf16(g32, same, rms), 5e-3)
    if P:           # prefix rows are plain linear attention, bit for bit
        dq, dk, dv = (to_device(x, True) for x in (q, k, v))
        plain = torch.empty_like(o32)
        binding.jv_linear_attn_fwd(dq, dk, dv, plain, (H, W))
        assert torch.equal(plain[:, :, :P], o32[:, :, :P])


@pytest.mark.parametrize("ksize", [3, 5])
@pytest.mark.parametrize("B,heads,H,W,P", [(2, 3, 13, 11, 0), (1, 2, 5, 7, 3), (1, 1, 1, 1, 0), (1, 5, 9, 40, 0)])
def test_fp32_token_wise_dynamic(B, heads, H, W, P, ksize):
    """The token-wise variant on fp32 tensors (plain fp32 kernels), at the fp32 bar; prefix rows
    are plain linear attention bit for bit."""
    C, hidden = heads * 64, 64
    q, k, v = synth.qkv(35, B, heads, P + H * W, 64, 0.5, False)
    tok = synth.squeeze_weights(C, hidden, ksize, 3700 + ksize)
    ref = oracle.linear_block(q, k, v, H, W, 1e-6, ksize=ksize, token=tok)
    got = _block(q, k, v, H, W, False, torch.float32, ksize=ksize, token=_dev(*tok))
    check(err_fp32(to_host(got), ref), FP32_TOL)
    if P:
        dq, dk, dv = (to_device(x, False) for x in (q, k, v))
        plain = torch.empty_like(got)
        binding.jv_linear_attn_fwd(dq, dk, dv, plain, (H, W))
        assert torch.equal(plain[:, :, :P], got[:, :, :P])


def test_token_wise_special_filters():
    """W2 = 0 makes every token's filters the static bank b2: the static block's result up to the
    order of the fp32 additions."""
    B, heads, H, W = 1, 2, 12, 9
    C, hidden = heads * 64, 64
    q, k, v = synth.qkv(34, B, heads, H * W, 64, 0.5, True)
    w1, b1, w2, b2 = synth.squeeze_weights(C, hidden, 3, 3600)
    b2 = synth.round_to_bf16(b2)
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    static = torch.empty_like(dq, dtype=torch.float32)
    binding.jv_linear_block_fwd(dq, dk, dv, static, (H, W), static_kernel=_dev(b2.reshape(C, 3, 3))[0])
    tok = torch.empty_like(static)
    binding.jv_linear_block_fwd(dq, dk, dv, tok, (H, W), token=_dev(w1, b1, np.zeros_like(w2), b2))
    assert float((tok - static).abs().max()) <= 1e-5 * float(static.abs().max())


def test_token_wise_reads_v_in_place_from_fused_rows():
    """Q, K, V as strided views of one [B, N, 3, heads, 64] buffer (the layout a fused QKV
    projection leaves): the generator reads V's rows in place; same bits as from packed tensors."""
    B, heads, H, W, P = 2, 3, 13, 11, 2
    N = P + H * W
    q, k, v = synth.qkv(35, B, heads, N, 64, 0.5, True)
    tok = _dev(*synth.squeeze_weights(heads * 64, 64, 3, 3700))
    dq, dk, dv = (to_device(x, True) for x in (q, k, v))
    packed = torch.empty(dq.shape, dtype=torch.float32, device="cuda")
    binding.jv_linear_block_fwd(dq, dk, dv, packed, (H, W), token=tok)
    fused = torch.empty(B, N, 3, heads, 64, dtype=torch.bfloat16, device="cuda")
    for i, t in enumerate((dq, dk, dv)):
        fused[:, :, i] = t.permute(0, 2, 1, 3)
    fq, fk, fv = (fused[:, :, i].permute(0, 2, 1, 3) for i in range(3))
    in_place = torch.full_like(packed, float("nan"))
    binding.jv_linear_block_fwd(fq, fk, fv, in_place, (H, W), token=tok)
    assert torch.equal(packed, in_place)


def test_token_wise_rejects_unsupported():
    qb = torch.zeros(1, 1, 16, 64, device="cuda", dtype=torch.bfloat16)
    with pytest.raises(binding.JvError) as e:     # hidden not a multiple of 64
        binding.jv_linear_block_fwd(qb, qb.clone(), qb.clone(), torch.empty_like(qb), (4, 4),
                                    token=_dev(*synth.squeeze_weights(64, 8, 3, 2)))
    assert e.value.status == binding.JV_ERR_UNSUPPORTED


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
