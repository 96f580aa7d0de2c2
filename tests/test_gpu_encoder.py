"""GPU parity of the encoder pieces (LayerNorm, GEMM with fused epilogues) and of encoder blocks
against the CPU oracle.  bf16 operands, fp32 accumulation: max |g - r| / RMS(r) <= 2e-2."""
import numpy as np
import pytest
import torch

import oracle
from paper_2605_26636_amd import binding, synth
from parity import BF16_TOL, check, err_bf16, err_bf16_stored, err_fp32, to_host

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("rows,cols", [(37, 1024), (5, 64), (300, 4096), (3, 8), (64, 1000)])
def test_layernorm(rows, cols):
    x = synth.normal((rows, cols), 500 + cols) * 2.0 + 0.5
    g, b = 1.0 + 0.1 * synth.normal((cols,), 501), 0.1 * synth.normal((cols,), 502)
    ref = oracle.layernorm(x.astype(np.float64), g, b, 1e-6)
    dx, dg, db = (torch.from_numpy(t).cuda() for t in (x, g, b))
    y32 = torch.empty(rows, cols, device="cuda")
    binding.jv_layernorm_fwd(dx, dg, db, y32, 1e-6)
    check(err_fp32(to_host(y32), ref), 1e-4)
    y16 = torch.empty(rows, cols, device="cuda", dtype=torch.bfloat16)
    binding.jv_layernorm_fwd(dx, dg, db, y16, 1e-6)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    xb = synth.round_to_bf16(x)
    binding.jv_layernorm_fwd(torch.from_numpy(xb).cuda().to(torch.bfloat16), dg, db, y32, 1e-6)
    check(err_fp32(to_host(y32), oracle.layernorm(xb.astype(np.float64), g, b, 1e-6)), 1e-4)


@pytest.mark.parametrize("M,N,K", [
    (256, 256, 64),      # one tile, one K step
    (300, 520, 192),     # ragged M and N, three K steps
    (1, 8, 64),          # smallest
    (1024, 768, 1024),   # several tiles per XCD slot
    (515, 1024, 4096),   # long K
    (4600, 4360, 128),   # 324 ragged tiles: workgroups run two tiles as one stream of K blocks
    (6400, 6200, 64),    # 625 tiles of a single K block each: three tiles per workgroup in flight
])
def test_gemm_epilogues(M, N, K):
    a = synth.round_to_bf16(synth.normal((M, K), 600 + M))
    w = synth.round_to_bf16(synth.normal((N, K), 601 + N, 1.0 / np.sqrt(K)))
    bias = synth.normal((N,), 602) * 0.5
    res = synth.normal((M, N), 603)
    da, dw = (torch.from_numpy(t).cuda().to(torch.bfloat16) for t in (a, w))
    db, dr = torch.from_numpy(bias).cuda(), torch.from_numpy(res).cuda()
    plain = oracle.linear(a.astype(np.float64), w, bias)
    y32 = torch.full((M, N), float("nan"), device="cuda")
    binding.jv_gemm_bias_act(da, dw, db, None, y32, binding.JV_EPI_NONE)
    check(err_bf16(to_host(y32), plain), 1e-4)           # exact bf16 products, fp32 accumulation
    y16 = torch.full((M, N), float("nan"), device="cuda", dtype=torch.bfloat16)
    binding.jv_gemm_bias_act(da, dw, db, None, y16, binding.JV_EPI_NONE)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    binding.jv_gemm_bias_act(da, dw, None, None, y32, binding.JV_EPI_NONE)
    check(err_bf16(to_host(y32), plain - bias), 1e-4)
    binding.jv_gemm_bias_act(da, dw, db, None, y32, binding.JV_EPI_GELU)
    check(err_bf16(to_host(y32), oracle.gelu(plain)), 2e-4)   # erf approximated to 2.5e-5
    binding.jv_gemm_bias_act(da, dw, db, dr, y32, binding.JV_EPI_RESIDUAL)
    check(err_bf16(to_host(y32), plain + res), 1e-4)
    inplace = dr.clone()
    binding.jv_gemm_bias_act(da, dw, db, inplace, inplace, binding.JV_EPI_RESIDUAL)
    assert torch.equal(inplace, y32)
    # bf16 output takes a bf16 residual: the fp32 sum with the same (bf16-valued) residual, rounded once
    r16 = dr.to(torch.bfloat16)
    binding.jv_gemm_bias_act(da, dw, db, r16.float(), y32, binding.JV_EPI_RESIDUAL)
    binding.jv_gemm_bias_act(da, dw, db, r16, y16, binding.JV_EPI_RESIDUAL)
    assert torch.equal(y32.to(torch.bfloat16), y16)
    inplace16 = r16.clone()
    binding.jv_gemm_bias_act(da, dw, db, inplace16, inplace16, binding.JV_EPI_RESIDUAL)
    assert torch.equal(inplace16, y16)
    binding.jv_gemm_bias_act(da, dw, db, None, y32, binding.JV_EPI_SILU)
    check(err_bf16(to_host(y32), plain / (1.0 + np.exp(-plain))), 1e-4)


def test_gemm_rows_beyond_32_bit_offsets_and_rerun_bits():
    """A above 2^30 elements (270 336 rows of 4096: the fc2 shape of a 256 x 256 grid at batch 4):
    row tiles are addressed from 64-bit bases.  A is one 4096-row block repeated, so every block
    of y must repeat the first one bit for bit, and the first one is checked against the oracle.
    The same launch repeated gives the same bits (the operand ring is ordered by counted waits)."""
    rep, M0, K, N = 66, 4096, 4096, 64
    a = synth.round_to_bf16(synth.normal((M0, K), 640))
    w = synth.round_to_bf16(synth.normal((N, K), 641, 1.0 / np.sqrt(K)))
    bias = synth.normal((N,), 642)
    da = torch.from_numpy(a).cuda().to(torch.bfloat16).repeat(rep, 1)
    assert da.numel() > (1 << 30)
    dw, db = torch.from_numpy(w).cuda().to(torch.bfloat16), torch.from_numpy(bias).cuda()
    y = torch.full((rep * M0, N), float("nan"), device="cuda")
    binding.jv_gemm_bias_act(da, dw, db, None, y, binding.JV_EPI_NONE)
    check(err_bf16(to_host(y[:M0]), oracle.linear(a.astype(np.float64), w, bias)), 1e-4)
    assert torch.equal(y.view(rep, M0, N), y[:M0].expand(rep, M0, N))
    for _ in range(3):
        y2 = torch.empty_like(y)
        binding.jv_gemm_bias_act(da, dw, db, None, y2, binding.JV_EPI_NONE)
        assert torch.equal(y2, y)
    res = torch.from_numpy(synth.normal((M0, N), 643)).cuda().repeat(rep, 1)
    z = torch.empty_like(y)
    binding.jv_gemm_bias_act(da, dw, db, res, z, binding.JV_EPI_RESIDUAL)
    assert torch.equal(z, y + res)


def test_gemm_rejects_unsupported_shapes():
    a = torch.zeros(8, 96, device="cuda", dtype=torch.bfloat16)
    w = torch.zeros(16, 96, device="cuda", dtype=torch.bfloat16)
    y = torch.zeros(8, 16, device="cuda")
    with pytest.raises(binding.JvError) as e:
        binding.jv_gemm_bias_act(a, w, None, None, y)
    assert e.value.status == binding.JV_ERR_UNSUPPORTED


def _device_blocks(blocks):
    out = []
    for b in blocks:
        d = {}
        for k, v in b.items():
            if k == "dwc":      # convolution branch of a linear-attention block: fp32 device tensors
                d[k] = {"ksize": v.get("ksize", 3)}
                if v.get("static_kernel") is not None:
                    d[k]["static_kernel"] = torch.from_numpy(v["static_kernel"]).cuda()
                for kind in ("squeeze", "token"):
                    if v.get(kind) is not None:
                        d[k][kind] = tuple(torch.from_numpy(a).cuda() for a in v[kind])
                continue
            t = torch.from_numpy(v).cuda()
            d[k] = t.to(torch.bfloat16) if k.startswith("w_") else t
        out.append(d)
    return out


@pytest.mark.parametrize("fold", [False, True], ids=["layernorm passes", "layernorm folded"])
def test_small_encoder_each_mixer_and_pattern(fold):
    B, H, W, heads, hidden = 2, 8, 8, 2, 256
    C = heads * 64
    x = synth.normal((B, H * W, C), 700)
    blocks = [synth.block_weights(C, hidden, 710 + i) for i in range(3)]
    for b in blocks:                                    # non-trivial biases and LayerNorm parameters
        for key in ("b_qkv", "b_o", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
            b[key] = synth.normal(b[key].shape, 720 + len(key)) * 0.1
        b["ln1_g"] = 1.0 + 0.1 * synth.normal((C,), 730)
        b["ln2_g"] = 1.0 + 0.1 * synth.normal((C,), 731)
    dev = _device_blocks(blocks)
    dx = torch.from_numpy(x).cuda()
    for pattern in ([0, 0, 0], [1, 1, 1], [2, 2, 2], [0, 1, 2]):
        enc = binding.Encoder(dev, pattern, heads, hidden, window=(4, 4), fold_layernorm=fold)
        y = torch.empty_like(dx)
        enc.forward(dx, y, (H, W))
        ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 4))
        check(err_bf16(to_host(y), ref), BF16_TOL)
        y2 = dx.clone()
        enc.forward(y2, y2, (H, W))                     # in place
        assert torch.equal(y, y2)
        enc.close()


@pytest.mark.parametrize("stream_dtype", [torch.float32, torch.bfloat16], ids=["fp32 stream", "bf16 stream"])
def test_encoder_fused_linear_projection(stream_dtype):
    """The apply pass of the linear-attention blocks folded into their output projection
    (jv_encoder_fuse_linear_projection): the same block as a function, so the same oracle and
    the same bar; images of 256 and of 512 tokens (one and two GEMM row tiles per image), a
    pattern with all three mixers, in place, and the blocks the option does not apply to (a
    convolution branch; an image that is not a multiple of 256 tokens) unchanged by it."""
    heads, hidden = 3, 256
    C = heads * 64
    blocks = [synth.block_weights(C, hidden, 910 + i) for i in range(3)]
    for b in blocks:
        for key in ("b_qkv", "b_o", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
            b[key] = synth.normal(b[key].shape, 920 + len(key)) * 0.1
        b["ln1_g"] = 1.0 + 0.1 * synth.normal((C,), 930)
        b["ln2_g"] = 1.0 + 0.1 * synth.normal((C,), 931)
    dev = _device_blocks(blocks)
    # (a stream stored in bf16 is judged beyond the storage format's own rounding, as in its own test)
    err = err_bf16 if stream_dtype == torch.float32 else err_bf16_stored
    for (B, H, W), pattern in (((3, 16, 16), [0, 0, 0]), ((2, 16, 32), [0, 1, 0]), ((2, 16, 16), [2, 0, 1])):
        if stream_dtype == torch.bfloat16:   # two blocks at a time: the error of a bf16 stream grows with depth
            pattern = pattern[:2]
        x = synth.normal((B, H * W, C), 900 + H * W)
        dx = torch.from_numpy(x).cuda().to(stream_dtype)
        ref = oracle.encoder_forward(dx.float().cpu().numpy().astype(np.float64), blocks[:len(pattern)], pattern, H, W, heads, window=(8, 8))
        enc = binding.Encoder(dev[:len(pattern)], pattern, heads, hidden, window=(8, 8), stream_dtype=stream_dtype)
        plain = torch.empty_like(dx)
        enc.forward(dx, plain, (H, W))
        ws_plain = enc.workspace_bytes(B, (H, W))
        enc.fuse_linear_projection(True)
        assert enc.workspace_bytes(B, (H, W)) > ws_plain
        y = torch.empty_like(dx)
        enc.forward(dx, y, (H, W))
        e = err(to_host(y), ref)
        print(f"fused projection, {B} x {H * W} tokens, pattern {pattern}: {e:.2e}")
        check(e, BF16_TOL)
        assert not torch.equal(y, plain)                 # the fused path did run
        y2 = dx.clone()
        enc.forward(y2, y2, (H, W))                      # in place
        assert torch.equal(y, y2)
        enc.fuse_linear_projection(False)
        y3 = torch.empty_like(dx)
        enc.forward(dx, y3, (H, W))
        assert torch.equal(y3, plain)
        enc.close()
    # blocks the option does not apply to run as without it: 18 x 18 = 324 tokens per image
    B, H, W = 2, 18, 18
    x = synth.normal((B, H * W, C), 950)
    dx = torch.from_numpy(x).cuda().to(stream_dtype)
    enc = binding.Encoder(dev, [0, 0, 0], heads, hidden, window=(8, 8), stream_dtype=stream_dtype)
    plain = torch.empty_like(dx)
    enc.forward(dx, plain, (H, W))
    ws_plain = enc.workspace_bytes(B, (H, W))
    enc.fuse_linear_projection(True)
    assert enc.workspace_bytes(B, (H, W)) == ws_plain
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    assert torch.equal(y, plain)
    enc.close()


def test_vit_l_blocks_teacher_forced():
    """One ViT-L block per mixer type at the encoder workload's width (1024, 16 heads, MLP 4096)
    on a 32 x 32 grid, each fed the same input: per-block parity at full width."""
    B, H, W, heads, hidden = 1, 32, 32, 16, 4096
    C = heads * 64
    x = synth.normal((B, H * W, C), 800)
    wts = synth.block_weights(C, hidden, 810)
    dev = _device_blocks([wts])
    dx = torch.from_numpy(x).cuda()
    for mixer in (0, 1, 2):
        enc = binding.Encoder(dev, [mixer], heads, hidden, window=(16, 16))
        y = torch.empty_like(dx)
        enc.forward(dx, y, (H, W))
        ref = oracle.encoder_block(x.astype(np.float64), wts, mixer, H, W, heads, (16, 16))
        check(err_bf16(to_host(y), ref), BF16_TOL)
        # the block's own contribution (output minus input) is what the kernels computed
        check(err_bf16(to_host(y) - x, ref - x), BF16_TOL)
        if mixer == 0:  # the same block with the apply pass folded into the output projection
            enc.fuse_linear_projection(True)
            yf = torch.empty_like(dx)
            enc.forward(dx, yf, (H, W))
            assert not torch.equal(yf, y)
            check(err_bf16(to_host(yf), ref), BF16_TOL)
            check(err_bf16(to_host(yf) - x, ref - x), BF16_TOL)
        enc.close()
    # the same block with the stream carried in bf16 (input rounded first, output stored in bf16)
    xb = synth.round_to_bf16(x)
    dxb = torch.from_numpy(xb).cuda().to(torch.bfloat16)
    for mixer in (0, 1, 2):
        enc = binding.Encoder(dev, [mixer], heads, hidden, window=(16, 16), stream_dtype=torch.bfloat16)
        y = torch.empty_like(dxb)
        enc.forward(dxb, y, (H, W))
        ref = oracle.encoder_block(xb.astype(np.float64), wts, mixer, H, W, heads, (16, 16))
        check(err_bf16_stored(to_host(y), ref), BF16_TOL)
        enc.close()


def test_vit_l_block_fc2_with_split_k():
    """Few tokens leave fc2 (K = 4096, 1024 output features) with fewer output tiles than half
    the compute units; the encoder then splits its K loop over two or four workgroups per tile
    and adds the partial results in a second pass.  6 144 tokens (96 tiles: two parts) and 2 304
    tokens (36 tiles: four parts), a linear-attention block at ViT-L width, both stream types;
    a second run gives the same bits (the partial results are added in a fixed order)."""
    heads, hidden = 16, 4096
    C = heads * 64
    wts = synth.block_weights(C, hidden, 830)
    wts["b_fc2"] = synth.normal(wts["b_fc2"].shape, 831) * 0.1
    dev = _device_blocks([wts])
    for H, W in ((64, 96), (48, 48)):
        x = synth.round_to_bf16(synth.normal((1, H * W, C), 832 + H))
        ref = oracle.encoder_block(x.astype(np.float64), wts, 0, H, W, heads, (16, 16))
        for sd in (torch.float32, torch.bfloat16):
            dx = torch.from_numpy(x).cuda().to(sd)
            enc = binding.Encoder(dev, [0], heads, hidden, window=(16, 16), stream_dtype=sd)
            y = torch.empty_like(dx)
            enc.forward(dx, y, (H, W))
            check((err_bf16 if sd == torch.float32 else err_bf16_stored)(to_host(y), ref), BF16_TOL)
            z = dx.clone()
            enc.forward(z, z, (H, W))     # in place: the residual is the output
            assert torch.equal(z, y)
            enc.close()


@pytest.mark.parametrize("fold", [False, True], ids=["layernorm passes", "layernorm folded"])
def test_config5_first_six_blocks_full_size(fold):
    """The encoder workload at its real shape (64 x 64 grid, width 1024, 16 heads, MLP 4096),
    image 0, through blocks 0..5 of the benchmark pattern (window, linear, window, linear,
    window, full): every mixer and every GEMM shape at full size against the oracle."""
    H = W = 64
    heads, hidden, C = 16, 4096, 1024
    pattern = synth.encoder_pattern(24)[:6]
    assert pattern == [1, 0, 1, 0, 1, 2]
    x = synth.normal((4, H * W, C), 5003)[:1]
    blocks = [synth.block_weights(C, hidden, 5000 + l) for l in range(6)]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(16, 16), fold_layernorm=fold)
    dx = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(16, 16))
    check(err_bf16(to_host(y), ref), BF16_TOL)
    check(err_bf16(to_host(y) - x, ref - x), BF16_TOL)   # what the six blocks added
    enc.close()


@pytest.mark.parametrize("fold", [False, True], ids=["layernorm passes", "layernorm folded"])
def test_config5_full_depth_against_oracle(fold):
    """All 24 blocks of the encoder workload (4 full / 12 window / 8 linear) on image 0 at full
    size against the oracle's fp64 forward: the end-to-end drift, printed, and held to the same
    2e-2 RMS bar as a single block (measured: 1.2e-2 at every tap and at the end; the stream's
    own RMS grows with depth as fast as the roundings the blocks add)."""
    H = W = 64
    heads, hidden, C, L = 16, 4096, 1024, 24
    pattern = synth.encoder_pattern(L)
    x = synth.normal((4, H * W, C), 5003)[:1]
    blocks = [synth.block_weights(C, hidden, 5000 + l) for l in range(L)]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(16, 16), fold_layernorm=fold)
    dx = torch.from_numpy(np.ascontiguousarray(x)).cuda()
    y = torch.empty_like(dx)
    taps = {l: torch.empty_like(dx) for l in (5, 11, 17)}
    enc.forward(dx, y, (H, W), taps=taps)
    ref, kept = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(16, 16), taps={5, 11, 17})
    for l in (5, 11, 17):
        e = err_bf16(to_host(taps[l]), kept[l])
        rms = float(np.sqrt(np.mean((to_host(taps[l]) - kept[l]) ** 2)) / np.sqrt(np.mean(kept[l] ** 2)))
        print(f"    after block {l}: max |g - r| / RMS {e:.3e}, RMS error / RMS {rms:.3e}")
    got = to_host(y)
    rms = float(np.sqrt(np.mean((got - ref) ** 2)) / np.sqrt(np.mean(ref ** 2)))
    print(f"    after block 23: RMS error / RMS {rms:.3e}")
    check(err_bf16(got, ref), BF16_TOL)
    enc.close()


def test_refused_forward_touches_nothing():
    """A (batch, grid) the pass cannot run is refused before the first launch: y keeps its
    bytes, and the workspace query answers 0 for it."""
    heads, hidden = 2, 256
    C = heads * 64
    enc = binding.Encoder(_device_blocks([synth.block_weights(C, hidden, 1100)]), [1], heads, hidden, window=(1, 1))
    H = W = 300                       # 90 000 windows of one token: above the 65 535 the kernels index
    assert enc.workspace_bytes(1, (H, W)) == 0
    assert enc.workspace_bytes(1, (200, 200)) > 0
    x = torch.zeros(1, H * W, C, device="cuda")
    y = torch.full_like(x, 3.25)
    ws = torch.empty(enc.workspace_bytes(1, (200, 200)) * 4, dtype=torch.uint8, device="cuda")
    with pytest.raises(binding.JvError) as e:
        enc.forward(x, y, (H, W), ws)
    assert e.value.status == binding.JV_ERR_UNSUPPORTED
    torch.cuda.synchronize()
    assert float(y.min()) == 3.25 and float(y.max()) == 3.25
    enc.close()


def test_config5_full_depth_batch_properties():
    """All 24 blocks on the whole batch of 4: the result is finite, and every image comes out
    as it does when it is run alone (images never mix; only the split of the linear-attention
    state reduction depends on the batch size, hence tolerances instead of equality)."""
    H = W = 64
    heads, hidden, C, L = 16, 4096, 1024, 24
    pattern = synth.encoder_pattern(L)
    assert (pattern.count(2), pattern.count(1), pattern.count(0)) == (4, 12, 8)
    blocks = _device_blocks([synth.block_weights(C, hidden, 5000 + l) for l in range(L)])
    enc = binding.Encoder(blocks, pattern, heads, hidden, window=(16, 16))
    dx = torch.from_numpy(synth.normal((4, H * W, C), 5003)).cuda()
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    assert torch.isfinite(y).all()
    for img in (0, 3):
        y1 = torch.empty(1, H * W, C, device="cuda")
        enc.forward(dx[img:img + 1].contiguous(), y1, (H, W))
        rms = float(y1.pow(2).mean().sqrt())
        diff = y1[0] - y[img]
        err_max, err_rms = float(diff.abs().max()) / rms, float(diff.pow(2).mean().sqrt()) / rms
        print(f"    image {img}: |batch - alone| / RMS: max {err_max:.2e}, rms {err_rms:.2e}")
        # a different summation order moves a few bf16 roundings, which 24 blocks then carry along
        assert err_rms <= 5e-3 and err_max <= 5e-2
    enc.close()


def test_encoder_linear_blocks_with_convolution_branch():
    """Linear-attention blocks carrying the paper's convolution branch (squeeze-dynamic and
    static filters) inside the encoder, next to a window block, against the oracle."""
    B, H, W, heads, hidden = 2, 12, 10, 2, 256
    C = heads * 64
    x = synth.normal((B, H * W, C), 900)
    blocks = [synth.block_weights(C, hidden, 910 + i) for i in range(3)]
    blocks[0]["dwc"] = {"squeeze": synth.squeeze_weights(C, 8, 3, 920), "ksize": 3}
    blocks[2]["dwc"] = {"static_kernel": synth.dwc_static_kernel(C, 5, 921), "ksize": 5}
    pattern = [0, 1, 0]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(4, 5))
    dx = torch.from_numpy(x).cuda()
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 5))
    check(err_bf16(to_host(y), ref), BF16_TOL)
    # the branch really ran: without it the result differs
    for b in blocks:
        b.pop("dwc", None)
    plain = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 5))
    assert err_bf16(to_host(y), plain) > 10 * BF16_TOL
    enc.close()


def test_encoder_token_wise_dynamic_filters():
    """A linear-attention block with per-token dynamic filters (the variant Tab. 1 lists as
    "Token-wise Dynamic DWC") inside the encoder, where V is read in place from the fused QKV
    rows; with and without prefix tokens."""
    H, W, heads, hidden = 9, 11, 2, 256
    C = heads * 64
    blocks = [synth.block_weights(C, hidden, 930 + i) for i in range(2)]
    # generator weights scaled down so that the branch adds about as much as the stream holds
    # (at full scale it is 5x the stream, and the result is the branch's own bf16 chain)
    for l, (hid, ks) in enumerate(((64, 3), (128, 5))):
        w1, b1, w2, b2 = synth.squeeze_weights(C, hid, ks, 940 + l)
        quarter = np.float32(0.25)
        blocks[l]["dwc"] = {"token": (w1 * quarter, b1, w2 * quarter, b2 * quarter), "ksize": ks}
    pattern = [0, 0]
    dev = _device_blocks(blocks)
    for B, P in ((2, 0), (1, 3)):
        x = synth.normal((B, P + H * W, C), 950 + P)
        enc = binding.Encoder(dev, pattern, heads, hidden, n_prefix=P)
        dx = torch.from_numpy(x).cuda()
        y = torch.empty_like(dx)
        enc.forward(dx, y, (H, W))
        ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, n_prefix=P)
        check(err_bf16(to_host(y), ref), BF16_TOL)
        plain = oracle.encoder_forward(x, [{k: v for k, v in b.items() if k != "dwc"} for b in blocks],
                                       pattern, H, W, heads, n_prefix=P)
        assert err_bf16(to_host(y), plain) > 10 * BF16_TOL
        enc.close()


def test_encoder_bf16_residual_stream():
    """The residual stream carried in bf16 (x, y and the taps are bf16; each block rounds the
    stream twice): every mixer, prefix tokens and a tap, two blocks at a time (the error of a
    stream stored in bf16 grows by about half a percent of its RMS per block of this small
    width), against the fp64 oracle run on the bf16-valued input."""
    B, H, W, heads, hidden, P = 2, 8, 9, 2, 256, 3
    C = heads * 64
    x = synth.round_to_bf16(synth.normal((B, P + H * W, C), 975))
    dx = torch.from_numpy(x).cuda().to(torch.bfloat16)
    for pattern, seed in (([0, 1], 960), ([2, 0], 962)):
        blocks = [synth.block_weights(C, hidden, seed + i) for i in range(2)]
        if pattern[0] == 0:
            blocks[0]["dwc"] = {"squeeze": synth.squeeze_weights(C, 8, 3, 970), "ksize": 3}
        enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(4, 3), n_prefix=P,
                              stream_dtype=torch.bfloat16)
        y = torch.full_like(dx, float("nan"))
        tap = torch.full_like(dx, float("nan"))
        enc.forward(dx, y, (H, W), taps={0: tap})
        ref, kept = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 3), taps=[0], n_prefix=P)
        # stored in bf16: the bar is 2e-2 RMS beyond the storage format's own rounding (2^-8 |r|)
        check(err_bf16_stored(to_host(tap), kept[0]), BF16_TOL)
        check(err_bf16_stored(to_host(y), ref), BF16_TOL)
        # in place, and the same bits as out of place
        z = dx.clone()
        enc.forward(z, z, (H, W))
        assert torch.equal(z, y)
        with pytest.raises(ValueError):   # an fp32 tensor for a bf16 stream
            enc.forward(dx.float(), y, (H, W))
        enc.close()


def test_folded_layernorm_variants():
    """LayerNorms folded into the products behind them: non-trivial gamma and beta, a stream whose
    tokens have a mean of the size of their spread (the case the folded form is most sensitive to),
    prefix tokens, taps, ragged token counts, fp32 and bf16 streams, in place; and switching the
    fold off again gives back the bits of the separate passes."""
    B, H, W, heads, hidden, P = 2, 7, 9, 3, 320, 2
    C = heads * 64
    x = synth.normal((B, P + H * W, C), 1200) + 0.8
    blocks = [synth.block_weights(C, hidden, 1210 + i) for i in range(4)]
    for i, b in enumerate(blocks):
        for key in ("b_qkv", "b_o", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
            b[key] = synth.normal(b[key].shape, 1220 + 7 * i + len(key)) * 0.2
        b["ln1_g"] = 1.0 + 0.3 * synth.normal((C,), 1230 + i)
        b["ln2_g"] = 0.7 + 0.3 * synth.normal((C,), 1240 + i)
    pattern = [1, 0, 2, 0]
    dev = _device_blocks(blocks)
    ref, kept = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 3), taps=[1], n_prefix=P)
    dx = torch.from_numpy(x).cuda()
    enc = binding.Encoder(dev, pattern, heads, hidden, window=(4, 3), n_prefix=P)
    plain = torch.empty_like(dx)
    enc.forward(dx, plain, (H, W))
    enc.fold_layernorm()
    y, tap = torch.full_like(dx, float("nan")), torch.full_like(dx, float("nan"))
    enc.forward(dx, y, (H, W), taps={1: tap})
    check(err_bf16(to_host(y), ref), BF16_TOL)
    check(err_bf16(to_host(tap), kept[1]), BF16_TOL)
    assert not torch.equal(y, plain)                    # another rounding order: the fold really ran
    z = dx.clone()
    enc.forward(z, z, (H, W))                           # in place
    assert torch.equal(z, y)
    enc.fold_layernorm(False)
    again = torch.empty_like(dx)
    enc.forward(dx, again, (H, W))
    assert torch.equal(again, plain)
    enc.close()
    # bf16 stream: the residual products' own output is what the folded products read
    xb = synth.round_to_bf16(x)
    dxb = torch.from_numpy(xb).cuda().to(torch.bfloat16)
    refb = oracle.encoder_forward(xb, blocks[:2], pattern[:2], H, W, heads, window=(4, 3), n_prefix=P)
    enc = binding.Encoder(dev[:2], pattern[:2], heads, hidden, window=(4, 3), n_prefix=P,
                          stream_dtype=torch.bfloat16, fold_layernorm=True)
    yb = torch.full_like(dxb, float("nan"))
    enc.forward(dxb, yb, (H, W))
    check(err_bf16_stored(to_host(yb), refb), BF16_TOL)
    enc.close()


def test_encoder_taps_intermediate_streams():
    """jv_encoder_forward_taps: the residual stream after chosen blocks (what a dense-prediction
    head reads), against the oracle; the final output is bit-identical to the untapped run; a tap
    on the last block equals y; invalid tap lists are rejected before any launch."""
    B, H, W, heads, hidden = 2, 8, 6, 2, 256
    C = heads * 64
    x = synth.normal((B, H * W, C), 950)
    blocks = [synth.block_weights(C, hidden, 960 + i) for i in range(5)]
    pattern = [0, 1, 2, 1, 0]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(4, 3))
    dx = torch.from_numpy(x).cuda()
    y_plain = torch.empty_like(dx)
    enc.forward(dx, y_plain, (H, W))
    ref, kept = oracle.encoder_forward(x, blocks, pattern, H, W, heads, window=(4, 3), taps={0, 2, 4})
    taps = {l: torch.full_like(dx, float("nan")) for l in (0, 2, 4)}
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W), taps=taps)
    assert torch.equal(y, y_plain)
    assert torch.equal(taps[4], y)
    for l in (0, 2, 4):
        check(err_bf16(to_host(taps[l]), kept[l]), BF16_TOL)
    check(err_bf16(to_host(y), ref), BF16_TOL)
    # in place (y is x) with taps
    y2 = dx.clone()
    t2 = {1: torch.empty_like(dx)}
    enc.forward(y2, y2, (H, W), taps=t2)
    assert torch.equal(y2, y_plain)
    # rejected: block index out of range, tap buffer aliasing y
    with pytest.raises(binding.JvError):
        enc.forward(dx, y, (H, W), taps={5: torch.empty_like(dx)})
    with pytest.raises(binding.JvError):
        enc.forward(dx, y, (H, W), taps={1: y})
    enc.close()


def test_encoder_focused_feature_map_variant():
    """la_focus_p: linear-attention blocks with the focused map (and a static convolution
    branch), the variant of the paper's block ablation, against the oracle."""
    B, H, W, heads, hidden = 2, 9, 7, 2, 256
    C = heads * 64
    x = synth.normal((B, H * W, C), 970)
    blocks = [synth.block_weights(C, hidden, 980 + i) for i in range(2)]
    blocks[1]["dwc"] = {"static_kernel": synth.dwc_static_kernel(C, 3, 990), "ksize": 3}
    pattern = [0, 0]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, la_focus_p=3)
    dx = torch.from_numpy(x).cuda()
    y = torch.empty_like(dx)
    enc.forward(dx, y, (H, W))
    ref = oracle.encoder_forward(x, blocks, pattern, H, W, heads, la_focus_p=3)
    check(err_bf16(to_host(y), ref), BF16_TOL)
    relu = oracle.encoder_forward(x, blocks, pattern, H, W, heads)
    assert err_bf16(to_host(y), relu) > 5 * BF16_TOL   # the map really differs from ReLU
    enc.close()


def test_encoder_forward_under_graph_capture():
    """The forward pass allocates nothing and never synchronises, so it can be captured in a HIP
    graph (after one eager call, which raises the kernels' LDS limits): every replay, with new
    input copied into the captured buffers and eager work in between, equals the eager result."""
    B, H, W, heads, hidden = 1, 16, 16, 2, 256
    C = heads * 64
    blocks = [synth.block_weights(C, hidden, 1010 + i) for i in range(3)]
    blocks[0]["dwc"] = {"squeeze": synth.squeeze_weights(C, 8, 3, 1020), "ksize": 3}
    pattern = [0, 1, 2]
    enc = binding.Encoder(_device_blocks(blocks), pattern, heads, hidden, window=(16, 16))
    xs = [torch.from_numpy(synth.normal((B, H * W, C), 1030 + i)).cuda() for i in range(3)]
    eager = []
    ws = torch.empty(enc.workspace_bytes(B, (H, W)), dtype=torch.uint8, device="cuda")
    for x in xs:
        y = torch.empty_like(x)
        enc.forward(x, y, (H, W), ws)
        eager.append(y)
    torch.cuda.synchronize()
    x_cap, y_cap, tap_cap = torch.empty_like(xs[0]), torch.empty_like(xs[0]), torch.empty_like(xs[0])
    x_cap.copy_(xs[0])
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            enc.forward(x_cap, y_cap, (H, W), ws, stream=side, taps={1: tap_cap})
    torch.cuda.current_stream().wait_stream(side)
    for rep in range(2):
        for x, want in zip(xs, eager):
            x_cap.copy_(x)
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(y_cap, want)
            scratch = torch.empty_like(x)
            enc.forward(x, scratch, (H, W), ws)        # eager work between the replays
            torch.cuda.synchronize()
            assert torch.equal(scratch, want)
    enc.close()


def test_gemm_random_shapes_all_epilogues():
    """Seeded sweep of ragged GEMM shapes (M arbitrary, N a multiple of 8, K a multiple of 64:
    edge tiles in both directions, one to nine K blocks, one or several tiles per workgroup
    slot), every epilogue with both output types, against the oracle's fp64 product."""
    rng = np.random.Generator(np.random.Philox(20260527))
    for case in range(10):
        M = int(rng.integers(1, 900))
        N = 8 * int(rng.integers(1, 110))
        K = 64 * int(rng.integers(1, 10))
        a = synth.round_to_bf16(synth.normal((M, K), 7000 + case))
        w = synth.round_to_bf16(synth.normal((N, K), 7100 + case, 1.0 / np.sqrt(K)))
        bias = synth.normal((N,), 7200 + case) * 0.5
        res = synth.normal((M, N), 7300 + case)
        da, dw = (torch.from_numpy(t).cuda().to(torch.bfloat16) for t in (a, w))
        db, dr = torch.from_numpy(bias).cuda(), torch.from_numpy(res).cuda()
        plain = oracle.linear(a.astype(np.float64), w, bias)
        want = {binding.JV_EPI_NONE: plain, binding.JV_EPI_GELU: oracle.gelu(plain),
                binding.JV_EPI_RESIDUAL: plain + res, binding.JV_EPI_SILU: plain / (1.0 + np.exp(-plain))}
        print(f"  case {case}: M {M} N {N} K {K}", flush=True)
        for epi, ref in want.items():
            # guard rows around y: nothing may be written outside [M, N]
            pad32 = torch.full((M + 2, N), 768.0, device="cuda")
            y32 = pad32[1:M + 1]
            binding.jv_gemm_bias_act(da, dw, db, dr if epi == binding.JV_EPI_RESIDUAL else None, y32, epi)
            check(err_bf16(to_host(y32), ref), 2e-4)
            assert float(pad32[0].min()) == 768.0 and float(pad32[M + 1].max()) == 768.0
            pad16 = torch.full((M + 2, N), 768.0, device="cuda", dtype=torch.bfloat16)
            y16 = pad16[1:M + 1]
            if epi == binding.JV_EPI_RESIDUAL:   # a bf16 residual; reference: the same values in fp32
                r16 = dr.to(torch.bfloat16)
                binding.jv_gemm_bias_act(da, dw, db, r16.float(), y32, epi)
                binding.jv_gemm_bias_act(da, dw, db, r16, y16, epi)
            else:
                binding.jv_gemm_bias_act(da, dw, db, None, y16, epi)
            assert torch.equal(y32.to(torch.bfloat16), y16)
            assert float(pad16[0].float().min()) == 768.0 and float(pad16[M + 1].float().max()) == 768.0
