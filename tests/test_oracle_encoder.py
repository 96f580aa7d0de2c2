"""Pins for the oracle's encoder pieces (LayerNorm, linear, GELU, block) and the DWC branch."""
import numpy as np
import torch
import torch.nn.functional as F

import oracle
from paper_2605_26636_amd import synth


def test_layernorm_properties_and_library():
    x = synth.normal((7, 33), 1).astype(np.float64) * 3 + 2
    ones, zeros = np.ones(33, np.float32), np.zeros(33, np.float32)
    y = oracle.layernorm(x, ones, zeros, eps=0.0)
    assert np.abs(y.mean(-1)).max() < 1e-14 and np.abs(y.var(-1) - 1).max() < 1e-13
    g, b = synth.normal((33,), 2), synth.normal((33,), 3)
    ref = F.layer_norm(torch.from_numpy(x), (33,), torch.from_numpy(g).double(),
                       torch.from_numpy(b).double(), eps=1e-6).numpy()
    assert np.abs(oracle.layernorm(x, g, b, 1e-6) - ref).max() < 1e-13
    # constant row: variance 0 -> output = beta exactly (eps keeps the division finite)
    assert np.array_equal(oracle.layernorm(np.full((1, 33), 4.0), g, b, 1e-6)[0], b.astype(np.float64))


def test_linear_against_library_matmul():
    a = synth.normal((5, 17), 4).astype(np.float64)
    w, b = synth.normal((9, 17), 5), synth.normal((9,), 6)
    ref = a @ w.astype(np.float64).T + b
    assert np.abs(oracle.linear(a, w, b) - ref).max() < 1e-13
    assert np.abs(oracle.linear(a, w) - (ref - b)).max() < 1e-13
    # identity weight reproduces the input; a transposed operand would fail on a non-square W
    assert np.array_equal(oracle.linear(a, np.eye(17, dtype=np.float32)), a)


def test_gelu_values(golden):
    g = golden("gelu_values.txt")
    assert np.abs(oracle.gelu(np.array(g["x"])) - np.array(g["gelu"])).max() < 1e-15
    x = synth.normal((100,), 7).astype(np.float64) * 3
    assert np.abs(oracle.gelu(x) - F.gelu(torch.from_numpy(x)).numpy()).max() < 1e-14


def test_dwc_hand_case_and_library(golden):
    g = golden("dwc_hand_case.txt")
    v = np.array(g["v"], dtype=np.float32).reshape(1, 1, 9, 1)
    for name in ("plus", "corner"):
        kern = np.array(g["kernel_" + name]).reshape(1, 1, 3, 3)
        assert oracle.dwc(v, kern, 3, 3).reshape(-1).tolist() == g["out_" + name]
    # against conv2d (a cross-correlation) with groups = C, on a ragged grid, k = 3 and 5
    B, heads, H, W, d = 2, 2, 5, 7, 4
    v = synth.normal((B, heads, H * W, d), 8)
    img = torch.from_numpy(v).double().permute(0, 1, 3, 2).reshape(B, heads * d, H, W)
    for k in (3, 5):
        kern = synth.normal((1, heads * d, k, k), 9).astype(np.float64)
        ref = F.conv2d(img, torch.from_numpy(kern[0])[:, None], padding=k // 2, groups=heads * d)
        ref = ref.reshape(B, heads, d, H * W).permute(0, 1, 3, 2).numpy()
        assert np.abs(oracle.dwc(v, kern, H, W) - ref).max() < 1e-13
        per_image = np.concatenate([kern, 2 * kern])
        got = oracle.dwc(v, per_image, H, W)
        assert np.abs(got[0] - ref[0]).max() < 1e-13 and np.abs(got[1] - 2 * ref[1]).max() < 1e-13


def test_linear_block_special_kernels():
    B, heads, H, W, d = 1, 2, 4, 5, 8
    q, k, v = synth.qkv(50, B, heads, H * W, d, 1.0, False)
    C = heads * d
    la = oracle.linear_attn_quadratic(q, k, v, 1e-6)
    assert np.array_equal(oracle.linear_block(q, k, v, H, W, static_kernel=np.zeros((C, 3, 3))), la)
    delta = np.zeros((C, 3, 3)); delta[:, 1, 1] = 1
    assert np.abs(oracle.linear_block(q, k, v, H, W, static_kernel=delta) - (la + v)).max() < 1e-15


def test_squeeze_kernel_generator():
    B, heads, N, d, k, hidden = 2, 2, 12, 4, 3, 5
    C = heads * d
    v = synth.normal((B, heads, N, d), 60)
    w1, b1 = synth.normal((hidden, C), 61), synth.normal((hidden,), 62)
    w2, b2 = synth.normal((C * k * k, hidden), 63), synth.normal((C * k * k,), 64)
    kap = oracle.squeeze_kernel(v, w1, b1, w2, b2, k)
    g = torch.from_numpy(v).double().mean(dim=2).reshape(B, C)          # channel = head*d + c
    u = F.silu(g @ torch.from_numpy(w1).double().T + torch.from_numpy(b1).double())
    ref = (u @ torch.from_numpy(w2).double().T + torch.from_numpy(b2).double()).reshape(B, C, k, k)
    assert np.abs(kap - ref.numpy()).max() < 1e-13
    # W2 = 0: the dynamic kernel is the static kernel b2, for every image
    kap0 = oracle.squeeze_kernel(v, w1, b1, np.zeros_like(w2), b2, k)
    assert np.array_equal(kap0[0], b2.astype(np.float64).reshape(C, k, k)) and np.array_equal(kap0[0], kap0[1])
    # the kernel depends on V only through its token mean: permuting tokens changes nothing
    perm = np.random.Generator(np.random.Philox(3)).permutation(N)
    assert np.abs(oracle.squeeze_kernel(v[:, :, perm], w1, b1, w2, b2, k) - kap).max() < 1e-13


def _block_weights(C, hidden, seed):
    return synth.block_weights(C, hidden, seed, bf16=False)


def test_encoder_block_against_torch_modules():
    B, H, W, C, heads, hidden = 2, 4, 4, 32, 2, 64
    x = synth.normal((B, H * W, C), 70).astype(np.float64)
    wts = _block_weights(C, hidden, 71)
    for key in ("b_qkv", "b_o", "b_fc1", "b_fc2", "ln1_b", "ln2_b"):
        wts[key] = synth.normal(wts[key].shape, 80 + len(key)) * 0.1        # non-zero biases
    got = oracle.encoder_block(x, wts, oracle.MIX_FULL, H, W, heads)
    t = {k: torch.from_numpy(v).double() for k, v in wts.items()}
    xt = torch.from_numpy(x)
    a = F.layer_norm(xt, (C,), t["ln1_g"], t["ln1_b"], 1e-6)
    o, _ = F.multi_head_attention_forward(
        a.transpose(0, 1), a.transpose(0, 1), a.transpose(0, 1), C, heads, t["w_qkv"], t["b_qkv"],
        None, None, False, 0.0, t["w_o"], t["b_o"], need_weights=False)
    xt = xt + o.transpose(0, 1)
    m = F.layer_norm(xt, (C,), t["ln2_g"], t["ln2_b"], 1e-6)
    xt = xt + F.linear(F.gelu(F.linear(m, t["w_fc1"], t["b_fc1"])), t["w_fc2"], t["b_fc2"])
    assert np.abs(got - xt.numpy()).max() < 1e-5       # q, k, v pass through float32 in the oracle


def test_encoder_patterns():
    B, H, W, C, heads, hidden = 1, 4, 4, 32, 2, 64
    x = synth.normal((B, H * W, C), 90)
    blocks = [_block_weights(C, hidden, 91 + i) for i in range(3)]
    full = oracle.encoder_forward(x, blocks, [oracle.MIX_FULL] * 3, H, W, heads)
    whole = oracle.encoder_forward(x, blocks, [oracle.MIX_WINDOW] * 3, H, W, heads, window=(H, W))
    assert np.abs(full - whole).max() < 1e-12
    pattern = synth.encoder_pattern(24)
    assert pattern.count(oracle.MIX_FULL) == 4 and pattern.count(oracle.MIX_WINDOW) == 12
    assert pattern.count(oracle.MIX_LINEAR) == 8
    assert [i for i, p in enumerate(pattern) if p == oracle.MIX_FULL] == [5, 11, 17, 23]


def test_linear_block_with_prefix_tokens():
    """Prefix tokens are ordinary tokens of the linear attention and of the filter generator's
    token average; the convolution runs over the grid tokens only."""
    P, H, W, heads, d = 2, 4, 5, 2, 16
    N, C = P + H * W, heads * d
    q, k, v = (synth.normal((1, heads, N, d), 500 + i) for i in range(3))
    kern = synth.dwc_static_kernel(C, 3, 510)
    o = oracle.linear_block(q, k, v, H, W, static_kernel=kern)
    la = oracle.linear_attn_quadratic(q, k, v)
    assert np.abs(o[:, :, :P] - la[:, :, :P]).max() < 1e-15          # prefix rows: no convolution term
    conv = oracle.dwc(np.ascontiguousarray(v[:, :, P:]), kern[None], H, W)
    assert np.abs(o[:, :, P:] - (la[:, :, P:] + conv)).max() < 1e-12
    # changing a prefix value row changes the convolution term of no grid token ...
    v2 = v.copy(); v2[:, :, 0] += 1.0
    conv_part = lambda vv: oracle.linear_block(q, k, vv, H, W, static_kernel=kern) - oracle.linear_attn_quadratic(q, k, vv)
    assert np.abs(conv_part(v2) - conv_part(v)).max() < 1e-12
    # ... but it moves the token average the dynamic filters are generated from
    sq = synth.squeeze_weights(C, 4, 3, 520)
    ka, kb = oracle.squeeze_kernel(v, *sq, 3), oracle.squeeze_kernel(v2, *sq, 3)
    assert np.abs(ka - kb).max() > 1e-6
    g = v.astype(np.float64).transpose(0, 2, 1, 3).reshape(1, N, C).mean(1)     # mean over all N tokens
    u = sq[0].astype(np.float64) @ g[0] + sq[1]
    u = u / (1.0 + np.exp(-u))
    want = (sq[2].astype(np.float64) @ u + sq[3]).reshape(C, 3, 3)
    assert np.abs(ka[0] - want).max() < 1e-12


def test_tokenwise_dynamic_filters():
    """Pins of the per-token dynamic convolution (Sec. 3.2.1; Tab. 1, "Token-wise Dynamic DWC")."""
    B, heads, H, W, d, k, hidden = 2, 2, 4, 5, 4, 3, 6
    C, N = heads * d, H * W
    v = synth.normal((B, heads, N, d), 70)
    w1, b1 = synth.normal((hidden, C), 71), synth.normal((hidden,), 72)
    w2, b2 = synth.normal((C * k * k, hidden), 73), synth.normal((C * k * k,), 74)
    # (1) W2 = 0: every token's filters are the static bank b2 -> the static convolution
    kap0 = oracle.tokenwise_kernels(v, w1, b1, np.zeros_like(w2), b2, k)
    static = b2.astype(np.float64).reshape(1, C, k, k)
    assert np.abs(oracle.dwc_tokenwise(v, kap0, H, W) - oracle.dwc(v, static, H, W)).max() < 1e-14
    # (2) an image whose tokens are all equal: each token equals the token average, so the
    # per-token filters are the per-image filters of the squeeze generator
    flat = np.ascontiguousarray(np.broadcast_to(v[:, :, :1], v.shape))
    kap = oracle.tokenwise_kernels(flat, w1, b1, w2, b2, k)
    per_image = oracle.squeeze_kernel(flat, w1, b1, w2, b2, k)
    assert np.abs(kap - per_image[:, None]).max() < 1e-6      # squeeze_kernel reads V as fp32
    assert np.abs(oracle.dwc_tokenwise(flat, kap, H, W) - oracle.dwc(flat, per_image, H, W)).max() < 1e-5
    # (3) the generator against library modules, token by token
    rows = torch.from_numpy(v).double().permute(0, 2, 1, 3).reshape(B, N, C)
    u = F.silu(rows @ torch.from_numpy(w1).double().T + torch.from_numpy(b1).double())
    ref = (u @ torch.from_numpy(w2).double().T + torch.from_numpy(b2).double()).reshape(B, N, C, k, k)
    full = oracle.tokenwise_kernels(v, w1, b1, w2, b2, k)
    assert np.abs(full - ref.numpy()).max() < 1e-13
    # (4) brute force of the convolution: the OUTPUT token's filters weight its neighbourhood
    want = np.zeros((B, heads, N, d))
    for b in range(B):
        for n in range(N):
            r, s = divmod(n, W)
            for ch in range(C):
                hh, c = divmod(ch, d)
                for di in range(k):
                    for dj in range(k):
                        r2, s2 = r + di - k // 2, s + dj - k // 2
                        if 0 <= r2 < H and 0 <= s2 < W:
                            want[b, hh, n, c] += full[b, n, ch, di, dj] * float(v[b, hh, r2 * W + s2, c])
    assert np.abs(oracle.dwc_tokenwise(v, full, H, W) - want).max() < 1e-13
    # (5) closed form with one live path: hidden unit 0 reads channel c0, filter entry
    # (channel c1, tap (0, 2)) reads hidden unit 0 -> out[n, c1] = w silu(a v[n, c0] + bias) v[n - W + 1, c1]
    c0, c1, a, bias, w = 1, 6, 0.7, -0.2, 1.3
    w1s = np.zeros((hidden, C)); w1s[0, c0] = a
    b1s = np.zeros(hidden); b1s[0] = bias
    w2s = np.zeros((C * k * k, hidden)); w2s[c1 * k * k + 0 * k + 2, 0] = w
    got = oracle.dwc_tokenwise(v, oracle.tokenwise_kernels(v, w1s, b1s, w2s, np.zeros(C * k * k), k), H, W)
    for n in range(N):
        r, s = divmod(n, W)
        pre = a * float(v[0, c0 // d, n, c0 % d]) + bias
        nb = float(v[0, c1 // d, (r - 1) * W + s + 1, c1 % d]) if r >= 1 and s + 1 < W else 0.0
        assert abs(got[0, c1 // d, n, c1 % d] - w * pre / (1 + np.exp(-pre)) * nb) < 1e-14
    assert np.count_nonzero(np.delete(got.transpose(0, 2, 1, 3).reshape(B, N, C), c1, axis=2)) == 0
    # (6) in the block: added on the grid tokens only; a prefix token changes nothing there
    q, kk_, vv = synth.qkv(75, 1, heads, 2 + N, d, 1.0, False)
    tok = (w1, b1, w2, b2)
    out = oracle.linear_block(q, kk_, vv, H, W, token=tok)
    la = oracle.linear_attn_quadratic(q, kk_, vv, 1e-6)
    assert np.array_equal(out[:, :, :2], la[:, :, :2])
    vg = np.ascontiguousarray(vv[:, :, 2:])
    conv = oracle.dwc_tokenwise(vg, oracle.tokenwise_kernels(vg, *tok, k), H, W)
    assert np.abs(out[:, :, 2:] - la[:, :, 2:] - conv).max() < 1e-13


def test_layernorm_folded_into_the_next_product_is_the_same_function():
    """The identity the encoder's folded LayerNorm rests on (Sec. 3.2.3's inherited pre-LN block):
    W LN(x) + b = (1/sigma) ((W gamma) x - mean (W gamma) 1) + (W beta + b), with the row
    statistics merged from groups of 64 features by the pairwise update of mean and squared
    deviations -- checked against the oracle's LayerNorm followed by its linear layer."""
    T, C, N, eps = 9, 192, 40, 1e-6
    x = synth.normal((T, C), 41).astype(np.float64) * 2.0 + 0.7
    gamma, beta = 1.0 + 0.2 * synth.normal((C,), 42), 0.3 * synth.normal((C,), 43)
    w, b = synth.normal((N, C), 44) / 8, synth.normal((N,), 45)
    want = oracle.linear(oracle.layernorm(x, gamma, beta, eps), w, b)
    # statistics per group of 64 features, then merged group by group
    cnt, mean, m2 = 0.0, np.zeros(T), np.zeros(T)
    for g0 in range(0, C, 64):
        part = x[:, g0:g0 + 64]
        gmean = part.mean(-1)
        gm2 = ((part - gmean[:, None]) ** 2).sum(-1)
        delta, total = gmean - mean, cnt + 64.0
        mean = mean + delta * 64.0 / total
        m2 = m2 + gm2 + delta * delta * cnt * 64.0 / total
        cnt = total
    assert np.abs(mean - x.mean(-1)).max() < 1e-13 and np.abs(m2 / cnt - x.var(-1)).max() < 1e-12
    # equal group sizes: the same statistics without a running merge (what the kernel does)
    gmeans = np.stack([x[:, g0:g0 + 64].mean(-1) for g0 in range(0, C, 64)], -1)
    gm2s = np.stack([((x[:, g0:g0 + 64] - x[:, g0:g0 + 64].mean(-1, keepdims=True)) ** 2).sum(-1) for g0 in range(0, C, 64)], -1)
    mean2 = gmeans.mean(-1)
    m2b = (gm2s + 64.0 * (gmeans - mean2[:, None]) ** 2).sum(-1)
    assert np.abs(mean2 - mean).max() < 1e-13 and np.abs(m2b - m2).max() < 1e-10
    rstd = 1.0 / np.sqrt(m2 / cnt + eps)
    wg = w.astype(np.float64) * gamma.astype(np.float64)[None, :]
    c1, c2 = wg.sum(-1), w.astype(np.float64) @ beta.astype(np.float64) + b
    got = rstd[:, None] * (x @ wg.T - mean[:, None] * c1[None, :]) + c2[None, :]
    assert np.abs(got - want).max() < 1e-11
