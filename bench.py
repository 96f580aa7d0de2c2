#!/usr/bin/env python3
"""Benchmark of the JetViT token-mixer hot path on one MI355X.

One "step" = one linear-attention layer + one 16x16 window-attention layer + one full-attention
layer on the ViT-L attention workload (bf16, batch 8, 64x64 grid = 4096 tokens, 16 heads x 64),
all inputs resident in HBM.  value = tokens pushed through a mixer layer per second
(3 layers x 32 768 tokens / step time).  Each mixer (and the paper's linear-attention block with
its squeeze-dynamic convolution branch) is also timed on its own with events on the launch
stream and priced against its roofline (HBM for linear and window attention, bf16 MFMA for full
attention); the dominant kernel of the step is full attention.  The hybrid ViT-L encoder
forward (24 blocks, batch 4, 64x64 grid) is timed in the same run and reported under "encoder".

Prints ONE JSON line.  Use --gpus 1 only: the library is a single-GPU path.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
TRAFFIC_FILE = os.path.join(ROOT, "profiles", "hbm_traffic.txt")


def kernel_sources_hash():
    """sha256 over the HIP sources of the library (file names and bytes, sorted): the build the
    counter traffic in profiles/hbm_traffic.txt was measured on is identified by it."""
    import glob
    import hashlib
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2605_26636_amd", "csrc")
    for path in sorted(glob.glob(os.path.join(csrc, "*.hip")) + glob.glob(os.path.join(csrc, "*.h"))):
        h.update(os.path.basename(path).encode())
        h.update(open(path, "rb").read())
    return h.hexdigest()[:16]


TRAFFIC_SOURCE = {"file": "profiles/hbm_traffic.txt"}


def read_traffic():
    """HBM bytes per launch measured with rocprofv3 counters (profiles/hbm_traffic.txt holds
    'kernel-key: bytes' lines, the commands that produced them and the hash of the kernel sources
    they were measured on).  The figures are handed out only while that hash is the hash of the
    present sources: after a kernel change the file is stale and every traffic is null until
    the counters are collected again.  {} when absent or stale; TRAFFIC_SOURCE says which."""
    out, measured_on = {}, None
    if os.path.exists(TRAFFIC_FILE):
        for line in open(TRAFFIC_FILE):
            line = line.split("#", 1)[0].strip()
            if ":" in line:
                key, val = line.split(":", 1)
                if key.strip() == "sources_sha256":
                    measured_on = val.strip()
                    continue
                try:
                    out[key.strip()] = float(val)
                except ValueError:
                    pass
    now = kernel_sources_hash()
    TRAFFIC_SOURCE.update({"measured_on_sources": measured_on, "present_sources": now,
                           "stale": measured_on != now})
    return out if measured_on == now else {}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=30)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--config", type=int, default=2, help="mixer workload (2 = headline)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-encoder", action="store_true", help="skip the encoder leg")
    ap.add_argument("--buffers", type=int, default=6, help="rotating input/output sets")
    ap.add_argument("--encoder", action="store_true",
                    help="run only the hybrid ViT-L encoder forward (config 5)")
    ap.add_argument("--paper-ratio", action="store_true",
                    help="encoder latency of all-full-attention vs hybrid patterns on a 64x128 grid "
                         "(the resolution of the paper's speed tables), as ratios")
    ap.add_argument("--model", choices=["L", "B", "H", "G", "7B"], default="L",
                    help="ViT size for --paper-ratio (7B: 40 blocks, width 4096, 32 heads x 128, MLP 8192)")
    ap.add_argument("--graph", action="store_true",
                    help="--paper-ratio: replay each forward pass as one captured HIP graph")
    ap.add_argument("--la-ablation", action="store_true",
                    help="time the linear-attention block variants of the paper's Tab. 1 in a pure "
                         "linear-attention ViT-L and print their ratios")
    ap.add_argument("--stream-bf16", action="store_true",
                    help="--encoder: carry the residual stream in bf16 instead of fp32")
    ap.add_argument("--fold-layernorm", action="store_true",
                    help="--encoder: fold the LayerNorms into the products behind them "
                         "(jv_encoder_fold_layernorm)")
    ap.add_argument("--fuse-linear-projection", action="store_true",
                    help="--encoder: fold the apply pass of the linear-attention blocks into their output "
                         "projection (jv_encoder_fuse_linear_projection)")
    ap.add_argument("--gemm", action="store_true",
                    help="time the encoder's four GEMM shapes alone (this library, and the vendor "
                         "library's plain GEMM through torch as a reference point)")
    ap.add_argument("--sweep", action="store_true",
                    help="time linear, window 16x16 (and full, up to 16 384 tokens) attention over the "
                         "token-count sweep at 32 768 tokens per call: 1 024 ... 65 536 tokens per image")
    ap.add_argument("--head-dim", type=int, choices=[64, 128], default=64,
                    help="--sweep: channels per head (1024 channels per token either way: 16 x 64 or 8 x 128)")
    ap.add_argument("--only", choices=["linear", "window", "full", "block"], default=None,
                    help="run only this mixer's launches (for counter collection)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain 256 MiB device copy (reference point for HBM counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build is a single-GPU path (no sharding, no collectives); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2605_26636_amd import binding, synth

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    binding.lib()
    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst
    if args.la_ablation:
        print(json.dumps(bench_la_ablation(args.steps, args.warmup)))
        return
    if args.sweep:
        print(json.dumps(bench_sweep(args.steps, args.warmup, args.buffers, args.head_dim)))
        return
    if args.gemm:
        print(json.dumps(bench_gemm(args.steps, args.warmup)))
        return
    if args.paper_ratio:
        print(json.dumps(bench_paper_ratio(args.steps, args.warmup, args.model, args.graph)))
        return
    if args.encoder:
        enc = bench_encoder(args.steps, args.warmup, args.stream_bf16, args.fold_layernorm, args.fuse_linear_projection)
        print(json.dumps({
            "metric": "hybrid ViT-L encoder forward, tokens/s per encoder",
            "value": enc["tokens_per_s"], "unit": "tokens/s", "n_gpus": 1, "steps": args.steps,
            "warmup": args.warmup, "ms_per_step": enc["ms_per_encoder"], "higher_is_better": True,
            "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
            "config": {"workload": enc["workload"]},
            "roofline": {"bound": "mfma", "achieved": enc["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                         "unit": "TFLOP/s", "frac": enc["mfma_frac"], "traffic": read_traffic().get("encoder")},
            "encoder": enc, "cpu_baseline": None}))
        return
    c = synth.CONFIGS[args.config]
    B, heads, H, W, d = c["B"], c["heads"], c["H"], c["W"], c["d"]
    N = H * W
    window = c["window"]
    tokens = B * N
    dt = torch.bfloat16 if c["bf16"] else torch.float32
    esz = 2 if c["bf16"] else 4

    q, k, v = synth.config_qkv(args.config)
    base = [torch.from_numpy(x).cuda().to(dt) for x in (q, k, v)]
    # Rotating buffer sets so that the last-level cache cannot hold the working set.
    sets = []
    for i in range(args.buffers):
        qs, ks, vs = (t.clone() if i else t for t in base)
        sets.append((qs, ks, vs, torch.empty_like(qs)))
    C = heads * d
    squeeze = tuple(torch.from_numpy(a).cuda() for a in synth.squeeze_weights(C, C // 16, 3, 2500))
    dwc = binding.make_dwc_params(squeeze=squeeze, ksize=3)
    ws = torch.empty(max(256, binding.jv_linear_block_workspace_bytes(
        binding.make_desc(*sets[0], (H, W)), dwc)), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()

    def linear(s):
        binding.jv_linear_attn_fwd(s[0], s[1], s[2], s[3], (H, W), 1e-6, ws, stream)

    def block(s):
        binding.jv_linear_block_fwd(s[0], s[1], s[2], s[3], (H, W), 1e-6, squeeze=squeeze, ksize=3,
                                    workspace=ws, stream=stream)

    def win(s):
        binding.jv_window_attn_fwd(s[0], s[1], s[2], s[3], (H, W), window, 0.0, stream)

    def full(s):
        binding.jv_full_attn_fwd(s[0], s[1], s[2], s[3], (H, W), 0.0, stream)

    mixers = {"linear": linear, "window": win, "full": full, "block": block}
    if args.only:
        fn = mixers[args.only]
        for i in range(args.warmup + args.steps):
            fn(sets[i % len(sets)])
        torch.cuda.synchronize()
        print(json.dumps({"only": args.only, "launches": args.warmup + args.steps}))
        return

    def step(i):
        s = sets[i % len(sets)]
        linear(s); win(s); full(s)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps

    # Per-mixer timing with events on the launch stream (average over the timed launches).
    per = {}
    for name, fn in mixers.items():
        for i in range(3):
            fn(sets[i % len(sets)])
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
               for _ in range(args.steps)]
        torch.cuda.synchronize()
        for i, (a, b) in enumerate(evs):
            s = sets[i % len(sets)]
            a.record(stream); fn(s); b.record(stream)
        torch.cuda.synchronize()
        t = np.array([a.elapsed_time(b) for a, b in evs])
        per[name] = {"ms_avg": float(t.mean()), "ms_min": float(t.min()),
                     "ms_median": float(np.median(t))}

    bytes_layer = 4 * tokens * heads * d * esz                 # read Q, K, V; write O
    flops = {"full": 4.0 * N * N * d * B * heads,              # QK^T and PV
             "window": 4.0 * N * (window[0] * window[1]) * d * B * heads,
             "linear": (4.0 * d * d + 2 * d) * tokens * heads,
             "block": (4.0 * d * d + 2 * d + 2 * 9) * tokens * heads}
    traffic = read_traffic()
    # the block also reads V a second time for its convolution: 5 tensor passes instead of 4
    mixer_bytes = {name: bytes_layer for name in per}
    mixer_bytes["block"] = 5 * tokens * heads * d * esz
    for name in per:
        ms = per[name]["ms_avg"]
        per[name]["tokens_per_s"] = tokens / (ms * 1e-3)
        per[name]["hbm_GBs"] = mixer_bytes[name] / (ms * 1e-3) / 1e9
        per[name]["hbm_frac"] = per[name]["hbm_GBs"] / HBM_PEAK_GBS
        per[name]["TFLOPs"] = flops[name] / (ms * 1e-3) / 1e12
        per[name]["mfma_frac"] = per[name]["TFLOPs"] / MFMA_BF16_PEAK_TFLOPS
    per["block"]["note"] = "linear attention + squeeze-dynamic 3x3 convolution of V (Eq. 4)"

    def hbm_roof(name, kernels):
        return {"kernel": kernels, "bound": "hbm", "achieved": per[name]["hbm_GBs"],
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": per[name]["hbm_frac"],
                "traffic": traffic.get(name), "algorithmic_bytes": mixer_bytes[name],
                "mfma_frac": per[name]["mfma_frac"]}

    roofline = {"kernel": "attn_ring_bf16 (full attention)", "bound": "mfma",
                "achieved": per["full"]["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                "unit": "TFLOP/s", "frac": per["full"]["mfma_frac"], "traffic": traffic.get("full"),
                "traffic_source": dict(TRAFFIC_SOURCE),
                "algorithmic_flops": flops["full"], "avg_launch_ms": per["full"]["ms_avg"]}
    rooflines = {
        "linear": hbm_roof("linear", "la_state_bf16 + la_apply_bf16"),
        "block": hbm_roof("block", "la_state_bf16 + squeeze_* + la_apply_bf16 (convolution fused)"),
        "window": hbm_roof("window", "attn_window8_bf16"),
        "full": dict(roofline),
    }

    encoder = None
    if not args.no_encoder and args.config == 2:
        del sets, base
        torch.cuda.empty_cache()
        encoder = bench_encoder(10, 3)
        encoder["bf16_residual_stream"] = {k: v for k, v in bench_encoder(10, 3, stream_bf16=True).items()
                                           if k in ("ms_per_encoder", "tokens_per_s", "TFLOPs", "mfma_frac")}
        rooflines["encoder"] = {"kernel": "gemm_bf16_kernel (+ mixers, LayerNorm)", "bound": "mfma",
                                "achieved": encoder["TFLOPs"], "peak": MFMA_BF16_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": encoder["mfma_frac"], "traffic": traffic.get("encoder")}

    cpu = None
    if not args.no_cpu_baseline:
        cpu = cpu_baseline(q, k, v, H, W, window)

    out = {
        "metric": "attention tokens/s per layer at ViT-L 4096 tokens; % of HBM or MFMA peak",
        "value": 3 * tokens / (ms_per_step * 1e-3), "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16" if c["bf16"] else "f32", "data": "synthetic",
        "config": {"workload": f"config{args.config}: B{B} {H}x{W} grid (N={N}) heads{heads} d{d} "
                               f"{'bf16' if c['bf16'] else 'fp32'}; step = linear + "
                               f"window{window[0]}x{window[1]} + full attention layer",
                   "tokens_per_layer": tokens},
        "per_mixer": per, "roofline": roofline, "rooflines": rooflines, "encoder": encoder,
        "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def bench_encoder(steps, warmup, stream_bf16=False, fold=False, fuse_linear=False):
    """Config 5: 24 pre-LN blocks of width 1024 (16 heads, MLP 4096), batch 4 on a 64x64 grid;
    full attention at blocks 5, 11, 17, 23, window 16x16 at the other even blocks, linear
    attention at the rest.  Random-init (Xavier-normal, seeded) bf16 weights; the residual stream
    in fp32, or in bf16 with stream_bf16 (what a network converted to bf16 as a whole carries)."""
    import torch
    from paper_2605_26636_amd import binding, synth
    B, H, W, heads, hidden, L = 4, 64, 64, 16, 4096, 24
    C, N = heads * 64, H * W
    pattern = synth.encoder_pattern(L)
    blocks = []
    for l in range(L):
        wts = synth.block_weights(C, hidden, 5000 + l)
        blocks.append({k: (torch.from_numpy(v).cuda().to(torch.bfloat16) if k.startswith("w_")
                           else torch.from_numpy(v).cuda()) for k, v in wts.items()})
    sd = torch.bfloat16 if stream_bf16 else torch.float32
    enc = binding.Encoder(blocks, pattern, heads, hidden, window=(16, 16), stream_dtype=sd, fold_layernorm=fold)
    if fuse_linear:
        enc.fuse_linear_projection(True)
    x = torch.from_numpy(synth.normal((B, N, C), 5003)).cuda().to(sd)
    y = torch.empty_like(x)
    ws = torch.empty(enc.workspace_bytes(B, (H, W)), dtype=torch.uint8, device="cuda")
    stream = torch.cuda.current_stream()
    for _ in range(warmup):
        enc.forward(x, y, (H, W), ws, stream)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        enc.forward(x, y, (H, W), ws, stream)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) * 1e3 / steps
    enc.close()
    T = B * N
    gemm_flops = 2.0 * T * C * (3 * C + C + 2 * hidden) * L
    n_full, n_win, n_lin = pattern.count(2), pattern.count(1), pattern.count(0)
    mix_flops = B * heads * (n_full * 4.0 * N * N * 64 + n_win * 4.0 * N * 256 * 64 +
                             n_lin * (4.0 * 64 * 64 + 128) * N)
    flops = gemm_flops + mix_flops
    tf = flops / (ms * 1e-3) / 1e12
    return {"workload": f"config5: 24-block hybrid ViT-L encoder, B{B} {H}x{W} grid, width {C}, "
                        f"{n_full} full / {n_win} window16x16 / {n_lin} linear blocks, "
                        f"{'bf16' if stream_bf16 else 'fp32'} residual stream",
            "ms_per_encoder": ms, "ms_per_layer": ms / L, "tokens_per_s": T / (ms * 1e-3),
            "steps": steps, "warmup": warmup, "flops_per_encoder": flops, "gemm_flops": gemm_flops,
            "TFLOPs": tf, "mfma_frac": tf / MFMA_BF16_PEAK_TFLOPS}


def bench_paper_ratio(steps, warmup, model="L", graph=False):
    """The paper's speed comparison re-created with random weights: a 24-block ViT-L on a 64x128
    token grid (1024x2048 px at patch 16, the resolution of its Tab. 1 and Tab. 3), batch 1,
    all blocks full attention against hybrids that keep 0, 1 or 2 full-attention blocks (at
    blocks 14 and 22, where the paper's search puts them for segmentation, Sec. 4.4); the first
    block is linear attention, the others alternate window 16x16 and linear attention; linear
    blocks carry the squeeze-dynamic 3x3 convolution branch (hidden width C/16).  model "B": the
    same with ViT-B (12 blocks, width 768, 12 heads), full attention kept at blocks 7 and 11, or
    "H" (32 blocks, width 1280, 20 heads, MLP 5120), blocks 19 and 29, or "G" (40 blocks, width
    1536, 24 heads, MLP 6144), blocks 24 and 37 (the paper prints positions for ViT-L only: scaled
    to the other depths).  "7B": the shape of the paper's largest teacher (Tab. 3: 40 blocks, width
    4096, 32 heads of 128 channels, MLP 8192), full attention kept at blocks 24 and 37; its weights
    (10.7 GB) are drawn on the device."""
    import torch
    from paper_2605_26636_amd import binding, synth
    B, H, W = 1, 64, 128
    heads, hidden, L, full_at_two = {"L": (16, 4096, 24, (14, 22)), "B": (12, 3072, 12, (7, 11)),
                                     "H": (20, 5120, 32, (19, 29)), "G": (24, 6144, 40, (24, 37)),
                                     "7B": (32, 8192, 40, (24, 37))}[model]
    wide = model == "7B"
    C, N = heads * (128 if wide else 64), H * W
    dev = []
    gen = torch.Generator(device="cuda")
    gen.manual_seed(5000)
    for l in range(L):
        if wide:  # Xavier-normal weights drawn on the device, zero biases, unit LayerNorm scale
            def w(rows, cols, fan):
                return (torch.randn(rows, cols, generator=gen, device="cuda") * (2.0 / fan) ** 0.5).to(torch.bfloat16)
            zeros = lambda n: torch.zeros(n, device="cuda")
            dev.append({"ln1_g": torch.ones(C, device="cuda"), "ln1_b": zeros(C), "w_qkv": w(3 * C, C, 2 * C),
                        "b_qkv": zeros(3 * C), "w_o": w(C, C, 2 * C), "b_o": zeros(C),
                        "ln2_g": torch.ones(C, device="cuda"), "ln2_b": zeros(C), "w_fc1": w(hidden, C, C + hidden),
                        "b_fc1": zeros(hidden), "w_fc2": w(C, hidden, C + hidden), "b_fc2": zeros(C)})
            hid = C // 16  # the squeeze-dynamic 3x3 branch, weights scaled as synth.squeeze_weights does
            rnd = lambda shape, scale: torch.randn(*shape, generator=gen, device="cuda") * scale
            dev[-1]["dwc"] = {"squeeze": (rnd((hid, C), 4.0 / C ** 0.5), rnd((hid,), 0.5),
                                          rnd((C * 9, hid), 1.0 / (3 * hid ** 0.5)), rnd((C * 9,), 0.5 / 3)), "ksize": 3}
            continue
        wts = synth.block_weights(C, hidden, 5000 + l)
        d = {k: (torch.from_numpy(v).cuda().to(torch.bfloat16) if k.startswith("w_")
                 else torch.from_numpy(v).cuda()) for k, v in wts.items()}
        d["dwc"] = {"squeeze": tuple(torch.from_numpy(a).cuda()
                                     for a in synth.squeeze_weights(C, C // 16, 3, 6000 + l)), "ksize": 3}
        dev.append(d)

    def hybrid(full_at):
        out = []
        for l in range(L):
            if l in full_at:
                out.append(synth.MIX_FULL)
            else:
                out.append(synth.MIX_LINEAR if l % 2 == 0 else synth.MIX_WINDOW)
        return out

    patterns = {"all_full": [synth.MIX_FULL] * L, "hybrid_0_full": hybrid(()),
                "hybrid_1_full": hybrid(full_at_two[:1]), "hybrid_2_full": hybrid(full_at_two)}
    x = torch.from_numpy(synth.normal((B, N, C), 5003)).cuda()
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    ms = {}
    for name, pattern in patterns.items():
        enc = binding.Encoder(dev, pattern, heads, hidden, window=(16, 16))
        ws = torch.empty(enc.workspace_bytes(B, (H, W)), dtype=torch.uint8, device="cuda")
        for _ in range(warmup):
            enc.forward(x, y, (H, W), ws, stream)
        torch.cuda.synchronize()
        run = lambda: enc.forward(x, y, (H, W), ws, stream)
        if graph:  # the whole forward as one HIP graph: no per-kernel launch cost on the host
            g = torch.cuda.CUDAGraph()
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            with torch.cuda.stream(side):
                with torch.cuda.graph(g, stream=side):
                    enc.forward(x, y, (H, W), ws, side)
            stream.wait_stream(side)
            run = g.replay
            run()
            torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            run()
        torch.cuda.synchronize()
        ms[name] = (time.perf_counter() - t0) * 1e3 / steps
        enc.close()
    base = ms["all_full"]
    return {"metric": "encoder latency ratio, all-full-attention ViT-%s vs hybrid (64x128 grid, batch 1)" % model,
            "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup, "dtype": "bf16",
            "data": "synthetic", "hip_graph": bool(graph), "ms": ms, "speedup_vs_all_full": {k: base / v for k, v in ms.items()},
            "paper_context_h100": {"DINOv3-L -> JetViT-L (2 full-attention blocks), whole model": "35.07 ms -> 18.77 ms (1.87x)",
                                   "DINOv3-B -> JetViT-B 0/1/2 full-attention blocks": "12.86 ms -> 7.37 / 7.69 / 8.27 ms"}}


def bench_gemm(steps, warmup):
    """The four GEMMs of a ViT-L block at 16 384 tokens (batch 4, 64x64 grid), each alone, same
    buffers every launch (operands warm in the last-level cache, as inside the encoder): QKV
    (bias), fc1 (bias + GELU), output projection and fc2 (bias + residual, in fp32 and in bf16).  The
    vendor library's plain bf16 GEMM (torch.nn.functional.linear: no GELU, no residual) is timed
    on the same shapes as a reference point."""
    import torch
    from paper_2605_26636_amd import binding
    M = 16384
    shapes = [("qkv", 3072, 1024, binding.JV_EPI_NONE), ("fc1_gelu", 4096, 1024, binding.JV_EPI_GELU),
              ("proj_residual", 1024, 1024, binding.JV_EPI_RESIDUAL), ("fc2_residual", 1024, 4096, binding.JV_EPI_RESIDUAL),
              ("proj_residual_bf16", 1024, 1024, binding.JV_EPI_RESIDUAL), ("fc2_residual_bf16", 1024, 4096, binding.JV_EPI_RESIDUAL)]
    gen = torch.Generator(device="cuda").manual_seed(5)
    out = {}
    for name, N, K, epi in shapes:
        a = torch.randn(M, K, device="cuda", generator=gen).to(torch.bfloat16)
        w = (torch.randn(N, K, device="cuda", generator=gen) / K ** 0.5).to(torch.bfloat16)
        bias = torch.zeros(N, device="cuda")
        rd = torch.bfloat16 if name.endswith("_bf16") else torch.float32      # residual and output alike
        res = torch.zeros(M, N, device="cuda", dtype=rd) if epi == binding.JV_EPI_RESIDUAL else None
        y = torch.empty(M, N, device="cuda", dtype=rd if res is not None else torch.bfloat16)

        def timed(fn):
            for _ in range(warmup):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(steps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / steps

        ms = timed(lambda: binding.jv_gemm_bias_act(a, w, bias, res, y, epi))
        ms_ref = timed(lambda: torch.nn.functional.linear(a, w))
        flops = 2.0 * M * N * K
        out[name] = {"M": M, "N": N, "K": K, "us": ms * 1e3, "TFLOPs": flops / (ms * 1e-3) / 1e12,
                     "mfma_frac": flops / (ms * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS,
                     "vendor_plain_gemm_us": ms_ref * 1e3, "vendor_plain_gemm_TFLOPs": flops / (ms_ref * 1e-3) / 1e12}
    return {"metric": "GEMMs of a ViT-L block at 16 384 tokens, each alone", "unit": "us", "n_gpus": 1,
            "steps": steps, "warmup": warmup, "dtype": "bf16", "data": "synthetic", "gemm": out}


def bench_sweep(steps, warmup, buffers, head_dim=64):
    """Token-count sweep of the crossover experiment (bf16, 16 heads x 64, or 8 heads x 128 with
    --head-dim 128: the same bytes and flops per token): 32 768 tokens per call
    as 32 images of 1 024 tokens ... 2 images of 16 384, and one image of 65 536 tokens.  Linear and
    16x16 window attention move the same bytes per token at every size; full attention (timed up
    to 16 384 tokens per image) grows with the image.  Events on the launch stream, rotating
    buffer sets."""
    import torch
    from paper_2605_26636_amd import binding, synth
    heads, d = 1024 // head_dim, head_dim
    stream = torch.cuda.current_stream()
    rows = []
    for B, H, W in synth.SWEEP:
        N = H * W
        q, k, v = synth.qkv(3, B, heads, N, d, 0.125, True)
        base = [torch.from_numpy(x).cuda().to(torch.bfloat16) for x in (q, k, v)]
        sets = []
        for i in range(buffers):
            qs, ks, vs = (t.clone() if i else t for t in base)
            sets.append((qs, ks, vs, torch.empty_like(qs)))
        ws = torch.empty(max(256, binding.jv_linear_attn_workspace_bytes(binding.make_desc(*sets[0], (H, W)))),
                         dtype=torch.uint8, device="cuda")
        mixers = {"linear": lambda s_: binding.jv_linear_attn_fwd(s_[0], s_[1], s_[2], s_[3], (H, W), 1e-6, ws, stream),
                  "window": lambda s_: binding.jv_window_attn_fwd(s_[0], s_[1], s_[2], s_[3], (H, W), (16, 16), 0.0, stream)}
        if N <= 16384:
            mixers["full"] = lambda s_: binding.jv_full_attn_fwd(s_[0], s_[1], s_[2], s_[3], (H, W), 0.0, stream)
        tokens = B * N
        bytes_layer = 4 * tokens * heads * d * 2
        row = {"tokens_per_image": N, "batch": B, "grid": [H, W]}
        for name, fn in mixers.items():
            n_timed = steps if name != "full" else max(3, min(steps, 10))
            for i in range(warmup):
                fn(sets[i % len(sets)])
            evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True))
                   for _ in range(n_timed)]
            torch.cuda.synchronize()
            for i, (a, b) in enumerate(evs):
                a.record(stream); fn(sets[i % len(sets)]); b.record(stream)
            torch.cuda.synchronize()
            t = np.array([a.elapsed_time(b) for a, b in evs])
            ms = float(np.median(t))
            row[name] = {"ms_median": ms, "ms_min": float(t.min()), "ns_per_token": ms * 1e6 / tokens}
            if name == "full":
                tf = 4.0 * N * N * d * B * heads / (ms * 1e-3) / 1e12
                row[name].update({"TFLOPs": tf, "mfma_frac": tf / MFMA_BF16_PEAK_TFLOPS})
            else:
                gbs = bytes_layer / (ms * 1e-3) / 1e9
                row[name].update({"hbm_GBs": gbs, "hbm_frac": gbs / HBM_PEAK_GBS})
        rows.append(row)
        del sets, base, ws
        torch.cuda.empty_cache()
    return {"metric": f"mixer time over the token-count sweep (bf16, {heads} heads x {d}, 16x16 windows)",
            "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup, "dtype": "bf16",
            "data": "synthetic", "sweep": rows}


def bench_la_ablation(steps, warmup):
    """The paper's linear-attention block ablation (Tab. 1) re-created for speed only, with random
    weights: a pure linear-attention ViT-L (24 blocks) on a 64x128 token grid, batch 1, with the
    block variants the table lists: ReLU linear attention; + static 3x3 convolution on V;
    + the focused feature map (p = 3) on top of that; + squeeze-dynamic convolution instead (the
    paper's block); + token-wise dynamic convolution (the same generator run on every token, the
    variant the paper rejects for its cost)."""
    import torch
    from paper_2605_26636_amd import binding, synth
    B, H, W, heads, hidden, L = 1, 64, 128, 16, 4096, 24
    C, N = heads * 64, H * W
    base_blocks = []
    for l in range(L):
        wts = synth.block_weights(C, hidden, 5000 + l)
        base_blocks.append({k: (torch.from_numpy(v).cuda().to(torch.bfloat16) if k.startswith("w_")
                                else torch.from_numpy(v).cuda()) for k, v in wts.items()})
    static = [{"static_kernel": torch.from_numpy(synth.dwc_static_kernel(C, 3, 6100 + l)).cuda(), "ksize": 3}
              for l in range(L)]
    squeeze = [{"squeeze": tuple(torch.from_numpy(a).cuda() for a in synth.squeeze_weights(C, C // 16, 3, 6000 + l)),
                "ksize": 3} for l in range(L)]

    def with_dwc(dwc):
        return [dict(b, dwc=dwc[l]) if dwc else dict(b) for l, b in enumerate(base_blocks)]

    variants = {"relu": (with_dwc(None), 1), "relu+static_dwc": (with_dwc(static), 1),
                "focused_p3+static_dwc": (with_dwc(static), 3), "relu+squeeze_dwc": (with_dwc(squeeze), 1),
                "relu+token_dwc": (with_dwc([{"token": d["squeeze"], "ksize": 3} for d in squeeze]), 1)}
    x = torch.from_numpy(synth.normal((B, N, C), 5003)).cuda()
    y = torch.empty_like(x)
    stream = torch.cuda.current_stream()
    ms = {}
    for name, (blocks, focus_p) in variants.items():
        enc = binding.Encoder(blocks, [synth.MIX_LINEAR] * L, heads, hidden, la_focus_p=focus_p)
        ws = torch.empty(enc.workspace_bytes(B, (H, W)), dtype=torch.uint8, device="cuda")
        for _ in range(warmup):
            enc.forward(x, y, (H, W), ws, stream)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            enc.forward(x, y, (H, W), ws, stream)
        torch.cuda.synchronize()
        ms[name] = (time.perf_counter() - t0) * 1e3 / steps
        enc.close()
    base = ms["relu"]
    return {"metric": "pure linear-attention ViT-L latency by block variant (64x128 grid, batch 1)",
            "unit": "ms", "n_gpus": 1, "steps": steps, "warmup": warmup, "dtype": "bf16",
            "data": "synthetic", "ms": ms, "relative_to_relu": {k: v / base for k, v in ms.items()},
            "paper_context_h100": {"latency ms (ReLU, +DWC, +DWC+focusing, token-wise dynamic, squeeze-dynamic)":
                                   "5.33, 5.72, 6.00, 8.94, 5.88 (1.00 : 1.07 : 1.13 : 1.68 : 1.10)"}}


def cpu_baseline(q, k, v, H, W, window):
    """The CPU oracle as it stands on a bounded sample of the same inputs: the whole linear and
    window layers (all images) and the full-attention layer of batch element 0."""
    import oracle
    B, heads, N = q.shape[0], q.shape[1], q.shape[2]
    cores = len(os.sched_getaffinity(0))
    t0 = time.perf_counter(); oracle.linear_attn_state(q, k, v, 1e-6); t_lin = time.perf_counter() - t0
    t0 = time.perf_counter(); oracle.window_attn(q, k, v, H, W, *window); t_win = time.perf_counter() - t0
    # full attention: image 0 first, then as many further images as fit in about 20 s
    t0 = time.perf_counter(); oracle.full_attn(q[:1], k[:1], v[:1]); t_one = time.perf_counter() - t0
    n_img, t_full_all = 1, t_one
    more = int(min(B - 1, 20.0 // max(t_one, 1e-3)))
    if more > 0:
        t0 = time.perf_counter(); oracle.full_attn(q[1:1 + more], k[1:1 + more], v[1:1 + more])
        t_full_all += time.perf_counter() - t0
        n_img += more
    t_full = t_full_all / n_img
    per_image = t_lin / B + t_win / B + t_full
    return {"value": 3 * N / per_image, "unit": "tokens/s", "cores": cores, "kind": "oracle",
            "sample": f"same seeded inputs: linear layer on all {B} images ({t_lin:.2f}s), window "
                      f"layer on all {B} images ({t_win:.2f}s), full-attention layer on {n_img} image(s) "
                      f"({t_full_all:.2f}s); value = 3 layers x {N} tokens / time per image",
            "tokens_per_s": {"linear": B * N / t_lin, "window": B * N / t_win, "full": N / t_full}}


if __name__ == "__main__":
    main()
