"""Seeded synthetic inputs shared by the tests, the smoke check and the benchmark.

This module holds no arithmetic of the method: it draws normal variates from a
counter-based generator, scales them, and (for bf16 workloads) rounds them once
to bfloat16 with round-to-nearest-even.  The oracle and the GPU path both
receive exactly these values.

Seed convention: seed = 1000 * config + role, role 0 = Q, 1 = K, 2 = V,
3 = encoder input, 10+ = weights.
"""
import numpy as np


def normal(shape, seed, scale=1.0):
    """float32 N(0, scale^2) array from numpy's Philox generator."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    a = rng.standard_normal(size=shape, dtype=np.float32)
    if scale != 1.0:
        a *= np.float32(scale)
    return a


def to_bf16_bits(a):
    """Round float32 -> bfloat16 (nearest even); returns the uint16 bit patterns."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(bits):
    """Widen bfloat16 bit patterns exactly to float32."""
    return (np.ascontiguousarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def round_to_bf16(a):
    """float32 values that are exactly representable in bfloat16 (nearest even)."""
    return bf16_bits_to_f32(to_bf16_bits(a))


def qkv(config, B, heads, N, d, scale, bf16):
    """Q, K, V as float32 arrays [B, heads, N, d]; bf16-representable when bf16=True."""
    out = []
    for role in range(3):
        a = normal((B, heads, N, d), 1000 * config + role, scale)
        out.append(round_to_bf16(a) if bf16 else a)
    return out


# The mixer workloads of the benchmark definition (grid, window, value scale).
CONFIGS = {
    1: dict(B=1, heads=6, H=16, W=16, d=64, scale=1.0, bf16=False, window=(8, 8)),
    2: dict(B=8, heads=16, H=64, W=64, d=64, scale=0.125, bf16=True, window=(16, 16)),
    3: dict(B=2, heads=16, H=128, W=128, d=64, scale=0.125, bf16=True, window=(16, 16)),
    4: dict(B=32, heads=16, H=37, W=37, d=64, scale=0.125, bf16=True, window=(8, 8)),
}
# N-sweep of config 3 for the linear and window mixers: (B, H, W).
SWEEP = [(32, 32, 32), (8, 64, 64), (2, 128, 128), (1, 256, 256)]


def config_qkv(config):
    c = CONFIGS[config]
    return qkv(config, c["B"], c["heads"], c["H"] * c["W"], c["d"], c["scale"], c["bf16"])


def sample_rows(B, heads, N, count, seed):
    """`count` distinct-ish (b, head, i) triples, seeded; always includes the corners."""
    rng = np.random.Generator(np.random.Philox(int(seed)))
    rows = np.stack([rng.integers(0, B, count), rng.integers(0, heads, count),
                     rng.integers(0, N, count)], axis=1).astype(np.int64)
    rows[0] = (0, 0, 0)
    rows[-1] = (B - 1, heads - 1, N - 1)
    return rows


# ---------------------------------------------------------------------------
# Encoder workload (config 5): random-init ViT-L weights and the block pattern
# ---------------------------------------------------------------------------
MIX_LINEAR, MIX_WINDOW, MIX_FULL = 0, 1, 2


def encoder_pattern(n_blocks=24):
    """Full attention at blocks 5, 11, 17, 23 (every sixth); of the rest, even-indexed blocks
    take window attention and odd-indexed blocks linear attention."""
    out = []
    for i in range(n_blocks):
        if i % 6 == 5:
            out.append(MIX_FULL)
        else:
            out.append(MIX_WINDOW if i % 2 == 0 else MIX_LINEAR)
    return out


def block_weights(C, hidden, seed, bf16=True):
    """Xavier-normal weights of one pre-LN block (std = sqrt(2 / (fan_in + fan_out)), Q, K, V
    drawn as three C x C matrices), zero biases, LayerNorm gamma = 1 and beta = 0; float32
    arrays, rounded to bf16-representable values when bf16=True."""
    def xavier(shape, s):
        w = normal(shape, s, np.sqrt(2.0 / (shape[0] + shape[1])))
        return round_to_bf16(w) if bf16 else w
    w_qkv = np.concatenate([xavier((C, C), seed * 16 + i) for i in range(3)], axis=0)
    return {
        "ln1_g": np.ones(C, np.float32), "ln1_b": np.zeros(C, np.float32),
        "w_qkv": w_qkv, "b_qkv": np.zeros(3 * C, np.float32),
        "w_o": xavier((C, C), seed * 16 + 3), "b_o": np.zeros(C, np.float32),
        "ln2_g": np.ones(C, np.float32), "ln2_b": np.zeros(C, np.float32),
        "w_fc1": xavier((hidden, C), seed * 16 + 4), "b_fc1": np.zeros(hidden, np.float32),
        "w_fc2": xavier((C, hidden), seed * 16 + 5), "b_fc2": np.zeros(C, np.float32),
    }


# ---------------------------------------------------------------------------
# Convolution branch of the linear-attention block
# ---------------------------------------------------------------------------
def dwc_static_kernel(C, ksize, seed):
    """Depth-wise filter bank [C, k, k], N(0, 1/k^2)."""
    return normal((C, ksize, ksize), seed, 1.0 / ksize)


def squeeze_weights(C, hidden, ksize, seed):
    """Generator weights of the dynamic filters: w1 [hidden, C], b1 [hidden],
    w2 [C*k*k, hidden], b2 [C*k*k]; scaled so that the generated filters are O(1/k)."""
    return (normal((hidden, C), seed, 4.0 / np.sqrt(C)), normal((hidden,), seed + 1, 0.5),
            normal((C * ksize * ksize, hidden), seed + 2, 1.0 / (ksize * np.sqrt(hidden))),
            normal((C * ksize * ksize,), seed + 3, 0.5 / ksize))
