"""Pins for the oracle's full softmax attention (Eq. 1)."""
import numpy as np
import torch

import oracle
from paper_2605_26636_amd import synth


def _qkv(seed, B=2, h=3, N=37, d=16, scale=1.0):
    return [synth.normal((B, h, N, d), seed + i, scale) for i in range(3)]


def test_hand_case(golden):
    g = golden("full_attn_hand_case.txt")
    q = np.array(g["q"], dtype=np.float32).reshape(1, 1, 1, 1)
    # ln 3 is not a float32; the case is checked at float32(ln 3), whose exp is 3(1 + 1e-8).
    k = np.array(g["k"], dtype=np.float32).reshape(1, 1, 2, 1)
    v = np.array(g["v"], dtype=np.float32).reshape(1, 1, 2, 1)
    # one query against two keys: use N = 2 by repeating the query row
    q2 = np.repeat(q, 2, axis=2)
    o = oracle.full_attn(q2, k, v, scale=g["scale"][0])
    assert np.allclose(o[0, 0, :, 0], g["o"][0], rtol=0, atol=1e-6)
    p = oracle.full_attn_probs(q2[0, 0], k[0, 0], scale=g["scale"][0])
    assert np.allclose(p[0], g["p"], atol=1e-7)


def test_probability_rows_sum_to_one():
    q, k, _ = _qkv(11, B=1, h=1, N=53, d=8, scale=2.0)
    p = oracle.full_attn_probs(q[0, 0], k[0, 0])
    assert p.min() >= 0.0
    assert np.abs(p.sum(axis=1) - 1.0).max() < 1e-14


def test_zero_query_gives_mean_of_values():
    q, k, v = _qkv(21)
    o = oracle.full_attn(np.zeros_like(q), k, v)
    mean = v.astype(np.float64).mean(axis=2, keepdims=True)
    assert np.abs(o - mean).max() < 1e-14


def test_key_shift_invariance():
    q, k, v = _qkv(31)
    t = synth.normal((1, 1, 1, q.shape[-1]), 99).astype(np.float64)
    # work on float64-exact float32 shifts: choose t on a coarse binary grid, k likewise
    k = np.round(k * 64) / 64
    t = (np.round(t * 64) / 64).astype(np.float32)
    o0 = oracle.full_attn(q, k.astype(np.float32), v)
    o1 = oracle.full_attn(q, (k + t).astype(np.float32), v)
    assert np.abs(o0 - o1).max() < 1e-12


def test_permutation_of_keys_and_queries():
    q, k, v = _qkv(41)
    N = q.shape[2]
    perm = np.random.Generator(np.random.Philox(7)).permutation(N)
    o = oracle.full_attn(q, k, v)
    assert np.abs(oracle.full_attn(q, k[:, :, perm], v[:, :, perm]) - o).max() < 1e-13
    assert np.abs(oracle.full_attn(q[:, :, perm], k, v) - o[:, :, perm]).max() < 1e-15


def test_one_hot_limit_picks_the_matching_value():
    # keys = large multiples of unit vectors; query aligned with key j -> output -> v_j
    d = 8
    k = (np.eye(d, dtype=np.float32) * 200.0).reshape(1, 1, d, d)
    q = k.copy()
    v = synth.normal((1, 1, d, d), 5)
    o = oracle.full_attn(q, k, v, scale=1.0)
    assert np.abs(o - v).max() < 1e-12


def test_against_library_sdpa_fp64():
    q, k, v = _qkv(51, B=2, h=2, N=65, d=32)
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double()).numpy()
    assert np.abs(oracle.full_attn(q, k, v) - ref).max() < 1e-13
    # non-default scale and the rows entry point
    ref2 = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double(),
        scale=0.37).numpy()
    rows = synth.sample_rows(2, 2, 65, 9, seed=3)
    got = oracle.full_attn_rows(q, k, v, rows, scale=0.37)
    want = np.stack([ref2[b, h, i] for b, h, i in rows])
    assert np.abs(got - want).max() < 1e-13


def test_masked_attn_with_full_mask_is_full_attn_and_rejects_empty_rows():
    q, k, v = _qkv(61, B=1, h=2, N=19, d=8)
    allow = np.ones((19, 19), dtype=np.uint8)
    assert np.array_equal(oracle.masked_attn(q, k, v, allow), oracle.full_attn(q, k, v))
    allow[4, :] = 0
    try:
        oracle.masked_attn(q, k, v, allow)
        assert False, "an empty softmax row must be an error"
    except ValueError:
        pass


def test_masked_attn_against_library_mask():
    q, k, v = _qkv(71, B=1, h=2, N=23, d=8)
    rng = np.random.Generator(np.random.Philox(9))
    allow = (rng.random((23, 23)) < 0.4).astype(np.uint8)
    allow[np.arange(23), np.arange(23)] = 1
    ref = torch.nn.functional.scaled_dot_product_attention(
        torch.from_numpy(q).double(), torch.from_numpy(k).double(), torch.from_numpy(v).double(),
        attn_mask=torch.from_numpy(allow.astype(bool))).numpy()
    assert np.abs(oracle.masked_attn(q, k, v, allow) - ref).max() < 1e-13
