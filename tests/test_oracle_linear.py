"""Pins for the oracle's ReLU linear attention (Eq. 2, key-sum normaliser)."""
import numpy as np

import oracle
from paper_2605_26636_amd import synth


def _qkv(seed, B=2, h=3, N=45, d=16, scale=1.0):
    return [synth.normal((B, h, N, d), seed + i, scale) for i in range(3)]


def test_hand_case(golden):
    g = golden("linear_attn_hand_case.txt")
    k = np.array(g["k"], dtype=np.float32).reshape(1, 1, 3, 2)
    v = np.array(g["v"], dtype=np.float32).reshape(1, 1, 3, 2)
    q = np.array(g["q"], dtype=np.float32).reshape(1, 1, 3, 2)
    want = np.array(g["o"]).reshape(3, 2)
    o, S, z = oracle.linear_attn_state(q, k, v, eps=1e-30)
    assert np.array_equal(S[0, 0], np.array(g["S"]).reshape(2, 2))
    assert np.array_equal(z[0, 0], np.array(g["z"]))
    assert np.abs(o[0, 0] - want).max() < 1e-15
    oq = oracle.linear_attn_quadratic(q, k, v, eps=1e-30)
    assert np.abs(oq[0, 0] - want).max() < 1e-15


def test_state_form_equals_quadratic_form():
    q, k, v = _qkv(100)
    o_state, _, _ = oracle.linear_attn_state(q, k, v, eps=1e-6)
    o_quad = oracle.linear_attn_quadratic(q, k, v, eps=1e-6)
    assert np.abs(o_state - o_quad).max() < 1e-12
    rows = synth.sample_rows(2, 3, 45, 11, seed=5)
    got = oracle.linear_attn_rows(q, k, v, rows, eps=1e-6)
    want = np.stack([o_quad[b, h, i] for b, h, i in rows])
    assert np.array_equal(got, want)


def test_against_matrix_product_form():
    # (relu(Q) relu(K)^T) V / rowsum, with library matmuls in float64
    q, k, v = _qkv(110, B=1, h=2, N=33, d=8)
    qd, kd, vd = (np.maximum(q, 0).astype(np.float64), np.maximum(k, 0).astype(np.float64),
                  v.astype(np.float64))
    a = qd @ np.swapaxes(kd, -1, -2)
    want = (a @ vd) / (a.sum(-1, keepdims=True) + 1e-6)
    assert np.abs(oracle.linear_attn_quadratic(q, k, v, eps=1e-6) - want).max() < 1e-13


def test_positive_rescaling_of_q_or_k_changes_nothing():
    q, k, v = _qkv(120)
    o = oracle.linear_attn_quadratic(q, k, v, eps=0.0)
    # powers of two keep every product exact, so only the cancellation is tested
    assert np.abs(oracle.linear_attn_quadratic(q * 4, k, v, eps=0.0) - o).max() < 1e-13
    assert np.abs(oracle.linear_attn_quadratic(q, k * 0.25, v, eps=0.0) - o).max() < 1e-13
    assert np.abs(oracle.linear_attn_state(q * 3.0, k * 0.7, v, eps=0.0)[0] - o).max() < 1e-6


def test_constant_values_are_reproduced():
    q, k, _ = _qkv(130)
    ones = np.ones_like(q)
    o = oracle.linear_attn_quadratic(q, k, ones, eps=1e-9)
    assert np.abs(o - 1.0).max() < 1e-7


def test_identical_keys_give_the_mean_of_values():
    q, _, v = _qkv(140)
    key = np.abs(synth.normal((1, 1, 1, q.shape[-1]), 7)) + 0.1
    k = np.broadcast_to(key, q.shape).copy()
    o = oracle.linear_attn_quadratic(q, k, v, eps=0.0)
    mean = np.broadcast_to(v.astype(np.float64).mean(axis=2, keepdims=True), o.shape)
    live = (np.maximum(q, 0).sum(-1) > 0)
    assert live.all()
    assert np.abs(o - mean).max() < 1e-13


def test_outputs_are_convex_combinations_of_values():
    q, k, v = _qkv(150)
    o = oracle.linear_attn_quadratic(q, k, v, eps=0.0)
    lo = v.min(axis=2, keepdims=True) - 1e-12
    hi = v.max(axis=2, keepdims=True) + 1e-12
    assert (o >= lo).all() and (o <= hi).all()


def test_all_negative_query_gives_zero():
    q, k, v = _qkv(160, B=1, h=1, N=9, d=4)
    q = -np.abs(q)
    assert np.array_equal(oracle.linear_attn_quadratic(q, k, v, eps=1e-6), np.zeros(q.shape))
    assert np.array_equal(oracle.linear_attn_state(q, k, v, eps=1e-6)[0], np.zeros(q.shape))


def test_eps_enters_the_denominator_additively():
    q, k, v = _qkv(170, B=1, h=1, N=5, d=4)
    q[..., 0] = np.abs(q[..., 0]) + 0.1           # keep every denominator away from 0/0
    k[..., 0] = np.abs(k[..., 0]) + 0.1
    o0 = oracle.linear_attn_quadratic(q, k, v, eps=0.0)
    o1 = oracle.linear_attn_quadratic(q, k, v, eps=0.5)
    den = (np.maximum(q, 0).astype(np.float64) @ np.maximum(k, 0).astype(np.float64).sum(2)[..., None])
    assert np.abs(o1 * (den + 0.5) - o0 * den).max() < 1e-13
