"""Pins for the oracle's elementary operations: closed forms, invariants and
library routines that special cases reduce to.  None of these re-uses the
oracle's own formula as the expected value."""
import math

import numpy as np
import pytest
import torch

import oracle
from oracle import Shape


# ------------------------------------------------------------------ RMSNorm
def test_rmsnorm_constant_vector_closed_form():
    # x = c*1  ->  y_k = g_k * c / sqrt(c^2 + eps)
    H, c, eps = 64, -2.5, 1e-5
    g = np.linspace(0.5, 1.5, H).astype(np.float32)
    y = oracle.rmsnorm(np.full((1, H), c), g, eps)[0]
    assert np.allclose(y, g.astype(np.float64) * c / math.sqrt(c * c + eps), rtol=1e-14, atol=0)


def test_rmsnorm_three_four():
    # mean square of (3,4) is 12.5
    y = oracle.rmsnorm(np.array([[3.0, 4.0]]), np.array([1.0, 2.0], dtype=np.float32), 0.0)[0]
    assert np.allclose(y, [3 / math.sqrt(12.5), 8 / math.sqrt(12.5)], rtol=1e-15)


def test_rmsnorm_scale_invariant_without_eps_and_eps_matters():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((3, 96)); g = rng.standard_normal(96).astype(np.float32)
    assert np.allclose(oracle.rmsnorm(7.0 * x, g, 0.0), oracle.rmsnorm(x, g, 0.0), rtol=1e-13)
    tiny = 1e-3 * x
    with_eps = oracle.rmsnorm(tiny, g, 1e-5)
    assert np.all(np.abs(with_eps) < np.abs(oracle.rmsnorm(tiny, g, 0.0)) + 1e-300)
    # eps enters inside the square root, added to the mean (not the sum)
    ms = (tiny ** 2).mean(axis=1, keepdims=True)
    assert np.allclose(with_eps, tiny * g / np.sqrt(ms + 1e-5), rtol=1e-13)


def test_rmsnorm_matches_torch_float64():
    rng = np.random.default_rng(1)
    x = rng.standard_normal((5, 128)); g = rng.standard_normal(128).astype(np.float32)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (128,), torch.from_numpy(g).double(), eps=1e-5)
    assert np.allclose(oracle.rmsnorm(x, g, 1e-5), ref.numpy(), rtol=1e-13, atol=1e-15)


# ------------------------------------------------------------------ linear
def test_linear_matches_float64_matmul_and_orientation():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((7, 40)); W = rng.standard_normal((24, 40)).astype(np.float32)
    y = oracle.linear(x, W)
    assert y.shape == (7, 24)
    assert np.allclose(y, x @ W.astype(np.float64).T, rtol=1e-13, atol=1e-13)


def test_linear_identity_and_one_hot_rows():
    x = np.arange(12, dtype=np.float64).reshape(3, 4)
    assert np.array_equal(oracle.linear(x, np.eye(4, dtype=np.float32)), x)
    W = np.zeros((2, 4), dtype=np.float32); W[0, 3] = 1; W[1, 1] = -2   # y0 = x3, y1 = -2 x1
    assert np.array_equal(oracle.linear(x, W), np.stack([x[:, 3], -2 * x[:, 1]], axis=1))


# ------------------------------------------------------------------ RoPE
def test_rope_position_zero_is_identity():
    u = np.random.default_rng(3).standard_normal(64)
    assert np.array_equal(oracle.rope(u, 0, 10000.0), u)


def test_rope_first_pair_rotates_by_position_in_radians():
    # d = 0 has angle pos * base^0 = pos; the pair is (u_0, u_{D/2})
    D, pos = 8, 3
    u = np.zeros(D); u[0] = 1.0
    r = oracle.rope(u, pos, 10000.0)
    expect = np.zeros(D); expect[0] = math.cos(3.0); expect[D // 2] = math.sin(3.0)
    assert np.allclose(r, expect, atol=1e-15)
    u = np.zeros(D); u[D // 2] = 1.0
    r = oracle.rope(u, pos, 10000.0)
    expect = np.zeros(D); expect[0] = -math.sin(3.0); expect[D // 2] = math.cos(3.0)
    assert np.allclose(r, expect, atol=1e-15)


def test_rope_frequency_schedule():
    # D = 4, base = 10000: d = 1 has angle pos * 10000^(-2/4) = pos / 100
    u = np.array([0.0, 1.0, 0.0, 0.0])
    r = oracle.rope(u, 50, 10000.0)
    assert np.allclose(r, [0.0, math.cos(0.5), 0.0, math.sin(0.5)], atol=1e-15)
    # last pair of D = 128: exponent -2*63/128
    D = 128
    u = np.zeros(D); u[63] = 1.0
    r = oracle.rope(u, 1000, 10000.0)
    ang = 1000 * 10000.0 ** (-126 / 128)
    assert np.allclose([r[63], r[127]], [math.cos(ang), math.sin(ang)], atol=1e-13)


def test_rope_preserves_pair_norms_and_relative_position():
    rng = np.random.default_rng(4)
    D = 64
    q, k = rng.standard_normal(D), rng.standard_normal(D)
    rq = oracle.rope(q, 37, 10000.0)
    assert np.allclose(rq[: D // 2] ** 2 + rq[D // 2:] ** 2, q[: D // 2] ** 2 + q[D // 2:] ** 2, rtol=1e-13)
    base_dot = oracle.rope(q, 37, 1e4) @ oracle.rope(k, 12, 1e4)
    for delta in (1, 100, 4000):
        assert abs(oracle.rope(q, 37 + delta, 1e4) @ oracle.rope(k, 12 + delta, 1e4) - base_dot) < 1e-10


def test_rope_equals_complex_multiplication():
    rng = np.random.default_rng(5)
    D, pos, base = 32, 77, 500.0
    u = rng.standard_normal(D)
    z = (u[: D // 2] + 1j * u[D // 2:]) * np.exp(1j * pos * base ** (-np.arange(D // 2) * 2.0 / D))
    r = oracle.rope(u, pos, base)
    assert np.allclose(r[: D // 2], z.real, atol=1e-13) and np.allclose(r[D // 2:], z.imag, atol=1e-13)


# ------------------------------------------------------------------ SiLU / softmax
def test_silu_special_values():
    assert oracle.silu(0.0) == 0.0
    assert abs(oracle.silu(40.0) - 40.0) < 1e-12
    assert abs(oracle.silu(-40.0)) < 1e-12
    for z in (0.3, 1.7, 5.0):                      # silu(z) - silu(-z) = z
        assert abs(oracle.silu(z) - oracle.silu(-z) - z) < 1e-14
    assert abs(oracle.silu(1.0) - 1.0 / (1.0 + math.exp(-1.0))) < 1e-15
    assert abs(oracle.silu(2.0) - float(torch.nn.functional.silu(torch.tensor(2.0, dtype=torch.float64)))) < 1e-15


def test_softmax_properties():
    rng = np.random.default_rng(6)
    s = rng.standard_normal(50) * 5
    p = oracle.softmax(s)
    assert abs(p.sum() - 1.0) < 1e-14 and np.all(p > 0)
    assert np.allclose(oracle.softmax(s + 1000.0), p, rtol=1e-12)        # shift invariance, no overflow
    assert np.allclose(oracle.softmax(np.array([0.0, math.log(3.0)])), [0.25, 0.75], rtol=1e-15)
    assert np.allclose(p, torch.softmax(torch.from_numpy(s), 0).numpy(), rtol=1e-13)


# ------------------------------------------------------------------ attention over the paged cache
def _paged(shape, K, V, table_row, num_blocks):
    """Place dense K,V [n][Hkv][D] into a fresh one-layer pool through table_row."""
    pool = oracle.new_pool(shape, 1, num_blocks)
    bs = shape.kv_block_size
    for r in range(K.shape[0]):
        pool[0, table_row[r // bs], 0, :, r % bs, :] = K[r]
        pool[0, table_row[r // bs], 1, :, r % bs, :] = V[r]
    return pool


def test_attention_single_key_returns_v0():
    sh = Shape(hidden=8, n_q_heads=2, n_kv_heads=2, head_dim=4, ffn=8, kv_block_size=4)
    rng = np.random.default_rng(7)
    K = rng.standard_normal((1, 2, 4)).astype(np.float32); V = rng.standard_normal((1, 2, 4)).astype(np.float32)
    pool = _paged(sh, K, V, [2], 3)
    o, p = oracle.attend_token(sh, pool, 0, [2], 0, rng.standard_normal((2, 4)), want_probs=True)
    assert np.array_equal(o, V[0].astype(np.float64)) and np.array_equal(p, np.ones((2, 1)))


def test_attention_equal_keys_gives_mean_of_values():
    sh = Shape(hidden=8, n_q_heads=2, n_kv_heads=2, head_dim=4, ffn=8, kv_block_size=4)
    rng = np.random.default_rng(8)
    n = 10
    K = np.repeat(rng.standard_normal((1, 2, 4)), n, axis=0).astype(np.float32)
    V = rng.standard_normal((n, 2, 4)).astype(np.float32)
    table = [4, 0, 2]
    pool = _paged(sh, K, V, table, 5)
    o = oracle.attend_token(sh, pool, 0, table, n - 1, rng.standard_normal((2, 4)))
    assert np.allclose(o, V.astype(np.float64).mean(axis=0), rtol=1e-13)


@pytest.mark.parametrize("hq,hkv", [(4, 4), (8, 2), (6, 1)])
def test_attention_matches_torch_sdpa_float64(hq, hkv):
    D, bs, n = 16, 4, 23
    sh = Shape(hidden=hq * D, n_q_heads=hq, n_kv_heads=hkv, head_dim=D, ffn=8, kv_block_size=bs)
    rng = np.random.default_rng(9)
    K = rng.standard_normal((n, hkv, D)).astype(np.float32); V = rng.standard_normal((n, hkv, D)).astype(np.float32)
    table = rng.permutation(9)[:6].astype(np.int32)
    pool = _paged(sh, K, V, table, 9)
    q = rng.standard_normal((hq, D))
    pos = n - 1
    o, p = oracle.attend_token(sh, pool, 0, table, pos, q, want_probs=True)
    rep = hq // hkv
    Kt = torch.from_numpy(K).double().permute(1, 0, 2).repeat_interleave(rep, dim=0)   # [hq, n, D]
    Vt = torch.from_numpy(V).double().permute(1, 0, 2).repeat_interleave(rep, dim=0)
    ref = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[:, None, :], Kt, Vt)[:, 0, :]
    assert np.allclose(o, ref.numpy(), rtol=1e-12, atol=1e-13)
    assert np.allclose(p.sum(axis=1), 1.0, rtol=1e-14)
    # probabilities against the definition with the 1/sqrt(D) scale
    s = torch.einsum("hd,hnd->hn", torch.from_numpy(q), Kt) / math.sqrt(D)
    assert np.allclose(p, torch.softmax(s, dim=1).numpy(), rtol=1e-12)


def test_attention_is_causal_and_ignores_other_blocks():
    sh = Shape(hidden=8, n_q_heads=2, n_kv_heads=1, head_dim=4, ffn=8, kv_block_size=4)
    rng = np.random.default_rng(10)
    n = 11
    K = rng.standard_normal((n, 1, 4)).astype(np.float32); V = rng.standard_normal((n, 1, 4)).astype(np.float32)
    table = [3, 1, 5]
    pool = _paged(sh, K, V, table, 6)
    q = rng.standard_normal((2, 4))
    o6 = oracle.attend_token(sh, pool, 0, table, 6, q)
    # garbage in later positions and in blocks the sequence does not own changes nothing
    pool2 = pool.copy()
    pool2[0, 1, :, :, 3, :] = 99.0          # position 7 (block index 1, slot 3)
    pool2[0, 5] = -77.0                     # positions 8..11
    pool2[0, [0, 2, 4]] = 1e6               # foreign blocks
    assert np.array_equal(oracle.attend_token(sh, pool2, 0, table, 6, q), o6)
    # ... and equals dense attention over the first 7 keys
    s = (K[:7, 0].astype(np.float64) @ q.T).T / 2.0
    pr = np.exp(s - s.max(axis=1, keepdims=True)); pr /= pr.sum(axis=1, keepdims=True)
    assert np.allclose(o6, pr @ V[:7, 0].astype(np.float64), rtol=1e-13)


def test_grouped_heads_equal_replicated_heads():
    D, bs, n = 8, 4, 9
    rng = np.random.default_rng(11)
    K = rng.standard_normal((n, 2, D)).astype(np.float32); V = rng.standard_normal((n, 2, D)).astype(np.float32)
    q = rng.standard_normal((6, D))
    table = [1, 0, 2]
    gqa = Shape(hidden=48, n_q_heads=6, n_kv_heads=2, head_dim=D, ffn=8, kv_block_size=bs)
    mha = Shape(hidden=48, n_q_heads=6, n_kv_heads=6, head_dim=D, ffn=8, kv_block_size=bs)
    o_g = oracle.attend_token(gqa, _paged(gqa, K, V, table, 3), 0, table, n - 1, q)
    o_m = oracle.attend_token(mha, _paged(mha, np.repeat(K, 3, axis=1), np.repeat(V, 3, axis=1), table, 3),
                              0, table, n - 1, q)
    assert np.array_equal(o_g, o_m)
