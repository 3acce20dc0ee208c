"""Pins for the oracle's dense and sparse attention (Eq. 1 and its restriction to rho)."""
import numpy as np
import pytest

import oracle
from helpers import bits_to_f64, dense_attention_f64, f32_to_bf16_bits, rand_qkv


@pytest.mark.parametrize("H,G,L,d", [(4, 2, 37, 128), (8, 8, 64, 128), (6, 2, 5, 64), (4, 1, 300, 128)])
def test_dense_matches_independent_float64_softmax(H, G, L, d):
    rng = np.random.default_rng(1)
    q, K, V = rand_qkv(rng, H, G, L, d)
    _, o64 = oracle.attention(q, K, V, want_f64=True)
    ref = dense_attention_f64(q, K, V)
    np.testing.assert_allclose(o64, ref, rtol=1e-12, atol=1e-13)


def test_gqa_head_to_kv_head_mapping():
    """Head h must read KV head h // g: make each KV head's V a distinct constant."""
    rng = np.random.default_rng(2)
    H, G, L, d = 8, 4, 16, 128
    q, K, V = rand_qkv(rng, H, G, L, d)
    Vc = np.empty((G, L, d), dtype=np.float32)
    for kv in range(G):
        Vc[kv] = float(kv + 1)
    _, o64 = oracle.attention(q, K, f32_to_bf16_bits(Vc), want_f64=True)
    for h in range(H):
        np.testing.assert_allclose(o64[h], h // (H // G) + 1, rtol=1e-14)


def test_single_token_returns_its_value_row():
    rng = np.random.default_rng(3)
    q, K, V = rand_qkv(rng, 4, 2, 9)
    out = oracle.attention(q, K, V, idx=np.array([5], dtype=np.int32))
    for h in range(4):
        np.testing.assert_array_equal(out[h], V[h // 2, 5])


def test_equal_keys_give_mean_of_values():
    rng = np.random.default_rng(4)
    q, K, V = rand_qkv(rng, 2, 1, 11)
    K[:] = K[:, :1]
    _, o64 = oracle.attention(q, K, V, want_f64=True)
    np.testing.assert_allclose(o64[0], bits_to_f64(V)[0].mean(axis=0), rtol=1e-13, atol=1e-15)


def test_scale_is_one_over_sqrt_d_by_default():
    rng = np.random.default_rng(5)
    q, K, V = rand_qkv(rng, 2, 1, 20, 64)
    _, a = oracle.attention(q, K, V, want_f64=True)
    _, b = oracle.attention(q, K, V, sm_scale=1 / 8.0, want_f64=True)
    np.testing.assert_array_equal(a, b)
    _, c = oracle.attention(q, K, V, sm_scale=1.0, want_f64=True)
    assert np.abs(a - c).max() > 1e-3


def test_sparse_equals_dense_on_gathered_cache():
    rng = np.random.default_rng(6)
    H, G, L = 8, 2, 200
    q, K, V = rand_qkv(rng, H, G, L)
    idx = np.sort(rng.choice(L, size=33, replace=False)).astype(np.int32)
    out, o64 = oracle.attention(q, K, V, idx=idx, want_f64=True)
    ref = dense_attention_f64(q, K, V, tokens=idx)
    np.testing.assert_allclose(o64, ref, rtol=1e-12, atol=1e-13)
    # same result as dense attention over a cache that physically holds only those tokens
    out2 = oracle.attention(q, np.ascontiguousarray(K[:, idx]), np.ascontiguousarray(V[:, idx]))
    np.testing.assert_array_equal(out, out2)


def test_sparse_over_all_tokens_is_dense_bit_for_bit():
    rng = np.random.default_rng(7)
    q, K, V = rand_qkv(rng, 4, 2, 77)
    a = oracle.attention(q, K, V)
    b = oracle.attention(q, K, V, idx=np.arange(77, dtype=np.int32))
    np.testing.assert_array_equal(a, b)


def test_bf16_rounding_of_output_is_nearest_even():
    """A one-token attention returns exp(0) * v / 1 = v; craft V so o needs rounding via 2 tokens."""
    # two tokens with equal keys: o = (v0 + v1) / 2.  Choose v0, v1 so the mean is a bf16 midpoint.
    q = f32_to_bf16_bits(np.ones((1, 128), dtype=np.float32))
    K = f32_to_bf16_bits(np.ones((1, 2, 128), dtype=np.float32))
    v0 = np.full(128, 1.0, dtype=np.float32)
    v1 = np.full(128, 1.0 + 2.0 ** -7, dtype=np.float32)     # next bf16 after 1.0
    V = f32_to_bf16_bits(np.stack([v0, v1])[None])
    out = oracle.attention(q, K, V)
    # mean = 1 + 2^-8: midpoint of 1.0 (even mantissa) and 1 + 2^-7 -> rounds to 1.0
    assert (out == 0x3F80).all()
    v0[:] = 1.0 + 2.0 ** -7
    v1[:] = 1.0 + 2.0 ** -6
    V = f32_to_bf16_bits(np.stack([v0, v1])[None])
    out = oracle.attention(q, K, V)
    # mean = 1 + 3*2^-8: midpoint of 0x3F81 (odd) and 0x3F82 (even) -> 0x3F82
    assert (out == 0x3F82).all()


def test_bf16_output_is_within_half_ulp_of_float64_result():
    rng = np.random.default_rng(8)
    q, K, V = rand_qkv(rng, 8, 2, 50)
    out, o64 = oracle.attention(q, K, V, want_f64=True)
    r = bits_to_f64(out)
    ulp = 2.0 ** (np.floor(np.log2(np.abs(o64))) - 7)
    assert (np.abs(r - o64) <= ulp / 2).all()


def test_recall_definition():
    rng = np.random.default_rng(9)
    H, G, L = 4, 2, 60
    q, K, _ = rand_qkv(rng, H, G, L)
    idx = np.sort(rng.choice(L, size=17, replace=False)).astype(np.int32)
    r = oracle.recall(q, K, idx)
    qf, Kf = bits_to_f64(q), bits_to_f64(K)
    for h in range(H):
        w = (Kf[h // 2] @ qf[h]) / np.sqrt(128)
        p = np.exp(w - w.max())
        p /= p.sum()
        np.testing.assert_allclose(r[h], p[idx].sum(), rtol=1e-12)
    np.testing.assert_allclose(oracle.recall(q, K, np.arange(L, dtype=np.int32)), 1.0, rtol=1e-13)


# ---------------------------------------------------------------- head-to-head (per-head) variant

def test_per_head_attention_with_one_shared_list_is_the_unified_sparse_attention():
    rng = np.random.default_rng(71)
    H, G, L = 8, 2, 90
    q, K, V = rand_qkv(rng, H, G, L)
    idx = np.sort(rng.choice(L, size=20, replace=False)).astype(np.int32)
    got = oracle.attention_per_head(q, K, V, np.tile(idx, (H, 1)))
    np.testing.assert_array_equal(got, oracle.attention(q, K, V, idx))


def test_per_head_attention_is_dense_attention_on_each_heads_gathered_rows():
    """Head h with list T_h must equal dense attention of q_h over K[h // g, T_h], V[h // g, T_h]."""
    rng = np.random.default_rng(72)
    H, G, L, n = 6, 3, 70, 17
    q, K, V = rand_qkv(rng, H, G, L)
    idx_head = np.stack([np.sort(rng.choice(L, size=n, replace=False)) for _ in range(H)]).astype(np.int32)
    got = bits_to_f64(oracle.attention_per_head(q, K, V, idx_head))
    for h in range(H):
        kv = h // (H // G)
        ref = dense_attention_f64(q[h:h + 1], K[kv:kv + 1, idx_head[h]], V[kv:kv + 1, idx_head[h]])[0]
        np.testing.assert_allclose(got[h], ref, rtol=2 ** -8, atol=1e-30)      # bf16 rounding of the output
