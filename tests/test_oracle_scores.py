"""Pins for the oracle's selection scores P = q . K^T (Alg. 1, selection layer)."""
import numpy as np
import pytest

import oracle
from helpers import bits_to_f64, f32_to_bf16_bits, rand_qkv


def _scalar_left_to_right(q, K, h, kv, t):
    acc = np.float32(0.0)
    qf = oracle.bf16_bits_to_f32(q[h])
    kf = oracle.bf16_bits_to_f32(K[kv, t])
    for i in range(qf.size):
        acc = np.float32(acc + np.float32(qf[i] * kf[i]))
    return acc


def test_bitwise_equal_to_scalar_float32_left_to_right_sum():
    rng = np.random.default_rng(11)
    H, G, L, d = 4, 2, 9, 128
    q, K, _ = rand_qkv(rng, H, G, L, d)
    P = oracle.scores(q, K, L - 2)
    assert P.shape == (H, L - 2) and P.dtype == np.float32
    for h in range(H):
        for t in range(L - 2):
            assert P[h, t].view(np.uint32) == _scalar_left_to_right(q, K, h, h // 2, t).view(np.uint32)


def test_within_error_bound_of_float64_dot_and_unscaled():
    rng = np.random.default_rng(12)
    H, G, L, d = 8, 2, 257, 128
    q, K, _ = rand_qkv(rng, H, G, L, d)
    P = oracle.scores(q, K, L)
    qf, Kf = bits_to_f64(q), bits_to_f64(K)
    for h in range(H):
        exact = Kf[h // 4] @ qf[h]                   # no 1/sqrt(d)
        bound = d * 2.0 ** -24 * (np.abs(Kf[h // 4]) @ np.abs(qf[h]))
        assert (np.abs(P[h] - exact) <= bound).all()
    assert np.abs(P).std() > 5.0                      # ~sqrt(128) = 11.3, not ~1


def test_summation_runs_left_to_right():
    """2^24 + 1 + 1 = 2^24 left to right (two ties to even), but 1 + 1 + 2^24 = 2^24 + 2."""
    d = 128
    q = f32_to_bf16_bits(np.ones((1, d), dtype=np.float32))
    k = np.zeros((1, 2, d), dtype=np.float32)
    k[0, 0, :3] = [2.0 ** 24, 1.0, 1.0]
    k[0, 1, :3] = [1.0, 1.0, 2.0 ** 24]
    P = oracle.scores(q, f32_to_bf16_bits(k), 2)
    assert P[0, 0] == np.float32(2.0 ** 24)
    assert P[0, 1] == np.float32(2.0 ** 24 + 2.0)
    # the same at the far end of the row (no blocking of the head dimension)
    k[:] = 0
    k[0, 0, [0, 126, 127]] = [2.0 ** 24, 1.0, 1.0]
    k[0, 1, [0, 1, 127]] = [1.0, 1.0, 2.0 ** 24]
    P = oracle.scores(q, f32_to_bf16_bits(k), 2)
    assert P[0, 0] == np.float32(2.0 ** 24)
    assert P[0, 1] == np.float32(2.0 ** 24 + 2.0)


def test_products_are_exact_so_only_additions_round():
    """A single non-zero product must come out exactly (16-bit significand fits binary32)."""
    d = 128
    a, b = np.float32(1.9921875), np.float32(-1.9921875)       # 0xFF * 2^-7, full 8-bit significands
    q = np.zeros((1, d), dtype=np.float32)
    k = np.zeros((1, 1, d), dtype=np.float32)
    q[0, 77], k[0, 0, 77] = a, b
    P = oracle.scores(f32_to_bf16_bits(q), f32_to_bf16_bits(k), 1)
    assert float(P[0, 0]) == float(a) * float(b)


def test_candidate_range_and_gqa_mapping():
    rng = np.random.default_rng(13)
    H, G, L = 6, 3, 40
    q, K, _ = rand_qkv(rng, H, G, L)
    P_all = oracle.scores(q, K, L)
    P_c = oracle.scores(q, K, L - 7)
    np.testing.assert_array_equal(P_all[:, : L - 7], P_c)
    # swapping two KV heads' keys swaps the scores of the head groups that read them
    K2 = K.copy()
    K2[[0, 2]] = K[[2, 0]]
    P2 = oracle.scores(q, K2, L)
    qf, Kf = bits_to_f64(q), bits_to_f64(K2)
    for h in range(H):
        np.testing.assert_allclose(P2[h], Kf[h // 2] @ qf[h], rtol=0, atol=1e-3)


@pytest.mark.parametrize("d", [64, 128])
def test_zero_rows_score_plus_zero(d):
    q = f32_to_bf16_bits(-np.ones((1, d), dtype=np.float32))
    K = np.zeros((1, 3, d), dtype=np.uint16)
    P = oracle.scores(q, K, 3)
    assert (P.view(np.uint32) == 0).all()          # +0.0, never -0.0
