"""Pins for per-head top-k, the cross-head union / global rank and the recency window
(Sec. 3.2, Sec. 3.3, Alg. 1 selection layer)."""
import numpy as np
import pytest

import oracle
from helpers import f32_to_bf16_bits, rand_qkv

# ----------------------------------------------------------------- per-head top-k


def _brute_topk(P, k):
    H, Lc = P.shape
    out = []
    for h in range(H):
        order = sorted(range(Lc), key=lambda t: (-float(P[h, t]), t))
        out.append(order[: min(k, Lc)])
    return np.array(out, dtype=np.int32)


@pytest.mark.parametrize("Lc,k", [(50, 7), (64, 64), (10, 30), (333, 100)])
def test_topk_matches_full_sort(Lc, k):
    rng = np.random.default_rng(21)
    P = rng.standard_normal((5, Lc)).astype(np.float32)
    np.testing.assert_array_equal(oracle.topk(P, k), _brute_topk(P, k))


def test_topk_ties_go_to_the_lowest_position():
    rng = np.random.default_rng(22)
    P = rng.integers(-3, 4, size=(6, 200)).astype(np.float32)   # heavy ties
    rho = oracle.topk(P, 50)
    np.testing.assert_array_equal(rho, _brute_topk(P, 50))
    P[:] = 1.5                                                    # everything ties
    np.testing.assert_array_equal(oracle.topk(P, 9), np.tile(np.arange(9, dtype=np.int32), (6, 1)))


def test_topk_signed_zeros_compare_equal():
    P = np.array([[0.0, -0.0, -0.0, 0.0, -1.0]], dtype=np.float32)
    np.testing.assert_array_equal(oracle.topk(P, 4), [[0, 1, 2, 3]])


def test_topk_is_ranked_best_first():
    rng = np.random.default_rng(23)
    P = rng.standard_normal((3, 100)).astype(np.float32)
    rho = oracle.topk(P, 20)
    for h in range(3):
        s = P[h, rho[h]]
        assert (np.diff(s) <= 0).all()
        assert set(rho[h]) == set(np.argsort(-P[h], kind="stable")[:20])

# ------------------------------------------------------------ union / rank / window


def _brute_unify(rho_head, P, L, K, W, mode):
    """Independent re-statement with python containers."""
    if L <= K:
        return list(range(L))
    H, k_eff = rho_head.shape
    info = {}
    for h in range(H):
        for j in range(k_eff):
            t = int(rho_head[h, j])
            e = info.setdefault(t, {"first": j * H + h, "votes": 0, "best": j, "max": -np.inf})
            e["first"] = min(e["first"], j * H + h)
            e["votes"] += 1
            e["best"] = min(e["best"], j)
            if P is not None:
                e["max"] = max(e["max"], float(P[h, t]))
    if mode == 0:
        ranked = sorted(info, key=lambda t: info[t]["first"])
    elif mode == 1:
        ranked = sorted(info, key=lambda t: (-info[t]["votes"], info[t]["best"], t))
    else:
        ranked = sorted(info, key=lambda t: (-info[t]["max"], t))
    keep = ranked[: K - W]
    return sorted(set(keep) | set(range(L - W, L)))


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("H,L,K,W,k", [(4, 64, 16, 4, 12), (2, 40, 4, 1, 3), (8, 100, 32, 8, 24),
                                       (3, 30, 10, 0, 10), (4, 50, 12, 12, 5), (4, 64, 16, 4, 20)])
def test_unify_matches_dictionary_brute_force(mode, H, L, K, W, k):
    rng = np.random.default_rng(100 * mode + H + L)
    for _ in range(5):
        # correlated heads so that the union really has duplicates
        base = rng.standard_normal(L - W).astype(np.float32)
        P = (base[None] + 0.7 * rng.standard_normal((H, L - W))).astype(np.float32)
        rho_head = oracle.topk(P, k)
        got = oracle.unify(rho_head, L, K, W, mode, P)
        assert got.tolist() == _brute_unify(rho_head, P, L, K, W, mode)


def test_first_occurrence_order_is_rank_major_then_head():
    """Hand-worked case, H = 2, k = 3, K - W = 3.
    head 0 ranks [7, 2, 5], head 1 ranks [2, 9, 7]: rank-major flattening is
    7, 2 | 2, 9 | 5, 7 -> distinct in order 7, 2, 9, 5 -> keep 7, 2, 9."""
    rho_head = np.array([[7, 2, 5], [2, 9, 7]], dtype=np.int32)
    got = oracle.unify(rho_head, L=20, K=5, W=2, rank_mode=0)
    assert got.tolist() == [2, 7, 9, 18, 19]
    # head-major flattening (7,2,5,...) or a position-sorted unique (2,5,7) would give other sets
    assert got.tolist() != sorted({7, 2, 5, 18, 19}) and got.tolist() != sorted({2, 5, 7, 18, 19})
    # votes: 7 and 2 have two votes (best ranks 0, 0 -> position breaks the tie), then 9 (rank 1) beats 5 (rank 2)
    assert oracle.unify(rho_head, 20, 5, 2, 1).tolist() == [2, 7, 9, 18, 19]
    rho_head = np.array([[7, 2, 5], [3, 9, 5]], dtype=np.int32)
    assert oracle.unify(rho_head, 20, 5, 2, 0).tolist() == [2, 3, 7, 18, 19]   # 7, 3, 2
    assert oracle.unify(rho_head, 20, 5, 2, 1).tolist() == [3, 5, 7, 18, 19]   # 5 (2 votes), 3, 7


def test_pipeline_figure_shape_K4_r025():
    """The pipeline figure's shape: K = 4, r = 0.25 -> k = 3 per head and one recent token."""
    rng = np.random.default_rng(31)
    H, G, L, K, W = 4, 2, 12, 4, 1
    q, Kc, _ = rand_qkv(rng, H, G, L)
    rho, rho_head, P = oracle.select(q, Kc, K, W, return_all=True)
    assert rho_head.shape == (H, 3) and P.shape == (H, L - 1)
    assert len(rho) == 4 and rho[-1] == L - 1
    assert set(rho[:-1]) <= set(rho_head.ravel())


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_invariants_of_the_selected_set(mode):
    rng = np.random.default_rng(32 + mode)
    H, G, L, K, W, k = 8, 2, 300, 64, 16, 48
    q, Kc, _ = rand_qkv(rng, H, G, L)
    rho, rho_head, P = oracle.select(q, Kc, K, W, k, mode, return_all=True)
    assert len(rho) == K and (np.diff(rho) > 0).all()                 # |rho| = K, ascending, distinct
    assert set(range(L - W, L)) <= set(rho)                           # window always kept
    hist = [t for t in rho if t < L - W]
    assert len(hist) == K - W
    assert set(hist) <= set(rho_head.ravel())                         # from some head's top-k
    assert rho_head.max() < L - W                                     # candidates exclude the window
    if mode == 0:
        assert set(rho_head[:, 0]) <= set(rho)                        # every head's best pick survives


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_identical_heads_reduce_to_one_heads_topk(mode):
    rng = np.random.default_rng(35)
    G, L, K, W = 1, 120, 40, 10
    q1, Kc, _ = rand_qkv(rng, 1, G, L)
    q = np.repeat(q1, 4, axis=0)
    rho, rho_head, _ = oracle.select(q, Kc, K, W, return_all=True, rank_mode=mode)
    assert sorted(rho[: K - W]) == sorted(rho_head[0, : K - W])
    rho1 = oracle.select(q1, Kc, K, W, rank_mode=mode)              # H = 1: plain top-(K-W) + window
    np.testing.assert_array_equal(rho, rho1)
    P = oracle.scores(q1, Kc, L - W)
    want = sorted(np.argsort(-P[0], kind="stable")[: K - W].tolist() + list(range(L - W, L)))
    assert rho1.tolist() == want


def test_window_only_and_no_window():
    rng = np.random.default_rng(36)
    q, Kc, _ = rand_qkv(rng, 4, 2, 90)
    np.testing.assert_array_equal(oracle.select(q, Kc, 20, 20), np.arange(70, 90))   # r = 1
    rho = oracle.select(q, Kc, 20, 0)                                                # r = 0
    assert len(rho) == 20
    P = oracle.scores(q, Kc, 90)
    assert set(np.argmax(P, axis=1)) <= set(rho)


def test_budget_covering_the_context_selects_everything():
    rng = np.random.default_rng(37)
    q, Kc, _ = rand_qkv(rng, 4, 2, 33)
    for K in (33, 34, 100):
        np.testing.assert_array_equal(oracle.select(q, Kc, K, K // 4), np.arange(33))


def test_planted_heavy_keys_are_selected():
    rng = np.random.default_rng(38)
    H, G, L, K, W = 8, 2, 512, 64, 16
    q, Kc, _ = rand_qkv(rng, H, G, L)
    qf = oracle.bf16_bits_to_f32(q).reshape(G, H // G, 128)
    planted = np.sort(rng.choice(L - W, size=6, replace=False))
    for kv in range(G):
        Kc[kv, planted] = f32_to_bf16_bits((3.0 / 2.0) * qf[kv].sum(axis=0))
    rho, rho_head, _ = oracle.select(q, Kc, K, W, return_all=True)
    assert set(planted) <= set(rho)
    for h in range(H):
        assert set(rho_head[h, :6]) == set(planted)                  # ranks 0..5 of every head

# ----------------------------------------------------------------- decode step walk


def test_decode_step_walks_the_schedule():
    rng = np.random.default_rng(39)
    H, G, L, K, W = 4, 2, 80, 16, 4
    layers = [rand_qkv(rng, H, G, L) for _ in range(4)]
    qs, Ks, Vs = zip(*layers)
    kinds = [oracle.LAYER_FULL, oracle.LAYER_SELECT, oracle.LAYER_SPARSE, oracle.LAYER_SPARSE]
    outs, rho = oracle.decode_step(kinds, qs, Ks, Vs, K, W)
    np.testing.assert_array_equal(rho, oracle.select(qs[1], Ks[1], K, W))   # from the selection layer's q, K
    np.testing.assert_array_equal(outs[0], oracle.attention(qs[0], Ks[0], Vs[0]))
    np.testing.assert_array_equal(outs[1], oracle.attention(qs[1], Ks[1], Vs[1]))   # selection layer: full
    for i in (2, 3):                                                         # own K/V, shared positions
        np.testing.assert_array_equal(outs[i], oracle.attention(qs[i], Ks[i], Vs[i], rho))
    with pytest.raises(ValueError):
        oracle.decode_step([oracle.LAYER_SPARSE], qs[:1], Ks[:1], Vs[:1], K, W)


def test_decode_step_with_budget_at_least_context_is_dense_everywhere():
    rng = np.random.default_rng(40)
    H, G, L = 4, 2, 50
    layers = [rand_qkv(rng, H, G, L) for _ in range(3)]
    qs, Ks, Vs = zip(*layers)
    kinds = [oracle.LAYER_SELECT, oracle.LAYER_SPARSE, oracle.LAYER_SPARSE]
    outs, rho = oracle.decode_step(kinds, qs, Ks, Vs, budget=64, window=16)
    np.testing.assert_array_equal(rho, np.arange(L))
    for i in range(3):
        np.testing.assert_array_equal(outs[i], oracle.attention(qs[i], Ks[i], Vs[i]))


def test_paged_view_resolution():
    rng = np.random.default_rng(41)
    G, page, d, L = 2, 16, 128, 45
    n_pages = 7
    pool = rng.integers(0, 2 ** 16, size=(n_pages, G, page, d), dtype=np.uint16)
    bt = np.array([4, 0, 6], dtype=np.int32)
    view = oracle.resolve_paged(pool, bt, L)
    for kv in range(G):
        for t in range(L):
            np.testing.assert_array_equal(view[kv, t], pool[bt[t // page], kv, t % page])


# ---------------------------------------------------------------- head-to-head (per-head) variant

def test_per_head_selection_is_each_heads_own_topk_plus_window():
    rng = np.random.default_rng(61)
    H, G, L, K, W = 8, 2, 400, 64, 16
    q, Kc, _ = rand_qkv(rng, H, G, L)
    rho_h = oracle.select_per_head(q, Kc, K, W)
    assert rho_h.shape == (H, K) and (np.diff(rho_h, axis=1) > 0).all()
    P = oracle.scores(q, Kc, L - W)
    for h in range(H):
        want = sorted(np.argsort(-P[h], kind="stable")[: K - W].tolist() + list(range(L - W, L)))
        assert rho_h[h].tolist() == want
    # the unified set takes every token from some head's own set
    rho = oracle.select(q, Kc, K, W)
    assert set(rho) <= set(rho_h.ravel())


def test_per_head_selection_with_one_head_is_the_unified_selection():
    rng = np.random.default_rng(62)
    q, Kc, _ = rand_qkv(rng, 1, 1, 250)
    np.testing.assert_array_equal(oracle.select_per_head(q, Kc, 48, 12)[0], oracle.select(q, Kc, 48, 12))
    np.testing.assert_array_equal(oracle.select_per_head(q, Kc, 300, 12)[0], np.arange(250))   # budget covers L


# ---------------------------------------------------------------- attention sinks (Sec. 4.1)

@pytest.mark.parametrize("mode", [0, 1, 2])
def test_sinks_are_always_kept_and_never_ranked(mode):
    rng = np.random.default_rng(81 + mode)
    H, G, L, K, W, S = 8, 2, 300, 64, 16, 4
    q, Kc, _ = rand_qkv(rng, H, G, L)
    rho, rho_head, P = oracle.select(q, Kc, K, W, rank_mode=mode, return_all=True, n_sink=S)
    assert len(rho) == K and (np.diff(rho) > 0).all()
    assert rho[:S].tolist() == list(range(S)) and set(range(L - W, L)) <= set(rho)
    assert rho_head.min() >= S and rho_head.max() < L - W              # sinks and window are no candidates
    for h in range(H):                                                 # each head: its best among [S, L-W)
        want = (np.argsort(-P[h, S:], kind="stable")[: rho_head.shape[1]] + S).tolist()
        assert rho_head[h].tolist() == want
    # the same problem with the sink keys cut out of the cache, shifted back: same picks
    rho_cut = oracle.select(q, Kc[:, S:], K - S, W, topk_per_head=K - W, rank_mode=mode)   # same k per head
    assert (rho_cut + S).tolist() == rho[S:].tolist()


def test_sinks_zero_is_the_plain_selection_and_sinks_fill_the_history():
    rng = np.random.default_rng(85)
    q, Kc, _ = rand_qkv(rng, 4, 2, 200)
    np.testing.assert_array_equal(oracle.select(q, Kc, 40, 10, n_sink=0), oracle.select(q, Kc, 40, 10))
    rho = oracle.select(q, Kc, 40, 10, n_sink=30)                       # K - W - S = 0: sinks + window only
    assert rho.tolist() == list(range(30)) + list(range(190, 200))
    np.testing.assert_array_equal(oracle.select(q, Kc, 300, 10, n_sink=4), np.arange(200))   # budget covers L


def test_per_head_selection_with_sinks():
    rng = np.random.default_rng(86)
    H, G, L, K, W, S = 4, 2, 260, 48, 12, 4
    q, Kc, _ = rand_qkv(rng, H, G, L)
    rho_h = oracle.select_per_head(q, Kc, K, W, n_sink=S)
    P = oracle.scores(q, Kc, L - W)
    for h in range(H):
        want = sorted(list(range(S)) + (np.argsort(-P[h, S:], kind="stable")[: K - W - S] + S).tolist()
                      + list(range(L - W, L)))
        assert rho_h[h].tolist() == want
