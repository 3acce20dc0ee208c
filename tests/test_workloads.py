"""The seeded generators: shapes, determinism, planted structure, paged tables (CPU)."""
import numpy as np
import torch

import oracle
from helpers import host_view
from paper_2508_07101_amd import workloads as wl


def _tiny(**kw):
    base = dict(name="tiny", n_layers=2, batch=3, n_q_heads=8, n_kv_heads=2, head_dim=128, seq_len=200,
                budget=32, window=8, topk_per_head=0, schedule=(1, 2), seed=5)
    base.update(kw)
    return wl.Workload(**base)


def test_five_workloads_have_the_stated_shapes():
    c = wl.WORKLOADS
    assert [c[n].n_layers for n in ("c2", "c3", "c5")] == [32, 36, 4]
    assert c["c2"].schedule[:3] == (0, 0, 1) and set(c["c2"].schedule[3:]) == {2} and len(c["c2"].schedule) == 32
    assert c["c3"].schedule.count(2) == 33 and c["c5"].schedule == (1, 2, 2, 2)
    assert (c["c1"].k_eff, c["c2"].k_eff, c["c4"].k_eff) == (1024, 1536, 3072)
    assert c["c4"].n_q_heads // c["c4"].n_kv_heads == 8 and c["c5"].paged and c["c5"].page_size == 16
    lens = wl.draw_lengths(c["c5"])
    assert len(lens) == 64 and min(lens) >= 8192 and max(lens) <= 32768 and lens == wl.draw_lengths(c["c5"])


def test_draws_are_seeded_and_free_of_tiny_values():
    a = wl.make_inputs(_tiny(), "cpu")
    b = wl.make_inputs(_tiny(), "cpu")
    for la, lb in zip(a.layers, b.layers):
        assert torch.equal(la.k, lb.k) and torch.equal(la.q, lb.q) and torch.equal(la.v, lb.v)
    c = wl.make_inputs(_tiny(seed=6), "cpu")
    assert not torch.equal(a.layers[0].k, c.layers[0].k)
    k = a.layers[0].k.float()
    assert ((k == 0) | (k.abs() >= 2.0 ** -30)).all()
    assert abs(float(k.std()) - 1.0) < 0.05


def test_planted_keys_rank_first_for_every_head():
    w = _tiny(n_planted=4, seq_len=400)
    inp = wl.make_inputs(w, "cpu")
    for b in range(w.batch):
        q, K, _ = host_view(inp, 0, b)
        P = oracle.scores(q, K, w.seq_len - w.window)
        top = oracle.topk(P, 4)
        planted = set(inp.layers[0].planted[b].tolist())
        assert max(planted) < w.seq_len - w.window
        for h in range(w.n_q_heads):
            assert set(top[h]) == planted


def test_paged_pool_and_block_table():
    w = _tiny(paged=True, lengths=(200, 17, 96))
    inp = wl.make_inputs(w, "cpu")
    pages = [(n + 15) // 16 for n in w.lengths]
    assert inp.n_pages == sum(pages) and inp.layers[0].k.shape == (sum(pages), 2, 16, 128)
    used = np.concatenate([inp.block_table[b, :n].numpy() for b, n in enumerate(pages)])
    assert sorted(used.tolist()) == list(range(sum(pages)))          # a permutation of all pool pages
    assert not (np.diff(used) == 1).all()                             # shuffled
    q, K, V = host_view(inp, 0, 2)
    pool = wl.bf16_bits(inp.layers[0].k)
    for t in (0, 15, 16, 95):
        page = int(inp.block_table[2, t // 16])
        np.testing.assert_array_equal(K[1, t], pool[page, 1, t % 16])


def test_lowrank_component_correlates_heads():
    w = _tiny(lowrank=8, lowrank_scale=2.0, seq_len=600, n_q_heads=8, n_kv_heads=8)
    inp = wl.make_inputs(w, "cpu")
    q, K, _ = host_view(inp, 0, 0)
    P = oracle.scores(q, K, 600).astype(np.float64)
    c = np.corrcoef(P)
    off = c[~np.eye(8, dtype=bool)]
    assert off.mean() > 0.2                                           # independent heads would give ~0


def test_loop_workload_has_the_papers_settings_and_room_to_grow():
    w = wl.WORKLOADS["loop"]
    assert w.n_layers == 36 and len(w.schedule) == 36 and w.n_sink == 4
    assert [i for i, k in enumerate(w.schedule) if k == 1] == [2, 12]     # selection layer and re-selection layer
    assert w.schedule[:2] == (0, 0) and w.window * 4 == w.budget          # two full layers first; r = 0.25
    assert wl.draw_lengths(w)[0] + w.grow_room <= w.seq_len


def test_grow_room_reserves_pages_and_cache_rows():
    w = _tiny(paged=True, lengths=(100, 17, 96), grow_room=40)
    inp = wl.make_inputs(w, "cpu")
    pages = [(n + 40 + 15) // 16 for n in w.lengths]
    assert inp.n_pages == sum(pages) and inp.block_table.shape[1] == max(pages)
    used = np.concatenate([inp.block_table[b, :n].numpy() for b, n in enumerate(pages)])
    assert sorted(used.tolist()) == list(range(sum(pages)))          # the reserved pages are distinct pool pages too
    c = wl.make_inputs(_tiny(lengths=(100, 17, 96), grow_room=40), "cpu")
    assert c.layers[0].k.shape[2] >= 140                             # contiguous caches hold the grown length


def test_decode_step_oracle_passes_the_sinks_on():
    rng = np.random.default_rng(3)
    from helpers import rand_qkv
    q, K, V = rand_qkv(rng, 4, 2, 150)
    outs, rho = oracle.decode_step([1, 2], [q, q], [K, K], [V, V], budget=32, window=8, n_sink=4)
    np.testing.assert_array_equal(rho, oracle.select(q, K, 32, 8, n_sink=4))
    np.testing.assert_array_equal(outs[1], oracle.attention(q, K, V, rho))
    assert rho[:4].tolist() == [0, 1, 2, 3]
