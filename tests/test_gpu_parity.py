"""Parity of the HIP path (through the C ABI) against the CPU oracle on the same seeded inputs.

Bars: selection scores, ranked per-head lists, idx and cnt bit-exact; attention outputs within
|gpu - oracle| <= 2e-2 + 1e-2 |oracle| on the bf16 values.
"""
import numpy as np
import pytest
import torch

import oracle
from helpers import assert_close_bf16, host_view
from paper_2508_07101_amd import binding as cb
from paper_2508_07101_amd import workloads as wl
from paper_2508_07101_amd.runner import StepRunner
from paper_2508_07101_amd.workloads import LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, bf16_bits

pytestmark = pytest.mark.gpu
DEV = "cuda"


def _say(msg):
    print(f"[parity] {msg}", flush=True)


def small(name="t", **kw):
    base = dict(name=name, n_layers=2, batch=2, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=1500,
                budget=256, window=64, topk_per_head=0, schedule=(LAYER_SELECT, LAYER_SPARSE), seed=777)
    base.update(kw)
    return wl.Workload(**base)


def check_select(inp, runner, layer_pos, seqs=None, check_scores=True, rank_mode=0):
    w = inp.workload
    torch.cuda.synchronize()
    idx = runner.idx.cpu().numpy()
    cnt = runner.cnt.cpu().numpy()
    P_dev, rho_dev = runner.scores(), runner.rho_head()
    for b in (range(w.batch) if seqs is None else seqs):
        q, K, _ = host_view(inp, layer_pos, b)
        L = inp.seq_lens_host[b]
        rho, rho_head, P = oracle.select(q, K, w.budget, w.window, w.topk_per_head, rank_mode, return_all=True,
                                         n_sink=w.n_sink)
        if L > w.budget:
            Lc = L - w.window
            if check_scores and runner.scores_valid:
                got = P_dev[b, :, :Lc].cpu().numpy()
                assert (got.view(np.uint32) == P.view(np.uint32)).all(), f"scores differ, seq {b}"
            k_eff = rho_head.shape[1]
            got = rho_dev[b, :k_eff, :].cpu().numpy().T
            assert (got == rho_head).all(), f"ranked per-head lists differ, seq {b}: {(got != rho_head).sum()} entries"
        assert cnt[b] == len(rho) == min(w.budget, L), f"cnt seq {b}: {cnt[b]} vs {len(rho)}"
        assert (idx[b, : cnt[b]] == rho).all(), f"idx differs, seq {b}"


def check_attention(inp, runner, layer_pos, kind, seqs=None):
    w = inp.workload
    torch.cuda.synchronize()
    out = bf16_bits(runner.outs[layer_pos])
    idx = runner.idx.cpu().numpy()
    cnt = runner.cnt.cpu().numpy()
    for b in (range(w.batch) if seqs is None else seqs):
        q, K, V = host_view(inp, layer_pos, b)
        rho = idx[b, : cnt[b]] if kind == LAYER_SPARSE else None
        want = oracle.attention(q, K, V, rho)
        assert_close_bf16(out[b], want, f"layer {layer_pos} kind {kind} seq {b}")


def run_and_check(w, layers=None, seqs=None, check_scores=True):
    inp = wl.make_inputs(w, DEV, layers)
    sched = list(w.schedule) if layers is None else [w.schedule[i] for i in layers]
    r = StepRunner(inp, sched)
    _say(f"{w.name}: decode step over {len(sched)} layers, lens {inp.seq_lens_host[:6]}...")
    r.run()
    torch.cuda.synchronize()
    sel = max(i for i, k in enumerate(sched) if k == LAYER_SELECT)
    # a selection layer on the filtered fast path writes no score array: the scores are then checked on cusa_select's
    check_select(inp, r, sel, seqs, check_scores)
    if check_scores and r.filtered_select():
        _say(f"{w.name}: filtered selection layer; scores from cusa_select")
        r.select(sel)
        check_select(inp, r, sel, seqs, True)
    return inp, r, sched


# ------------------------------------------------------------------ small shapes

@pytest.mark.parametrize("H,G", [(8, 8), (16, 8), (32, 8), (64, 8)])
def test_small_contiguous_all_group_sizes(H, G):
    w = small(f"g{H // G}", n_q_heads=H, n_kv_heads=G, batch=3, seq_len=1500, min_seq_len=900, n_planted=5)
    inp, r, sched = run_and_check(w)
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)


def test_small_paged_ragged_with_short_sequences():
    # lengths from below the budget (rho = everything) to several score tiles with a ragged tail
    w = small("paged", batch=6, seq_len=2100, lengths=(100, 2100, 256, 257, 1033, 777), paged=True,
              budget=256, window=64)
    inp, r, sched = run_and_check(w)
    assert min(inp.seq_lens_host) <= w.budget < max(inp.seq_lens_host)
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)


def test_lowrank_correlated_heads_and_wider_topk():
    w = small("lowrank", batch=2, seq_len=3000, lowrank=8, budget=512, window=128, topk_per_head=512)
    inp, r, sched = run_and_check(w)
    check_attention(inp, r, 1, LAYER_SPARSE)


def test_four_layer_schedule_full_full_select_sparse():
    w = small("sched", n_layers=5, schedule=(LAYER_FULL, LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, LAYER_SPARSE),
              batch=2, seq_len=1200)
    inp, r, sched = run_and_check(w)
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)


@pytest.mark.parametrize("L,K,W,k", [
    (300, 256, 64, 0),      # L just above K
    (257, 256, 64, 0),      # L = K + 1
    (256, 256, 64, 0),      # L = K: everything
    (5, 256, 64, 0),        # tiny
    (1, 256, 64, 0),        # the current token only
    (330, 256, 64, 300),    # Lc = 266 < k: k clamps to Lc
    (1000, 128, 0, 0),      # no window
    (1000, 128, 128, 0),    # window only
    (1000, 64, 16, 1024),   # k far above K - W
    (1777, 1000, 250, 0),   # sizes that are multiples of nothing
    (4099, 333, 77, 401),
    (777, 37, 5, 33),
    (500, 1, 0, 0),         # budget of one token: the single best-ranked pick
    (500, 1, 1, 0),         # budget of one token: the current token
])
def test_edge_lengths_and_budgets(L, K, W, k):
    w = small(f"edge{L}_{K}_{W}_{k}", batch=2, seq_len=L, budget=K, window=W, topk_per_head=k)
    inp, r, sched = run_and_check(w)
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)


def _with_keys(w, fn, rank_mode=0):
    inp = wl.make_inputs(w, DEV)
    fn(inp.layers[0].k)
    r = StepRunner(inp, rank_mode=rank_mode)
    r.run()
    check_select(inp, r, 0, rank_mode=rank_mode)
    return inp, r


def test_ties_duplicated_keys_go_to_lowest_position():
    w = small("dup", batch=2, seq_len=1400, budget=256, window=64)

    def dup(k):
        k[:, :, 500:1000] = k[:, :, 0:500]      # every score in [0,500) appears again 500 later
    _with_keys(w, dup)


def test_ties_all_keys_equal():
    w = small("alleq", batch=1, seq_len=2500, budget=256, window=64)

    def alleq(k):
        k[:] = k[:, :, :1].clone()               # every candidate ties: ranks are positions 0,1,2,...
    inp, r = _with_keys(w, alleq)
    torch.cuda.synchronize()
    rho = r.rho_head()[0].cpu().numpy()          # [k, H]
    assert (rho == np.arange(rho.shape[0])[:, None]).all()


def test_ties_quantised_keys():
    w = small("quant", batch=2, seq_len=3000, budget=512, window=128)

    def quant(k):
        k.copy_(torch.sign(k) * (k.abs() > 0.8))   # keys in {-1, 0, 1}: scores collide heavily
    _with_keys(w, quant)


@pytest.mark.parametrize("L", [12000, 40000])
def test_ties_on_long_rows_overflow_the_candidate_list(L):
    """Rows long enough for the top-k kernel's LDS candidate list (keys in registers, and streamed
    from memory), with so many equal scores that the list cannot hold the candidates."""
    w = small(f"longties{L}", batch=1, seq_len=L, budget=512, window=128)

    def quant(k):
        k.copy_(torch.sign(k) * (k.abs() > 1.5))   # most keys are zero: most scores are exactly 0
    _with_keys(w, quant)

    def alleq(k):
        k[:] = k[:, :, :1].clone()
    inp, r = _with_keys(small(f"longeq{L}", batch=1, seq_len=L, budget=512, window=128), alleq)
    torch.cuda.synchronize()
    rho = r.rho_head()[0].cpu().numpy()
    assert (rho == np.arange(rho.shape[0])[:, None]).all()


@pytest.mark.parametrize("L", [12000, 40000])
def test_long_rows_with_distinct_scores_use_the_candidate_list(L):
    w = small(f"long{L}", batch=2, seq_len=L, min_seq_len=L - 3000, budget=1024, window=256, n_planted=8)
    inp, r, sched = run_and_check(w)
    check_attention(inp, r, 1, LAYER_SPARSE)


def test_large_topk_per_head_uses_the_widest_sort():
    """k between 4097 and 8192: eight sorted composites per thread and the largest LDS footprint."""
    w = small("bigk", batch=1, seq_len=20000, budget=6144, window=1024, n_planted=8)
    inp, r, sched = run_and_check(w)
    check_attention(inp, r, 1, LAYER_SPARSE)


def test_group_of_eight_on_long_paged_rows():
    w = small("g8long", n_q_heads=64, n_kv_heads=8, batch=2, seq_len=36000, min_seq_len=30000, paged=True,
              budget=1024, window=256)
    inp, r, sched = run_and_check(w)
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind, seqs=[1])


def test_repeated_steps_are_bit_identical():
    """Races between waves or workgroups would show up as run-to-run differences."""
    w = small("repeat", n_layers=3, schedule=(LAYER_FULL, LAYER_SELECT, LAYER_SPARSE), batch=5, seq_len=6000,
              lengths=(6000, 700, 2049, 4097, 300), paged=True, budget=512, window=128, lowrank=4)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    ref = None
    for _ in range(12):
        r.idx.fill_(-1)
        for o in r.outs:
            o.zero_()
        r.run()
        torch.cuda.synchronize()
        cur = [r.idx.clone(), r.cnt.clone()] + [o.clone() for o in r.outs]
        cnt = cur[1].cpu().numpy()
        for b in range(w.batch):
            cur[0][b, cnt[b]:] = -1                      # entries past cnt are unspecified
        if ref is not None:
            assert all(torch.equal(a, b_) for a, b_ in zip(cur, ref))
        ref = cur


def test_selection_is_deterministic_across_runs():
    w = small("det", batch=2, seq_len=4000, budget=512, window=128)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    ref = None
    for _ in range(3):
        r.idx.fill_(-1)
        r.select(0)
        torch.cuda.synchronize()
        cur = (r.idx.clone(), r.rho_head().clone())
        if ref is not None:
            assert torch.equal(cur[0], ref[0]) and torch.equal(cur[1], ref[1])
        ref = cur


def test_separate_entry_points_match_the_decode_step():
    w = small("entry", batch=2, seq_len=1700, n_planted=4)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.run()
    torch.cuda.synchronize()
    idx, outs = r.idx.clone(), [o.clone() for o in r.outs]
    r.idx.fill_(-1)
    r.select(0)
    r.full(0)
    r.sparse(1)
    torch.cuda.synchronize()
    assert torch.equal(r.idx, idx)
    assert torch.equal(r.outs[1], outs[1])
    # the step's selection layer sums q.k in the scoring order (it also emits P); the stand-alone
    # full attention sums it four elements at a time: same result up to binary32 rounding order
    torch.testing.assert_close(r.outs[0].float(), outs[0].float(), atol=2e-2, rtol=1e-2)


@pytest.mark.parametrize("H,paged,L", [(8, False, 1500), (16, True, 1500), (32, False, 1500), (64, True, 1500),
                                       (32, True, 21000), (64, False, 21000)])
def test_standalone_entry_points_match_the_oracle(H, paged, L):
    """cusa_select scores with its own kernel (the decode step takes the scores from the selection
    layer's attention pass); cusa_full_attn and cusa_sparse_attn are called one by one."""
    w = small(f"alone{H}", n_q_heads=H, n_kv_heads=8, batch=3, seq_len=L, min_seq_len=L * 3 // 5, paged=paged,
              n_planted=5)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    _say(f"{w.name}: select, full, sparse one by one, lens {inp.seq_lens_host}")
    r.scores().zero_()
    r.select(0)
    seqs = None if L < 4000 else [2]
    check_select(inp, r, 0, seqs)
    r.full(0)
    check_attention(inp, r, 0, LAYER_FULL, seqs)
    r.sparse(1)
    check_attention(inp, r, 1, LAYER_SPARSE, seqs)


@pytest.mark.parametrize("H,paged,lengths,sinks", [(8, False, (1500, 900, 1211), 0), (16, True, (100, 1500, 257), 0),
                                                   (32, False, (1500, 256, 1033), 4), (64, True, (1400, 1500, 700), 0),
                                                   (32, True, (9000, 300, 7001), 4)])
def test_per_head_selection_and_attention_match_the_oracle(H, paged, lengths, sinks):
    """Head-to-head variant: every head its own top-(K-W) + window, and sparse attention over it."""
    w = small(f"perhead{H}", n_q_heads=H, n_kv_heads=8, batch=len(lengths), seq_len=max(lengths), lengths=lengths,
              paged=paged, n_planted=5, n_sink=sinks)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    _say(f"{w.name}: per-head select + sparse attention, lens {inp.seq_lens_host}")
    idx_head = r.make_idx_head()
    r.select_per_head(0, idx_head)
    r.sparse_per_head(1, idx_head)
    torch.cuda.synchronize()
    got_idx, got_cnt = idx_head.cpu().numpy(), r.cnt.cpu().numpy()
    out = bf16_bits(r.outs[1])
    for b in range(w.batch):
        q, K, _ = host_view(inp, 0, b)
        rho_h = oracle.select_per_head(q, K, w.budget, w.window, w.n_sink)
        assert got_cnt[b] == rho_h.shape[1] == min(w.budget, inp.seq_lens_host[b])
        assert (got_idx[b, :, : got_cnt[b]] == rho_h).all(), f"per-head sets differ, seq {b}"
        q, K, V = host_view(inp, 1, b)
        assert_close_bf16(out[b], oracle.attention_per_head(q, K, V, rho_h), f"per-head attention seq {b}")


def test_per_head_attention_with_one_shared_list_equals_the_unified_kernel():
    w = small("perhead_shared", batch=2, seq_len=3000, budget=512, window=128)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.select(0)
    r.sparse(1)
    torch.cuda.synchronize()
    want = r.outs[1].clone()
    idx_head = r.idx[:, None, :].expand(-1, w.n_q_heads, -1).contiguous()
    r.outs[1].zero_()
    r.sparse_per_head(1, idx_head)
    torch.cuda.synchronize()
    # same tokens, same order of accumulation inside a tile; the split of the list over workgroups differs
    torch.testing.assert_close(r.outs[1].float(), want.float(), atol=2e-2, rtol=1e-2)


@pytest.mark.parametrize("mode", [1, 2])
@pytest.mark.parametrize("kw", [
    dict(n_q_heads=32, batch=3, seq_len=1500, lengths=(1500, 200, 1033)),
    dict(n_q_heads=64, batch=2, seq_len=2600, paged=True, lowrank=4, budget=512, window=128, topk_per_head=700),
    dict(n_q_heads=8, batch=2, seq_len=9000, min_seq_len=7000, budget=1024, window=0),
    dict(n_q_heads=16, batch=2, seq_len=700, budget=128, window=128),
], ids=["ragged", "correlated_paged_widek", "long_no_window", "window_only"])
def test_votes_and_max_score_rankings_match_the_oracle(mode, kw):
    """The other two readings of the global ranking (number of proposing heads; best proposing score)."""
    base = dict(n_kv_heads=8, n_planted=6)
    base.update(kw)
    w = small(f"rank{mode}", **base)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp, rank_mode=mode)
    _say(f"{w.name}: rank mode {mode}, decode step then stand-alone select, lens {inp.seq_lens_host}")
    r.run()
    check_select(inp, r, 0, rank_mode=mode)
    check_attention(inp, r, 1, LAYER_SPARSE)
    step_idx = r.idx.clone()
    r.idx.fill_(-1)
    r.select(0)
    torch.cuda.synchronize()
    assert torch.equal(r.idx, step_idx)


def test_quantised_scores_tie_in_every_ranking():
    """Few distinct score values: the rankings are decided by their tie rules (position, best rank)."""
    def quant(k):
        k.copy_(torch.sign(k) * (k.abs() > 0.8))   # keys in {-1, 0, 1}: scores collide heavily
    for mode in (1, 2):
        _with_keys(small(f"rankties{mode}", batch=2, seq_len=2000, budget=256, window=64), quant, rank_mode=mode)


@pytest.mark.parametrize("kw", [
    dict(n_q_heads=32, batch=3, seq_len=1500, lengths=(1500, 200, 1033)),
    dict(n_q_heads=64, batch=2, seq_len=6000, min_seq_len=5000, paged=True, budget=512, window=128),
], ids=["ragged", "g8_paged_long"])
def test_attention_recall_matches_the_oracle(kw):
    """Eq. 3 for the unified set and for per-head sets, from the kernels' softmax denominators."""
    base = dict(n_kv_heads=8, n_planted=6)
    base.update(kw)
    w = small("recall", **base)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.select(0)
    rec = r.recall(0)
    idx_head = r.make_idx_head()
    r.select_per_head(0, idx_head)
    rec_h = r.recall(0, idx_head)
    torch.cuda.synchronize()
    idx, cnt = r.idx.cpu().numpy(), r.cnt.cpu().numpy()
    ih = idx_head.cpu().numpy()
    g = w.n_q_heads // w.n_kv_heads
    for b in range(w.batch):
        q, K, _ = host_view(inp, 0, b)
        want = oracle.recall(q, K, idx[b, : cnt[b]])
        np.testing.assert_allclose(rec[b].cpu().numpy(), want, atol=1e-3, rtol=0)
        want_h = np.array([oracle.recall(q[h:h + 1], K[h // g:h // g + 1], ih[b, h, : cnt[b]])[0]
                           for h in range(w.n_q_heads)])
        np.testing.assert_allclose(rec_h[b].cpu().numpy(), want_h, atol=1e-3, rtol=0)
        if inp.seq_lens_host[b] <= w.budget:
            np.testing.assert_allclose(want, 1.0)                       # the set is every token
        else:
            assert (want_h >= want - 1e-12).all()                      # a head's own top-k is its best set of that size


@pytest.mark.parametrize("mode", [0, 1, 2])
@pytest.mark.parametrize("kw", [
    dict(n_q_heads=32, batch=3, seq_len=1500, lengths=(1500, 200, 1033), n_sink=4),
    dict(n_q_heads=64, batch=2, seq_len=2600, paged=True, lowrank=4, budget=512, window=128, n_sink=4),
    dict(n_q_heads=16, batch=2, seq_len=5000, min_seq_len=4000, budget=256, window=64, n_sink=40),
    dict(n_q_heads=16, batch=2, seq_len=700, budget=128, window=64, n_sink=64),
], ids=["ragged", "correlated_paged", "many_sinks", "sinks_fill_the_history"])
def test_attention_sinks_are_kept_and_not_ranked(mode, kw):
    """Sec. 4.1 reserves four sink tokens: positions below n_sink are always in rho and no candidates."""
    base = dict(n_kv_heads=8, n_planted=6)
    base.update(kw)
    w = small(f"sinks{mode}", **base)
    inp = wl.make_inputs(w, DEV)
    # make the sink keys attractive, so that leaving them out of the ranking matters
    inp.layers[0].k[:, :, : w.n_sink, :] = inp.layers[0].k[:, :, : w.n_sink, :] * 4
    r = StepRunner(inp, rank_mode=mode)
    _say(f"{w.name}: {w.n_sink} sinks, rank mode {mode}, lens {inp.seq_lens_host}")
    r.run()
    check_select(inp, r, 0, rank_mode=mode)
    check_attention(inp, r, 1, LAYER_SPARSE)
    torch.cuda.synchronize()
    for b, L in enumerate(inp.seq_lens_host):
        if L > w.budget:
            assert r.idx[b, : w.n_sink].tolist() == list(range(w.n_sink))


@pytest.mark.parametrize("paged", [False, True])
def test_decode_loop_growing_sequences_with_reselection(paged):
    """Consecutive decode steps: every sequence one token longer after each step, rho rebuilt by the
    selection layer and again by a re-selection layer (Sec. 4.1), four sink tokens.  One sequence
    crosses the budget (L = K: everything, L = K + 1: selection) on the way."""
    sched = (LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, LAYER_SELECT, LAYER_SPARSE)
    w = small("loop", n_layers=5, schedule=sched, batch=3, seq_len=1500, lengths=(1490, 700, 255), grow_room=4,
              paged=paged, n_sink=4, n_planted=5)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    for step in range(4):
        _say(f"loop step {step}: lens {inp.seq_lens_host}")
        r.idx.fill_(-1)
        r.run()
        check_select(inp, r, 3)                        # rho of the re-selection layer is the one left in idx
        check_attention(inp, r, 0, LAYER_FULL)
        check_attention(inp, r, 3, LAYER_SELECT)
        check_attention(inp, r, 4, LAYER_SPARSE)
        if step < 3:
            r.grow(1)
    assert inp.seq_lens_host == [1493, 703, 258] and inp.seq_lens.tolist() == inp.seq_lens_host


def test_decode_loop_first_selection_feeds_the_layers_before_the_reselection():
    """Layer 2 must attend the rho of layer 1's selection, not the re-selection's."""
    sched = (LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, LAYER_SELECT, LAYER_SPARSE)
    w = small("resel", n_layers=5, schedule=sched, batch=2, seq_len=1400, n_planted=5)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.run()
    torch.cuda.synchronize()
    out = bf16_bits(r.outs[2])
    for b in range(w.batch):
        q, K, _ = host_view(inp, 1, b)
        rho1 = oracle.select(q, K, w.budget, w.window, w.topk_per_head)
        q, K, V = host_view(inp, 2, b)
        assert_close_bf16(out[b], oracle.attention(q, K, V, rho1), f"layer 2 seq {b}")


@pytest.mark.parametrize("paged", [False, True])
def test_selection_layer_entry_point_equals_the_decode_step(paged):
    """cusa_select_layer + cusa_sparse_attn, called layer by layer, give what cusa_decode_step gives."""
    w = small("layercall", batch=3, seq_len=2300, lengths=(2300, 180, 1290), paged=paged, n_planted=4, n_sink=4)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.run()
    torch.cuda.synchronize()
    idx, cnt, outs = r.idx.clone(), r.cnt.clone(), [o.clone() for o in r.outs]
    r.idx.fill_(-1)
    for o in r.outs:
        o.zero_()
    r.select_layer(0)
    r.sparse(1)
    torch.cuda.synchronize()
    assert torch.equal(r.cnt, cnt)
    for b in range(w.batch):
        assert torch.equal(r.idx[b, : int(cnt[b])], idx[b, : int(cnt[b])])
    assert torch.equal(r.outs[0], outs[0]) and torch.equal(r.outs[1], outs[1])
    check_select(inp, r, 0)
    check_attention(inp, r, 0, LAYER_SELECT)


def test_strided_contiguous_cache_view():
    """K/V given as [B, L, G, d] storage viewed as [B, G, L, d] (token stride G*d)."""
    w = small("strided", batch=2, seq_len=900)
    inp = wl.make_inputs(w, DEV)
    for lay in inp.layers:
        lay.k = lay.k.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
        lay.v = lay.v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    r = StepRunner(inp)
    r.run()
    check_select(inp, r, 0)
    check_attention(inp, r, 1, LAYER_SPARSE)
    check_attention(inp, r, 0, LAYER_FULL)


def test_planted_heavy_keys_are_selected_on_gpu():
    w = small("planted", batch=2, seq_len=4096, budget=256, window=64, n_planted=16)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    r.run()
    torch.cuda.synchronize()
    idx = r.idx.cpu().numpy()
    planted = inp.layers[0].planted.numpy()
    for b in range(w.batch):
        assert set(planted[b]) <= set(idx[b])


@pytest.mark.parametrize("mode", [0, 1, 2])
def test_few_long_ragged_rows_are_ranked_in_slices(mode):
    """Few rows longer than 32768 candidates: the per-head top-k cuts a row into slices and merges their picks.
    One sequence is so much shorter that its last slice is empty; equal scores sit on both sides of a slice
    boundary; the votes / max-score rankings rank their one key row per sequence the same way."""
    w = small(f"slices{mode}", n_q_heads=8, n_kv_heads=8, batch=2, seq_len=90000, lengths=(90000, 41000),
              budget=512, window=128)

    def dup(k):
        k[:, :, 30000:36000] = k[:, :, 0:6000]           # 6000 scores again, across the first slice boundary
    _with_keys(w, dup, rank_mode=mode)


def _kernel_calls(fn):
    cb.profile_reset()
    cb.profile_enable(True)
    fn()
    torch.cuda.synchronize()
    prof = cb.profile_read()
    cb.profile_enable(False)
    return {k: v["calls"] for k, v in prof.items()}


def test_filtered_selection_layer_fast_path_and_its_second_chance():
    """A selection layer with many scores keeps only the candidates above a sampled threshold.  The result must
    not depend on the guess: random scores (the guess holds), massive ties (far more candidates than the lists
    hold), and a sequence whose large scores all sit where the sample does not look (fewer candidates than k)."""
    lens = (18000, 9000, 17011, 12345, 16000, 15999, 9777, 18000, 11000, 13579, 10001, 17500, 14000, 9100, 16384, 12800)
    w = small("filter", batch=16, seq_len=18000, lengths=lens, budget=2048, window=512, n_planted=9)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    assert r.filtered_select()
    calls = _kernel_calls(r.run)
    assert calls["sample_threshold_kernel"] == 1 and calls["topk_kernel<filtered>"] == 1
    assert r.second_chance_heads() == 0                  # random scores: every guess holds
    check_select(inp, r, 0, check_scores=False)
    for i, kind in enumerate(w.schedule):
        check_attention(inp, r, i, kind, seqs=[0, 7])
    # massive ties: most keys zero -> most scores exactly 0 and equal
    k = inp.layers[0].k
    saved = k.clone()
    k.copy_(torch.sign(k) * (k.abs() > 1.5))
    r.run()
    check_select(inp, r, 0, check_scores=False)
    # Where the sample does not look.  Sequence 3: every key OUTSIDE the sampled tiles is made to score high, so the
    # threshold (from ordinary scores) lets nearly everything through: more candidates than the buffers hold.
    # Sequence 5: only the keys INSIDE the sampled tiles score high, so the threshold is far too high and fewer
    # than k candidates pass.  Both heads' worth are found out and ranked again the ordinary way.
    k.copy_(saved)
    q = inp.layers[0].q
    for b, inside in ((3, False), (5, True)):
        Lb = inp.seq_lens_host[b]
        pos = torch.arange(Lb, device=k.device)
        sampled = (pos // 64) % 16 == 0                                               # the library samples every 16th tile of 64 tokens at this length
        chosen = sampled if inside else ~sampled
        boost = 4.0 * q[b].float().view(8, 4, 128).mean(dim=1)                        # [G, d], along the group's queries
        rows = k[b, :, :Lb][:, chosen].float() * 0.05 + boost[:, None, :]
        k[b, :, torch.nonzero(chosen).squeeze(1)] = rows.to(torch.bfloat16)
    r.run()
    assert r.second_chance_heads() >= w.n_q_heads        # the two sequences' heads were found out
    check_select(inp, r, 0, check_scores=False)
    check_attention(inp, r, 1, LAYER_SPARSE, seqs=[3, 5])


@pytest.mark.parametrize("H,paged,sinks,k", [(8, True, 4, 0), (16, False, 0, 0), (32, True, 40, 2048)])
def test_filtered_selection_layer_group_sizes_layouts_sinks(H, paged, sinks, k):
    """The fast path for query groups of 1, 2 and 4 heads, both cache layouts, with sinks, and with a per-head k
    above K - W; ragged lengths, one sequence within the budget."""
    B = 32 * 32 // H if H < 32 else 28
    rng = np.random.default_rng(H)
    lens = [int(x) for x in rng.integers(9000, 11000, size=B)]
    lens[1], lens[2] = 11000, 300
    w = small(f"filter_g{H // 8}", batch=B, n_q_heads=H, seq_len=11000, lengths=tuple(lens), budget=1024, window=256,
              paged=paged, n_sink=sinks, topk_per_head=k, n_planted=6)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    assert r.filtered_select()
    calls = _kernel_calls(r.run)
    assert calls["sample_threshold_kernel"] == 1 and calls["topk_kernel<filtered>"] == 1
    check_select(inp, r, 0, seqs=range(0, B, 3), check_scores=False)
    check_attention(inp, r, 0, LAYER_SELECT, seqs=[1, 2])
    check_attention(inp, r, 1, LAYER_SPARSE, seqs=[0, 2])


def test_filtered_selection_with_a_capacity_far_above_the_lengths():
    """The bound max_seq_len is a capacity (here 8 times the longest sequence): the sample of a sequence is
    taken at the density its own length allows, so the thresholds hold and no head needs the second chance."""
    lens = tuple(int(x) for x in np.random.default_rng(5).integers(9000, 12000, size=16))
    w = small("filter_cap", batch=16, seq_len=12000, lengths=lens, budget=1024, window=256, n_planted=5)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp, max_len=96000)
    assert r.filtered_select()
    r.run()
    check_select(inp, r, 0, seqs=range(0, 16, 3), check_scores=False)
    n_failed = r.second_chance_heads()
    assert n_failed == 0, f"{n_failed} heads took the second chance"


def test_many_rows_take_the_lean_streamed_topk():
    """512 rows of more than 8192 candidates: the per-head top-k runs its register-lean streamed form, two rows
    at a time per CU (ragged lengths, so that rows end inside a batch of keys)."""
    w = small("manyrows", batch=16, seq_len=9700, min_seq_len=8400, budget=512, window=128, n_planted=7)
    inp, r, sched = run_and_check(w)
    check_attention(inp, r, 1, LAYER_SPARSE, seqs=[0, 9])


def test_decode_step_with_different_length_bounds_per_layer():
    """Layers of one step may carry different host-side bounds max_seq_len (here 4096 / 4097 / 4096 around a
    place where the attention kernels' tiling changes); the workspace is sized once, for the largest."""
    w = small("bounds", n_layers=3, schedule=(LAYER_FULL, LAYER_SELECT, LAYER_SPARSE), batch=1, seq_len=4097,
              lengths=(4090,), budget=512, window=128)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    bounds = [4096, 4097, 4096]
    kvs = [cb.KvCache(l.k, l.v, inp.seq_lens, m, None) for l, m in zip(inp.layers, bounds)]
    ws = cb.alloc_workspace(r.params, max(bounds), DEV)
    assert cb.workspace_bytes(r.params, 4096) <= cb.workspace_bytes(r.params, 4097)
    cb.decode_step(r.params, list(w.schedule), [l.q for l in inp.layers], kvs, r.outs, r.idx, r.cnt, ws)
    torch.cuda.synchronize()
    r.ws, r.max_len = ws, max(bounds)                    # where check_select reads the intermediates from
    check_select(inp, r, 1)
    for i, kind in enumerate(w.schedule):
        check_attention(inp, r, i, kind)
    # and the other way round: a workspace sized for a capacity serves a shorter bound
    ws_big = cb.alloc_workspace(r.params, 65536, DEV)
    cb.full_attn(r.params, inp.layers[0].q, kvs[0], r.outs[0], ws_big)
    check_attention(inp, r, 0, LAYER_FULL)


# ------------------------------------------------------------------ the five workloads at full size

def test_c1_full_size():
    inp, r, sched = run_and_check(wl.WORKLOADS["c1"])
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)
    planted = inp.layers[0].planted.numpy()
    assert set(planted[0]) <= set(r.idx.cpu().numpy()[0])


def test_c2_full_size_whole_step_sampled_layers():
    w = wl.WORKLOADS["c2"]
    inp, r, sched = run_and_check(w)
    for i in (0, 2, 3, 17, 31):
        _say(f"c2: oracle attention for layer {i}")
        check_attention(inp, r, i, sched[i])


def test_c3_full_size_every_sequence_selected_layers():
    """c3 at full size: two full layers, the selection layer, the first and the LAST sparse layer (35).  The
    selection (scores, ranked lists, idx, cnt) is compared with the oracle for every sequence; attention on
    two sequences per layer."""
    w = wl.WORKLOADS["c3"]
    layers = [0, 2, 3, 35]
    inp, r, sched = run_and_check(w, layers)             # seqs=None: all eight sequences
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind, seqs=[0, 5])


def test_c4_full_size():
    inp, r, sched = run_and_check(wl.WORKLOADS["c4"])
    for i, kind in enumerate(sched):
        check_attention(inp, r, i, kind)


def test_c5_full_size_whole_step_every_sequence():
    """c5 at full size, the whole four-layer step as the bench runs it.  The selection is compared with the
    oracle for every one of the 64 sequences; attention on sampled sequences: the selection layer's own output
    and the first and last sparse layers."""
    w = wl.WORKLOADS["c5"]
    inp = wl.make_inputs(w, DEV)
    lens = inp.seq_lens_host
    seqs = sorted({int(np.argmin(lens)), int(np.argmax(lens)), 17})
    r = StepRunner(inp)
    _say(f"c5: whole step, {len(inp.layers)} layers; attention on sequences {seqs}")
    r.run()
    assert r.filtered_select()                           # the step's selection layer takes the filtered fast path here
    check_select(inp, r, 0, check_scores=False)          # every sequence
    _say("c5: selection equal to the oracle's for all sequences")
    check_attention(inp, r, 0, LAYER_FULL, seqs[:1])
    check_attention(inp, r, 1, LAYER_SPARSE, seqs)
    check_attention(inp, r, 3, LAYER_SPARSE, seqs)
    # properties that hold for every sequence, checked without the oracle
    torch.cuda.synchronize()
    idx, cnt = r.idx.cpu().numpy(), r.cnt.cpu().numpy()
    for b in range(w.batch):
        assert cnt[b] == w.budget
        row = idx[b]
        assert (np.diff(row) > 0).all() and row[0] >= 0
        assert (row[-w.window:] == np.arange(lens[b] - w.window, lens[b])).all()


def test_c2_full_size_per_head_variant():
    """Head-to-head sets and their sparse attention at c2's shape, in the launch configuration the bench times."""
    w = wl.WORKLOADS["c2"]
    inp = wl.make_inputs(w, DEV, layers=[2, 3])
    r = StepRunner(inp, [LAYER_SELECT, LAYER_SPARSE])
    idx_head = r.make_idx_head()
    r.select_per_head(0, idx_head)
    r.sparse_per_head(1, idx_head)
    torch.cuda.synchronize()
    q, K, _ = host_view(inp, 0, 0)
    rho_h = oracle.select_per_head(q, K, w.budget, w.window)
    assert int(r.cnt[0]) == w.budget and (idx_head[0].cpu().numpy() == rho_h).all()
    q, K, V = host_view(inp, 1, 0)
    assert_close_bf16(bf16_bits(r.outs[1])[0], oracle.attention_per_head(q, K, V, rho_h), "c2 per-head attention")


@pytest.mark.parametrize("mode", [1, 2])
def test_c3_full_size_other_rankings_sampled_sequences(mode):
    """Votes / max-score rankings on c3's correlated heads at full size (two of the eight sequences checked)."""
    w = wl.WORKLOADS["c3"]
    inp = wl.make_inputs(w, DEV, layers=[2, 3])
    r = StepRunner(inp, [LAYER_SELECT, LAYER_SPARSE], rank_mode=mode)
    r.run()
    check_select(inp, r, 0, seqs=[0, 5], rank_mode=mode)
    check_attention(inp, r, 1, LAYER_SPARSE, seqs=[5])


def test_loop_workload_full_size_two_steps():
    """The decode-loop workload's shape (re-selection layer, sinks), two consecutive steps on a layer subset."""
    w = wl.scaled(wl.WORKLOADS["loop"], n_layers=5,
                  schedule=(LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, LAYER_SELECT, LAYER_SPARSE))
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    for step in range(2):
        r.run()
        check_select(inp, r, 3)
        check_attention(inp, r, 4, LAYER_SPARSE)
        r.grow(1)


def test_longest_supported_selection():
    """The longest sequence the selection accepts (its bitmap over candidate positions fills the LDS it may
    use): 1 179 648 candidates plus the window, one sequence, eight heads."""
    W = 64
    L = 144 * 1024 * 8 + W
    w = small("longest", n_q_heads=8, n_kv_heads=8, batch=1, seq_len=L, budget=256, window=W, n_planted=8)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    _say(f"longest: L = {L}")
    r.run()
    check_select(inp, r, 0)
    check_attention(inp, r, 1, LAYER_SPARSE)
    # the per-head emission and the votes ranking use the same bitmap at the same size
    idx_head = r.make_idx_head()
    r.select_per_head(0, idx_head)
    torch.cuda.synchronize()
    q, K, _ = host_view(inp, 0, 0)
    assert (idx_head[0].cpu().numpy() == oracle.select_per_head(q, K, w.budget, w.window)).all()
    r1 = StepRunner(inp, rank_mode=1)
    r1.select(0)
    check_select(inp, r1, 0, rank_mode=1, check_scores=False)
    # one token more is refused on the host, before anything is launched
    kv = r.kvs[0]
    kv.max_seq_len += 1
    with pytest.raises(cb.CusaError) as e:
        cb.select(r.params, inp.layers[0].q, kv, r.idx, r.cnt, r.ws)
    assert e.value.status in (cb.ERR_UNSUPPORTED, cb.ERR_WORKSPACE_TOO_SMALL)


def test_random_small_configurations():
    """Forty seeded draws of the whole parameter space at small sizes: group size, batch, ragged lengths on
    both sides of the budget, budgets and windows that are multiples of nothing, k above K - W, sinks, the
    three rankings, both cache layouts."""
    rng = np.random.default_rng(20250807)
    for case in range(40):
        g = int(rng.choice([1, 2, 4, 8]))
        G = int(rng.choice([1, 2, 8]))
        B = int(rng.integers(1, 5))
        K = int(rng.integers(2, 700))
        W = int(rng.integers(0, K + 1))
        sinks = int(rng.integers(0, min(6, K - W) + 1))
        k = 0 if rng.random() < 0.5 else int(rng.integers(max(K - W - sinks, 1), K - W + 400))
        Lmax = int(rng.integers(K + 2, 3200))
        lengths = tuple(int(v) for v in rng.integers(1, Lmax + 1, size=B))
        lengths = (Lmax,) + lengths[1:]
        mode = int(rng.integers(0, 3))
        paged = bool(rng.random() < 0.5)
        w = small(f"rand{case}", n_q_heads=G * g, n_kv_heads=G, batch=B, seq_len=Lmax, lengths=lengths, budget=K,
                  window=W, topk_per_head=k, n_sink=sinks, paged=paged, n_planted=int(rng.integers(0, 4)),
                  lowrank=int(rng.choice([0, 4])), seed=1000 + case)
        _say(f"random case {case}: g={g} G={G} lens={lengths} K={K} W={W} k={k} sinks={sinks} mode={mode} paged={paged}")
        inp = wl.make_inputs(w, DEV)
        r = StepRunner(inp, rank_mode=mode)
        r.run()
        check_select(inp, r, 0, rank_mode=mode)
        check_attention(inp, r, 0, LAYER_SELECT)
        check_attention(inp, r, 1, LAYER_SPARSE)
        if case % 4 == 0:                              # the per-head variant and the recall diagnostic as well
            rec = r.recall(0)
            idx_head = r.make_idx_head()
            r.select_per_head(0, idx_head)
            r.sparse_per_head(1, idx_head)
            torch.cuda.synchronize()
            idx, cnt, ih = r.idx.cpu().numpy(), r.cnt.cpu().numpy(), idx_head.cpu().numpy()
            out = bf16_bits(r.outs[1])
            for b in range(B):
                q, Kc, _ = host_view(inp, 0, b)
                rho_h = oracle.select_per_head(q, Kc, K, W, sinks)
                assert (ih[b, :, : cnt[b]] == rho_h).all(), f"case {case}: per-head sets differ, seq {b}"
                np.testing.assert_allclose(rec[b].cpu().numpy(), oracle.recall(q, Kc, idx[b, : cnt[b]]), atol=1e-3, rtol=0)
                q, Kc, Vc = host_view(inp, 1, b)
                assert_close_bf16(out[b], oracle.attention_per_head(q, Kc, Vc, rho_h), f"case {case}: per-head attention seq {b}")


@pytest.mark.parametrize("filtered", [False, True])
def test_decode_step_captured_in_a_hip_graph_replays_like_the_eager_step(filtered):
    """The library only enqueues kernels (no allocation, no memset, no synchronisation), so a step can be
    captured once and replayed; every replay must give what the eager step gives -- whatever the workspace
    holds when it starts (it is scribbled over between the replays), also on the filtered selection, whose
    counters and flags live there."""
    if filtered:
        w = small("graphf", n_layers=3, schedule=(LAYER_SELECT, LAYER_SPARSE, LAYER_SPARSE), batch=20, seq_len=14000,
                  min_seq_len=12000, budget=1024, window=256, paged=True, n_planted=4, n_sink=4)
    else:
        w = small("graph", n_layers=4, schedule=(LAYER_FULL, LAYER_SELECT, LAYER_SPARSE, LAYER_SPARSE), batch=3,
                  seq_len=2600, lengths=(2600, 140, 1777), paged=True, n_planted=4, n_sink=4)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    assert r.filtered_select() == filtered
    r.run()                                            # eager: also warms the library (LDS attributes) before capture
    torch.cuda.synchronize()
    want_idx, want_outs = r.idx.clone(), [o.clone() for o in r.outs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        r.run()
    for replay in range(3):
        r.idx.fill_(-1)                                # eager work between the replays
        r.ws.fill_(0xA5 if replay % 2 else 0)
        for o in r.outs:
            o.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for b in range(w.batch):
            n = int(r.cnt[b])
            assert torch.equal(r.idx[b, :n], want_idx[b, :n]), f"replay {replay}: rho differs, seq {b}"
        for got, ref in zip(r.outs, want_outs):
            assert torch.equal(got, ref), f"replay {replay}: outputs differ"


def test_sparse_attention_clamps_indices_outside_the_sequence():
    """idx entries must lie in [0, L) (the caller's duty); the kernel still never reads outside the cache:
    it clamps, so the result is attention over the clamped list."""
    w = small("clamp", batch=2, seq_len=900, lengths=(900, 650), budget=64, window=16)
    inp = wl.make_inputs(w, DEV)
    r = StepRunner(inp)
    rng = np.random.default_rng(9)
    idx = np.stack([np.sort(rng.choice(L, size=64, replace=False)) for L in inp.seq_lens_host]).astype(np.int32)
    idx[0, :3] = (-7, -1, -2_000_000_000)
    idx[1, -2:] = (650, 2_000_000_000)
    r.idx.copy_(torch.from_numpy(idx))
    r.cnt.fill_(64)
    r.sparse(1)
    torch.cuda.synchronize()
    out = bf16_bits(r.outs[1])
    for b, L in enumerate(inp.seq_lens_host):
        q, K, V = host_view(inp, 1, b)
        assert_close_bf16(out[b], oracle.attention(q, K, V, np.clip(idx[b], 0, L - 1)), f"clamped list, seq {b}")
