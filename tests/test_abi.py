"""The C-ABI library loads, exports every symbol cusa.h declares, and rejects bad
arguments on the host (no kernel is launched by anything in this file)."""
import ctypes
import os
import re

import pytest

from paper_2508_07101_amd import binding as cb

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "cusa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cusa_[a-z_0-9]+)\s*\(", text)))


def test_header_symbols_are_exported():
    lib = cb.load()
    names = _declared_symbols()
    assert set(names) == set(cb.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror_covers_every_status():
    seen = {cb.strerror(s) for s in range(5)}
    assert len(seen) == 5 and "unknown status" not in seen
    assert cb.strerror(99) == "unknown status"


def test_workspace_bytes_grows_with_the_problem():
    p = cb.make_params(1, 32, 8, 2048, 512)
    a = cb.workspace_bytes(p, 32768)
    b = cb.workspace_bytes(p, 65536)
    assert 0 < a < b and a % 256 == 0
    lay = cb.workspace_layout(p, 32768)
    assert lay.k == 1536 and lay.ld_scores >= 32768 - 512 and lay.total_bytes == a
    assert lay.scores_offset % 256 == 0 and lay.rho_head_offset % 256 == 0


@pytest.mark.parametrize("kw,status", [
    (dict(n_q_heads=30), cb.ERR_INVALID_ARG),              # H % G != 0
    (dict(head_dim=64), cb.ERR_UNSUPPORTED),
    (dict(n_q_heads=48, n_kv_heads=8), cb.ERR_UNSUPPORTED),  # g = 6
    (dict(window=4096), cb.ERR_INVALID_ARG),               # W > K
    (dict(topk_per_head=100), cb.ERR_INVALID_ARG),         # k < K - W
    (dict(topk_per_head=10000), cb.ERR_UNSUPPORTED),
    (dict(n_sink=-1), cb.ERR_INVALID_ARG),
    (dict(n_sink=1537), cb.ERR_INVALID_ARG),               # more sinks than K - W
    (dict(rank_mode=7), cb.ERR_INVALID_ARG),
    (dict(sm_scale=0.0), cb.ERR_INVALID_ARG),
    (dict(batch=0), cb.ERR_INVALID_ARG),
])
def test_bad_params_are_rejected(kw, status):
    base = dict(batch=1, n_q_heads=32, n_kv_heads=8, budget=2048, window=512)
    base.update(kw)
    p = cb.make_params(**base)
    n = ctypes.c_size_t(0)
    assert cb.load().cusa_workspace_bytes(ctypes.byref(p), 4096, ctypes.byref(n)) == status


def test_null_and_misshapen_arguments_are_rejected_before_any_launch():
    lib = cb.load()
    p = cb.make_params(1, 32, 8, 2048, 512)
    kv = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 128, None, 0, 0, 0, 0x3000, 4096)
    fake = ctypes.c_void_p(0x10000)
    # NULL q
    assert lib.cusa_full_attn(ctypes.byref(p), None, ctypes.byref(kv), fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    # workspace too small / NULL / misaligned
    assert lib.cusa_full_attn(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    assert lib.cusa_full_attn(ctypes.byref(p), fake, ctypes.byref(kv), fake, None, 1 << 30, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_full_attn(ctypes.byref(p), fake, ctypes.byref(kv), fake, ctypes.c_void_p(0x10010), 1 << 30, None) == cb.ERR_INVALID_ARG
    # token stride below the row length
    bad = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 64, None, 0, 0, 0, 0x3000, 4096)
    assert lib.cusa_select(ctypes.byref(p), fake, ctypes.byref(bad), fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    # paged: wrong page size, missing table, table too short for max_seq_len
    pg = cb.CusaKv(0x1000, 0x2000, cb.KV_PAGED, 0, 0, 0, 0x4000, 256, 32, 100, 0x3000, 4096)
    assert lib.cusa_select(ctypes.byref(p), fake, ctypes.byref(pg), fake, fake, fake, 1 << 30, None) == cb.ERR_UNSUPPORTED
    pg = cb.CusaKv(0x1000, 0x2000, cb.KV_PAGED, 0, 0, 0, None, 256, 16, 100, 0x3000, 4096)
    assert lib.cusa_select(ctypes.byref(p), fake, ctypes.byref(pg), fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    pg = cb.CusaKv(0x1000, 0x2000, cb.KV_PAGED, 0, 0, 0, 0x4000, 10, 16, 100, 0x3000, 4096)
    assert lib.cusa_select(ctypes.byref(p), fake, ctypes.byref(pg), fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    # selection on sequences longer than the union kernel's on-chip bitmap covers
    lng = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 2_000_000 * 128, 128, None, 0, 0, 0, 0x3000, 2_000_000)
    assert lib.cusa_select(ctypes.byref(p), fake, ctypes.byref(lng), fake, fake, fake, 1 << 40, None) == cb.ERR_UNSUPPORTED
    # unknown layout, missing seq_lens
    bad = cb.CusaKv(0x1000, 0x2000, 5, 0, 4096 * 128, 128, None, 0, 0, 0, 0x3000, 4096)
    assert lib.cusa_sparse_attn(ctypes.byref(p), fake, ctypes.byref(bad), fake, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    bad = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 128, None, 0, 0, 0, None, 4096)
    assert lib.cusa_sparse_attn(ctypes.byref(p), fake, ctypes.byref(bad), fake, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG


def test_per_head_entry_points_reject_bad_arguments_before_any_launch():
    lib = cb.load()
    p = cb.make_params(1, 32, 8, 2048, 512)
    kv = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 128, None, 0, 0, 0, 0x3000, 4096)
    fake = ctypes.c_void_p(0x10000)
    assert lib.cusa_select_per_head(ctypes.byref(p), fake, ctypes.byref(kv), None, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_select_per_head(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    lng = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 2_000_000 * 128, 128, None, 0, 0, 0, 0x3000, 2_000_000)
    assert lib.cusa_select_per_head(ctypes.byref(p), fake, ctypes.byref(lng), fake, fake, fake, 1 << 40, None) == cb.ERR_UNSUPPORTED
    assert lib.cusa_sparse_attn_per_head(ctypes.byref(p), fake, ctypes.byref(kv), fake, None, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_sparse_attn_per_head(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    assert lib.cusa_select_layer(ctypes.byref(p), fake, ctypes.byref(kv), None, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_select_layer(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    assert lib.cusa_select_layer(ctypes.byref(p), fake, ctypes.byref(lng), fake, fake, fake, fake, 1 << 40, None) == cb.ERR_UNSUPPORTED
    assert lib.cusa_attention_recall(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, 0, None, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_attention_recall(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, 1, fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    bad = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 64, None, 0, 0, 0, 0x3000, 4096)
    assert lib.cusa_sparse_attn_per_head(ctypes.byref(p), fake, ctypes.byref(bad), fake, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG


def test_decode_step_rejects_sparse_before_select_and_unknown_kinds():
    lib = cb.load()
    p = cb.make_params(1, 32, 8, 2048, 512)
    n = 2
    kvs = (cb.CusaKv * n)(*[cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 0, 4096 * 128, 128, None, 0, 0, 0, 0x3000, 4096)] * n)
    ptrs = (ctypes.c_void_p * n)(0x10000, 0x20000)
    fake = ctypes.c_void_p(0x10000)
    for kinds in ([cb.LAYER_SPARSE, cb.LAYER_SELECT], [cb.LAYER_FULL, cb.LAYER_SPARSE], [cb.LAYER_FULL, 9]):
        arr = (ctypes.c_int32 * n)(*kinds)
        assert lib.cusa_decode_step(ctypes.byref(p), n, arr, ptrs, kvs, ptrs, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG
    arr = (ctypes.c_int32 * n)(cb.LAYER_SELECT, cb.LAYER_SPARSE)
    assert lib.cusa_decode_step(ctypes.byref(p), n, arr, ptrs, kvs, ptrs, fake, fake, fake, 16, None) == cb.ERR_WORKSPACE_TOO_SMALL
    assert lib.cusa_decode_step(ctypes.byref(p), 0, arr, ptrs, kvs, ptrs, fake, fake, fake, 1 << 30, None) == cb.ERR_INVALID_ARG


@pytest.mark.parametrize("B,H,G,K,W", [(1, 32, 8, 2048, 512), (1, 64, 8, 4096, 1024), (8, 32, 8, 4096, 1024),
                                        (3, 16, 8, 256, 64), (64, 32, 8, 2048, 512)])
def test_workspace_bytes_never_shrink_with_capacity(B, H, G, K, W):
    """A workspace sized for a capacity must serve every shorter bound: bytes(m) <= bytes(M) for m <= M
    (checked densely around the places where the attention kernels' tiling changes)."""
    p = cb.make_params(B, H, G, K, W)
    lens = sorted(set([1, 2, 63, 64, 65, 255, 256, 257, 1000] +
                      [c + d for c in range(1024, 40000, 1024) for d in (-1, 0, 1)] +
                      [c + d for c in (65536, 131072, 262144) for d in (-1, 0, 1)]))
    prev = 0
    for m in lens:
        n = cb.workspace_bytes(p, m)
        assert n >= prev, f"workspace shrinks from {prev} to {n} at max_seq_len {m}"
        prev = n


def test_layout_reports_the_filtered_fast_path():
    """The layout says whether a selection layer of this size keeps only the scores that can matter: many scores,
    groups of at most four heads, the default ranking, a sample dense enough for the longest sequence."""
    c5 = dict(batch=64, n_q_heads=32, n_kv_heads=8, budget=2048, window=512)
    assert cb.workspace_layout(cb.make_params(**c5), 32768).filtered_select == 1
    assert cb.workspace_layout(cb.make_params(**c5), 8192).filtered_select == 1
    assert cb.workspace_layout(cb.make_params(**c5), 4096).filtered_select == 0          # few scores, k a large share
    assert cb.workspace_layout(cb.make_params(**dict(c5, batch=1)), 32768).filtered_select == 0
    assert cb.workspace_layout(cb.make_params(**dict(c5, n_q_heads=64)), 32768).filtered_select == 0   # groups of 8
    assert cb.workspace_layout(cb.make_params(**dict(c5, rank_mode=cb.RANK_VOTES)), 32768).filtered_select == 0
    # a bound so long that the 64 sampled tiles are too thin a sample for k = 1536: the ordinary way, same buffers
    far = cb.workspace_layout(cb.make_params(**c5), 1 << 20)
    assert far.filtered_select == 0 and far.total_bytes >= cb.workspace_bytes(cb.make_params(**c5), 32768)


def test_build_id_matches_the_sources():
    from paper_2508_07101_amd import build
    assert cb.load().cusa_build_id().decode() == build.source_id() == cb.built_from()


def test_probe_rejects_bad_arguments():
    lib = cb.load()
    fake = ctypes.c_void_p(0x10000)
    assert lib.cusa_probe_stream_read(None, 1 << 20, fake, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_probe_stream_read(fake, 8, fake, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_probe_stream_read(ctypes.c_void_p(0x10008), 1 << 20, fake, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_probe_stream_read(fake, 1 << 20, None, None) == cb.ERR_INVALID_ARG


def test_traffic_probe_rejects_bad_arguments():
    lib = cb.load()
    fake = ctypes.c_void_p(0x10000)
    assert lib.cusa_probe_traffic(-1, fake, 1 << 22, fake, 1 << 20, None) == cb.ERR_INVALID_ARG     # no such pattern
    assert lib.cusa_probe_traffic(4, fake, 1 << 22, fake, 1 << 20, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_probe_traffic(2, None, 1 << 22, fake, 1 << 20, None) == cb.ERR_INVALID_ARG
    assert lib.cusa_probe_traffic(2, fake, 1 << 19, fake, 1 << 20, None) == cb.ERR_INVALID_ARG      # under one chunk
    assert lib.cusa_probe_traffic(1, fake, 1 << 21, fake, 1 << 20, None) == cb.ERR_INVALID_ARG      # gather needs 4 MiB
    assert lib.cusa_probe_traffic(3, fake, 1 << 25, fake, 1 << 19, None) == cb.ERR_INVALID_ARG      # results do not fit
