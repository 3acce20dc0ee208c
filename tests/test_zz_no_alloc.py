"""The allocation-free sparse-attention entry point against cusa_sparse_attn (same kernels, the
split-K partials in the library's static device array instead of a caller workspace): two calls in
a row, the second on a smaller problem, so that whatever the first left in the array is there when
the second runs.  Also: the oracle bar on the outputs, and the size limit's error."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
from helpers import assert_close_bf16, host_view
from paper_2508_07101_amd import binding as cb
from paper_2508_07101_amd import workloads as wl
from paper_2508_07101_amd.runner import StepRunner
from paper_2508_07101_amd.workloads import LAYER_SELECT, LAYER_SPARSE, bf16_bits

pytestmark = pytest.mark.gpu


def _case(name, batch, seq_len, budget, window, seed, **kw):
    return wl.Workload(name=name, n_layers=2, batch=batch, n_q_heads=32, n_kv_heads=8, head_dim=128, seq_len=seq_len,
                       budget=budget, window=window, topk_per_head=0, schedule=(LAYER_SELECT, LAYER_SPARSE), seed=seed, **kw)


def _run_both(w):
    print(f"[no-alloc] {w.name}: batch {w.batch}, L {w.seq_len}, budget {w.budget}", flush=True)
    inp = wl.make_inputs(w, "cuda")
    r = StepRunner(inp)
    r.run()                                              # rho from the selection layer; layer 1 by cusa_sparse_attn
    torch.cuda.synchronize()
    want = bf16_bits(r.outs[1]).copy()
    got_t = torch.zeros_like(r.outs[1])
    cb.sparse_attn_noalloc(r.params, inp.layers[1].q, r.kvs[1], r.idx, r.cnt, got_t)
    torch.cuda.synchronize()
    got = bf16_bits(got_t)
    assert (got == want).all(), f"{w.name}: {(got != want).sum()} of {got.size} outputs differ from cusa_sparse_attn"
    idx, cnt = r.idx.cpu().numpy(), r.cnt.cpu().numpy()
    for b in range(w.batch):
        q, K, V = host_view(inp, 1, b)
        assert_close_bf16(got[b], oracle.attention(q, K, V, idx[b, : cnt[b]]), f"{w.name} seq {b}")


def test_two_calls_in_a_row_the_second_smaller():
    # several splits per head (partials go through the static array), ragged, then a smaller problem
    _run_both(_case("na_big", 3, 6000, 2048, 512, 4242, min_seq_len=2500))
    _run_both(_case("na_small", 2, 1500, 512, 128, 4243, lengths=(1500, 300)))
    # and a paged one on top of what the two left behind
    _run_both(_case("na_paged", 2, 3000, 1024, 256, 4244, paged=True, lengths=(3000, 1111)))


def test_problem_beyond_the_static_array_is_refused():
    lib = cb.load()
    cap = cb.noalloc_max_scratch_bytes()
    assert cap == 8 << 20
    # batch 1024 x 32 heads x at least one split x 520 B > 8 MiB
    p = cb.make_params(1024, 32, 8, 2048, 512)
    kv = cb.CusaKv(0x1000, 0x2000, cb.KV_CONTIGUOUS, 4096 * 128 * 8, 4096 * 128, 128, None, 0, 0, 0, 0x3000, 4096)
    fake = ctypes.c_void_p(0x10000)
    assert lib.cusa_sparse_attn_noalloc(ctypes.byref(p), fake, ctypes.byref(kv), fake, fake, fake, None) == cb.ERR_UNSUPPORTED
