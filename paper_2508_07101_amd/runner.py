"""Glue between a drawn workload and the C-ABI calls: allocates outputs, index
buffers and workspace with torch and marshals the per-layer descriptors.  No
arithmetic of the method happens here."""
from __future__ import annotations

from typing import List, Optional

import torch

from . import binding as cb
from .workloads import Inputs


def params_of(inp: Inputs, rank_mode: int = cb.RANK_FIRST_OCCURRENCE) -> cb.CusaParams:
    w = inp.workload
    return cb.make_params(w.batch, w.n_q_heads, w.n_kv_heads, w.budget, w.window, w.topk_per_head,
                          head_dim=w.head_dim, rank_mode=rank_mode, n_sink=w.n_sink)


def kv_of(inp: Inputs, layer_pos: int, max_len: Optional[int] = None) -> cb.KvCache:
    lay = inp.layers[layer_pos]
    bound = max(inp.seq_lens_host) + inp.workload.grow_room if max_len is None else max_len
    return cb.KvCache(lay.k, lay.v, inp.seq_lens, bound, inp.block_table)


class StepRunner:
    """One decode step (attention part of Alg. 1) over ``inp.layers`` with ``schedule``."""

    def __init__(self, inp: Inputs, schedule: Optional[List[int]] = None, rank_mode: int = cb.RANK_FIRST_OCCURRENCE,
                 max_len: Optional[int] = None):
        w = inp.workload
        self.inp = inp
        self.schedule = list(w.schedule if schedule is None else schedule)
        assert len(self.schedule) == len(inp.layers)
        dev = inp.seq_lens.device
        self.params = params_of(inp, rank_mode)
        # capacity: the lengths may grow up to it (max_len: a bound above what the caches hold, which no kernel reads up to)
        self.max_len = max(inp.seq_lens_host) + w.grow_room if max_len is None else max_len
        assert self.max_len >= max(inp.seq_lens_host)
        self.kvs = [kv_of(inp, i, self.max_len) for i in range(len(inp.layers))]
        self.outs = [torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.bfloat16, device=dev)
                     for _ in inp.layers]
        self.idx = torch.full((w.batch, w.budget), -1, dtype=torch.int32, device=dev)
        self.cnt = torch.zeros((w.batch,), dtype=torch.int32, device=dev)
        self.ws = cb.alloc_workspace(self.params, self.max_len, dev)
        self.scores_valid = False     # whether the workspace holds the selection scores of the last call
        self.step = cb.DecodeStep(self.params, self.schedule, [l.q for l in inp.layers], self.kvs, self.outs,
                                  self.idx, self.cnt, self.ws)

    def run(self):
        self.step.run()
        # a selection layer on the filtered fast path writes no score array
        self.scores_valid = not self.filtered_select()

    def grow(self, n: int = 1):
        """Every sequence gets n more tokens (already present in the drawn caches), as after n decode steps."""
        assert max(self.inp.seq_lens_host) + n <= self.max_len, "no room left in the caches"
        self.inp.seq_lens.add_(n)
        self.inp.seq_lens_host[:] = [v + n for v in self.inp.seq_lens_host]

    # single entry points on one layer (by position in inp.layers)
    def select(self, layer_pos: int):
        cb.select(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], self.idx, self.cnt, self.ws)
        self.scores_valid = True

    def select_layer(self, layer_pos: int):
        cb.select_layer(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], self.outs[layer_pos], self.idx,
                        self.cnt, self.ws)
        self.scores_valid = not self.filtered_select()

    def sparse(self, layer_pos: int):
        cb.sparse_attn(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], self.idx, self.cnt,
                       self.outs[layer_pos], self.ws)

    # head-to-head variant: every head its own token set, idx_head [B, H, budget]
    def make_idx_head(self) -> torch.Tensor:
        w = self.inp.workload
        return torch.full((w.batch, w.n_q_heads, w.budget), -1, dtype=torch.int32, device=self.idx.device)

    def select_per_head(self, layer_pos: int, idx_head: torch.Tensor):
        cb.select_per_head(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], idx_head, self.cnt, self.ws)

    def sparse_per_head(self, layer_pos: int, idx_head: torch.Tensor):
        cb.sparse_attn_per_head(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], idx_head, self.cnt,
                                self.outs[layer_pos], self.ws)

    def recall(self, layer_pos: int, idx: Optional[torch.Tensor] = None) -> torch.Tensor:
        """Eq. 3 on this layer's q and K for the current rho (idx None) or for per-head sets idx [B, H, budget]."""
        w = self.inp.workload
        out = torch.empty((w.batch, w.n_q_heads), dtype=torch.float32, device=self.idx.device)
        cb.attention_recall(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos],
                            self.idx if idx is None else idx, self.cnt, out, self.ws, per_head=idx is not None)
        return out

    def full(self, layer_pos: int):
        cb.full_attn(self.params, self.inp.layers[layer_pos].q, self.kvs[layer_pos], self.outs[layer_pos], self.ws)

    def second_chance_heads(self) -> int:
        """Heads of the last filtered selection layer whose threshold failed (they were scored and ranked again)."""
        lay = cb.workspace_layout(self.params, self.max_len)
        assert lay.filtered_select
        return int(self.ws[lay.second_chance_offset: lay.second_chance_offset + 4].view(torch.int32).item())

    def filtered_select(self) -> bool:
        """Whether a selection layer of this size keeps candidates instead of writing the score array."""
        return bool(cb.workspace_layout(self.params, self.max_len).filtered_select)

    # selection intermediates, for parity tests
    def scores(self) -> torch.Tensor:
        lay = cb.workspace_layout(self.params, self.max_len)
        w = self.inp.workload
        n = w.batch * w.n_q_heads * lay.ld_scores
        flat = self.ws[lay.scores_offset: lay.scores_offset + 4 * n].view(torch.float32)
        return flat.view(w.batch, w.n_q_heads, lay.ld_scores)

    def rho_head(self) -> torch.Tensor:
        """[B, k, H] rank-major ranked picks."""
        lay = cb.workspace_layout(self.params, self.max_len)
        w = self.inp.workload
        n = w.batch * lay.k * w.n_q_heads
        flat = self.ws[lay.rho_head_offset: lay.rho_head_offset + 4 * n].view(torch.int32)
        return flat.view(w.batch, lay.k, w.n_q_heads)
