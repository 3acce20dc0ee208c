"""Algorithmic bytes and flops of the hot path (what the method itself must move).

These are the numerators of the achieved-bandwidth figures.  They reproduce the
paper's kernel-metrics table (budget 2K, context 16K, d = 128, 2-byte elements):
global-to-shared traffic is counted per KV head, flops per query head.
"""
from __future__ import annotations

from typing import Iterable, Sequence

ELT = 2  # bytes per bf16 element
LAYER_FULL, LAYER_SELECT, LAYER_SPARSE = 0, 1, 2


def attn_bytes_per_kv_head(n_tokens: int, d: int = 128) -> int:
    """K and V rows of n_tokens tokens, read once."""
    return 2 * n_tokens * d * ELT


def attn_flops_per_q_head(n_tokens: int, d: int = 128) -> int:
    """q.K^T and P.V, one multiply and one add per element each."""
    return 4 * n_tokens * d


def full_attn_bytes(G: int, L: int, d: int = 128) -> int:
    return G * attn_bytes_per_kv_head(L, d)


def sparse_attn_bytes(G: int, budget: int, L: int, d: int = 128) -> int:
    n = min(budget, L)
    return G * attn_bytes_per_kv_head(n, d) + 4 * n


def per_head_sparse_attn_bytes(H: int, budget: int, L: int, d: int = 128) -> int:
    """Head-to-head variant: every query head reads the K and V rows of its own list."""
    n = min(budget, L)
    return H * (attn_bytes_per_kv_head(n, d) + 4 * n)


def score_bytes(G: int, L: int, budget: int, window: int, d: int = 128) -> int:
    """K rows of the candidate range [0, L-W), read once; nothing when the budget covers L."""
    if L <= budget:
        return 0
    return G * (L - window) * d * ELT


def step_bytes(schedule: Sequence[int], seq_lens: Iterable[int], G: int, budget: int,
               window: int, d: int = 128, fused_select: bool = True) -> dict:
    """Per-kind and total algorithmic bytes of one decode step over all sequences.

    fused_select: the selection layer scores its tokens in the same pass that computes its output
    (as the decode step does), so its K rows count once; False counts the separate scoring pass of
    a stand-alone selection call as well."""
    out = {"full": 0, "score": 0, "sparse": 0}
    lens = list(seq_lens)
    for kind in schedule:
        for L in lens:
            if kind in (LAYER_FULL, LAYER_SELECT):
                out["full"] += full_attn_bytes(G, L, d)
            if kind == LAYER_SELECT and not fused_select:
                out["score"] += score_bytes(G, L, budget, window, d)
            if kind == LAYER_SPARSE:
                out["sparse"] += sparse_attn_bytes(G, budget, L, d)
    out["total"] = out["full"] + out["score"] + out["sparse"]
    return out
