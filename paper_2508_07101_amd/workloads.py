"""Seeded synthetic workloads with the shapes of the paper's efficiency runs.

This module only DRAWS inputs (q, K/V caches, lengths, block tables); it holds
none of the method's arithmetic, and both the CPU oracle's callers and the HIP
path's callers take their inputs from here.  The paper measures on real model
attention (Llama-3-8B / Qwen3-8B shaped GQA, d = 128, Sec. 4.3); those weights
are not available, so the five workloads below are i.i.d. bf16 stand-ins with
planted structure:

* c1  one layer, B1 H32 G8 L4096, K1024 W256 k1024, 16 planted heavy keys
* c2  32 layers (full, full, select, 29 x sparse), B1 L32768, K2048 W512,
      64 planted keys per layer
* c3  36 layers (full, full, select, 33 x sparse), B8 L16384, K4096 W1024,
      rank-8 component shared by all heads of a sequence
* c4  one layer, H64 G8 (g = 8), L131072, K4096 W1024, 256 planted keys
* c5  4 layers (select, 3 x sparse), B64, L ~ U[8192, 32768], 16-token pages
      behind a shuffled block table, K2048 W512

A planted key at position p of KV head kv is 3 * sum_{h in group kv} q_h / sqrt(g)
(bf16), which every head of the group scores far above the N(0,1) background.
Values smaller than 2^-30 in magnitude are flushed to zero so that no product
of two inputs is subnormal in binary32.
"""
from __future__ import annotations

from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional

import numpy as np
import torch

LAYER_FULL, LAYER_SELECT, LAYER_SPARSE = 0, 1, 2
BASE_SEED = 20250807


@dataclass(frozen=True)
class Workload:
    name: str
    n_layers: int
    batch: int
    n_q_heads: int
    n_kv_heads: int
    head_dim: int
    seq_len: int                 # fixed length, or the upper bound when ragged
    budget: int                  # K
    window: int                  # W
    topk_per_head: int           # k (0 -> K - W)
    schedule: tuple              # layer kinds, len n_layers
    min_seq_len: int = 0         # > 0: lengths uniform in [min_seq_len, seq_len]
    n_planted: int = 0           # planted heavy keys per layer and sequence
    lowrank: int = 0             # rank of the per-sequence shared component
    lowrank_scale: float = 0.5
    paged: bool = False
    page_size: int = 16
    seed: int = BASE_SEED
    same_layer_sparse: bool = False   # single-layer configs: sparse pass on the selection layer's KV
    lengths: tuple = ()               # explicit per-sequence lengths (tests); overrides the draw
    n_sink: int = 0                   # first positions always kept in rho (attention sinks, Sec. 4.1)
    grow_room: int = 0                # cache capacity beyond the drawn lengths (decode loops: L grows by one per step)

    @property
    def k_eff(self) -> int:
        return self.topk_per_head if self.topk_per_head > 0 else self.budget - self.window


def _sched(n_full: int, n_sparse: int) -> tuple:
    return (LAYER_FULL,) * n_full + (LAYER_SELECT,) + (LAYER_SPARSE,) * n_sparse


WORKLOADS: Dict[str, Workload] = {
    "c1": Workload("c1", 2, 1, 32, 8, 128, 4096, 1024, 256, 1024, _sched(0, 1),
                   n_planted=16, seed=BASE_SEED + 1, same_layer_sparse=True),
    "c2": Workload("c2", 32, 1, 32, 8, 128, 32768, 2048, 512, 0, _sched(2, 29),
                   n_planted=64, seed=BASE_SEED + 2),
    "c3": Workload("c3", 36, 8, 32, 8, 128, 16384, 4096, 1024, 0, _sched(2, 33),
                   lowrank=8, seed=BASE_SEED + 3),
    "c4": Workload("c4", 2, 1, 64, 8, 128, 131072, 4096, 1024, 0, _sched(0, 1),
                   n_planted=256, seed=BASE_SEED + 4, same_layer_sparse=True),
    "c5": Workload("c5", 4, 64, 32, 8, 128, 32768, 2048, 512, 0, _sched(0, 3),
                   min_seq_len=8192, paged=True, seed=BASE_SEED + 5),
    # Steady-state decode loop (not one of the quoted configurations): the c2 model shape with the
    # paper's experimental settings of Sec. 4.1 -- two full layers, a selection layer, a re-selection
    # layer at layer 12, four sink tokens -- and room for the sequence to grow by one token per step.
    "loop": Workload("loop", 36, 1, 32, 8, 128, 32768, 2048, 512, 0,
                     _sched(2, 9) + (LAYER_SELECT,) + (LAYER_SPARSE,) * 23,
                     n_planted=64, seed=BASE_SEED + 6, n_sink=4, lengths=(32768 - 256,), grow_room=256),
}


def scaled(w: Workload, **kw) -> Workload:
    """A smaller (or otherwise altered) copy of a workload for parity tests."""
    return replace(w, **kw)


@dataclass
class Layer:
    """One layer's inputs.  bf16 torch tensors on ``device``.

    contiguous: k, v are [B, G, Lmax, d].   paged: k, v are pools
    [n_pages, G, page_size, d] addressed through ``Inputs.block_table``.
    """
    q: torch.Tensor
    k: torch.Tensor
    v: torch.Tensor
    planted: Optional[torch.Tensor] = None   # [B, n_planted] int64 positions (selection tests)


@dataclass
class Inputs:
    workload: Workload
    seq_lens: torch.Tensor                   # [B] int32 on device
    seq_lens_host: List[int]
    layers: List[Layer] = field(default_factory=list)
    block_table: Optional[torch.Tensor] = None   # [B, max_pages] int32 on device
    n_pages: int = 0


def _gen(device, seed: int) -> torch.Generator:
    g = torch.Generator(device=device)
    g.manual_seed(seed)
    return g


def _normal_bf16(shape, gen, device, add: Optional[torch.Tensor] = None) -> torch.Tensor:
    x = torch.randn(shape, generator=gen, device=device, dtype=torch.float32)
    if add is not None:
        x += add
    x = torch.where(x.abs() < 2.0 ** -30, torch.zeros_like(x), x)
    return x.to(torch.bfloat16)


def draw_lengths(w: Workload) -> List[int]:
    if w.lengths:
        assert len(w.lengths) == w.batch and max(w.lengths) <= w.seq_len
        return [int(v) for v in w.lengths]
    if w.min_seq_len <= 0:
        return [w.seq_len] * w.batch
    rng = np.random.default_rng(w.seed)
    return [int(v) for v in rng.integers(w.min_seq_len, w.seq_len + 1, size=w.batch)]


def make_layer(w: Workload, layer: int, seq_lens_host: List[int], device,
               n_pages: int = 0) -> Layer:
    """Draw q, K, V of one layer (its own seeded stream, independent of other layers)."""
    gen = _gen(device, w.seed * 1000 + layer)
    B, H, G, d = w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim
    g = H // G
    q_add = k_add = v_add = None
    if w.lowrank > 0:
        r = w.lowrank
        M = torch.randn((B, r, d), generator=gen, device=device)
        c = torch.randn((B, 1, r), generator=gen, device=device)
        q_add = (w.lowrank_scale / r ** 0.5) * torch.bmm(c, M)             # [B,1,d] -> all heads
        a = torch.randn((B, w.seq_len, r), generator=gen, device=device)
        k_add = (w.lowrank_scale * torch.bmm(a, M)).unsqueeze(1)             # [B,1,L,d] -> all KV heads
        a2 = torch.randn((B, w.seq_len, r), generator=gen, device=device)
        v_add = (w.lowrank_scale * torch.bmm(a2, M)).unsqueeze(1)
    q = _normal_bf16((B, H, d), gen, device, q_add)
    if w.paged:
        shape = (n_pages, G, w.page_size, d)
        return Layer(q, _normal_bf16(shape, gen, device), _normal_bf16(shape, gen, device))
    k = _normal_bf16((B, G, w.seq_len, d), gen, device, k_add)
    v = _normal_bf16((B, G, w.seq_len, d), gen, device, v_add)
    planted = None
    if w.n_planted > 0:
        heavy = (3.0 / g ** 0.5) * q.float().view(B, G, g, d).sum(dim=2)     # [B,G,d]
        heavy = heavy.to(torch.bfloat16)
        rng = np.random.default_rng(w.seed * 1000 + layer)
        rows = []
        for b in range(B):
            hi = max(seq_lens_host[b] - w.window, 1)
            n = min(w.n_planted, hi)
            rows.append(np.sort(rng.choice(hi, size=n, replace=False)))
            pos = torch.as_tensor(rows[-1], device=device, dtype=torch.long)
            k[b, :, pos, :] = heavy[b].unsqueeze(1)
        if all(len(r_) == len(rows[0]) for r_ in rows):
            planted = torch.as_tensor(np.stack(rows), dtype=torch.long)
    return Layer(q, k, v, planted)


def make_inputs(w: Workload, device="cpu", layers: Optional[List[int]] = None) -> Inputs:
    """Draw the whole workload (or only the listed layer numbers) on ``device``."""
    lens = draw_lengths(w)
    assert max(lens) + w.grow_room <= w.seq_len, "the drawn caches hold seq_len tokens"
    inp = Inputs(w, torch.tensor(lens, dtype=torch.int32, device=device), lens)
    if w.paged:
        pages = [(n + w.grow_room + w.page_size - 1) // w.page_size for n in lens]
        inp.n_pages = int(sum(pages))
        perm = torch.randperm(inp.n_pages, generator=_gen("cpu", w.seed)).to(torch.int32)
        table = torch.zeros((w.batch, max(pages)), dtype=torch.int32)
        off = 0
        for b, n in enumerate(pages):
            table[b, :n] = perm[off:off + n]
            off += n
        inp.block_table = table.to(device)
    for layer in (range(w.n_layers) if layers is None else layers):
        if w.same_layer_sparse and layer > 0:
            inp.layers.append(inp.layers[0])
            continue
        inp.layers.append(make_layer(w, layer, lens, device, inp.n_pages))
    return inp


def bf16_bits(t: torch.Tensor) -> np.ndarray:
    """Host uint16 bit patterns of a bf16 tensor (what the oracle consumes)."""
    return t.detach().contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def bits_to_bf16(a: np.ndarray, device="cpu") -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a).view(np.int16)).view(torch.bfloat16).to(device)
