"""CPU oracle for the CUSA decode hot path -- TEST INFRASTRUCTURE ONLY.

A ctypes front-end to ``cusa_oracle.c`` plus the walk over layers of Alg. 1
(attention part).  Only ``tests/``, ``__graft_entry__.smoke()`` and the
``cpu_baseline`` leg of ``bench.py`` may import this package; the product path
never does, and nothing here imports the product package.

Arrays are numpy; bf16 tensors are ``uint16`` bit patterns.  One call handles
one sequence given as its logical view ``q[H,d]``, ``K[G,L,d]``, ``V[G,L,d]``.

Parity status: every function (the head-to-head variant included) is pinned by CPU tests except the CHOICE of the
global-ranking reading (``rank_mode``), which is "parity unpinned" -- the paper
defines no ranking key and prints no worked example.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "cusa_oracle.c")
_LIB = os.path.join(_HERE, "libcusa_oracle.so")

LAYER_FULL, LAYER_SELECT, LAYER_SPARSE = 0, 1, 2
RANK_FIRST_OCCURRENCE, RANK_VOTES, RANK_MAX_SCORE = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no contraction) and return the path."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(
            ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-fopenmp", "-fno-fast-math",
             "-ffp-contract=off", "-Wall", "-Wextra", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        c_i, c_i64, c_d, vp = ctypes.c_int, ctypes.c_int64, ctypes.c_double, ctypes.c_void_p
        lib.cusa_oracle_num_threads.restype = c_i
        lib.cusa_oracle_resolve_paged.argtypes = [vp, vp, c_i, c_i, c_i, c_i, vp]
        lib.cusa_oracle_scores.argtypes = [vp, vp, c_i, c_i, c_i, c_i, c_i, vp, c_i64]
        lib.cusa_oracle_topk.argtypes = [vp, c_i64, c_i, c_i, c_i, vp]
        lib.cusa_oracle_unify.argtypes = [vp, vp, c_i64, c_i, c_i, c_i, c_i, c_i, c_i, vp]
        lib.cusa_oracle_unify.restype = c_i
        lib.cusa_oracle_attention.argtypes = [vp, vp, vp, c_i, c_i, c_i, c_i, vp, c_i, c_d, vp, vp]
        lib.cusa_oracle_recall.argtypes = [vp, vp, c_i, c_i, c_i, c_i, vp, c_i, c_d, vp]
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().cusa_oracle_num_threads())


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def bf16_bits_to_f32(a: np.ndarray) -> np.ndarray:
    """Exact widening of bf16 bit patterns to float32."""
    return (np.asarray(a, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def resolve_paged(pool: np.ndarray, block_table_row: np.ndarray, L: int) -> np.ndarray:
    """Logical [G, L, d] view of one sequence from a pool [n_pages, G, page, d]."""
    pool = _u16(pool)
    _, G, page, d = pool.shape
    bt = np.ascontiguousarray(block_table_row, dtype=np.int32)
    assert bt.size * page >= L
    out = np.empty((G, L, d), dtype=np.uint16)
    _load().cusa_oracle_resolve_paged(_p(pool), _p(bt), G, page, d, L, _p(out))
    return out


def scores(q: np.ndarray, K: np.ndarray, Lc: int) -> np.ndarray:
    """P[H, Lc] = q . K^T, unscaled, float32, summed left to right (Alg. 1, selection layer)."""
    q, K = _u16(q), _u16(K)
    H, d = q.shape
    G, L, d2 = K.shape
    assert d == d2 and H % G == 0 and 0 <= Lc <= L
    P = np.empty((H, Lc), dtype=np.float32)
    _load().cusa_oracle_scores(_p(q), _p(K), H, G, d, L, Lc, _p(P), Lc)
    return P


def topk(P: np.ndarray, k: int) -> np.ndarray:
    """rho_head[H, min(k, Lc)]: ranked positions, score desc then position asc (Sec. 3.2)."""
    P = np.ascontiguousarray(P, dtype=np.float32)
    H, Lc = P.shape
    k_eff = min(k, Lc)
    rho = np.empty((H, k_eff), dtype=np.int32)
    _load().cusa_oracle_topk(_p(P), Lc, H, Lc, k_eff, _p(rho))
    return rho


def unify(rho_head: np.ndarray, L: int, K: int, W: int, rank_mode: int = 0,
          P: Optional[np.ndarray] = None) -> np.ndarray:
    """rho (ascending positions): unified[:K-W] U Recent(W); all of [0,L) when L <= K."""
    rho_head = np.ascontiguousarray(rho_head, dtype=np.int32)
    H, k_eff = rho_head.shape
    ldp = 0
    if P is not None:
        P = np.ascontiguousarray(P, dtype=np.float32)
        ldp = P.shape[1]
    elif rank_mode == RANK_MAX_SCORE:
        raise ValueError("rank_mode 2 needs the scores P")
    idx = np.empty(max(K, 1) + 8, dtype=np.int32)
    n = _load().cusa_oracle_unify(_p(rho_head), _p(P), ldp, H, k_eff, L, K, W, rank_mode, _p(idx))
    return idx[:n].copy()


def select(q: np.ndarray, K: np.ndarray, budget: int, window: int, topk_per_head: int = 0,
           rank_mode: int = 0, return_all: bool = False, n_sink: int = 0):
    """Token selection of Alg. 1 for one sequence: scores -> per-head top-k -> rho.

    n_sink (Sec. 4.1 reserves four tokens as attention sinks; reading: inside the budget): the
    first n_sink positions are always in rho and are no candidates; the heads rank the positions
    [n_sink, L-W) and the unified list keeps K - W - n_sink of them, so |rho| stays K."""
    L = K.shape[1]
    k = topk_per_head if topk_per_head > 0 else budget - window
    assert 0 <= n_sink <= budget - window
    if L <= budget:
        rho = np.arange(L, dtype=np.int32)
        return (rho, None, None) if return_all else rho
    Lc = L - window
    P = scores(q, K, Lc)
    rho_head = topk(P[:, n_sink:], k) + n_sink                       # ranked picks among [n_sink, Lc)
    hist_and_recent = unify(rho_head, L, budget - n_sink, window, rank_mode, P)
    rho = np.concatenate([np.arange(n_sink, dtype=np.int32), hist_and_recent]).astype(np.int32)
    return (rho, rho_head, P) if return_all else rho


def attention(q: np.ndarray, K: np.ndarray, V: np.ndarray, idx: Optional[np.ndarray] = None,
              sm_scale: Optional[float] = None, want_f64: bool = False):
    """Eq. 1 over all tokens (idx None) or over rho (Eq. 2's restriction); bf16 bits out."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    H, d = q.shape
    G, L, _ = K.shape
    assert K.shape == V.shape and H % G == 0
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    if idx is None:
        n, ip = L, None
    else:
        idx = np.ascontiguousarray(idx, dtype=np.int32)
        assert idx.size == 0 or (idx.min() >= 0 and idx.max() < L)
        n, ip = idx.size, _p(idx)
    out = np.empty((H, d), dtype=np.uint16)
    o64 = np.empty((H, d), dtype=np.float64) if want_f64 else None
    _load().cusa_oracle_attention(_p(q), _p(K), _p(V), H, G, d, L, ip, n, float(sm_scale),
                                  _p(out), _p(o64))
    return (out, o64) if want_f64 else out


def select_per_head(q: np.ndarray, K: np.ndarray, budget: int, window: int, n_sink: int = 0) -> np.ndarray:
    """Head-to-head selection (the per-head variant CUSA is compared with, Sec. 3.2 and the
    generalization figure): head h keeps its own top-(K-W) candidates plus the last W positions.
    Returns rho_h[H, min(K, L)], every row ascending."""
    H, L = q.shape[0], K.shape[1]
    if L <= budget:
        return np.tile(np.arange(L, dtype=np.int32), (H, 1))
    Lc = L - window
    picks = topk(scores(q, K, Lc)[:, n_sink:], budget - window - n_sink) + n_sink   # ranked, distinct per row
    fixed = np.concatenate([np.arange(n_sink, dtype=np.int32), np.arange(Lc, L, dtype=np.int32)])
    return np.sort(np.concatenate([picks, np.tile(fixed, (H, 1))], axis=1), axis=1).astype(np.int32)


def attention_per_head(q: np.ndarray, K: np.ndarray, V: np.ndarray, idx_head: np.ndarray,
                       sm_scale: Optional[float] = None) -> np.ndarray:
    """Eq. 1 restricted, for head h, to its own token list idx_head[h]; bf16 bits out.
    Written as H single-head calls of ``attention`` on the head's KV group."""
    q, K, V = _u16(q), _u16(K), _u16(V)
    H, G = q.shape[0], K.shape[0]
    g = H // G
    return np.concatenate([attention(q[h:h + 1], K[h // g:h // g + 1], V[h // g:h // g + 1], idx_head[h], sm_scale)
                           for h in range(H)], axis=0)


def recall(q: np.ndarray, K: np.ndarray, idx: np.ndarray, sm_scale: Optional[float] = None):
    """Eq. 3: share of each head's softmax mass that falls on the token set idx."""
    q, K = _u16(q), _u16(K)
    H, d = q.shape
    G, L, _ = K.shape
    if sm_scale is None:
        sm_scale = 1.0 / np.sqrt(d)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    r = np.empty(H, dtype=np.float64)
    _load().cusa_oracle_recall(_p(q), _p(K), H, G, d, L, _p(idx), idx.size, float(sm_scale), _p(r))
    return r


def decode_step(layer_kind: Sequence[int], q_layers, k_layers, v_layers, budget: int,
                window: int, topk_per_head: int = 0, rank_mode: int = 0,
                sm_scale: Optional[float] = None, n_sink: int = 0):
    """Attention part of Alg. 1 for ONE sequence over all layers.

    q_layers[i]: [H,d]; k_layers[i], v_layers[i]: [G,L,d] (bf16 bits).  A full
    layer attends to everything; a selection layer also attends to everything
    and then sets rho from its own q and K; a sparse layer attends to rho at the
    same logical positions of its own K/V.  Returns (outs[list of [H,d]], rho).
    """
    rho = None
    outs = []
    for kind, q, K, V in zip(layer_kind, q_layers, k_layers, v_layers):
        if kind == LAYER_FULL:
            outs.append(attention(q, K, V, None, sm_scale))
        elif kind == LAYER_SELECT:
            outs.append(attention(q, K, V, None, sm_scale))
            rho = select(q, K, budget, window, topk_per_head, rank_mode, n_sink=n_sink)
        elif kind == LAYER_SPARSE:
            if rho is None:
                raise ValueError("sparse layer before any selection layer (rho is empty)")
            outs.append(attention(q, K, V, rho, sm_scale))
        else:
            raise ValueError(f"unknown layer kind {kind}")
    return outs, rho
