"""ctypes binding of libcusa's C ABI (include/cusa.h): argument marshalling only.

Every step of the path runs in the library's HIP kernels.  torch supplies device
memory (``tensor.data_ptr()``) and the stream.  If the library cannot be loaded
or built this module raises; there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import List, Optional, Sequence

import torch

from . import build as _build

LAYER_FULL, LAYER_SELECT, LAYER_SPARSE = 0, 1, 2
KV_CONTIGUOUS, KV_PAGED = 0, 1
RANK_FIRST_OCCURRENCE, RANK_VOTES, RANK_MAX_SCORE = 0, 1, 2
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_WORKSPACE_TOO_SMALL, ERR_LAUNCH = range(5)

EXPORTS = [
    "cusa_workspace_bytes", "cusa_workspace_layout", "cusa_select", "cusa_sparse_attn",
    "cusa_select_per_head", "cusa_sparse_attn_per_head", "cusa_attention_recall", "cusa_select_layer",
    "cusa_full_attn", "cusa_decode_step", "cusa_strerror", "cusa_profile_num_kernels",
    "cusa_profile_kernel_name", "cusa_profile_enable", "cusa_profile_reset", "cusa_profile_read",
    "cusa_build_id", "cusa_probe_stream_read", "cusa_probe_traffic", "cusa_sparse_attn_noalloc", "cusa_noalloc_max_scratch_bytes",
]


class CusaParams(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("n_q_heads", ctypes.c_int32), ("n_kv_heads", ctypes.c_int32),
                ("head_dim", ctypes.c_int32), ("budget", ctypes.c_int32), ("window", ctypes.c_int32),
                ("topk_per_head", ctypes.c_int32), ("n_sink", ctypes.c_int32), ("rank_mode", ctypes.c_int32),
                ("sm_scale", ctypes.c_float)]


class CusaKv(ctypes.Structure):
    _fields_ = [("k", ctypes.c_void_p), ("v", ctypes.c_void_p), ("layout", ctypes.c_int32),
                ("stride_batch", ctypes.c_int64), ("stride_head", ctypes.c_int64),
                ("stride_token", ctypes.c_int64), ("block_table", ctypes.c_void_p),
                ("max_pages", ctypes.c_int32), ("page_size", ctypes.c_int32), ("n_pages", ctypes.c_int64),
                ("seq_lens", ctypes.c_void_p), ("max_seq_len", ctypes.c_int32)]


class CusaWsLayout(ctypes.Structure):
    _fields_ = [("scores_offset", ctypes.c_size_t), ("ld_scores", ctypes.c_int64),
                ("rho_head_offset", ctypes.c_size_t), ("k", ctypes.c_int32), ("total_bytes", ctypes.c_size_t),
                ("filtered_select", ctypes.c_int32), ("second_chance_offset", ctypes.c_size_t)]


class CusaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {strerror(status)} (status {status})")


_lib = None


def lib_path() -> str:
    return _build.LIB


def built_from() -> str:
    """Build id of the library file, read from the file itself (nothing is mapped)."""
    marker = b"CUSA_BUILD_ID="
    with open(_build.LIB, "rb") as fh:
        data = fh.read()
    at = data.find(marker)
    if at < 0:
        return "none"
    return data[at + len(marker): at + len(marker) + 16].decode("ascii", "replace")


def load():
    """Load the built library.  It is built first when none exists, and rebuilt when the file found
    was compiled from other sources than those in the tree (its build id says so); if that rebuild
    is impossible the call raises rather than run kernels that do not match the sources."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_build.LIB):
        _build.build_lib(force=False)
    have, want = built_from(), _build.source_id()
    if have != want:
        try:
            _build.build_lib(force=True)
        except Exception as e:
            raise RuntimeError(f"libcusa.so was built from other sources (build id {have}, tree {want}) "
                               f"and cannot be rebuilt here: {e}; run __graft_entry__.build()") from e
    lib = ctypes.CDLL(_build.LIB)
    vp, i32, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_size_t
    P = ctypes.POINTER
    lib.cusa_workspace_bytes.argtypes = [P(CusaParams), i32, P(sz)]
    lib.cusa_workspace_layout.argtypes = [P(CusaParams), i32, P(CusaWsLayout)]
    lib.cusa_select.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, sz, vp]
    lib.cusa_sparse_attn.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, vp, sz, vp]
    lib.cusa_select_per_head.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, sz, vp]
    lib.cusa_sparse_attn_per_head.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, vp, sz, vp]
    lib.cusa_attention_recall.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, i32, vp, vp, sz, vp]
    lib.cusa_select_layer.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, vp, sz, vp]
    lib.cusa_full_attn.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, sz, vp]
    lib.cusa_decode_step.argtypes = [P(CusaParams), i32, P(i32), P(vp), P(CusaKv), P(vp), vp, vp, vp, sz, vp]
    for name in ("cusa_workspace_bytes", "cusa_workspace_layout", "cusa_select", "cusa_sparse_attn",
                 "cusa_select_per_head", "cusa_sparse_attn_per_head", "cusa_attention_recall", "cusa_select_layer",
                 "cusa_full_attn", "cusa_decode_step", "cusa_profile_read"):
        getattr(lib, name).restype = ctypes.c_int
    lib.cusa_strerror.argtypes = [ctypes.c_int]
    lib.cusa_strerror.restype = ctypes.c_char_p
    lib.cusa_profile_num_kernels.restype = i32
    lib.cusa_profile_kernel_name.argtypes = [i32]
    lib.cusa_profile_kernel_name.restype = ctypes.c_char_p
    lib.cusa_profile_enable.argtypes = [i32]
    lib.cusa_profile_reset.argtypes = []
    lib.cusa_profile_read.argtypes = [i32, P(ctypes.c_int64), P(ctypes.c_double)]
    lib.cusa_build_id.restype = ctypes.c_char_p
    lib.cusa_sparse_attn_noalloc.argtypes = [P(CusaParams), vp, P(CusaKv), vp, vp, vp, vp]
    lib.cusa_sparse_attn_noalloc.restype = ctypes.c_int
    lib.cusa_noalloc_max_scratch_bytes.argtypes = []
    lib.cusa_noalloc_max_scratch_bytes.restype = sz
    lib.cusa_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.cusa_probe_stream_read.restype = ctypes.c_int
    lib.cusa_probe_traffic.argtypes = [i32, vp, sz, vp, sz, vp]
    lib.cusa_probe_traffic.restype = ctypes.c_int
    _lib = lib
    return lib


def strerror(status: int) -> str:
    return load().cusa_strerror(int(status)).decode()


def _check(status: int, where: str):
    if status != OK:
        raise CusaError(status, where)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def make_params(batch, n_q_heads, n_kv_heads, budget, window, topk_per_head=0, head_dim=128,
                sm_scale=None, rank_mode=RANK_FIRST_OCCURRENCE, n_sink=0) -> CusaParams:
    if sm_scale is None:
        sm_scale = head_dim ** -0.5
    return CusaParams(batch, n_q_heads, n_kv_heads, head_dim, budget, window, topk_per_head, n_sink,
                      rank_mode, sm_scale)


@dataclass
class KvCache:
    """One layer's cache view; keeps the tensors alive and builds the C descriptor."""
    k: torch.Tensor
    v: torch.Tensor
    seq_lens: torch.Tensor                      # int32 [B] on device
    max_seq_len: int
    block_table: Optional[torch.Tensor] = None  # int32 [B, max_pages] -> paged

    def desc(self) -> CusaKv:
        if self.block_table is None:
            assert self.k.dim() == 4 and self.k.stride(3) == 1 and self.k.stride() == self.v.stride()
            sb, sh, st, _ = self.k.stride()
            return CusaKv(self.k.data_ptr(), self.v.data_ptr(), KV_CONTIGUOUS, sb, sh, st, None, 0, 0, 0,
                          self.seq_lens.data_ptr(), self.max_seq_len)
        assert self.k.is_contiguous() and self.v.is_contiguous() and self.block_table.is_contiguous()
        n_pages, _, page, _ = self.k.shape
        return CusaKv(self.k.data_ptr(), self.v.data_ptr(), KV_PAGED, 0, 0, 0, self.block_table.data_ptr(),
                      self.block_table.shape[1], page, n_pages, self.seq_lens.data_ptr(), self.max_seq_len)


def workspace_bytes(params: CusaParams, max_seq_len: int) -> int:
    n = ctypes.c_size_t(0)
    _check(load().cusa_workspace_bytes(ctypes.byref(params), max_seq_len, ctypes.byref(n)), "cusa_workspace_bytes")
    return int(n.value)


def workspace_layout(params: CusaParams, max_seq_len: int) -> CusaWsLayout:
    lay = CusaWsLayout()
    _check(load().cusa_workspace_layout(ctypes.byref(params), max_seq_len, ctypes.byref(lay)),
           "cusa_workspace_layout")
    return lay


def alloc_workspace(params: CusaParams, max_seq_len: int, device="cuda") -> torch.Tensor:
    return torch.empty(workspace_bytes(params, max_seq_len), dtype=torch.uint8, device=device)


def select(params: CusaParams, q: torch.Tensor, kv: KvCache, idx: torch.Tensor, cnt: torch.Tensor,
           ws: torch.Tensor):
    d = kv.desc()
    _check(load().cusa_select(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx), _ptr(cnt), _ptr(ws),
                              ws.numel(), _stream()), "cusa_select")


def sparse_attn(params: CusaParams, q, kv: KvCache, idx, cnt, out, ws):
    d = kv.desc()
    _check(load().cusa_sparse_attn(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx), _ptr(cnt),
                                   _ptr(out), _ptr(ws), ws.numel(), _stream()), "cusa_sparse_attn")


def sparse_attn_noalloc(params: CusaParams, q, kv: KvCache, idx, cnt, out):
    """cusa_sparse_attn with the partials in the library's static scratch (no workspace argument)."""
    d = kv.desc()
    _check(load().cusa_sparse_attn_noalloc(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx), _ptr(cnt),
                                           _ptr(out), _stream()), "cusa_sparse_attn_noalloc")


def noalloc_max_scratch_bytes() -> int:
    return int(load().cusa_noalloc_max_scratch_bytes())


def select_per_head(params: CusaParams, q, kv: KvCache, idx_head, cnt, ws):
    """idx_head: int32 [B, H, budget]; every head keeps its own picks (head-to-head selection)."""
    d = kv.desc()
    _check(load().cusa_select_per_head(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx_head), _ptr(cnt),
                                       _ptr(ws), ws.numel(), _stream()), "cusa_select_per_head")


def sparse_attn_per_head(params: CusaParams, q, kv: KvCache, idx_head, cnt, out, ws):
    d = kv.desc()
    _check(load().cusa_sparse_attn_per_head(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx_head), _ptr(cnt),
                                            _ptr(out), _ptr(ws), ws.numel(), _stream()), "cusa_sparse_attn_per_head")


def attention_recall(params: CusaParams, q, kv: KvCache, idx, cnt, recall, ws, per_head: bool = False):
    """recall: float32 [B, H], Eq. 3 for the token set idx/cnt (idx [B, H, budget] when per_head)."""
    d = kv.desc()
    _check(load().cusa_attention_recall(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(idx), _ptr(cnt),
                                        1 if per_head else 0, _ptr(recall), _ptr(ws), ws.numel(), _stream()),
           "cusa_attention_recall")


def select_layer(params: CusaParams, q, kv: KvCache, out, idx, cnt, ws):
    """A selection layer in one call: full-attention output and rho from one pass over K."""
    d = kv.desc()
    _check(load().cusa_select_layer(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(out), _ptr(idx), _ptr(cnt),
                                    _ptr(ws), ws.numel(), _stream()), "cusa_select_layer")


def full_attn(params: CusaParams, q, kv: KvCache, out, ws):
    d = kv.desc()
    _check(load().cusa_full_attn(ctypes.byref(params), _ptr(q), ctypes.byref(d), _ptr(out), _ptr(ws),
                                 ws.numel(), _stream()), "cusa_full_attn")


class DecodeStep:
    """Marshals one decode step's per-layer pointers once, then replays cusa_decode_step."""

    def __init__(self, params: CusaParams, layer_kind: Sequence[int], q_layers: List[torch.Tensor],
                 kv_layers: List[KvCache], out_layers: List[torch.Tensor], idx, cnt, ws):
        n = len(layer_kind)
        assert len(q_layers) == len(kv_layers) == len(out_layers) == n
        self.params, self.n = params, n
        self._keep = (q_layers, kv_layers, out_layers, idx, cnt, ws)
        self.kinds = (ctypes.c_int32 * n)(*layer_kind)
        self.qs = (ctypes.c_void_p * n)(*[t.data_ptr() for t in q_layers])
        self.outs = (ctypes.c_void_p * n)(*[t.data_ptr() for t in out_layers])
        self.kvs = (CusaKv * n)(*[kv.desc() for kv in kv_layers])
        self.idx, self.cnt, self.ws = idx, cnt, ws

    def run(self):
        _check(load().cusa_decode_step(ctypes.byref(self.params), self.n, self.kinds, self.qs, self.kvs,
                                       self.outs, _ptr(self.idx), _ptr(self.cnt), _ptr(self.ws),
                                       self.ws.numel(), _stream()), "cusa_decode_step")


def decode_step(params, layer_kind, q_layers, kv_layers, out_layers, idx, cnt, ws):
    DecodeStep(params, layer_kind, q_layers, kv_layers, out_layers, idx, cnt, ws).run()


def probe_stream_read(src: torch.Tensor, sink: torch.Tensor):
    """Enqueue the streaming-read probe over the bytes of src (benchmark support)."""
    _check(load().cusa_probe_stream_read(_ptr(src), src.numel() * src.element_size(), _ptr(sink), _stream()),
           "cusa_probe_stream_read")


def probe_traffic(pattern: int, src: torch.Tensor, dst: torch.Tensor):
    """Enqueue a traffic probe (0 stream in tiles, 1 gathered rows, 2 stream + scattered writes, 3 stream + burst writes)."""
    _check(load().cusa_probe_traffic(pattern, _ptr(src), src.numel() * src.element_size(), _ptr(dst),
                                     dst.numel() * dst.element_size(), _stream()), "cusa_probe_traffic")


# ---- per-kernel timing ---------------------------------------------------------

def profile_enable(on: bool):
    load().cusa_profile_enable(1 if on else 0)


def profile_reset():
    load().cusa_profile_reset()


def profile_read() -> dict:
    lib = load()
    n = lib.cusa_profile_num_kernels()
    calls = (ctypes.c_int64 * n)()
    ms = (ctypes.c_double * n)()
    _check(lib.cusa_profile_read(n, calls, ms), "cusa_profile_read")
    return {lib.cusa_profile_kernel_name(i).decode(): {"calls": int(calls[i]), "total_ms": float(ms[i])}
            for i in range(n)}
