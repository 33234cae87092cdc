"""ctypes binding of libjq.so: argument marshalling only.

Every step of the eviction path (paper Section 4.3) runs in the HIP kernels of
libjq; this module turns torch tensors into device pointers, fills the
``jq_shape`` struct and raises on a non-zero status.  There is no CPU fallback:
if the library cannot be loaded the import of a function fails loudly.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass, field
from typing import Optional, Sequence

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_PKG, "libjq.so")
_lib = None

JQ_MAX_SEQ = 128
STATUS = {0: "JQ_OK", -1: "JQ_ERR_NULL", -2: "JQ_ERR_SHAPE", -3: "JQ_ERR_BUDGET", -4: "JQ_ERR_UNSUPPORTED",
          -5: "JQ_ERR_WORKSPACE", -6: "JQ_ERR_ALIAS", -7: "JQ_ERR_LAUNCH"}
EXPORTS = ("jq_workspace_bytes", "jq_score", "jq_score_lse", "jq_evict_lse", "jq_score_tail", "jq_evict_tail", "jq_pool", "jq_select_topk", "jq_compact", "jq_compact_inplace_workspace_bytes", "jq_compact_inplace", "jq_evict", "jq_evict_inplace_workspace_bytes", "jq_evict_inplace", "jq_evict_stream", "jq_evict_static", "jq_score_paged", "jq_evict_paged", "jq_evict_paged_inplace_workspace_bytes", "jq_evict_paged_inplace", "jq_evict_traced", "jq_hit_rate", "jq_map_mse", "jq_map_mse_fused_workspace_bytes", "jq_map_mse_fused",
           "jq_copy_probe", "jq_reload_knobs", "jq_status_string")
TRACE_KERNELS = ("jq_stats_kernel", "jq_score_kernel", "jq_pool_kernel", "jq_select_finalize_kernel")
TRACE_MARKS = 2 * len(TRACE_KERNELS)


class JQError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (%s)" % (what, STATUS.get(status, status), status_string(status)))


class _CShape(ctypes.Structure):
    _fields_ = [("n_layers", ctypes.c_int32), ("n_seq", ctypes.c_int32), ("n_q", ctypes.c_int32),
                ("h_q", ctypes.c_int32), ("h_kv", ctypes.c_int32), ("d", ctypes.c_int32),
                ("pool_k", ctypes.c_int32), ("scale", ctypes.c_float),
                ("cu_seqlens", ctypes.POINTER(ctypes.c_int32)), ("budgets", ctypes.POINTER(ctypes.c_int32)),
                ("keep_first", ctypes.c_int32), ("keep_last", ctypes.c_int32), ("window", ctypes.c_int32),
                ("layer_budgets", ctypes.c_void_p)]


class _CPages(ctypes.Structure):
    _fields_ = [("page_size", ctypes.c_int32), ("n_pages", ctypes.c_int32), ("max_pages_per_seq", ctypes.c_int32),
                ("block_table", ctypes.c_void_p)]


def lib() -> ctypes.CDLL:
    """Load libjq.so (building it first only when no built library is present)."""
    global _lib
    if _lib is None:
        # PyTorch provides device memory and streams, and ships its own HIP runtime: it must be in the
        # process before libjq so that both resolve to that one runtime (same SONAME) instead of two.
        import torch  # noqa: F401
        if not os.path.exists(_LIB_PATH):
            from . import _build
            _build.build()
        L = ctypes.CDLL(_LIB_PATH)
        vp, sz = ctypes.c_void_p, ctypes.c_size_t
        shp = ctypes.POINTER(_CShape)
        L.jq_workspace_bytes.argtypes = [shp, ctypes.POINTER(sz)]
        L.jq_score.argtypes = [shp, vp, vp, vp, vp, sz, vp]
        L.jq_score_lse.argtypes = [shp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_lse.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_hit_rate.argtypes = [shp, vp, vp, ctypes.POINTER(ctypes.c_int32), vp, vp]
        L.jq_map_mse.argtypes = [shp, vp, ctypes.c_float, vp, ctypes.c_float, vp, vp]
        L.jq_map_mse_fused_workspace_bytes.argtypes = [shp, ctypes.c_int32, ctypes.POINTER(sz)]
        L.jq_map_mse_fused.argtypes = [shp, vp, vp, ctypes.c_int32, vp, vp, vp, sz, vp]
        L.jq_score_tail.argtypes = [shp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_tail.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_pool.argtypes = [shp, vp, vp, vp]
        L.jq_select_topk.argtypes = [shp, vp, vp, vp, sz, vp]
        L.jq_compact.argtypes = [shp, vp, vp, vp, vp, vp, vp]
        L.jq_compact_inplace_workspace_bytes.argtypes = [shp, ctypes.POINTER(sz)]
        L.jq_compact_inplace.argtypes = [shp, vp, vp, vp, vp, sz, vp]
        L.jq_evict.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_static.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp]
        L.jq_evict_inplace_workspace_bytes.argtypes = [shp, ctypes.POINTER(sz)]
        L.jq_evict_inplace.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_stream.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        pgp = ctypes.POINTER(_CPages)
        L.jq_score_paged.argtypes = [shp, pgp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_paged.argtypes = [shp, pgp, pgp, vp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_paged_inplace_workspace_bytes.argtypes = [shp, pgp, ctypes.POINTER(sz)]
        L.jq_evict_paged_inplace.argtypes = [shp, pgp, pgp, vp, vp, vp, vp, vp, vp, vp, sz, vp]
        L.jq_evict_traced.argtypes = [shp, vp, vp, vp, vp, vp, vp, vp, vp, sz, vp, ctypes.POINTER(vp), ctypes.c_int]
        L.jq_copy_probe.argtypes = [vp, vp, sz, vp]
        L.jq_reload_knobs.argtypes = []
        L.jq_status_string.argtypes = [ctypes.c_int]
        L.jq_status_string.restype = ctypes.c_char_p
        for name in EXPORTS[:-1]:
            getattr(L, name).restype = ctypes.c_int
        _lib = L
    return _lib


def status_string(status: int) -> str:
    return lib().jq_status_string(int(status)).decode()


@dataclass
class Shape:
    """Host-side problem description; mirrors ``jq_shape`` in include/jq.h."""
    n_layers: int
    seq_lens: Sequence[int]
    n_q: int
    h_q: int
    h_kv: int
    d: int = 128
    pool_k: int = 7
    budgets: Optional[Sequence[int]] = None
    scale: float = 0.0
    keep_first: int = 0   # positions at the start / end of every sequence that the selection always keeps
    keep_last: int = 0
    window: bool = False  # the queries are the prompt's own last n_q tokens (causal inside them, always kept)
    layer_budgets: object = None  # int32 DEVICE tensor [n_layers, n_seq]: per-layer budgets (`budgets` = the largest)
    _keep: list = field(default_factory=list, repr=False)

    @property
    def n_seq(self) -> int:
        return len(self.seq_lens)

    @property
    def T(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def TB(self) -> int:
        return int(sum(self.budgets)) if self.budgets is not None else 0

    def c_struct(self) -> _CShape:
        key = (self.n_layers, tuple(self.seq_lens), self.n_q, self.h_q, self.h_kv, self.d, self.pool_k,
               None if self.budgets is None else tuple(self.budgets), float(self.scale), self.keep_first, self.keep_last, bool(self.window),
               None if self.layer_budgets is None else int(self.layer_budgets.data_ptr()))
        if self._keep and self._keep[0] == key:  # marshalled once per distinct description
            return self._keep[3]
        cu = np.concatenate([[0], np.cumsum(np.asarray(self.seq_lens, dtype=np.int64))]).astype(np.int32)
        bud = None if self.budgets is None else np.ascontiguousarray(self.budgets, dtype=np.int32)
        i32p = ctypes.POINTER(ctypes.c_int32)
        cs = _CShape(self.n_layers, self.n_seq, self.n_q, self.h_q, self.h_kv, self.d, self.pool_k,
                     float(self.scale), cu.ctypes.data_as(i32p),
                     bud.ctypes.data_as(i32p) if bud is not None else ctypes.cast(None, i32p),
                     int(self.keep_first), int(self.keep_last), int(bool(self.window)),
                     None if self.layer_budgets is None else int(self.layer_budgets.data_ptr()))
        self._keep = [key, cu, bud, cs]  # the host arrays must outlive the struct
        return cs


def _ptr(t) -> Optional[int]:
    return None if t is None else int(t.data_ptr())


def _stream(stream) -> Optional[int]:
    import torch
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream) or None


def _check(rc: int, what: str):
    if rc != 0:
        raise JQError(rc, what)


def workspace_bytes(shape: Shape) -> int:
    n = ctypes.c_size_t(0)
    cs = shape.c_struct()
    _check(lib().jq_workspace_bytes(ctypes.byref(cs), ctypes.byref(n)), "jq_workspace_bytes")
    return int(n.value)


def alloc_workspace(shape: Shape, device="cuda"):
    import torch
    return torch.empty(workspace_bytes(shape), dtype=torch.uint8, device=device)


def score(shape: Shape, Q, K, scores=None, ws=None, stream=None, lse=None, k_tail=None):
    """Unpooled scores; with `lse` ([n_layers, n_seq, n_q, h_q] fp32) the one-pass supplied-normaliser variant,
    with `k_tail` ([n_layers, n_seq, n_q, h_kv, d] bf16) the variant whose softmax covers the soft tokens' own keys."""
    import torch
    if scores is None:
        scores = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=K.device)
    if ws is None:
        ws = alloc_workspace(shape, K.device)
    cs = shape.c_struct()
    if lse is not None:
        _check(lib().jq_score_lse(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(lse), _ptr(scores), _ptr(ws), ws.numel(),
                                  _stream(stream)), "jq_score_lse")
        return scores
    if k_tail is not None:
        _check(lib().jq_score_tail(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(k_tail), _ptr(scores), _ptr(ws), ws.numel(),
                                   _stream(stream)), "jq_score_tail")
        return scores
    _check(lib().jq_score(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(scores), _ptr(ws), ws.numel(), _stream(stream)), "jq_score")
    return scores


def pool(shape: Shape, scores, pooled=None, stream=None):
    import torch
    if pooled is None:
        pooled = torch.empty_like(scores)
    cs = shape.c_struct()
    _check(lib().jq_pool(ctypes.byref(cs), _ptr(scores), _ptr(pooled), _stream(stream)), "jq_pool")
    return pooled


def select_topk(shape: Shape, pooled, idx=None, ws=None, stream=None):
    import torch
    if idx is None:
        idx = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=pooled.device)
    if ws is None:
        ws = alloc_workspace(shape, pooled.device)
    cs = shape.c_struct()
    _check(lib().jq_select_topk(ctypes.byref(cs), _ptr(pooled), _ptr(idx), _ptr(ws), ws.numel(), _stream(stream)), "jq_select_topk")
    return idx


def compact(shape: Shape, K, V, idx, K_out=None, V_out=None, stream=None):
    import torch
    if K_out is None:
        K_out = torch.empty((shape.n_layers, shape.TB, shape.h_kv, shape.d), dtype=K.dtype, device=K.device)
    if V_out is None:
        V_out = torch.empty_like(K_out)
    cs = shape.c_struct()
    _check(lib().jq_compact(ctypes.byref(cs), _ptr(K), _ptr(V), _ptr(idx), _ptr(K_out), _ptr(V_out), _stream(stream)), "jq_compact")
    return K_out, V_out


def compact_inplace(shape: Shape, K, V, idx, ws=None, stream=None):
    """Kept rows written over the front of K and V themselves (rows 0..TB-1 of every layer)."""
    import torch
    cs = shape.c_struct()
    if ws is None:
        n = ctypes.c_size_t(0)
        _check(lib().jq_compact_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(n)), "jq_compact_inplace_workspace_bytes")
        ws = torch.empty(int(n.value), dtype=torch.uint8, device=K.device)
    _check(lib().jq_compact_inplace(ctypes.byref(cs), _ptr(K), _ptr(V), _ptr(idx), _ptr(ws), ws.numel(), _stream(stream)),
           "jq_compact_inplace")
    return K, V


def evict(shape: Shape, Q, K, V, K_out=None, V_out=None, idx_out=None, scores_out=None, ws=None, stream=None,
          want_idx=True, want_scores=True, marks=None, lse=None, k_tail=None):
    """Fused score -> pool -> top-B -> gather.  Returns (K_out, V_out, idx_out, pooled scores).

    `marks`: optional list of TRACE_MARKS torch.cuda.Event(enable_timing=True) objects that have been
    recorded once (so that their handles exist); events 2i / 2i+1 receive the start / stop time of
    kernel TRACE_KERNELS[i]."""
    import torch
    dev = K.device
    if K_out is None:
        K_out = torch.empty((shape.n_layers, shape.TB, shape.h_kv, shape.d), dtype=K.dtype, device=dev)
    if V_out is None:
        V_out = torch.empty_like(K_out)
    if idx_out is None and want_idx:
        idx_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if scores_out is None and want_scores:
        scores_out = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=dev)
    if ws is None:
        ws = alloc_workspace(shape, dev)
    cs = shape.c_struct()
    if lse is not None:
        _check(lib().jq_evict_lse(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(lse), _ptr(K_out), _ptr(V_out),
                                  _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)), "jq_evict_lse")
        return K_out, V_out, idx_out, scores_out
    if k_tail is not None:
        _check(lib().jq_evict_tail(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(k_tail), _ptr(K_out), _ptr(V_out),
                                   _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)), "jq_evict_tail")
        return K_out, V_out, idx_out, scores_out
    if marks is not None:
        arr = (ctypes.c_void_p * len(marks))(*[int(ev.cuda_event) for ev in marks])
        _check(lib().jq_evict_traced(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(K_out), _ptr(V_out),
                                     _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream), arr,
                                     len(marks)), "jq_evict_traced")
        return K_out, V_out, idx_out, scores_out
    _check(lib().jq_evict(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(K_out), _ptr(V_out), _ptr(idx_out),
                          _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)), "jq_evict")
    return K_out, V_out, idx_out, scores_out


def evict_inplace(shape: Shape, Q, K, V, lse=None, idx_out=None, scores_out=None, ws=None, stream=None, want_idx=True,
                  want_scores=True):
    """Fused eviction whose pruned cache is written over the front of K and V themselves (rows 0..TB-1 of every
    layer).  Returns (K, V, idx_out, pooled scores)."""
    import torch
    dev = K.device
    if idx_out is None and want_idx:
        idx_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if scores_out is None and want_scores:
        scores_out = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=dev)
    cs = shape.c_struct()
    if ws is None:
        n = ctypes.c_size_t(0)
        _check(lib().jq_evict_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(n)), "jq_evict_inplace_workspace_bytes")
        ws = torch.empty(int(n.value), dtype=torch.uint8, device=dev)
    _check(lib().jq_evict_inplace(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(lse), _ptr(idx_out), _ptr(scores_out),
                                  _ptr(ws), ws.numel(), _stream(stream)), "jq_evict_inplace")
    return K, V, idx_out, scores_out


def evict_stream(shape: Shape, Q, K, V, pos, lse=None, K_out=None, V_out=None, pos_out=None, idx_out=None, scores_out=None,
                 ws=None, stream=None):
    """One eviction step during decoding on a pruned cache K, V [n_layers, T, h_kv, d] whose rows came from the
    tokens pos [n_layers, h_kv, T].  Returns (K_out, V_out, pos_out, idx_out, pooled scores)."""
    import torch
    dev = K.device
    if K_out is None:
        K_out = torch.empty((shape.n_layers, shape.TB, shape.h_kv, shape.d), dtype=K.dtype, device=dev)
    if V_out is None:
        V_out = torch.empty_like(K_out)
    if pos_out is None:
        pos_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if idx_out is None:
        idx_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if scores_out is None:
        scores_out = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=dev)
    if ws is None:
        ws = alloc_workspace(shape, dev)
    cs = shape.c_struct()
    _check(lib().jq_evict_stream(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(pos), _ptr(lse), _ptr(K_out), _ptr(V_out),
                                 _ptr(pos_out), _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)),
           "jq_evict_stream")
    return K_out, V_out, pos_out, idx_out, scores_out


STATIC_WS_BYTES = 32 << 20


def evict_static(shape: Shape, Q, K, V, K_out, V_out, idx_out=None, scores_out=None, stream=None):
    """jq_evict_static: the fused eviction with the library's built-in scratch array instead of a workspace.
    Every output the caller wants is passed in (this wrapper allocates nothing either)."""
    cs = shape.c_struct()
    _check(lib().jq_evict_static(ctypes.byref(cs), _ptr(Q), _ptr(K), _ptr(V), _ptr(K_out), _ptr(V_out), _ptr(idx_out),
                                 _ptr(scores_out), _stream(stream)), "jq_evict_static")
    return K_out, V_out, idx_out, scores_out


@dataclass
class Pages:
    """A paged K/V cache; mirrors ``jq_pages``.  `block_table`: int32 device tensor [n_seq, max_pages_per_seq]."""
    page_size: int
    n_pages: int
    block_table: object

    def c_struct(self) -> _CPages:
        bt = self.block_table
        return _CPages(int(self.page_size), int(self.n_pages), int(bt.shape[1]) if bt is not None else 0,
                       _ptr(bt) if bt is not None else None)


def score_paged(shape: Shape, pages: Pages, Q, K_pool, lse=None, scores=None, ws=None, stream=None):
    """Unpooled scores from a paged cache: K_pool [n_layers, n_pages, page_size, h_kv, d] bf16."""
    import torch
    if scores is None:
        scores = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=K_pool.device)
    if ws is None:
        ws = alloc_workspace(shape, K_pool.device)
    cs, cp = shape.c_struct(), pages.c_struct()
    _check(lib().jq_score_paged(ctypes.byref(cs), ctypes.byref(cp), _ptr(Q), _ptr(K_pool), _ptr(lse), _ptr(scores), _ptr(ws),
                                ws.numel(), _stream(stream)), "jq_score_paged")
    return scores


def evict_paged(shape: Shape, pages: Pages, Q, K_pool, V_pool, lse=None, K_out=None, V_out=None, idx_out=None,
                scores_out=None, ws=None, stream=None, want_idx=True, want_scores=True, out_pages: Optional[Pages] = None):
    """Fused eviction on a paged cache.  Returns (K_out, V_out, idx_out, pooled scores); K_out / V_out are dense, or
    pools [n_layers, out_pages.n_pages, out_pages.page_size, h_kv, d] when `out_pages` describes a paged output."""
    import torch
    dev = K_pool.device
    if K_out is None and out_pages is not None:
        K_out = torch.zeros((shape.n_layers, out_pages.n_pages, out_pages.page_size, shape.h_kv, shape.d), dtype=K_pool.dtype,
                            device=dev)
    if K_out is None:
        K_out = torch.empty((shape.n_layers, shape.TB, shape.h_kv, shape.d), dtype=K_pool.dtype, device=dev)
    if V_out is None:
        V_out = torch.zeros_like(K_out) if out_pages is not None else torch.empty_like(K_out)
    if idx_out is None and want_idx:
        idx_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if scores_out is None and want_scores:
        scores_out = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=dev)
    if ws is None:
        ws = alloc_workspace(shape, dev)
    cs, cp = shape.c_struct(), pages.c_struct()
    co = out_pages.c_struct() if out_pages is not None else None
    _check(lib().jq_evict_paged(ctypes.byref(cs), ctypes.byref(cp), ctypes.byref(co) if co is not None else None, _ptr(Q),
                                _ptr(K_pool), _ptr(V_pool), _ptr(lse),
                                _ptr(K_out), _ptr(V_out), _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(),
                                _stream(stream)), "jq_evict_paged")
    return K_out, V_out, idx_out, scores_out


def evict_paged_inplace(shape: Shape, pages: Pages, out_pages: Pages, Q, K_pool, V_pool, lse=None, idx_out=None, scores_out=None,
                        ws=None, stream=None):
    """Fused eviction on a paged cache whose kept rows are written into pages of the same pools (`out_pages`: same
    page size and pool size, its own block table).  Returns (K_pool, V_pool, idx_out, pooled scores)."""
    import torch
    dev = K_pool.device
    if idx_out is None:
        idx_out = torch.empty((shape.n_layers, shape.h_kv, shape.TB), dtype=torch.int32, device=dev)
    if scores_out is None:
        scores_out = torch.empty((shape.n_layers, shape.h_kv, shape.T), dtype=torch.float32, device=dev)
    cs, cp, co = shape.c_struct(), pages.c_struct(), out_pages.c_struct()
    if ws is None:
        n = ctypes.c_size_t(0)
        _check(lib().jq_evict_paged_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(cp), ctypes.byref(n)),
               "jq_evict_paged_inplace_workspace_bytes")
        ws = torch.empty(int(n.value), dtype=torch.uint8, device=dev)
    _check(lib().jq_evict_paged_inplace(ctypes.byref(cs), ctypes.byref(cp), ctypes.byref(co), _ptr(Q), _ptr(K_pool), _ptr(V_pool),
                                        _ptr(lse), _ptr(idx_out), _ptr(scores_out), _ptr(ws), ws.numel(), _stream(stream)),
           "jq_evict_paged_inplace")
    return K_pool, V_pool, idx_out, scores_out


def hit_rate(shape: Shape, idx_cur, idx_ref, ref_budgets=None, rate=None, stream=None):
    """Eq. 6 per (layer, sequence, head): |I_cur & I_ref| / |I_ref| for ascending position lists; returns
    rate [n_layers, n_seq, h_kv] fp32.  `ref_budgets`: list lengths of idx_ref per sequence (default: shape's)."""
    import torch
    if rate is None:
        rate = torch.empty((shape.n_layers, shape.n_seq, shape.h_kv), dtype=torch.float32, device=idx_cur.device)
    cs = shape.c_struct()
    rb = None
    if ref_budgets is not None:
        rb = np.ascontiguousarray(ref_budgets, dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    _check(lib().jq_hit_rate(ctypes.byref(cs), _ptr(idx_cur), _ptr(idx_ref),
                             rb.ctypes.data_as(i32p) if rb is not None else ctypes.cast(None, i32p), _ptr(rate),
                             _stream(stream)), "jq_hit_rate")
    return rate


def map_mse(shape: Shape, scores_a, rows_a: float, scores_b, rows_b: float, mse=None, stream=None):
    """Eq. 5 forward per (layer, sequence, head): mean over the prompt of (scores_a/rows_a - scores_b/rows_b)^2."""
    import torch
    if mse is None:
        mse = torch.empty((shape.n_layers, shape.n_seq, shape.h_kv), dtype=torch.float32, device=scores_a.device)
    cs = shape.c_struct()
    _check(lib().jq_map_mse(ctypes.byref(cs), _ptr(scores_a), float(rows_a), _ptr(scores_b), float(rows_b), _ptr(mse),
                            _stream(stream)), "jq_map_mse")
    return mse


def map_mse_fused(shape: Shape, Q_a, Q_b, K, mse=None, ws=None, stream=None):
    """Eq. 3-5 forward from the two query sets (Q_a [.., shape.n_q, h_q, d] soft tokens, Q_b [.., n_q_b, h_q, d] response
    tokens): the second map is compared with the first inside the launch that completes it and never stored."""
    import torch
    n_q_b = int(Q_b.shape[2])
    if mse is None:
        mse = torch.empty((shape.n_layers, shape.n_seq, shape.h_kv), dtype=torch.float32, device=K.device)
    cs = shape.c_struct()
    if ws is None:
        n = ctypes.c_size_t()
        _check(lib().jq_map_mse_fused_workspace_bytes(ctypes.byref(cs), n_q_b, ctypes.byref(n)), "jq_map_mse_fused_workspace_bytes")
        ws = torch.empty((n.value,), dtype=torch.uint8, device=K.device)
    _check(lib().jq_map_mse_fused(ctypes.byref(cs), _ptr(Q_a), _ptr(Q_b), n_q_b, _ptr(K), _ptr(mse), _ptr(ws), ws.numel(),
                                  _stream(stream)), "jq_map_mse_fused")
    return mse


def reload_knobs() -> None:
    """Make the library read its ablation knobs (JQ_CHUNK_KEYS, JQ_DEPTH_1, ...) from the environment again."""
    _check(lib().jq_reload_knobs(), "jq_reload_knobs")


def copy_probe(src, dst, stream=None):
    """Plain copy of src into dst (same byte size): the known-size kernel used to calibrate traffic counters."""
    nbytes = src.numel() * src.element_size()
    _check(lib().jq_copy_probe(_ptr(src), _ptr(dst), nbytes, _stream(stream)), "jq_copy_probe")
    return dst
