"""ctypes wrapper around the fp64 CPU oracle (``jq_oracle.c``) -- TEST INFRASTRUCTURE ONLY.

Only the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may
import this module.  It never touches the HIP library and shares nothing with
it.  Batched helpers here are plain Python loops over (layer, sequence) calling
the single-problem C functions, following Section 4.3 of the paper one problem
at a time.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "jq_oracle.c")
_LIB = os.path.join(_HERE, "libjq_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (-O2, OpenMP, no fast-math).  Returns the .so path."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c99", "-Wall", "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        u16p, f64p, i32p = (np.ctypeslib.ndpointer(dtype=t, flags="C_CONTIGUOUS") for t in (np.uint16, np.float64, np.int32))
        lib.jqo_num_threads.restype = ctypes.c_int
        lib.jqo_score.argtypes = [ctypes.c_int] * 4 + [ctypes.c_long, ctypes.c_double, u16p, u16p, f64p]
        lib.jqo_score_lse.argtypes = [ctypes.c_int] * 4 + [ctypes.c_long, ctypes.c_double, u16p, u16p, f64p, f64p]
        lib.jqo_score_tail.argtypes = [ctypes.c_int] * 4 + [ctypes.c_long, ctypes.c_double, u16p, u16p, u16p, f64p]
        lib.jqo_score_window.argtypes = [ctypes.c_int] * 4 + [ctypes.c_long, ctypes.c_double, u16p, u16p, f64p]
        lib.jqo_score_window.restype = ctypes.c_int
        lib.jqo_map_mse.argtypes = [ctypes.c_long, ctypes.c_int, ctypes.c_double, ctypes.c_double, f64p, f64p, f64p]
        lib.jqo_map_mse.restype = ctypes.c_int
        lib.jqo_pool.argtypes = [ctypes.c_long, ctypes.c_int, f64p, f64p]
        lib.jqo_select_topk.argtypes = [ctypes.c_long, ctypes.c_long, f64p, i32p]
        lib.jqo_select_topk_keep.argtypes = [ctypes.c_long] * 4 + [f64p, i32p]
        lib.jqo_select_topk_keep.restype = ctypes.c_int
        lib.jqo_compact.argtypes = [ctypes.c_long, ctypes.c_int, ctypes.c_int, ctypes.c_long, u16p, u16p, i32p, u16p, u16p]
        for f in (lib.jqo_score, lib.jqo_score_lse, lib.jqo_score_tail, lib.jqo_pool, lib.jqo_select_topk, lib.jqo_compact):
            f.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().jqo_num_threads())


def _check(rc: int, what: str):
    if rc != 0:
        raise ValueError("oracle %s rejected its arguments (rc=%d)" % (what, rc))


def score(Q: np.ndarray, K: np.ndarray, scale: float = 0.0) -> np.ndarray:
    """Q [n_q,h_q,d], K [L,h_kv,d] bf16 bits (uint16) -> score [h_kv, L] float64."""
    Q = np.ascontiguousarray(Q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    n_q, h_q, d = Q.shape
    L, h_kv, d2 = K.shape
    if d != d2:
        raise ValueError("head dims differ")
    out = np.empty((h_kv, L), dtype=np.float64)
    _check(_load().jqo_score(n_q, h_q, h_kv, d, L, float(scale), Q, K, out), "score")
    return out


def score_lse(Q: np.ndarray, K: np.ndarray, lse: np.ndarray, scale: float = 0.0) -> np.ndarray:
    """Scores as a slice of a wider softmax: lse [n_q, h_q] is the natural-log normaliser of each query row."""
    Q = np.ascontiguousarray(Q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    lse = np.ascontiguousarray(lse, dtype=np.float64)
    n_q, h_q, d = Q.shape
    L, h_kv, d2 = K.shape
    if d != d2 or lse.shape != (n_q, h_q):
        raise ValueError("shape mismatch")
    out = np.empty((h_kv, L), dtype=np.float64)
    _check(_load().jqo_score_lse(n_q, h_q, h_kv, d, L, float(scale), Q, K, lse, out), "score_lse")
    return out


def score_tail(Q: np.ndarray, K: np.ndarray, K_tail: np.ndarray, scale: float = 0.0) -> np.ndarray:
    """Scores with the soft tokens' own keys K_tail [n_q, h_kv, d] in each row's softmax, causally (i' <= i)."""
    Q = np.ascontiguousarray(Q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    K_tail = np.ascontiguousarray(K_tail, dtype=np.uint16)
    n_q, h_q, d = Q.shape
    L, h_kv, d2 = K.shape
    if d != d2 or K_tail.shape != (n_q, h_kv, d):
        raise ValueError("shape mismatch")
    out = np.empty((h_kv, L), dtype=np.float64)
    _check(_load().jqo_score_tail(n_q, h_q, h_kv, d, L, float(scale), Q, K, K_tail, out), "score_tail")
    return out


def score_window(Q: np.ndarray, K: np.ndarray, scale: float = 0.0) -> np.ndarray:
    """Scores of a prompt under its own last n_q tokens (causal inside the window; the window's own positions get 0).
    Q [n_q,h_q,d], K [L,h_kv,d] uint16 bf16 bits with the window's keys as its last n_q rows -> [h_kv, L] float64."""
    Q = np.ascontiguousarray(Q, dtype=np.uint16)
    K = np.ascontiguousarray(K, dtype=np.uint16)
    n_q, h_q, d = Q.shape
    L, h_kv, d2 = K.shape
    if d != d2:
        raise ValueError("head dimension mismatch")
    out = np.empty((h_kv, L), dtype=np.float64)
    _check(_load().jqo_score_window(n_q, h_q, h_kv, d, L, float(scale), Q, K, out), "score_window")
    return out


def pool(scores: np.ndarray, pool_k: int) -> np.ndarray:
    """scores [h_kv, L] (or [L]) float64 -> pooled, same shape."""
    s = np.ascontiguousarray(scores, dtype=np.float64)
    flat = s.reshape(-1, s.shape[-1])
    out = np.empty_like(flat)
    for g in range(flat.shape[0]):
        _check(_load().jqo_pool(flat.shape[1], int(pool_k), flat[g], out[g]), "pool")
    return out.reshape(s.shape)


def select_topk(pooled: np.ndarray, B: int, keep_first: int = 0, keep_last: int = 0) -> np.ndarray:
    """pooled [h_kv, L] (or [L]) float64 -> idx [h_kv, B] (or [B]) int32, ascending.

    With keep_first / keep_last the first / last positions are kept regardless of their scores and
    count towards B."""
    p = np.ascontiguousarray(pooled, dtype=np.float64)
    flat = p.reshape(-1, p.shape[-1])
    out = np.empty((flat.shape[0], int(B)), dtype=np.int32)
    for g in range(flat.shape[0]):
        if keep_first or keep_last:
            _check(_load().jqo_select_topk_keep(flat.shape[1], int(B), int(keep_first), int(keep_last), flat[g], out[g]),
                   "select_topk_keep")
        else:
            _check(_load().jqo_select_topk(flat.shape[1], int(B), flat[g], out[g]), "select_topk")
    return out.reshape(p.shape[:-1] + (int(B),))


def compact(K: np.ndarray, V: np.ndarray, idx: np.ndarray):
    """K,V [L,h_kv,d] uint16, idx [h_kv,B] int32 -> K_out,V_out [B,h_kv,d] uint16."""
    K = np.ascontiguousarray(K, dtype=np.uint16)
    V = np.ascontiguousarray(V, dtype=np.uint16)
    idx = np.ascontiguousarray(idx, dtype=np.int32)
    L, h_kv, d = K.shape
    B = idx.shape[1]
    Ko = np.empty((B, h_kv, d), dtype=np.uint16)
    Vo = np.empty_like(Ko)
    _check(_load().jqo_compact(L, h_kv, d, B, K, V, idx, Ko, Vo), "compact")
    return Ko, Vo


def evict(Q, K, V, B: int, pool_k: int, scale: float = 0.0, lse=None, K_tail=None, keep_first: int = 0,
          keep_last: int = 0, window: bool = False):
    """One (layer, sequence): score -> pool -> top-B -> gather.  Returns a dict.

    With `lse` the scores are the slice-of-a-wider-softmax variant (score_lse), with `K_tail` the
    variant whose softmax also covers the soft tokens' own keys (score_tail)."""
    if window:  # the queries are the prompt's own last n_q tokens, which are always kept
        s = score_window(Q, K, scale)
        keep_last = max(keep_last, Q.shape[0])
    elif lse is not None:
        s = score_lse(Q, K, lse, scale)
    elif K_tail is not None:
        s = score_tail(Q, K, K_tail, scale)
    else:
        s = score(Q, K, scale)
    p = pool(s, pool_k)
    idx = select_topk(p, B, keep_first, keep_last)
    Ko, Vo = compact(K, V, idx)
    return {"scores": s, "pooled": p, "idx": idx, "K_out": Ko, "V_out": Vo}


def evict_batch(Q, K, V, cu_seqlens, budgets, pool_k: int, scale: float = 0.0, keep_first: int = 0, keep_last: int = 0,
                window: bool = False, layer_budgets=None):
    """Layers x ragged sequences, one problem at a time.

    Q [nl,n_seq,n_q,h_q,d], K/V [nl,T,h_kv,d] uint16.  Returns pooled [nl,h_kv,T],
    scores [nl,h_kv,T], idx [nl,h_kv,TB] (sequence-local), K_out/V_out [nl,TB,h_kv,d].
    """
    nl, T, h_kv, d = K.shape
    cu = [int(x) for x in cu_seqlens]
    cb = np.concatenate([[0], np.cumsum(budgets)]).astype(np.int64)
    TB = int(cb[-1])
    scores = np.empty((nl, h_kv, T)); pooled = np.empty((nl, h_kv, T))
    idx = np.empty((nl, h_kv, TB), dtype=np.int32)
    Ko = np.empty((nl, TB, h_kv, d), dtype=np.uint16); Vo = np.empty_like(Ko)
    for l in range(nl):
        for s in range(len(cu) - 1):
            # budgets that differ from layer to layer (the depth-dependent allocation of the PyramidKV baseline,
            # Section 5.1): layer l keeps layer_budgets[l][s] positions and fills only that many slots
            b = int(budgets[s]) if layer_budgets is None else int(layer_budgets[l][s])
            r = evict(Q[l, s], K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], b, pool_k, scale,
                      keep_first=keep_first, keep_last=keep_last, window=window)
            scores[l, :, cu[s]:cu[s + 1]] = r["scores"]
            pooled[l, :, cu[s]:cu[s + 1]] = r["pooled"]
            idx[l, :, cb[s]:cb[s] + b] = r["idx"]
            Ko[l, cb[s]:cb[s] + b] = r["K_out"]
            Vo[l, cb[s]:cb[s] + b] = r["V_out"]
    return {"scores": scores, "pooled": pooled, "idx": idx, "K_out": Ko, "V_out": Vo}


def stream_step(Q, K, V, pos, B: int, pool_k: int = 1, scale: float = 0.0, lse=None, keep_first: int = 0, keep_last: int = 0):
    """One eviction step during decoding on a cache that earlier steps have pruned (the paper names streaming
    eviction in the decoding phase as future work in its closing paragraph and defines nothing; the reading is the
    Section 4.3 step applied to the cache as it stands).

    K, V [rows, h_kv, d]: row b of head g is that head's own b-th cached row; pos [h_kv, rows] int: the token each
    row came from.  The soft-token queries Q score the cached rows (softmax over the cached rows alone, or with the
    supplied normalisers `lse`), the scores are pooled along the cache rows, the top B rows per head are kept (the
    first keep_first and last keep_last rows always), and K, V and pos are gathered.  Returns a dict with idx (row
    numbers), pooled, K_out, V_out and pos_out [h_kv, B]."""
    r = evict(Q, K, V, B, pool_k, scale, lse=lse, keep_first=keep_first, keep_last=keep_last)
    pos = np.asarray(pos)
    h_kv = K.shape[1]
    pos_out = np.empty((h_kv, B), dtype=np.int32)
    for g in range(h_kv):
        for b in range(B):
            pos_out[g, b] = pos[g, r["idx"][g, b]]
    r["pos_out"] = pos_out
    return r


def map_mse(score_a: np.ndarray, rows_a: float, score_b: np.ndarray, rows_b: float) -> np.ndarray:
    """Eq. 5 forward per KV head: mean over the prompt of (score_a/rows_a - score_b/rows_b)^2; scores [h_kv, L]."""
    a = np.ascontiguousarray(score_a, dtype=np.float64)
    b = np.ascontiguousarray(score_b, dtype=np.float64)
    if a.shape != b.shape or a.ndim != 2:
        raise ValueError("shape mismatch")
    out = np.empty(a.shape[0], dtype=np.float64)
    _check(_load().jqo_map_mse(a.shape[1], a.shape[0], float(rows_a), float(rows_b), a, b, out), "map_mse")
    return out


def hit_rate(idx_cur, idx_ref) -> float:
    """Critical-KV hit rate (Eq. 6): |I_cur & I_ref| / |I_ref| for two index sets."""
    a, b = set(int(x) for x in np.ravel(idx_cur)), set(int(x) for x in np.ravel(idx_ref))
    return len(a & b) / float(len(b))
