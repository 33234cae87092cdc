"""CPU-only checks of the C-ABI library: it loads, exports every declared symbol, and rejects
malformed arguments on the host before touching a GPU (no compute call is made here)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2509_10798_amd as jq
from paper_2509_10798_amd.binding import _CShape

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_header_symbols_are_exported():
    header = open(os.path.join(ROOT, "include", "jq.h")).read()
    declared = set(re.findall(r"\b(jq_[a-z_]+)\s*\(", header))
    assert declared == set(jq.EXPORTS)
    L = jq.lib()
    for name in declared:
        assert hasattr(L, name), name


def test_status_strings():
    for code in range(0, -8, -1):
        assert jq.status_string(code) and jq.status_string(code) != "unknown status"
    assert jq.status_string(5) == "unknown status"


def shape(**kw):
    base = dict(n_layers=1, seq_lens=[64], n_q=4, h_q=4, h_kv=2, d=128, pool_k=7, budgets=[8])
    base.update(kw)
    return jq.Shape(**base)


def ws_status(sh):
    try:
        jq.workspace_bytes(sh)
        return 0
    except jq.JQError as e:
        return e.status


def test_workspace_size_grows_with_problem():
    a = jq.workspace_bytes(shape())
    b = jq.workspace_bytes(shape(seq_lens=[4096], budgets=[8]))
    assert 0 < a < b and a % 256 == 0


@pytest.mark.parametrize("kw,code", [
    (dict(h_q=3), -2), (dict(pool_k=4), -2), (dict(pool_k=0), -2), (dict(n_q=0), -2), (dict(n_layers=0), -2),
    (dict(scale=-1.0), -2), (dict(scale=float("nan")), -2),
    (dict(d=64), -4), (dict(seq_lens=[8] * 129, budgets=[1] * 129), -4), (dict(h_q=1028, h_kv=257), -4),
    (dict(budgets=[0]), -3), (dict(budgets=[65]), -3),
    (dict(seq_lens=[64, 0], budgets=[8, 1]), -2),
    (dict(seq_lens=[2200000], h_q=8, h_kv=8, n_q=2), -4),      # one sequence's keys reach 4 GiB
    (dict(seq_lens=[2097000], h_q=8, h_kv=8, n_q=2), 0),       # ... and just below
    (dict(keep_first=-1), -2), (dict(keep_last=-3), -2),
    (dict(keep_first=5, keep_last=4), -3),                       # more always-kept positions than the budget
    (dict(seq_lens=[64, 64], budgets=[40, 8], keep_last=9), -3), # ... in any sequence
    (dict(keep_first=4, keep_last=4), 0),
    (dict(window=True), 0),                                      # 4 window tokens inside a budget of 8
    (dict(window=True, budgets=[3]), -3),                        # the window alone exceeds the budget
    (dict(window=True, keep_first=5), -3),
    (dict(window=True, seq_lens=[64, 3], budgets=[8, 3]), -2),   # a sequence shorter than its window
])
def test_shape_errors(kw, code):
    assert ws_status(shape(**kw)) == code


def test_null_and_alias_errors_come_before_any_launch():
    L = jq.lib()
    sh = shape()
    cs = sh.c_struct()
    n = ctypes.c_size_t()
    assert L.jq_workspace_bytes(None, ctypes.byref(n)) == -1
    assert L.jq_workspace_bytes(ctypes.byref(cs), None) == -1
    assert L.jq_score(ctypes.byref(cs), None, None, None, None, 0, None) == -1
    assert L.jq_evict(ctypes.byref(cs), None, None, None, None, None, None, None, None, 0, None) == -1
    # fake, never dereferenced device addresses: validation is pure pointer arithmetic
    big = 1 << 40
    Q, K, V, Ko, Vo, ws = big, big + (1 << 30), big + (2 << 30), big + (3 << 30), big + (4 << 30), big + (5 << 30)
    need = jq.workspace_bytes(sh)
    assert L.jq_evict(ctypes.byref(cs), Q, K, V, Ko, Vo, None, None, ws, need - 1, None) == -5     # too small
    assert L.jq_evict(ctypes.byref(cs), Q, K, V, Ko, Vo, None, None, ws + 4, need, None) == -5     # misaligned
    assert L.jq_evict(ctypes.byref(cs), Q, K, V, K + 256, Vo, None, None, ws, need, None) == -6    # K_out inside K
    assert L.jq_evict(ctypes.byref(cs), Q, K, V, Ko, Ko, None, None, ws, need, None) == -6         # outputs overlap
    assert L.jq_evict(ctypes.byref(cs), Q + 2, K, V, Ko, Vo, None, None, ws, need, None) == -4     # misaligned Q
    lse = big + (6 << 30)
    assert L.jq_score_lse(ctypes.byref(cs), Q, K, None, Ko, ws, need, None) == -1                  # lse required
    assert L.jq_evict_lse(ctypes.byref(cs), Q, K, V, None, Ko, Vo, None, None, ws, need, None) == -1
    assert L.jq_evict_lse(ctypes.byref(cs), Q, K, V, lse + 2, Ko, Vo, None, None, ws, need, None) == -4
    assert L.jq_evict_lse(ctypes.byref(cs), Q, K, V, Ko, Ko, Vo, None, None, ws, need, None) == -6   # lse inside K_out
    kt = big + (7 << 30)
    assert L.jq_score_tail(ctypes.byref(cs), Q, K, None, Ko, ws, need, None) == -1                 # soft-token keys required
    assert L.jq_score_tail(ctypes.byref(cs), Q, K, kt + 2, Ko, ws, need, None) == -4
    assert L.jq_score_tail(ctypes.byref(cs), Q, K, ws + 512, Ko, ws, need, None) == -6             # keys inside the workspace
    cs_w = shape(window=True).c_struct()                                                           # the window's keys are in K already
    assert L.jq_score_tail(ctypes.byref(cs_w), Q, K, kt, Ko, ws, need, None) == -2
    assert L.jq_evict_tail(ctypes.byref(cs_w), Q, K, V, kt, Ko, Vo, None, None, ws, need, None) == -2
    assert L.jq_evict_tail(ctypes.byref(cs), Q, K, V, None, Ko, Vo, None, None, ws, need, None) == -1
    assert L.jq_evict_tail(ctypes.byref(cs), Q, K, V, Vo, Ko, Vo, None, None, ws, need, None) == -6   # keys inside V_out
    assert L.jq_evict_traced(ctypes.byref(cs), Q, K, V, Ko, Vo, None, None, ws, need, None, None, 10) == -1
    assert L.jq_hit_rate(ctypes.byref(cs), Ko, None, None, Vo, None) == -1
    assert L.jq_hit_rate(ctypes.byref(cs), Ko, Vo, None, Ko + 8, None) == -6                       # rate inside idx_cur
    too_many = (ctypes.c_int32 * sh.n_seq)(*([10 ** 9] * sh.n_seq))
    assert L.jq_hit_rate(ctypes.byref(cs), Ko, Vo, too_many, ws, None) == -3                       # reference budget > L
    assert L.jq_map_mse(ctypes.byref(cs), K, 1.0, None, 1.0, ws, None) == -1
    assert L.jq_map_mse(ctypes.byref(cs), K, 0.0, V, 1.0, ws, None) == -2                          # no rows
    assert L.jq_map_mse(ctypes.byref(cs), K, 1.0, V, 1.0, K + 64, None) == -6                      # result inside an input
    # the same objective from the two query sets
    nf = ctypes.c_size_t()
    assert L.jq_map_mse_fused_workspace_bytes(ctypes.byref(cs), 70, ctypes.byref(nf)) == 0 and nf.value > need
    assert L.jq_map_mse_fused_workspace_bytes(ctypes.byref(cs), 0, ctypes.byref(nf)) == -2          # no response tokens
    assert L.jq_map_mse_fused_workspace_bytes(ctypes.byref(cs), 70, None) == -1
    L.jq_map_mse_fused_workspace_bytes(ctypes.byref(cs), 70, ctypes.byref(nf))
    fused = lambda qa=Q, qb=Q + (1 << 22), k=K, out=V, w=ws, wb=None: L.jq_map_mse_fused(
        ctypes.byref(cs), qa, qb, 70, k, out, w, nf.value if wb is None else wb, None)
    assert fused(qb=None) == -1 and fused(out=None) == -1 and fused(w=None) == -1
    assert fused(wb=nf.value - 1) == -5
    assert fused(out=K + 64) == -6                                                                  # result inside the keys
    assert fused(qb=ws + 256) == -6                                                                 # queries inside the workspace
    assert fused(qa=Q + 2) == -4                                                                    # misaligned queries
    assert L.jq_copy_probe(K, K + 64, 1024, None) == -6 and L.jq_copy_probe(K, Ko, 24, None) == -2
    assert L.jq_compact(ctypes.byref(cs), K, V, ws, V, Vo, None) == -6
    assert L.jq_pool(ctypes.byref(cs), K, K, None) == -6
    n_in = ctypes.c_size_t()
    assert L.jq_compact_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(n_in)) == 0
    assert n_in.value == 2 * 8 * 2 * 128 * 2                                                       # K and V rows of the budget
    assert L.jq_compact_inplace_workspace_bytes(ctypes.byref(cs), None) == -1
    assert L.jq_compact_inplace(ctypes.byref(cs), K, V, Ko, None, n_in.value, None) == -1
    assert L.jq_compact_inplace(ctypes.byref(cs), K, V, Ko, ws, n_in.value - 1, None) == -5
    assert L.jq_evict_stream(ctypes.byref(cs), Q, K, V, None, None, Ko, Vo, ws + (1 << 29), None, None, ws, need, None) == -1   # positions required
    assert L.jq_evict_stream(ctypes.byref(cs), Q, K, V, lse, None, Ko, Vo, None, None, None, ws, need, None) == -1
    assert L.jq_evict_stream(ctypes.byref(cs), Q, K, V, lse, None, Ko, Vo, Ko + 64, None, None, ws, need, None) == -6          # pos_out inside K_out
    assert L.jq_evict_stream(ctypes.byref(cs), Q, K, V, lse + 2, None, Ko, Vo, kt, None, None, ws, need, None) == -4           # misaligned positions
    n_ev = ctypes.c_size_t()  # (paged in-place eviction: checked in test_paged_descriptor_errors)
    assert L.jq_evict_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(n_ev)) == 0 and n_ev.value >= need + n_in.value
    assert L.jq_evict_inplace_workspace_bytes(ctypes.byref(cs), None) == -1
    assert L.jq_evict_inplace(ctypes.byref(cs), Q, None, V, None, None, None, ws, n_ev.value, None) == -1
    assert L.jq_evict_inplace(ctypes.byref(cs), Q, K, V, None, None, None, ws, need, None) == -5              # no room for the staged rows
    assert L.jq_evict_inplace(ctypes.byref(cs), Q, K, K + 512, None, None, None, ws, n_ev.value, None) == -6  # V inside K
    assert L.jq_evict_inplace(ctypes.byref(cs), K + 64, K, V, None, None, None, ws, n_ev.value, None) == -6   # Q inside K (which is written)
    assert L.jq_evict_inplace(ctypes.byref(cs), Q, K, V, None, Ko, Ko + 16, ws, n_ev.value, None) == -6       # the two outputs overlap
    assert L.jq_compact_inplace(ctypes.byref(cs), K, K + 256, Ko, ws, n_in.value, None) == -6      # V inside K
    assert L.jq_compact_inplace(ctypes.byref(cs), K, V, K + 512, ws, n_in.value, None) == -6       # idx inside K
    assert L.jq_compact_inplace(ctypes.byref(cs), K, V, Ko, V + 1024, n_in.value, None) == -6      # staging inside V
    class _T:                                   # stands in for a device tensor: only its address is marshalled
        def __init__(self, addr): self.addr = addr
        def data_ptr(self): return self.addr
    cs_lb = shape(layer_budgets=_T(big + (10 << 30) + 2)).c_struct()
    assert L.jq_evict(ctypes.byref(cs_lb), Q, K, V, Ko, Vo, None, None, ws, need, None) == -4      # misaligned per-layer budgets
    cs_lb = shape(layer_budgets=_T(Ko + 64)).c_struct()
    assert L.jq_evict(ctypes.byref(cs_lb), Q, K, V, Ko, Vo, None, None, ws, need, None) == -6      # ... inside an output
    assert L.jq_compact(ctypes.byref(cs_lb), K, V, ws, Ko, Vo, None) == -6
    cs2 = shape(budgets=None).c_struct()
    assert L.jq_compact(ctypes.byref(cs2), K, V, ws, Ko, Vo, None) == -1                           # budgets required
    bad = _CShape(1, 1, 4, 4, 2, 128, 7, 0.0, ctypes.cast(None, ctypes.POINTER(ctypes.c_int32)),
                  ctypes.cast(None, ctypes.POINTER(ctypes.c_int32)))
    assert L.jq_pool(ctypes.byref(bad), K, V, None) == -1                                          # cu_seqlens NULL


def test_cu_seqlens_must_start_at_zero():
    L = jq.lib()
    cu = np.array([1, 65], dtype=np.int32); bud = np.array([8], dtype=np.int32)
    i32p = ctypes.POINTER(ctypes.c_int32)
    cs = _CShape(1, 1, 4, 4, 2, 128, 7, 0.0, cu.ctypes.data_as(i32p), bud.ctypes.data_as(i32p))
    n = ctypes.c_size_t()
    assert L.jq_workspace_bytes(ctypes.byref(cs), ctypes.byref(n)) == -2


def test_paged_descriptor_errors_come_before_any_launch():
    from paper_2509_10798_amd.binding import _CPages
    L = jq.lib()
    sh = shape(seq_lens=[300, 64], budgets=[8, 8])
    cs = sh.c_struct()
    need = jq.workspace_bytes(sh)
    big = 1 << 40
    Q, K, V, Ko, Vo, ws, tab, sc = (big + (i << 30) for i in range(8))

    def score(pg, table=tab, k=K):
        cp = _CPages(*pg, table)
        return L.jq_score_paged(ctypes.byref(cs), ctypes.byref(cp), Q, k, None, sc, ws, need, None)

    def evict(pg, table=tab, ko=Ko, out=None):
        cp = _CPages(*pg, table)
        co = ctypes.byref(_CPages(*out)) if out is not None else None
        return L.jq_evict_paged(ctypes.byref(cs), ctypes.byref(cp), co, Q, K, V, None, ko, Vo, None, None, ws, need, None)

    assert L.jq_score_paged(ctypes.byref(cs), None, Q, K, None, sc, ws, need, None) == -1          # no descriptor
    assert score((64, 16, 5), table=None) == -1                                                    # no block table
    assert score((48, 16, 8)) == -2 and score((16, 32, 32)) == -2 and score((1 << 17, 4, 1)) == -2  # page size
    assert score((64, 0, 5)) == -2 and score((64, 16, 0)) == -2
    assert score((64, 16, 4)) == -2                                     # 300 tokens need 5 pages of 64
    assert score((65536, 1 << 20, 5)) == -4                             # pool beyond the 32-bit offset range
    assert score((64, 16, 5), table=tab + 2) == -4                      # misaligned table
    assert score((64, 16, 5), table=ws + 1024) == -6                    # table inside the workspace (aliasing is checked
                                                                        # last, so this descriptor passed everything else)
    assert evict((64, 16, 5), ko=K + 256) == -6                         # K_out inside the pool
    assert evict((64, 16, 5), table=Ko) == -6                           # table inside an output
    otab = big + (9 << 30)
    assert evict((64, 16, 5), out=(16, 4, 1, None)) == -1               # output descriptor without a table
    assert evict((64, 16, 5), out=(24, 4, 1, otab)) == -2               # page size not a power of two
    assert evict((64, 16, 5), out=(4, 4, 1, otab)) == -2                # budgets of 8 need 2 pages of 4
    assert evict((64, 16, 5), out=(4, 4, 2, otab + 2)) == -4            # misaligned output table
    assert evict((64, 16, 5), out=(4, 4, 2, Ko + 64)) == -6             # output table inside the output pool
    assert evict((64, 16, 5), out=(4, 1 << 20, 2, otab), ko=K - (1 << 29)) == -6   # a large output pool reaches into K

    # the same eviction with the kept rows written into the input's own pools
    def inplace(pg, out, table=tab, q=Q, wsb=None):
        cp, co = _CPages(*pg, table), _CPages(*out)
        n = ctypes.c_size_t()
        assert L.jq_evict_paged_inplace_workspace_bytes(ctypes.byref(cs), ctypes.byref(cp), ctypes.byref(n)) == 0 and n.value > need
        return L.jq_evict_paged_inplace(ctypes.byref(cs), ctypes.byref(cp), ctypes.byref(co), q, K, V, None, None, None, ws,
                                        n.value if wsb is None else wsb, None)
    assert inplace((64, 16, 5), (32, 16, 1, otab)) == -2                # the output pages are pages of the same pool: same page size
    assert inplace((64, 16, 5), (64, 8, 1, otab)) == -2                 # ... and same pool size
    assert inplace((64, 16, 5), (64, 16, 1, None)) == -1
    assert inplace((64, 16, 5), (64, 16, 1, otab), wsb=need) == -5      # no room for the staged rows and the page map
    assert inplace((64, 16, 5), (64, 16, 1, otab), q=K + 64) == -6      # Q inside a pool that is written
    assert inplace((64, 16, 5), (64, 16, 1, ws + 256)) == -6            # output table inside the workspace


def test_knobs_are_read_once_and_again_on_request(monkeypatch):
    # the environment is not consulted by ordinary calls: a knob set after the first call has no effect until
    # jq_reload_knobs; the per-workgroup statistics area of the workspace shows which wave split is planned
    sh = shape(seq_lens=[8192], budgets=[8])
    jq.reload_knobs()
    base = jq.workspace_bytes(sh)
    monkeypatch.setenv("JQ_CHUNK_KEYS", "32")
    assert jq.workspace_bytes(sh) == base
    jq.reload_knobs()
    assert jq.workspace_bytes(sh) > base          # one wave per 32 keys: more workgroups, more partial statistics
    monkeypatch.setenv("JQ_CHUNK_KEYS", "33")     # not a multiple of the tile: ignored
    jq.reload_knobs()
    assert jq.workspace_bytes(sh) == base
    monkeypatch.undo()
    jq.reload_knobs()
    assert jq.workspace_bytes(sh) == base
