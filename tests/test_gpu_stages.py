"""GPU parity, stage by stage, through the C ABI: each HIP stage against the matching oracle
stage on identical seeded inputs, at sizes that span several tiles, chunks and ragged tails."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok, assert_kept_set_ok_keep, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import f32_to_bf16_bits, make_workload

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def run_score_case(n_layers, seq_lens, n_q, h_q, h_kv, seed, scale=0.0, spread=1.0):
    torch = torch_()
    rng = np.random.default_rng(seed)
    T, d = sum(seq_lens), 128
    Q = f32_to_bf16_bits(rng.standard_normal((n_layers, len(seq_lens), n_q, h_q, d)).astype(np.float32) * spread)
    K = f32_to_bf16_bits(rng.standard_normal((n_layers, T, h_kv, d)).astype(np.float32) * spread)
    sh = jq.Shape(n_layers=n_layers, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv, scale=scale)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    G = h_q // h_kv
    worst = 0.0
    for l in range(n_layers):
        for s, L in enumerate(seq_lens):
            ref = oracle.score(Q[l, s], K[l, cu[s]:cu[s + 1]], scale)
            seg = got[l, :, cu[s]:cu[s + 1]]
            worst = max(worst, assert_scores_close(seg, ref, n_q * G / L, "layer %d seq %d" % (l, s)))
            np.testing.assert_allclose(seg.sum(axis=1), n_q * G, rtol=1e-4)
    return worst


@pytest.mark.parametrize("n_layers,seq_lens,n_q,h_q,h_kv", [
    (1, [2048], 16, 8, 2),            # the tiny named workload's shape: 64 query rows, 2 row tiles
    (1, [1], 4, 4, 2),                # a single key
    (1, [31], 4, 4, 2),               # less than one tile
    (1, [33], 8, 8, 2),               # one full tile and a one-key tail
    (1, [1000], 32, 32, 8),           # 128 query rows (4 row tiles), ragged tail
    (2, [517, 64, 3001], 10, 8, 2),   # layers x ragged batch, 40 query rows (padded row tile)
    (1, [700], 40, 8, 2),             # 160 query rows: two passes over K
    (1, [300], 3, 6, 6),              # no grouping (G = 1), 3 query rows
    (1, [400, 77], 11, 6, 2),         # three query heads per KV head (not a power of two), 33 query rows
])
def test_score_matches_oracle(n_layers, seq_lens, n_q, h_q, h_kv):
    print("score case", n_layers, seq_lens, n_q, h_q, h_kv, flush=True)
    worst = run_score_case(n_layers, seq_lens, n_q, h_q, h_kv, seed=11)
    assert worst < 1.0


def test_score_with_peaked_softmax_and_custom_scale():
    # large logits: exercises the running-maximum rescaling and the split of -beta/c
    print("score peaked", flush=True)
    run_score_case(1, [1500], 16, 8, 2, seed=12, scale=0.35, spread=1.5)


@pytest.mark.parametrize("alpha,where,chunk", [(9.0, 3500, 1024), (9.0, 3, 1024), (7.0, 4999, 1024), (30.0, 2048, 1024), (9.0, 31, 1024),
                                               (9.0, 3500, None), (30.0, 4100, None)])
def test_score_with_one_dominant_key(knobs, alpha, where, chunk):
    # The statistics pass keeps the first tile's maximum as the softmax offset of a query row.  A key that
    # aligns with a query row, planted late, exceeds that offset by more than fp32 exp2 can hold
    # (alpha >= 9: the wave must fall back to the running maximum), by a large but representable factor
    # (alpha = 7), or sits in the first tile itself, so that every later term underflows.  chunk None: no knob at
    # all -- at the default work split this sequence gets 79 waves of two tiles each, and the planted key sits in
    # the second tile of its wave, so the fallback is reached the way a caller would reach it.
    print("score dominant key", alpha, where, chunk, flush=True)
    torch = torch_()
    if chunk:
        knobs(JQ_CHUNK_KEYS=str(chunk))                    # long waves: many tiles after the first
    rng = np.random.default_rng(15)
    L, n_q, h_q, h_kv, d = 5000, 16, 8, 2, 128
    Qf = rng.standard_normal((1, 1, n_q, h_q, d)).astype(np.float32)
    Kf = rng.standard_normal((1, L, h_kv, d)).astype(np.float32)
    Kf[0, where, 0] = alpha * Qf[0, 0, 5, 1]               # head 0 of K <- query row (token 5, head 1 of group 0)
    Kf[0, where, 1] = alpha * Qf[0, 0, 2, 6]
    Q, K = f32_to_bf16_bits(Qf), f32_to_bf16_bits(Kf)
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=n_q, h_q=h_q, h_kv=h_kv)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    got = got.cpu().numpy()[0]
    ref = oracle.score(Q[0, 0], K[0])
    assert np.isfinite(got).all()
    assert_scores_close(got, ref, n_q * (h_q // h_kv) / L, "dominant key")
    np.testing.assert_allclose(got.sum(axis=1), n_q * (h_q // h_kv), rtol=1e-4)
    assert ref[0, where] > 0.99 and got[0, where] > 0.99   # that query row's whole mass sits on the planted key


def test_score_several_chunks_per_sequence(knobs):
    # force 64-key chunks so that one sequence is split over many waves and partial statistics merge
    print("score chunked", flush=True)
    knobs(JQ_CHUNK_KEYS="64")
    run_score_case(1, [1111, 95], 16, 8, 2, seed=13)


def test_score_with_hundreds_of_partial_statistics(knobs):
    # a sequence cut into more than 256 waves leaves more partials than the second pass merges by itself: the
    # separate merge launch runs (here forced by 64-key chunks)
    print("score with a merge launch", flush=True)
    knobs(JQ_CHUNK_KEYS="64")
    run_score_case(1, [20000, 300], 16, 8, 2, seed=14)


def test_score_is_deterministic():
    torch = torch_()
    w = make_workload(1)
    Q, K, _ = w.assemble()
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv)
    Qd, Kd = to_dev_bf16(Q), to_dev_bf16(K)
    a = jq.score(sh, Qd, Kd).clone()
    b = jq.score(sh, Qd, Kd)
    torch.cuda.synchronize()
    assert torch.equal(a, b)


@pytest.mark.parametrize("seq_lens,k", [([1], 7), ([5], 7), ([4096], 7), ([100, 3, 2000], 7), ([777], 1), ([777], 5), ([50], 31)])
def test_pool_matches_oracle(seq_lens, k):
    torch = torch_()
    rng = np.random.default_rng(21)
    T, h_kv, nl = sum(seq_lens), 3, 2
    x = rng.random((nl, h_kv, T)).astype(np.float32) * np.float32(3.0)
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, pool_k=k)
    got = jq.pool(sh, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for s in range(len(seq_lens)):
        ref = oracle.pool(x[:, :, cu[s]:cu[s + 1]].astype(np.float64), k)
        np.testing.assert_allclose(got[:, :, cu[s]:cu[s + 1]], ref, rtol=2e-6, atol=0)


def run_select_case(x, seq_lens, budgets, keep_first=0, keep_last=0):
    torch = torch_()
    nl, h_kv, T = x.shape
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=budgets, keep_first=keep_first,
                  keep_last=keep_last)
    idx = jq.select_topk(sh, torch.from_numpy(x).cuda())
    torch.cuda.synchronize()
    idx = idx.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)]); cb = np.concatenate([[0], np.cumsum(budgets)])
    for s in range(len(seq_lens)):
        ref = oracle.select_topk(x[:, :, cu[s]:cu[s + 1]].astype(np.float64), budgets[s], keep_first, keep_last)
        np.testing.assert_array_equal(idx[:, :, cb[s]:cb[s + 1]], ref)


@pytest.mark.parametrize("seq_lens,budgets", [([1], [1]), ([7], [7]), ([100], [1]), ([5000], [256]),
                                               ([4097, 33, 9000], [512, 33, 1]), ([70000], [2048]),
                                               ([300000], [2048]),    # bitmaps beyond 64 KiB of LDS: the raised limit
                                               ([700000], [3000])])   # too long for the LDS bitmaps: streaming path
def test_select_is_exact_on_random_scores(seq_lens, budgets):
    print("select case", seq_lens, budgets, flush=True)
    rng = np.random.default_rng(31)
    x = rng.random((2, 3, sum(seq_lens))).astype(np.float32)
    run_select_case(x, seq_lens, budgets)


def test_select_with_heavy_ties_and_special_values():
    rng = np.random.default_rng(32)
    x = np.round(rng.random((1, 4, 6000)).astype(np.float32), 2)       # ~100 distinct values
    x[0, 1] = 0.5                                                      # all equal -> first B positions
    x[0, 2, ::3] = 0.0; x[0, 2, 1::7] = -0.0                           # signed zeros compare equal
    x[0, 3] = -x[0, 3]                                                 # negative scores are legal input
    run_select_case(x, [6000], [1000])
    run_select_case(x, [2500, 3500], [2500, 17])                       # B = L for the first sequence


def test_select_narrow_value_range():
    # all values inside one level-1 and one level-2 radix bin: only the last 10 bits differ
    base = np.float32(1.0).view(np.uint32)
    rng = np.random.default_rng(33)
    bits = (base + rng.integers(0, 1024, (1, 2, 9000)).astype(np.uint32)).astype(np.uint32)
    run_select_case(bits.view(np.float32), [9000], [700])


def test_select_wide_dynamic_range():
    # a peaked softmax spreads scores over hundreds of octaves, far below any block's histogram window;
    # with a large budget the threshold itself lies in that far tail
    rng = np.random.default_rng(34)
    x = np.exp(-np.abs(rng.standard_normal((2, 3, 20000))) * 60.0).astype(np.float32)   # down to denormals and 0
    x[1, 0, 5000:9000] = 0.0
    run_select_case(x, [20000], [64])
    run_select_case(x, [20000], [15000])
    run_select_case(x, [12000, 8000], [9000, 100])


@pytest.mark.parametrize("seq_lens,budgets,kf,kl", [
    ([5000], [256], 4, 32), ([5000], [36], 4, 32),            # the forced positions fill the budget exactly
    ([100], [10], 0, 10), ([100], [10], 10, 0), ([7], [7], 3, 4),
    ([4097, 40, 9000], [512, 40, 33], 1, 32),                  # ragged batch; a sequence kept whole; one nearly all forced
    ([70000], [2048], 16, 1000),
    ([700000], [3000], 4, 64),                                 # streaming path
])
def test_select_with_always_kept_ends(seq_lens, budgets, kf, kl):
    # sinks and local window of the Section 5.1 baselines: kept whatever they score, counted in the budget
    rng = np.random.default_rng(35)
    x = rng.random((2, 3, sum(seq_lens))).astype(np.float32)
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for s in range(len(seq_lens)):                             # make the forced positions the WORST candidates
        x[:, :, cu[s]:cu[s] + kf] = 0.0
        x[:, :, cu[s + 1] - kl:cu[s + 1]] = -1.0
    run_select_case(x, seq_lens, budgets, kf, kl)


def test_select_with_always_kept_ends_and_ties():
    rng = np.random.default_rng(36)
    x = np.round(rng.random((1, 4, 6000)).astype(np.float32), 2)
    x[0, 1] = 0.5                                              # all equal: forced ends, then the lowest free positions
    x[0, 2, :50] = 2.0                                         # forced positions that would have won anyway
    run_select_case(x, [6000], [1000], 8, 100)
    run_select_case(x, [2500, 3500], [2500, 120], 8, 100)


def test_compact_is_bit_exact():
    torch = torch_()
    rng = np.random.default_rng(41)
    nl, seq_lens, budgets, h_kv, d = 2, [300, 41], [64, 41], 4, 128
    T, TB = sum(seq_lens), sum(budgets)
    K = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    V = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    idx = np.empty((nl, h_kv, TB), dtype=np.int32)
    cu = np.concatenate([[0], np.cumsum(seq_lens)]); cb = np.concatenate([[0], np.cumsum(budgets)])
    for l in range(nl):
        for g in range(h_kv):
            for s in range(2):
                idx[l, g, cb[s]:cb[s + 1]] = np.sort(rng.choice(seq_lens[s], budgets[s], replace=False))
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=budgets)
    Ko, Vo = jq.compact(sh, to_dev_bf16(K), to_dev_bf16(V), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    Ko, Vo = from_dev_bf16(Ko), from_dev_bf16(Vo)
    for l in range(nl):
        for s in range(2):
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Ko[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo[l, cb[s]:cb[s + 1]], rv)


@pytest.mark.parametrize("seq_lens,budgets,mode", [
    ([3000], [500], "random"),            # sources on both sides of the overwritten front
    ([3000], [500], "front"),             # every source lies inside the front: all rows are staged
    ([3000], [500], "back"),              # no source inside the front
    ([900, 40, 2000], [300, 40, 700], "random"),   # a later sequence's rows land on an earlier sequence's sources
    ([64], [64], "random"),               # everything kept: a permutation-free identity
])
def test_compact_inplace_matches_out_of_place_gather(seq_lens, budgets, mode):
    torch = torch_()
    rng = np.random.default_rng(43)
    nl, h_kv, d = 2, 3, 128
    T, TB = sum(seq_lens), sum(budgets)
    K = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    V = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    idx = np.empty((nl, h_kv, TB), dtype=np.int32)
    cb = np.concatenate([[0], np.cumsum(budgets)]); cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for l in range(nl):
        for g in range(h_kv):
            for s, (L, B) in enumerate(zip(seq_lens, budgets)):
                if mode == "front":
                    pick = np.arange(B)
                elif mode == "back":
                    pick = np.arange(L - B, L)
                else:
                    pick = np.sort(rng.choice(L, size=B, replace=False))
                idx[l, g, cb[s]:cb[s + 1]] = pick
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=budgets)
    Kd, Vd = to_dev_bf16(K), to_dev_bf16(V)
    jq.compact_inplace(sh, Kd, Vd, torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    Kh, Vh = from_dev_bf16(Kd), from_dev_bf16(Vd)
    for l in range(nl):
        for s in range(len(seq_lens)):
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Kh[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vh[l, cb[s]:cb[s + 1]], rv)
    np.testing.assert_array_equal(Kh[:, TB:], K[:, TB:])        # the rest of the cache is untouched
    np.testing.assert_array_equal(Vh[:, TB:], V[:, TB:])


def test_compact_inplace_with_layer_dependent_budgets():
    torch = torch_()
    rng = np.random.default_rng(44)
    nl, h_kv, d, seq_lens, cap, lb = 2, 2, 128, [400, 300], [100, 50], [[100, 50], [30, 1]]
    T, TB = sum(seq_lens), sum(cap)
    K = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    V = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    idx = np.zeros((nl, h_kv, TB), dtype=np.int32)
    cb = np.concatenate([[0], np.cumsum(cap)]); cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for l in range(nl):
        for g in range(h_kv):
            for s in range(2):
                idx[l, g, cb[s]:cb[s] + lb[l][s]] = np.sort(rng.choice(seq_lens[s], size=lb[l][s], replace=False))
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=cap,
                  layer_budgets=torch.tensor(lb, dtype=torch.int32, device="cuda"))
    Kd, Vd = to_dev_bf16(K), to_dev_bf16(V)
    jq.compact_inplace(sh, Kd, Vd, torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    Kh, Vh = from_dev_bf16(Kd), from_dev_bf16(Vd)
    for l in range(nl):
        for s in range(2):
            b = lb[l][s]
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], np.ascontiguousarray(idx[l, :, cb[s]:cb[s] + b]))
            np.testing.assert_array_equal(Kh[l, cb[s]:cb[s] + b], rk)
            np.testing.assert_array_equal(Vh[l, cb[s]:cb[s] + b], rv)
            np.testing.assert_array_equal(Kh[l, cb[s] + b:cb[s + 1]], K[l, cb[s] + b:cb[s + 1]])   # unused slots keep their rows
    np.testing.assert_array_equal(Kh[:, TB:], K[:, TB:])


def test_sink_and_recent_window_retention_through_compact():
    # position-based retention (attention sinks + recent window, the StreamingLLM baseline of Section 5.1)
    # needs no scores: the caller writes the positions and jq_compact prunes the cache
    torch = torch_()
    rng = np.random.default_rng(42)
    nl, seq_lens, h_kv, d, sink, recent = 2, [500, 90], 4, 128, 4, 28
    budgets = [sink + recent] * 2
    T = sum(seq_lens)
    K = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    V = rng.integers(0, 65536, (nl, T, h_kv, d)).astype(np.uint16)
    idx = np.empty((nl, h_kv, sum(budgets)), dtype=np.int32)
    for s, L in enumerate(seq_lens):
        idx[:, :, s * 32:(s + 1) * 32] = np.concatenate([np.arange(sink), np.arange(L - recent, L)])
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=budgets)
    Ko, Vo = jq.compact(sh, to_dev_bf16(K), to_dev_bf16(V), torch.from_numpy(idx).cuda())
    torch.cuda.synchronize()
    Ko, Vo = from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for s, L in enumerate(seq_lens):
        seg = K[:, cu[s]:cu[s + 1]]
        np.testing.assert_array_equal(Ko[:, s * 32:s * 32 + sink], seg[:, :sink])
        np.testing.assert_array_equal(Ko[:, s * 32 + sink:(s + 1) * 32], seg[:, L - recent:])
        np.testing.assert_array_equal(Vo[:, s * 32 + sink:(s + 1) * 32], V[:, cu[s]:cu[s + 1]][:, L - recent:])


def test_layer_dependent_budgets_by_one_call_per_layer():
    # budgets that shrink with depth (the pyramid-shaped allocation among the Section 5.1 baselines):
    # budgets are uniform over the layers of one call, so such a schedule is one call per layer
    torch = torch_()
    w = make_workload(1, seq_lens=[1200], budget=[300], n_layers=3)
    Q, K, V = w.assemble()
    for layer, B in enumerate([300, 180, 60]):
        sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=[B])
        Ko, Vo, idx, pooled = jq.evict(sh, to_dev_bf16(Q[layer:layer + 1]), to_dev_bf16(K[layer:layer + 1]),
                                       to_dev_bf16(V[layer:layer + 1]))
        torch.cuda.synchronize()
        r = oracle.evict(Q[layer, 0], K[layer], V[layer], B, w.pool_k)
        for g in range(w.h_kv):
            assert_kept_set_ok(r["pooled"][g], r["idx"][g], idx[0, g].cpu().numpy(), "layer %d head %d" % (layer, g))
        rk, rv = oracle.compact(K[layer], V[layer], np.ascontiguousarray(idx[0].cpu().numpy()))
        np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
        np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)


def test_evict_with_always_kept_ends():
    # the fused call with attention sinks and a recent window forced into the kept set
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 700], budget=[200, 64], n_layers=2)
    Q, K, V = w.assemble()
    kf, kl = 4, 32
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets,
                  keep_first=kf, keep_last=kl)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd)
    i1 = jq.select_topk(sh, pooled)
    torch.cuda.synchronize()
    assert torch.equal(idx, i1)
    ref = oracle.evict_batch(Q, K, V, w.cu_seqlens, w.budgets, w.pool_k, keep_first=kf, keep_last=kl)
    pooled_h, idx_h = pooled.cpu().numpy(), idx.cpu().numpy()
    Ko_h, Vo_h = from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(2):
        for s in range(2):
            L = w.seq_lens[s]
            # the reported scores are the plain pooled scores: forcing changes the kept set only
            assert_scores_close(pooled_h[l, :, cu[s]:cu[s + 1]], ref["pooled"][l, :, cu[s]:cu[s + 1]], w.n_q * w.group / L)
            for g in range(w.h_kv):
                assert_kept_set_ok_keep(ref["pooled"][l, g, cu[s]:cu[s + 1]], ref["idx"][l, g, cb[s]:cb[s + 1]],
                                        idx_h[l, g, cb[s]:cb[s + 1]], kf, kl, "l%d s%d g%d" % (l, s, g))
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx_h[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s + 1]], rv)
    # the forced window really changes the outcome here: without it some of those rows are dropped
    sh0 = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    idx0 = jq.evict(sh0, Qd, Kd, Vd)[2]
    torch.cuda.synchronize()
    assert not torch.equal(idx0, idx)


def test_layer_dependent_budgets_in_one_call():
    # the same schedule as one fused call: `budgets` gives every sequence's largest budget (and the output layout),
    # a device array the budget of every (layer, sequence); slots beyond a layer's own budget stay untouched
    torch = torch_()
    seq_lens, cap, lb = [1200, 500], [300, 100], [[300, 100], [180, 64], [60, 7]]
    w = make_workload(1, seq_lens=seq_lens, budget=cap, n_layers=3)
    Q, K, V = w.assemble()
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    lb_d = torch.tensor(lb, dtype=torch.int32, device="cuda")
    sh = jq.Shape(n_layers=3, seq_lens=seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=cap,
                  layer_budgets=lb_d)
    TB = sum(cap)
    idx = torch.full((3, w.h_kv, TB), -7, dtype=torch.int32, device="cuda")
    Ko = torch.full((3, TB, w.h_kv, w.d), 1.5, dtype=torch.bfloat16, device="cuda"); Vo = Ko.clone()
    jq.evict(sh, Qd, Kd, Vd, K_out=Ko, V_out=Vo, idx_out=idx)
    # stage by stage as well
    pooled = jq.pool(sh, jq.score(sh, Qd, Kd))
    idx2 = torch.full_like(idx, -7)
    jq.select_topk(sh, pooled, idx=idx2)
    Ko2 = torch.full_like(Ko, 1.5); Vo2 = Ko2.clone()
    jq.compact(sh, Kd, Vd, idx2, K_out=Ko2, V_out=Vo2)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(Ko.view(torch.int16), Ko2.view(torch.int16))
    assert torch.equal(Vo.view(torch.int16), Vo2.view(torch.int16))
    ref = oracle.evict_batch(Q, K, V, w.cu_seqlens, cap, w.pool_k, layer_budgets=lb)
    idx_h, Ko_h, Vo_h = idx.cpu().numpy(), from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu, cb = w.cu_seqlens, w.cu_budgets
    filler = from_dev_bf16(torch.full((1,), 1.5, dtype=torch.bfloat16, device="cuda"))[0]
    for l in range(3):
        for s in range(2):
            b = lb[l][s]
            for g in range(w.h_kv):
                assert_kept_set_ok(ref["pooled"][l, g, cu[s]:cu[s + 1]], ref["idx"][l, g, cb[s]:cb[s] + b],
                                   idx_h[l, g, cb[s]:cb[s] + b], "l%d s%d g%d" % (l, s, g))
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], np.ascontiguousarray(idx_h[l, :, cb[s]:cb[s] + b]))
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s] + b], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s] + b], rv)
            assert (idx_h[l, :, cb[s] + b:cb[s + 1]] == -7).all()                  # unused slots are not written
            assert (Ko_h[l, cb[s] + b:cb[s + 1]] == filler).all() and (Vo_h[l, cb[s] + b:cb[s + 1]] == filler).all()
    # values outside 1..cap are clamped on the device
    lb_bad = torch.tensor([[0, 10 ** 6], [300, 100], [300, 100]], dtype=torch.int32, device="cuda")
    sh_bad = jq.Shape(n_layers=3, seq_lens=seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=cap,
                      layer_budgets=lb_bad)
    idx3 = torch.full_like(idx, -7)
    jq.select_topk(sh_bad, pooled, idx=idx3)
    torch.cuda.synchronize()
    i3 = idx3.cpu().numpy()
    assert (i3[0, :, 0] >= 0).all() and (i3[0, :, 1:cb[1]] == -7).all()            # 0 -> one kept position
    assert (i3[0, :, cb[1]:cb[2]] >= 0).all()                                      # 10^6 -> the sequence's cap


def test_layer_budget_below_the_always_kept_positions_is_raised_to_them():
    # a per-layer budget smaller than keep_first + keep_last cannot drop always-kept positions: it is raised to their
    # number, in the selection, the gather and the in-place gather alike
    torch = torch_()
    L, h_kv, kf, kl, cap = 3000, 2, 4, 32, 200
    rng = np.random.default_rng(38)
    x = rng.random((3, h_kv, L)).astype(np.float32)
    x[:, :, :kf] = 0.0; x[:, :, L - kl:] = -1.0                        # the forced positions score worst
    lb = [[10], [kf + kl], [120]]                                      # below, at, above the forced count
    lb_d = torch.tensor(lb, dtype=torch.int32, device="cuda")
    sh = jq.Shape(n_layers=3, seq_lens=[L], n_q=1, h_q=h_kv, h_kv=h_kv, budgets=[cap], keep_first=kf, keep_last=kl,
                  layer_budgets=lb_d)
    idx = torch.full((3, h_kv, cap), -7, dtype=torch.int32, device="cuda")
    jq.select_topk(sh, torch.from_numpy(x).cuda(), idx=idx)
    K = rng.integers(0, 65536, (3, L, h_kv, 128)).astype(np.uint16)
    V = rng.integers(0, 65536, (3, L, h_kv, 128)).astype(np.uint16)
    Kd, Vd = to_dev_bf16(K), to_dev_bf16(V)
    Ko = torch.full((3, cap, h_kv, 128), 1.5, dtype=torch.bfloat16, device="cuda"); Vo = Ko.clone()
    jq.compact(sh, Kd, Vd, idx, K_out=Ko, V_out=Vo)
    Ki, Vi = Kd.clone(), Vd.clone()
    jq.compact_inplace(sh, Ki, Vi, idx)
    torch.cuda.synchronize()
    idx_h, Ko_h, Vo_h, Ki_h = idx.cpu().numpy(), from_dev_bf16(Ko), from_dev_bf16(Vo), from_dev_bf16(Ki)
    filler = from_dev_bf16(torch.full((1,), 1.5, dtype=torch.bfloat16, device="cuda"))[0]
    for l, b in enumerate([kf + kl, kf + kl, 120]):                   # the budgets actually used
        ref = oracle.select_topk(x[l].astype(np.float64), b, kf, kl)
        np.testing.assert_array_equal(idx_h[l, :, :b], ref)
        assert (idx_h[l, :, b:] == -7).all()
        rk, rv = oracle.compact(K[l], V[l], np.ascontiguousarray(idx_h[l, :, :b]))
        np.testing.assert_array_equal(Ko_h[l, :b], rk)
        np.testing.assert_array_equal(Vo_h[l, :b], rv)
        assert (Ko_h[l, b:] == filler).all()
        np.testing.assert_array_equal(Ki_h[l, :b], rk)
        np.testing.assert_array_equal(Ki_h[l, b:], K[l, b:])           # rows beyond the layer's own budget stay


def test_evict_equals_stage_composition_and_oracle():
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 700], budget=[200, 64], n_layers=2)
    Q, K, V = w.assemble()
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd)
    s1 = jq.score(sh, Qd, Kd)
    p1 = jq.pool(sh, s1)
    i1 = jq.select_topk(sh, p1)
    Ko1, Vo1 = jq.compact(sh, Kd, Vd, i1)
    torch.cuda.synchronize()
    assert torch.equal(pooled, p1) and torch.equal(idx, i1) and torch.equal(Ko.view(torch.int16), Ko1.view(torch.int16))
    assert torch.equal(Vo.view(torch.int16), Vo1.view(torch.int16))
    # outputs may also be left in the workspace
    Ko2, Vo2, none_idx, none_sc = jq.evict(sh, Qd, Kd, Vd, want_idx=False, want_scores=False)
    torch.cuda.synchronize()
    assert none_idx is None and none_sc is None and torch.equal(Ko2.view(torch.int16), Ko.view(torch.int16))

    ref = oracle.evict_batch(Q, K, V, w.cu_seqlens, w.budgets, w.pool_k)
    pooled_h, idx_h = pooled.cpu().numpy(), idx.cpu().numpy()
    Ko_h, Vo_h = from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(2):
        for s in range(2):
            L = w.seq_lens[s]
            assert_scores_close(pooled_h[l, :, cu[s]:cu[s + 1]], ref["pooled"][l, :, cu[s]:cu[s + 1]], w.n_q * w.group / L)
            for g in range(w.h_kv):
                assert_kept_set_ok(ref["pooled"][l, g, cu[s]:cu[s + 1]], ref["idx"][l, g, cb[s]:cb[s + 1]],
                                   idx_h[l, g, cb[s]:cb[s + 1]], "l%d s%d g%d" % (l, s, g))
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx_h[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s + 1]], rv)


@pytest.mark.parametrize("seq_lens,budgets,n_layers,with_lse", [
    ([3000], [500], 2, False),                 # sources on both sides of the overwritten front
    ([900, 40, 2000], [300, 40, 700], 2, False),   # a later sequence's rows land on an earlier sequence's sources; one kept whole
    ([600], [600], 1, False),                  # everything kept: every source lies inside the front
    ([2500, 1300], [256, 100], 1, True),       # one pass with supplied normalisers
])
def test_evict_inplace_leaves_the_pruned_cache_at_the_front_of_k_and_v(seq_lens, budgets, n_layers, with_lse):
    # the fused call without a second cache equals jq_evict followed by a copy of its pruned cache over the front of K, V
    torch = torch_()
    print("evict in place", seq_lens, budgets, n_layers, with_lse, flush=True)
    w = make_workload(1, seq_lens=seq_lens, budget=budgets, n_layers=n_layers)
    Q, K, V = w.assemble()
    sh = jq.Shape(n_layers=n_layers, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    lse = None
    if with_lse:
        lse = torch.full((n_layers, len(seq_lens), w.n_q, w.h_q), 9.0, dtype=torch.float32, device="cuda")
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd, lse=lse)
    Ki, Vi = Kd.clone(), Vd.clone()
    _, _, idx2, pooled2 = jq.evict_inplace(sh, Qd, Ki, Vi, lse=lse)
    torch.cuda.synchronize()
    TB = sum(budgets)
    assert torch.equal(idx, idx2) and torch.equal(pooled, pooled2)
    assert torch.equal(Ki[:, :TB].view(torch.int16), Ko.view(torch.int16)) and torch.equal(Vi[:, :TB].view(torch.int16), Vo.view(torch.int16))
    assert torch.equal(Ki[:, TB:].view(torch.int16), Kd[:, TB:].view(torch.int16))       # the rest is untouched
    assert torch.equal(Vi[:, TB:].view(torch.int16), Vd[:, TB:].view(torch.int16))
    # and the pruned cache is the oracle's gather of those positions from the ORIGINAL cache
    idx_h, Ki_h = idx.cpu().numpy(), from_dev_bf16(Ki)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(n_layers):
        for s in range(len(seq_lens)):
            rk, _ = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], np.ascontiguousarray(idx_h[l, :, cb[s]:cb[s + 1]]))
            np.testing.assert_array_equal(Ki_h[l, cb[s]:cb[s + 1]], rk)


def test_evict_inplace_on_a_long_sequence_takes_the_streaming_selection():
    torch = torch_()
    L, h, n_q, B = 700000, 2, 2, 300
    torch.manual_seed(7)
    Kd = torch.randn((1, L, h, 128), device="cuda", dtype=torch.bfloat16)
    Vd = torch.randn((1, L, h, 128), device="cuda", dtype=torch.bfloat16)
    Qd = torch.randn((1, 1, n_q, h, 128), device="cuda", dtype=torch.bfloat16)
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=n_q, h_q=h, h_kv=h, budgets=[B])
    Ko, Vo, idx, _ = jq.evict(sh, Qd, Kd, Vd)
    Ki, Vi = Kd.clone(), Vd.clone()
    _, _, idx2, _ = jq.evict_inplace(sh, Qd, Ki, Vi)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2)
    assert torch.equal(Ki[:, :B].view(torch.int16), Ko.view(torch.int16)) and torch.equal(Vi[:, :B].view(torch.int16), Vo.view(torch.int16))
    assert torch.equal(Ki[:, B:].view(torch.int16), Kd[:, B:].view(torch.int16))
