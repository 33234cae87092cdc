"""GPU parity of the window-query mode: the prompt's own last n_q tokens are the queries (the observation
window of the window-query baselines of Section 5.1), causal inside the window, window always kept."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok_keep, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import f32_to_bf16_bits, make_workload, page_out

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def window_inputs(seed, n_layers, seq_lens, n_q, h_q, h_kv, q_spread=1.0):
    rng = np.random.default_rng(seed)
    T, d, ns = sum(seq_lens), 128, len(seq_lens)
    Q = f32_to_bf16_bits(rng.standard_normal((n_layers, ns, n_q, h_q, d)).astype(np.float32) * q_spread)
    K = f32_to_bf16_bits(rng.standard_normal((n_layers, T, h_kv, d)).astype(np.float32))
    V = f32_to_bf16_bits(rng.standard_normal((n_layers, T, h_kv, d)).astype(np.float32))
    return Q, K, V


def check_window_scores(n_layers, seq_lens, n_q, h_q, h_kv, seed=71, q_spread=1.0):
    torch = torch_()
    Q, K, _ = window_inputs(seed, n_layers, seq_lens, n_q, h_q, h_kv, q_spread)
    sh = jq.Shape(n_layers=n_layers, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv, window=True)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for l in range(n_layers):
        for s, L in enumerate(seq_lens):
            ref = oracle.score_window(Q[l, s], K[l, cu[s]:cu[s + 1]])
            seg = got[l, :, cu[s]:cu[s + 1]]
            assert not seg[:, L - n_q:].any(), "the window's own positions must report 0"
            if L > n_q:
                assert_scores_close(seg[:, :L - n_q], ref[:, :L - n_q], ref[:, :L - n_q].mean(), "layer %d seq %d" % (l, s))


@pytest.mark.parametrize("n_layers,seq_lens,n_q,h_q,h_kv", [
    (1, [2048], 16, 8, 2),            # window inside the last tile
    (1, [2060], 32, 8, 2),            # window across two tiles, partial last tile
    (1, [33], 8, 8, 2),               # one-key last tile
    (1, [1000], 32, 32, 8),           # 128 query rows
    (2, [517, 64, 3001], 10, 8, 2),   # layers x ragged batch, padded row tile
    (1, [700], 40, 8, 2),             # 160 query rows: two passes over K, window of 40 over three tiles
    (1, [40], 40, 8, 2),              # nothing in front of the window: every score is 0
    (1, [41, 300], 40, 6, 2),         # a single key in front of the window; three heads per group
])
def test_window_scores_match_oracle(n_layers, seq_lens, n_q, h_q, h_kv):
    print("window score case", n_layers, seq_lens, n_q, h_q, h_kv, flush=True)
    check_window_scores(n_layers, seq_lens, n_q, h_q, h_kv)


def test_window_scores_with_many_small_waves(knobs):
    # 64-key chunks: waves whose only tiles lie inside the window (some query rows then see none of their keys)
    knobs(JQ_CHUNK_KEYS="64")
    check_window_scores(1, [1000, 130], 48, 8, 2, seed=72)
    check_window_scores(1, [200], 32, 8, 2, seed=73, q_spread=3.0)


def test_window_eviction_matches_oracle_and_keeps_the_window():
    torch = torch_()
    n_q, h_q, h_kv, seq_lens, budgets = 32, 8, 2, [1500, 700], [200, 64]
    Q, K, V = window_inputs(74, 2, seq_lens, n_q, h_q, h_kv)
    sh = jq.Shape(n_layers=2, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv, pool_k=7, budgets=budgets, keep_first=4,
                  window=True)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd)
    # the same out of a paged cache
    Kp, Vp, table = page_out(K, V, seq_lens, 128, seed=5)
    pages = jq.Pages(page_size=128, n_pages=Kp.shape[1], block_table=torch.from_numpy(table).cuda())
    Ko2, Vo2, idx2, pooled2 = jq.evict_paged(sh, pages, Qd, to_dev_bf16(Kp), to_dev_bf16(Vp))
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(pooled, pooled2) and torch.equal(Ko.view(torch.int16), Ko2.view(torch.int16))
    cu = np.concatenate([[0], np.cumsum(seq_lens)]); cb = np.concatenate([[0], np.cumsum(budgets)])
    ref = oracle.evict_batch(Q, K, V, cu, budgets, 7, keep_first=4, window=True)
    idx_h, pooled_h = idx.cpu().numpy(), pooled.cpu().numpy()
    Ko_h, Vo_h = from_dev_bf16(Ko), from_dev_bf16(Vo)
    for l in range(2):
        for s, L in enumerate(seq_lens):
            P = L - n_q
            assert_scores_close(pooled_h[l, :, cu[s]:cu[s] + P], ref["pooled"][l, :, cu[s]:cu[s] + P],
                                ref["pooled"][l, :, cu[s]:cu[s] + P].mean(), "pooled l%d s%d" % (l, s))
            for g in range(h_kv):
                got = idx_h[l, g, cb[s]:cb[s + 1]]
                assert set(range(P, L)) <= set(got.tolist()) and set(range(4)) <= set(got.tolist())
                assert_kept_set_ok_keep(ref["pooled"][l, g, cu[s]:cu[s + 1]], ref["idx"][l, g, cb[s]:cb[s + 1]], got, 4, n_q,
                                        "l%d s%d g%d" % (l, s, g))
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx_h[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s + 1]], rv)


def test_window_with_supplied_normalisers():
    # one pass: the caller's log-sum-exp of every window row over the keys that row sees
    torch = torch_()
    n_q, h_q, h_kv, L = 16, 8, 2, 900
    Q, K, _ = window_inputs(75, 1, [L], n_q, h_q, h_kv)
    from workloads import bf16_bits_to_f64
    q, k = bf16_bits_to_f64(Q[0, 0]), bf16_bits_to_f64(K[0])
    lse = np.empty((1, 1, n_q, h_q), dtype=np.float32)
    for h in range(h_q):
        t = (q[:, h, :] @ k[:, h // (h_q // h_kv), :].T) / np.sqrt(128.0)
        for i in range(n_q):
            vis = t[i, :L - n_q + i + 1]
            lse[0, 0, i, h] = vis.max() + np.log(np.exp(vis - vis.max()).sum())
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=n_q, h_q=h_q, h_kv=h_kv, window=True)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K), lse=torch.from_numpy(lse).cuda())
    two_pass = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    ref = oracle.score_window(Q[0, 0], K[0])
    assert not got[0, :, L - n_q:].any()
    assert_scores_close(got[0, :, :L - n_q].cpu().numpy(), ref[:, :L - n_q], ref[:, :L - n_q].mean(), "one pass")
    assert_scores_close(two_pass[0, :, :L - n_q].cpu().numpy(), ref[:, :L - n_q], ref[:, :L - n_q].mean(), "two passes")
