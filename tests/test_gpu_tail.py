"""GPU parity of the entry points whose softmax also covers the soft tokens' own keys (causal tail),
against the oracle; the same call scores a prompt under its own last tokens (observation window)."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import f32_to_bf16_bits, make_workload

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


@pytest.mark.parametrize("n_layers,seq_lens,n_q,h_q,h_kv,tail_spread", [
    (1, [700], 16, 8, 2, 1.0),
    (2, [333, 1025, 40], 32, 32, 8, 1.0),     # 128 query rows, ragged batch, two layers
    (1, [90], 40, 8, 2, 1.0),                 # 160 query rows (two row groups), more soft tokens than partial-lanes
    (1, [500], 16, 8, 2, 3.0),                # soft-token keys that take most of the mass
    (1, [5], 3, 6, 6, 1.0),                   # tiny, no grouping
])
def test_score_tail_matches_oracle(n_layers, seq_lens, n_q, h_q, h_kv, tail_spread):
    print("score tail case", n_layers, seq_lens, n_q, h_q, h_kv, tail_spread, flush=True)
    torch = torch_()
    rng = np.random.default_rng(61)
    T, d, ns = sum(seq_lens), 128, len(seq_lens)
    Q = f32_to_bf16_bits(rng.standard_normal((n_layers, ns, n_q, h_q, d)).astype(np.float32))
    K = f32_to_bf16_bits(rng.standard_normal((n_layers, T, h_kv, d)).astype(np.float32))
    Kt = f32_to_bf16_bits(rng.standard_normal((n_layers, ns, n_q, h_kv, d)).astype(np.float32) * tail_spread)
    sh = jq.Shape(n_layers=n_layers, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K), k_tail=to_dev_bf16(Kt))
    plain = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    got, plain = got.cpu().numpy(), plain.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    G = h_q // h_kv
    for l in range(n_layers):
        for s, L in enumerate(seq_lens):
            ref = oracle.score_tail(Q[l, s], K[l, cu[s]:cu[s + 1]], Kt[l, s])
            seg = got[l, :, cu[s]:cu[s + 1]]
            # the absolute floor follows the scores' own scale, which the tail shrinks
            assert_scores_close(seg, ref, ref.mean(), "layer %d seq %d" % (l, s))
            assert (seg.sum(axis=1) < n_q * G).all()                       # the soft tokens took their share
            assert (seg <= plain[l, :, cu[s]:cu[s + 1]] * (1 + 1e-5)).all()  # a larger normaliser only lowers scores


def test_observation_window_scoring_of_a_prompt():
    # SnapKV-style use: the last 32 tokens of a prompt score the tokens before them; their own keys enter
    # the softmax causally.  Q and keys come from the same sequence here.
    torch = torch_()
    rng = np.random.default_rng(62)
    L, win, h_q, h_kv, d = 3000, 32, 8, 2, 128
    Qall = f32_to_bf16_bits(rng.standard_normal((L, h_q, d)).astype(np.float32))
    Kall = f32_to_bf16_bits(rng.standard_normal((L, h_kv, d)).astype(np.float32))
    Q = Qall[None, None, L - win:]                      # [1, 1, win, h_q, d]
    K = Kall[None, :L - win]                            # prompt without the window
    Kt = Kall[None, None, L - win:]                     # the window's own keys
    sh = jq.Shape(n_layers=1, seq_lens=[L - win], n_q=win, h_q=h_q, h_kv=h_kv)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K), k_tail=to_dev_bf16(Kt))
    torch.cuda.synchronize()
    ref = oracle.score_tail(Q[0, 0], K[0], Kt[0, 0])
    assert_scores_close(got.cpu().numpy()[0], ref, ref.mean(), "window")


def test_evict_tail_matches_oracle_end_to_end():
    torch = torch_()
    w = make_workload(1, seq_lens=[1800, 600], budget=[256, 100], n_layers=2)
    Q, K, V = w.assemble()
    rng = np.random.default_rng(63)
    Kt = f32_to_bf16_bits(rng.standard_normal((w.n_layers, w.n_seq, w.n_q, w.h_kv, w.d)).astype(np.float32) * 1.5)
    sh = jq.Shape(n_layers=w.n_layers, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k,
                  budgets=w.budgets)
    Ko, Vo, idx, pooled = jq.evict(sh, to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V), k_tail=to_dev_bf16(Kt))
    torch.cuda.synchronize()
    idx_h, pooled_h, Ko_h, Vo_h = idx.cpu().numpy(), pooled.cpu().numpy(), from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(w.n_layers):
        for s in range(w.n_seq):
            r = oracle.evict(Q[l, s], K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], w.budgets[s], w.pool_k, K_tail=Kt[l, s])
            assert_scores_close(pooled_h[l, :, cu[s]:cu[s + 1]], r["pooled"], r["pooled"].mean(), "pooled %d %d" % (l, s))
            for g in range(w.h_kv):
                assert_kept_set_ok(r["pooled"][g], r["idx"][g], idx_h[l, g, cb[s]:cb[s + 1]], "l%d s%d g%d" % (l, s, g))
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], np.ascontiguousarray(idx_h[l, :, cb[s]:cb[s + 1]]))
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s + 1]], rv)
