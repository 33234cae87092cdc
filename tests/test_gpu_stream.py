"""GPU parity of jq_evict_stream: eviction steps during decoding on a cache that earlier steps pruned, against
oracle.stream_step on the same state, over several steps with newly decoded rows appended in between."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok_keep, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import f32_to_bf16_bits, make_workload

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("with_lse,pool_k", [(False, 1), (True, 1), (False, 7)])
def test_stream_steps_match_the_oracle(with_lse, pool_k):
    import torch
    assert torch.cuda.is_available(), "this test needs the GPU"
    print("stream steps", with_lse, pool_k, flush=True)
    w = make_workload(1, seq_lens=[3000], budget=[400])
    Q0, K0, V0 = w.assemble()
    h_kv, h_q, n_q, d, B, n_new = w.h_kv, w.h_q, w.n_q, w.d, 400, 96
    rng = np.random.default_rng(99)
    K, V = K0[0], V0[0]                                              # [rows, h_kv, d]
    pos = np.tile(np.arange(K.shape[0], dtype=np.int32), (h_kv, 1))  # [h_kv, rows]
    next_tok = K.shape[0]
    for step in range(4):
        rows = K.shape[0]
        Q = Q0[0, 0] if step == 0 else f32_to_bf16_bits(rng.standard_normal((n_q, h_q, d)).astype(np.float32))
        kl = 0 if step == 0 else n_new                                # the tokens decoded since the last step stay
        lse_h = None
        if with_lse:                                                  # normalisers that cover more than the cache: prompt-only lse + 0.3
            from workloads import bf16_bits_to_f64
            q, k = bf16_bits_to_f64(Q), bf16_bits_to_f64(K)
            lse_h = np.empty((n_q, h_q))
            for h in range(h_q):
                s = q[:, h] @ k[:, h // w.group].T / np.sqrt(d)
                lse_h[:, h] = np.log(np.exp(s - s.max(1, keepdims=True)).sum(1)) + s.max(1) + 0.3
        ref = oracle.stream_step(Q, K, V, pos, B, pool_k=pool_k, lse=lse_h, keep_first=2, keep_last=kl)
        sh = jq.Shape(n_layers=1, seq_lens=[rows], n_q=n_q, h_q=h_q, h_kv=h_kv, pool_k=pool_k, budgets=[B], keep_first=2, keep_last=kl)
        lse_d = None if lse_h is None else torch.from_numpy(lse_h.astype(np.float32)).cuda().reshape(1, 1, n_q, h_q)
        Ko, Vo, po, idx, pooled = jq.evict_stream(sh, to_dev_bf16(Q[None, None]), to_dev_bf16(K[None]), to_dev_bf16(V[None]),
                                                  torch.from_numpy(pos[None].copy()).cuda(), lse=lse_d)
        torch.cuda.synchronize()
        idx_h, po_h = idx[0].cpu().numpy(), po[0].cpu().numpy()
        assert_scores_close(pooled[0].cpu().numpy(), ref["pooled"], n_q * w.group / rows, "step %d pooled" % step)
        for g in range(h_kv):
            assert_kept_set_ok_keep(ref["pooled"][g], ref["idx"][g], idx_h[g], 2, kl, "step %d head %d" % (step, g))
            np.testing.assert_array_equal(po_h[g], pos[g, idx_h[g]])            # positions follow the rows
        rk, rv = oracle.compact(K, V, np.ascontiguousarray(idx_h))
        np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
        np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)
        if step > 0:
            assert (po_h[:, -n_new:] == np.arange(next_tok - n_new, next_tok)).all()
        # the next step continues from the ORACLE's state (so that every step is judged on identical inputs)
        new_k = f32_to_bf16_bits(rng.standard_normal((n_new, h_kv, d)).astype(np.float32))
        new_v = f32_to_bf16_bits(rng.standard_normal((n_new, h_kv, d)).astype(np.float32))
        K = np.concatenate([ref["K_out"], new_k]); V = np.concatenate([ref["V_out"], new_v])
        pos = np.concatenate([ref["pos_out"], np.tile(np.arange(next_tok, next_tok + n_new, dtype=np.int32), (h_kv, 1))], axis=1)
        next_tok += n_new


def test_stream_step_on_a_batch_of_layers_and_sequences():
    import torch
    rng = np.random.default_rng(3)
    nl, seq_lens, budgets, h_kv, h_q, n_q, d = 2, [700, 300], [128, 64], 2, 4, 8, 128
    T = sum(seq_lens)
    Q = f32_to_bf16_bits(rng.standard_normal((nl, 2, n_q, h_q, d)).astype(np.float32))
    K = f32_to_bf16_bits(rng.standard_normal((nl, T, h_kv, d)).astype(np.float32))
    V = f32_to_bf16_bits(rng.standard_normal((nl, T, h_kv, d)).astype(np.float32))
    pos = np.sort(rng.integers(0, 10 ** 6, (nl, h_kv, T)), axis=2).astype(np.int32)
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv, pool_k=1, budgets=budgets, keep_last=16)
    Ko, Vo, po, idx, pooled = jq.evict_stream(sh, to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V), torch.from_numpy(pos).cuda())
    torch.cuda.synchronize()
    cu, cb = np.concatenate([[0], np.cumsum(seq_lens)]), np.concatenate([[0], np.cumsum(budgets)])
    for l in range(nl):
        for s in range(2):
            ref = oracle.stream_step(Q[l, s], K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], pos[l, :, cu[s]:cu[s + 1]], budgets[s],
                                     keep_last=16)
            idx_h = idx[l, :, cb[s]:cb[s + 1]].cpu().numpy()
            for g in range(h_kv):
                assert_kept_set_ok_keep(ref["pooled"][g], ref["idx"][g], idx_h[g], 0, 16, "l%d s%d g%d" % (l, s, g))
                np.testing.assert_array_equal(po[l, g, cb[s]:cb[s + 1]].cpu().numpy(), pos[l, g, cu[s]:cu[s + 1]][idx_h[g]])
