"""GPU parity of the supplied-normaliser (one pass over K) entry points against the oracle, plus the
measurement aids of the ABI (traced evict, copy probe)."""
import math

import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import bf16_bits_to_f64, f32_to_bf16_bits, make_workload

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def prefill_lse(Q, K, K_soft):
    """What a causal prefill attention kernel would keep for the soft-token rows: log-sum-exp over the prompt
    keys and the soft-token keys up to the row's own position.  Q [n_q,h_q,d], K [L,h_kv,d], K_soft [n_q,h_kv,d]."""
    n_q, h_q, d = Q.shape
    G = h_q // K.shape[1]
    Qd = bf16_bits_to_f64(Q)
    lse = np.empty((n_q, h_q))
    for h in range(h_q):
        s = Qd[:, h, :] @ bf16_bits_to_f64(K[:, h // G, :]).T / math.sqrt(d)             # [n_q, L]
        if K_soft is not None:
            st = Qd[:, h, :] @ bf16_bits_to_f64(K_soft[:, h // G, :]).T / math.sqrt(d)   # [n_q, n_q]
            st = np.where(np.tril(np.ones((n_q, n_q), dtype=bool)), st, -np.inf)
            s = np.concatenate([s, st], axis=1)
        m = s.max(axis=1)
        lse[:, h] = m + np.log(np.exp(s - m[:, None]).sum(axis=1))
    return lse


@pytest.mark.parametrize("seq_lens,n_q,h_q,h_kv", [([700], 16, 8, 2), ([333, 1025], 32, 32, 8), ([90], 40, 8, 2)])
def test_score_lse_matches_oracle(seq_lens, n_q, h_q, h_kv):
    torch = torch_()
    rng = np.random.default_rng(51)
    T, d, ns = sum(seq_lens), 128, len(seq_lens)
    Q = f32_to_bf16_bits(rng.standard_normal((1, ns, n_q, h_q, d)).astype(np.float32))
    K = f32_to_bf16_bits(rng.standard_normal((1, T, h_kv, d)).astype(np.float32))
    Ks = f32_to_bf16_bits(rng.standard_normal((ns, n_q, h_kv, d)).astype(np.float32))
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    lse = np.stack([prefill_lse(Q[0, s], K[0, cu[s]:cu[s + 1]], Ks[s]) for s in range(ns)])[None].astype(np.float32)
    sh = jq.Shape(n_layers=1, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv)
    got = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K), lse=torch.from_numpy(lse).cuda())
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    for s, L in enumerate(seq_lens):
        ref = oracle.score_lse(Q[0, s], K[0, cu[s]:cu[s + 1]], lse[0, s].astype(np.float64))
        assert_scores_close(got[0, :, cu[s]:cu[s + 1]], ref, n_q * (h_q // h_kv) / L, "seq %d" % s)
        assert (got[0, :, cu[s]:cu[s + 1]].sum(axis=1) < n_q * (h_q // h_kv)).all()      # the soft tail took its share


def test_score_lse_over_the_prompt_reproduces_two_pass_scores():
    torch = torch_()
    w = make_workload(1)
    Q, K, _ = w.assemble()
    lse = prefill_lse(Q[0, 0], K[0], None)[None, None].astype(np.float32)
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv)
    Qd, Kd = to_dev_bf16(Q), to_dev_bf16(K)
    one = jq.score(sh, Qd, Kd, lse=torch.from_numpy(lse).cuda())
    two = jq.score(sh, Qd, Kd)
    torch.cuda.synchronize()
    np.testing.assert_allclose(one.cpu().numpy(), two.cpu().numpy(), rtol=2e-4, atol=1e-9)


def test_evict_lse_on_the_128k_layer():
    torch = torch_()
    w = make_workload(3)
    Q, K, V = w.assemble()
    rng = np.random.default_rng(52)
    Ks = f32_to_bf16_bits(rng.standard_normal((w.n_q, w.h_kv, w.d)).astype(np.float32))
    lse = prefill_lse(Q[0, 0], K[0], Ks).astype(np.float32)
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Ko, Vo, idx, pooled = jq.evict(sh, to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V),
                                   lse=torch.from_numpy(lse[None, None]).cuda())
    torch.cuda.synchronize()
    ref = oracle.evict(Q[0, 0], K[0], V[0], w.budgets[0], w.pool_k, lse=lse.astype(np.float64))
    assert_scores_close(pooled[0].cpu().numpy(), ref["pooled"], w.n_q * w.group / w.seq_lens[0], "pooled")
    idx_h = idx[0].cpu().numpy()
    for g in range(w.h_kv):
        assert_kept_set_ok(ref["pooled"][g], ref["idx"][g], idx_h[g], "head %d" % g)
    rk, rv = oracle.compact(K[0], V[0], idx_h)
    np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
    np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)


def test_traced_evict_equals_evict_and_times_every_kernel():
    torch = torch_()
    w = make_workload(1)
    Q, K, V = w.assemble()
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(jq.TRACE_MARKS)]
    for ev in marks:
        ev.record()
    torch.cuda.synchronize()
    a = jq.evict(sh, Qd, Kd, Vd)
    b = jq.evict(sh, Qd, Kd, Vd, marks=marks)
    torch.cuda.synchronize()
    for x, y in zip(a, b):
        assert torch.equal(x.view(torch.int32) if x.dtype != torch.bfloat16 else x.view(torch.int16),
                           y.view(torch.int32) if y.dtype != torch.bfloat16 else y.view(torch.int16))
    for j, name in enumerate(jq.TRACE_KERNELS):
        ms = marks[2 * j].elapsed_time(marks[2 * j + 1])
        assert 0.0 < ms < 50.0, (name, ms)


def test_copy_probe_copies():
    torch = torch_()
    src = torch.randint(0, 255, (1 << 20,), dtype=torch.uint8, device="cuda")
    dst = torch.zeros_like(src)
    jq.copy_probe(src, dst)
    torch.cuda.synchronize()
    assert torch.equal(src, dst)


def test_hit_rate_matches_oracle_on_random_sets_and_on_two_scorers():
    # Eq. 6 between two kept sets, per (layer, sequence, head)
    torch = torch_()
    rng = np.random.default_rng(71)
    nl, h_kv, seq_lens, budgets, ref_budgets = 2, 3, [500, 64, 3000], [100, 64, 700], [80, 10, 1500]
    sh = jq.Shape(n_layers=nl, seq_lens=seq_lens, n_q=1, h_q=h_kv, h_kv=h_kv, budgets=budgets)

    def random_sets(buds):
        out = np.empty((nl, h_kv, sum(buds)), dtype=np.int32)
        cb = np.concatenate([[0], np.cumsum(buds)])
        for l in range(nl):
            for g in range(h_kv):
                for s, L in enumerate(seq_lens):
                    out[l, g, cb[s]:cb[s + 1]] = np.sort(rng.choice(L, buds[s], replace=False))
        return out, cb

    cur, cb = random_sets(budgets)
    for rb in (None, ref_budgets):
        ref, cr = random_sets(budgets if rb is None else rb)
        got = jq.hit_rate(sh, torch.from_numpy(cur).cuda(), torch.from_numpy(ref).cuda(), ref_budgets=rb)
        torch.cuda.synchronize()
        got = got.cpu().numpy()
        for l in range(nl):
            for s in range(len(seq_lens)):
                for g in range(h_kv):
                    want = oracle.hit_rate(cur[l, g, cb[s]:cb[s + 1]], ref[l, g, cr[s]:cr[s + 1]])
                    assert abs(float(got[l, s, g]) - want) <= 1e-7, (l, s, g)
    same = jq.hit_rate(sh, torch.from_numpy(cur).cuda(), torch.from_numpy(cur.copy()).cuda())
    torch.cuda.synchronize()
    assert (same.cpu().numpy() == 1.0).all()

    # the kept sets of the prompt-only softmax and of the softmax that also covers strong soft-token keys
    w = make_workload(1, seq_lens=[1500], budget=[200])
    Q, K, V = w.assemble()
    Kt = f32_to_bf16_bits(rng.standard_normal((1, 1, w.n_q, w.h_kv, w.d)).astype(np.float32) * 2.0)
    sh2 = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    _, _, idx_a, _ = jq.evict(sh2, Qd, Kd, Vd)
    _, _, idx_b, _ = jq.evict(sh2, Qd, Kd, Vd, k_tail=to_dev_bf16(Kt))
    rate = jq.hit_rate(sh2, idx_b, idx_a)
    torch.cuda.synchronize()
    ia, ib, rate = idx_a.cpu().numpy(), idx_b.cpu().numpy(), rate.cpu().numpy()
    for g in range(w.h_kv):
        assert abs(float(rate[0, 0, g]) - oracle.hit_rate(ib[0, g], ia[0, g])) <= 1e-7
    assert rate.min() > 0.5            # the planted heavy hitters stay in both sets


def test_map_mse_of_soft_and_response_maps_matches_oracle():
    # Eq. 3-5 forward: soft-token map (n = 8 tokens) against a response map (m = 70 tokens: 280 query rows, three
    # passes over K), both from jq_score, ragged batch of two prompts
    torch = torch_()
    rng = np.random.default_rng(81)
    seq_lens, h_q, h_kv, d, n, m = [900, 333], 8, 2, 128, 8, 70
    T = sum(seq_lens)
    K = f32_to_bf16_bits(rng.standard_normal((1, T, h_kv, d)).astype(np.float32))
    Qs = f32_to_bf16_bits(rng.standard_normal((1, 2, n, h_q, d)).astype(np.float32))
    Qr = f32_to_bf16_bits(rng.standard_normal((1, 2, m, h_q, d)).astype(np.float32))
    G = h_q // h_kv
    Kd = to_dev_bf16(K)
    sh_s = jq.Shape(n_layers=1, seq_lens=seq_lens, n_q=n, h_q=h_q, h_kv=h_kv)
    sh_r = jq.Shape(n_layers=1, seq_lens=seq_lens, n_q=m, h_q=h_q, h_kv=h_kv)
    sa = jq.score(sh_s, to_dev_bf16(Qs), Kd)
    sb = jq.score(sh_r, to_dev_bf16(Qr), Kd)
    got = jq.map_mse(sh_s, sa, n * G, sb, m * G)
    torch.cuda.synchronize()
    got = got.cpu().numpy()
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for s in range(2):
        ra = oracle.score(Qs[0, s], K[0, cu[s]:cu[s + 1]])
        rb = oracle.score(Qr[0, s], K[0, cu[s]:cu[s + 1]])
        want = oracle.map_mse(ra, n * G, rb, m * G)
        # the maps agree with the oracle's to 2e-3 relative per entry, so does their squared difference in the mean
        np.testing.assert_allclose(got[0, s], want, rtol=8e-3)
        # and the reduction itself is exact to fp32 rounding when fed the GPU's own maps
        own = oracle.map_mse(sa[0, :, cu[s]:cu[s + 1]].cpu().numpy(), n * G, sb[0, :, cu[s]:cu[s + 1]].cpu().numpy(), m * G)
        np.testing.assert_allclose(got[0, s], own, rtol=2e-6)


@pytest.mark.parametrize("n,m,seq_lens", [
    (8, 70, [900, 333]),      # response rows beyond 128 per head: two earlier row groups are summed, the third compares
    (32, 24, [4099]),         # one row group each; many workgroups, ragged last tile
    (4, 1, [31, 64, 1]),      # sub-tile sequences, surplus waves in every workgroup
])
def test_map_mse_fused_matches_oracle_and_the_two_call_composition(n, m, seq_lens):
    # Eq. 3-5 forward from the two query sets: the response's map is never stored
    torch = torch_()
    rng = np.random.default_rng(82 + n)
    h_q, h_kv, d = 8, 2, 128
    T, ns = sum(seq_lens), len(seq_lens)
    K = f32_to_bf16_bits(rng.standard_normal((2, T, h_kv, d)).astype(np.float32))
    Qs = f32_to_bf16_bits(rng.standard_normal((2, ns, n, h_q, d)).astype(np.float32))
    Qr = f32_to_bf16_bits(rng.standard_normal((2, ns, m, h_q, d)).astype(np.float32))
    G = h_q // h_kv
    Kd, Qsd, Qrd = to_dev_bf16(K), to_dev_bf16(Qs), to_dev_bf16(Qr)
    sh_s = jq.Shape(n_layers=2, seq_lens=seq_lens, n_q=n, h_q=h_q, h_kv=h_kv)
    sh_r = jq.Shape(n_layers=2, seq_lens=seq_lens, n_q=m, h_q=h_q, h_kv=h_kv)
    got = jq.map_mse_fused(sh_s, Qsd, Qrd, Kd)
    two = jq.map_mse(sh_s, jq.score(sh_s, Qsd, Kd), n * G, jq.score(sh_r, Qrd, Kd), m * G)
    torch.cuda.synchronize()
    got, two = got.cpu().numpy(), two.cpu().numpy()
    # same maps, same fp64 squares; only the order of the additions differs from the stand-alone reduction
    np.testing.assert_allclose(got, two, rtol=1e-5)
    cu = np.concatenate([[0], np.cumsum(seq_lens)])
    for layer in range(2):
        for s in range(ns):
            ra = oracle.score(Qs[layer, s], K[layer, cu[s]:cu[s + 1]])
            rb = oracle.score(Qr[layer, s], K[layer, cu[s]:cu[s + 1]])
            np.testing.assert_allclose(got[layer, s], oracle.map_mse(ra, n * G, rb, m * G), rtol=8e-3)
    # a second call on the same workspace gives the same bits (fixed summation order)
    again = jq.map_mse_fused(sh_s, Qsd, Qrd, Kd)
    torch.cuda.synchronize()
    assert np.array_equal(again.cpu().numpy(), got)


def test_map_mse_fused_of_identical_query_sets_is_zero():
    torch = torch_()
    rng = np.random.default_rng(90)
    K = to_dev_bf16(f32_to_bf16_bits(rng.standard_normal((1, 2000, 2, 128)).astype(np.float32)))
    Q = to_dev_bf16(f32_to_bf16_bits(rng.standard_normal((1, 1, 16, 8, 128)).astype(np.float32)))
    sh = jq.Shape(n_layers=1, seq_lens=[2000], n_q=16, h_q=8, h_kv=2)
    got = jq.map_mse_fused(sh, Q, Q.clone(), K)
    torch.cuda.synchronize()
    assert float(got.abs().max()) == 0.0
