"""GPU parity of the fused jq_evict on the five named workloads at their full sizes, in the
launch configuration bench.py times (one call per workload).  Every layer of the 32-layer workload
and every sequence of the ragged batch is compared with the oracle element by element (unpooled
scores from jq_score, pooled scores, kept sets, pruned cache); properties that hold at any size --
kept positions ascending and in range, the pruned cache bit-identical to a gather of the library's
own positions, pooled mass conserved -- are checked on the device on top of that."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import make_workload

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def shape_of(w):
    return jq.Shape(n_layers=w.n_layers, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k,
                    budgets=w.budgets)


def check_problem_against_oracle(w, Q, K, V, pooled_h, idx_h, Ko_h, Vo_h, what, raw_h=None):
    """One (layer, sequence): Q [n_q,h_q,d], K/V [L,h_kv,d] host bits; GPU outputs for that problem
    (`raw_h`: the unpooled scores of jq_score for the same problem, compared as well when given)."""
    L, B = K.shape[0], idx_h.shape[1]
    ref_s = oracle.score(Q, K)
    if raw_h is not None:
        assert_scores_close(raw_h, ref_s, w.n_q * w.group / L, what + " unpooled")
    ref_p = oracle.pool(ref_s, w.pool_k)
    assert_scores_close(pooled_h, ref_p, w.n_q * w.group / L, what + " pooled")
    ref_idx = oracle.select_topk(ref_p, B)
    verdicts = [assert_kept_set_ok(ref_p[g], ref_idx[g], idx_h[g], "%s head %d" % (what, g)) for g in range(w.h_kv)]
    rk, rv = oracle.compact(K, V, np.ascontiguousarray(idx_h))
    np.testing.assert_array_equal(Ko_h, rk)
    np.testing.assert_array_equal(Vo_h, rv)
    # Eq. 6 hit rate against the oracle's set: 1 when identical, and never far from it in contested cases
    assert min(oracle.hit_rate(idx_h[g], ref_idx[g]) for g in range(w.h_kv)) > 0.98
    return verdicts


def check_properties_on_device(torch, w, Kd, Vd, Ko, Vo, idx, pooled):
    """Every (layer, sequence, head) of the call, with torch ops on the device (test infrastructure only)."""
    cu, cb = w.cu_seqlens, w.cu_budgets
    for s in range(w.n_seq):
        L = w.seq_lens[s]
        seg = idx[:, :, cb[s]:cb[s + 1]].long()                      # [nl, h_kv, B]
        assert bool((seg[..., 1:] > seg[..., :-1]).all()) and int(seg.min()) >= 0 and int(seg.max()) < L
        for g in range(w.h_kv):
            src = seg[:, g, :] + int(cu[s])                          # [nl, B] token rows
            want_k = torch.gather(Kd[:, :, g, :].view(torch.int16), 1, src[..., None].expand(-1, -1, w.d))
            want_v = torch.gather(Vd[:, :, g, :].view(torch.int16), 1, src[..., None].expand(-1, -1, w.d))
            assert torch.equal(Ko[:, cb[s]:cb[s + 1], g, :].view(torch.int16), want_k)
            assert torch.equal(Vo[:, cb[s]:cb[s + 1], g, :].view(torch.int16), want_v)
        # average pooling with zero padding loses only the mass of the 3 positions next to each end
        mass = pooled[:, :, cu[s]:cu[s + 1]].double().sum(dim=2)
        total = float(w.n_q * w.group)
        assert bool((mass <= total * (1 + 1e-5)).all()) and bool((mass >= total * (1 - 6.0 * 50 / L)).all())
        assert bool((pooled[:, :, cu[s]:cu[s + 1]] >= 0).all())


def test_config1_tiny():
    torch = torch_()
    w = make_workload(1)
    Q, K, V = w.assemble()
    Ko, Vo, idx, pooled = jq.evict(shape_of(w), to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V))
    torch.cuda.synchronize()
    check_problem_against_oracle(w, Q[0, 0], K[0], V[0], pooled[0].cpu().numpy(), idx[0].cpu().numpy(),
                                 from_dev_bf16(Ko)[0], from_dev_bf16(Vo)[0], "config 1")
    for g, pos in enumerate(w.planted_positions(0, 0)):
        assert set(pos.tolist()) <= set(idx[0, g].cpu().numpy().tolist())     # planted heavy hitters are kept


def test_config2_llama_layer_three_budgets():
    torch = torch_()
    base = make_workload(2)
    Q, K, V = base.assemble()
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    ref_p = oracle.pool(oracle.score(Q[0, 0], K[0]), base.pool_k)
    for B in (128, 512, 2048):
        print("config 2 budget", B, flush=True)
        w = make_workload(2, budget=B)
        Ko, Vo, idx, pooled = jq.evict(shape_of(w), Qd, Kd, Vd)
        torch.cuda.synchronize()
        idx_h = idx[0].cpu().numpy()
        assert_scores_close(pooled[0].cpu().numpy(), ref_p, w.n_q * w.group / w.seq_lens[0], "config 2 pooled")
        ref_idx = oracle.select_topk(ref_p, B)
        for g in range(w.h_kv):
            assert_kept_set_ok(ref_p[g], ref_idx[g], idx_h[g], "config 2 B=%d head %d" % (B, g))
        rk, rv = oracle.compact(K[0], V[0], idx_h)
        np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
        np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)


def test_config3_mistral_layer_128k():
    torch = torch_()
    w = make_workload(3)
    Q, K, V = w.assemble()
    Kd, Vd = to_dev_bf16(K), to_dev_bf16(V)
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict(shape_of(w), Qd, Kd, Vd)
    raw = jq.score(shape_of(w), Qd, Kd)
    torch.cuda.synchronize()
    check_properties_on_device(torch, w, Kd, Vd, Ko, Vo, idx, pooled)
    check_problem_against_oracle(w, Q[0, 0], K[0], V[0], pooled[0].cpu().numpy(), idx[0].cpu().numpy(),
                                 from_dev_bf16(Ko)[0], from_dev_bf16(Vo)[0], "config 3", raw_h=raw[0].cpu().numpy())


def test_config3_paged_cache_with_sinks_and_window():
    # the headline layer again, out of a paged cache (256-token pages in random order) and with attention sinks
    # and a local window forced into the kept set: bit-identical to the dense call, whose kept sets are
    # checked against the oracle's forced selection on the oracle's own pooled scores
    torch = torch_()
    from workloads import page_out
    w = make_workload(3)
    Q, K, V = w.assemble()
    kf, kl = 4, 32
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets,
                  keep_first=kf, keep_last=kl)
    Qd, Kd, Vd = to_dev_bf16(Q), to_dev_bf16(K), to_dev_bf16(V)
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd)
    Kp, Vp, table = page_out(K, V, w.seq_lens, 256, seed=3)
    pages = jq.Pages(page_size=256, n_pages=Kp.shape[1], block_table=torch.from_numpy(table).cuda())
    Ko2, Vo2, idx2, pooled2 = jq.evict_paged(sh, pages, Qd, to_dev_bf16(Kp), to_dev_bf16(Vp))
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled2) and torch.equal(idx, idx2)
    assert torch.equal(Ko.view(torch.int16), Ko2.view(torch.int16)) and torch.equal(Vo.view(torch.int16), Vo2.view(torch.int16))
    check_properties_on_device(torch, w, Kd, Vd, Ko, Vo, idx, pooled)
    ref_p = oracle.pool(oracle.score(Q[0, 0], K[0]), w.pool_k)
    ref_idx = oracle.select_topk(ref_p, w.budgets[0], kf, kl)
    idx_h = idx[0].cpu().numpy()
    from parity import assert_kept_set_ok_keep
    for g in range(w.h_kv):
        assert_kept_set_ok_keep(ref_p[g], ref_idx[g], idx_h[g], kf, kl, "config 3 forced head %d" % g)


@pytest.fixture(scope="module")
def config4_call():
    """The 32-layer workload through ONE jq_evict call (and one jq_score call); host copies of the inputs are kept for the
    oracle (8 GiB), device tensors are dropped when the module's tests are done."""
    torch = torch_()
    w = make_workload(4)
    nl, L = w.n_layers, w.seq_lens[0]
    Qd = torch.empty((nl, 1, w.n_q, w.h_q, w.d), dtype=torch.bfloat16, device="cuda")
    Kd = torch.empty((nl, L, w.h_kv, w.d), dtype=torch.bfloat16, device="cuda")
    Vd = torch.empty_like(Kd)
    host = []
    for l in range(nl):                                  # 8 GiB of inputs: generated and uploaded layer by layer
        q, k, v = w.tensors(l, 0)
        Qd[l, 0].copy_(to_dev_bf16(q)); Kd[l].copy_(to_dev_bf16(k)); Vd[l].copy_(to_dev_bf16(v))
        host.append((q, k, v))
        if l % 8 == 7:
            print("config 4: layer", l, "generated", flush=True)
    Ko, Vo, idx, pooled = jq.evict(shape_of(w), Qd, Kd, Vd)
    raw = jq.score(shape_of(w), Qd, Kd)
    torch.cuda.synchronize()
    assert tuple(Ko.shape) == (32, 1024, 8, 128) and Ko.is_contiguous() and tuple(Vo.shape) == (32, 1024, 8, 128)
    check_properties_on_device(torch, w, Kd, Vd, Ko, Vo, idx, pooled)
    yield w, host, Ko, Vo, idx, pooled, raw
    del Qd, Kd, Vd, Ko, Vo, idx, pooled, raw, host
    torch.cuda.empty_cache()


@pytest.mark.timeout(600)
@pytest.mark.parametrize("first", [0, 8, 16, 24])
def test_config4_thirty_two_layers(config4_call, first):
    # every layer of the one 32-layer call against the oracle, eight layers per test
    w, host, Ko, Vo, idx, pooled, raw = config4_call
    for l in range(first, first + 8):
        q, k, v = host[l]
        check_problem_against_oracle(w, q, k, v, pooled[l].cpu().numpy(), idx[l].cpu().numpy(),
                                     from_dev_bf16(Ko[l]), from_dev_bf16(Vo[l]), "config 4 layer %d" % l,
                                     raw_h=raw[l].cpu().numpy())
        print("config 4: layer", l, "matches the oracle", flush=True)


@pytest.mark.timeout(600)
def test_config5_ragged_batch():
    torch = torch_()
    w = make_workload(5)
    T = w.total_tokens
    cu, cb = w.cu_seqlens, w.cu_budgets
    Qd = torch.empty((1, w.n_seq, w.n_q, w.h_q, w.d), dtype=torch.bfloat16, device="cuda")
    Kd = torch.empty((1, T, w.h_kv, w.d), dtype=torch.bfloat16, device="cuda")
    Vd = torch.empty_like(Kd)
    for s in range(w.n_seq):
        q, k, v = w.tensors(0, s)
        Qd[0, s].copy_(to_dev_bf16(q)); Kd[0, cu[s]:cu[s + 1]].copy_(to_dev_bf16(k)); Vd[0, cu[s]:cu[s + 1]].copy_(to_dev_bf16(v))
    print("config 5: %d tokens generated" % T, flush=True)
    Ko, Vo, idx, pooled = jq.evict(shape_of(w), Qd, Kd, Vd)        # a single fused call for all 16 sequences
    raw = jq.score(shape_of(w), Qd, Kd)
    torch.cuda.synchronize()
    check_properties_on_device(torch, w, Kd, Vd, Ko, Vo, idx, pooled)
    for s in range(w.n_seq):                                       # every sequence against the oracle
        q, k, v = w.tensors(0, s)
        check_problem_against_oracle(w, q, k, v, pooled[0, :, cu[s]:cu[s + 1]].cpu().numpy(),
                                     idx[0, :, cb[s]:cb[s + 1]].cpu().numpy(), from_dev_bf16(Ko[0, cb[s]:cb[s + 1]]),
                                     from_dev_bf16(Vo[0, cb[s]:cb[s + 1]]), "config 5 seq %d" % s,
                                     raw_h=raw[0, :, cu[s]:cu[s + 1]].cpu().numpy())
        print("config 5: sequence", s, "L =", w.seq_lens[s], "matches the oracle", flush=True)


def test_sequence_just_below_the_four_gib_limit():
    # the longest sequence the score kernels address (its keys stay below 4 GiB): byte offsets beyond 2^31 and
    # up to 2^32 - 2^18, heavy hitters planted where an overflowing offset would miss them; few query rows so
    # that the oracle can do the whole sequence
    torch = torch_()
    L, h, n_q, B, d = 2097000, 8, 2, 2048, 128
    assert L * h * d * 2 < 2 ** 32
    torch.manual_seed(250999)
    Kd = torch.randn((1, L, h, d), device="cuda", dtype=torch.bfloat16)
    Vd = torch.randn((1, L, h, d), device="cuda", dtype=torch.bfloat16)
    Qd = torch.randn((1, 1, n_q, h, d), device="cuda", dtype=torch.bfloat16)
    planted = [5, 1048575, 1048576, 1572864, L - 40, L - 1]            # 1048576 rows = byte offset 2^31
    for j in planted:
        Kd[0, j] = (3.0 * Qd[0, 0].float().mean(dim=0)).to(torch.bfloat16)   # [h, d]: aligned with each head's queries
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=n_q, h_q=h, h_kv=h, pool_k=7, budgets=[B])
    Ko, Vo, idx, pooled = jq.evict(sh, Qd, Kd, Vd)
    torch.cuda.synchronize()
    Q, K, V = from_dev_bf16(Qd), from_dev_bf16(Kd), from_dev_bf16(Vd)
    print("oracle on %d keys" % L, flush=True)
    ref_p = oracle.pool(oracle.score(Q[0, 0], K[0]), 7)
    pooled_h, idx_h = pooled[0].cpu().numpy(), idx[0].cpu().numpy()
    assert_scores_close(pooled_h, ref_p, n_q / L, "pooled, 2.1 M keys")
    ref_idx = oracle.select_topk(ref_p, B)
    for g in range(h):
        assert_kept_set_ok(ref_p[g], ref_idx[g], idx_h[g], "head %d" % g)
        assert set(planted) <= set(idx_h[g].tolist())
    rk, rv = oracle.compact(K[0], V[0], np.ascontiguousarray(idx_h))
    np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
    np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)
