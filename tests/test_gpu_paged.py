"""GPU parity of the paged-cache entry points: the same eviction (Section 4.3) when K and V live in pools of
fixed-size pages behind a block table.  The oracle sees the dense tensors the pools were filled from."""
import numpy as np
import pytest

import oracle
import paper_2509_10798_amd as jq
from parity import assert_kept_set_ok, assert_scores_close, from_dev_bf16, to_dev_bf16
from workloads import bf16_bits_to_f64, make_workload, page_out

pytestmark = pytest.mark.gpu


def torch_():
    import torch
    assert torch.cuda.is_available(), "these tests need the GPU"
    return torch


def paged_inputs(w, page_size, seed=0, n_layers=None):
    torch = torch_()
    Q, K, V = w.assemble()
    Kp, Vp, table = page_out(K, V, w.seq_lens, page_size, seed)
    pages = jq.Pages(page_size=page_size, n_pages=Kp.shape[1], block_table=torch.from_numpy(table).cuda())
    return Q, K, V, to_dev_bf16(Kp), to_dev_bf16(Vp), pages


@pytest.mark.parametrize("seq_lens,page_size,n_layers", [
    ([2048], 32, 1),            # one tile per page
    ([1000], 64, 1),            # ragged tail inside the last page
    ([517, 64, 3001], 256, 2),  # layers x ragged batch; a sequence shorter than a page
    ([5000], 1024, 1),
    ([33], 4096, 1),            # page far larger than the sequence
])
def test_score_paged_matches_oracle_and_dense(seq_lens, page_size, n_layers):
    torch = torch_()
    print("paged score case", seq_lens, page_size, n_layers, flush=True)
    w = make_workload(1, seq_lens=seq_lens, budget=[1] * len(seq_lens), n_layers=n_layers)
    Q, K, V, Kp, Vp, pages = paged_inputs(w, page_size, seed=page_size)
    sh = jq.Shape(n_layers=n_layers, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv)
    got = jq.score_paged(sh, pages, to_dev_bf16(Q), Kp)
    dense = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K))
    torch.cuda.synchronize()
    assert torch.equal(got, dense)          # same tiles, same arithmetic, same order: only the addresses differ
    got = got.cpu().numpy()
    cu = w.cu_seqlens
    for l in range(n_layers):
        for s, L in enumerate(seq_lens):
            ref = oracle.score(Q[l, s], K[l, cu[s]:cu[s + 1]])
            assert_scores_close(got[l, :, cu[s]:cu[s + 1]], ref, w.n_q * w.group / L, "layer %d seq %d" % (l, s))


def test_score_paged_with_supplied_normalisers():
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 300], budget=[1, 1], n_layers=1)
    Q, K, V, Kp, Vp, pages = paged_inputs(w, 128, seed=5)
    sh = jq.Shape(n_layers=1, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv)
    # normalisers of a softmax that is a little wider than the prompt: log-sum-exp over the prompt plus log(1.25)
    cu = w.cu_seqlens
    lse = np.empty((1, 2, w.n_q, w.h_q), dtype=np.float32)
    for s in range(2):
        q, k = bf16_bits_to_f64(Q[0, s]), bf16_bits_to_f64(K[0, cu[s]:cu[s + 1]])
        for h in range(w.h_q):
            t = (q[:, h, :] @ k[:, h // w.group, :].T) / np.sqrt(128.0)
            m = t.max(axis=1)
            lse[0, s, :, h] = m + np.log(np.exp(t - m[:, None]).sum(axis=1)) + np.log(1.25)
    lse_d = torch.from_numpy(lse).cuda()
    got = jq.score_paged(sh, pages, to_dev_bf16(Q), Kp, lse=lse_d)
    dense = jq.score(sh, to_dev_bf16(Q), to_dev_bf16(K), lse=lse_d)
    torch.cuda.synchronize()
    assert torch.equal(got, dense)
    for s, L in enumerate(w.seq_lens):
        ref = oracle.score_lse(Q[0, s], K[0, cu[s]:cu[s + 1]], lse[0, s].astype(np.float64))
        assert_scores_close(got[0, :, cu[s]:cu[s + 1]].cpu().numpy(), ref, w.n_q * w.group / L, "seq %d" % s)


@pytest.mark.parametrize("page_size", [32, 512])
def test_evict_paged_matches_oracle_and_dense(page_size):
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 700], budget=[200, 64], n_layers=2)
    Q, K, V, Kp, Vp, pages = paged_inputs(w, page_size, seed=page_size + 1)
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets,
                  keep_first=2, keep_last=8)
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, Kp, Vp)
    Ko1, Vo1, idx1, pooled1 = jq.evict(sh, Qd, to_dev_bf16(K), to_dev_bf16(V))
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled1) and torch.equal(idx, idx1)
    assert torch.equal(Ko.view(torch.int16), Ko1.view(torch.int16)) and torch.equal(Vo.view(torch.int16), Vo1.view(torch.int16))
    ref = oracle.evict_batch(Q, K, V, w.cu_seqlens, w.budgets, w.pool_k, keep_first=2, keep_last=8)
    idx_h, Ko_h, Vo_h = idx.cpu().numpy(), from_dev_bf16(Ko), from_dev_bf16(Vo)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(2):
        for s in range(2):
            rk, rv = oracle.compact(K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], idx_h[l, :, cb[s]:cb[s + 1]])
            np.testing.assert_array_equal(Ko_h[l, cb[s]:cb[s + 1]], rk)
            np.testing.assert_array_equal(Vo_h[l, cb[s]:cb[s + 1]], rv)
            assert_scores_close(pooled[l, :, cu[s]:cu[s + 1]].cpu().numpy(), ref["pooled"][l, :, cu[s]:cu[s + 1]],
                                w.n_q * w.group / w.seq_lens[s])


def test_block_table_entries_outside_the_pool_are_clamped_the_same_way_everywhere():
    # a -1 (and a too large) entry INSIDE a sequence's range: the keys that are scored and the rows that are gathered
    # must come from the same page, i.e. the call equals the call on the correspondingly clamped table
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 700], budget=[400, 200], n_layers=2)
    Q, K, V, Kp, Vp, pages = paged_inputs(w, 64, seed=77)
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    bad = pages.block_table.clone()
    bad[0, 3] = -1; bad[0, 7] = pages.n_pages + 5; bad[1, 2] = -(2 ** 31)
    good = bad.clone()
    good[0, 3] = 0; good[0, 7] = pages.n_pages - 1; good[1, 2] = 0
    Qd = to_dev_bf16(Q)
    a = jq.evict_paged(sh, jq.Pages(page_size=64, n_pages=pages.n_pages, block_table=bad), Qd, Kp, Vp)
    b = jq.evict_paged(sh, jq.Pages(page_size=64, n_pages=pages.n_pages, block_table=good), Qd, Kp, Vp)
    torch.cuda.synchronize()
    assert torch.equal(a[3], b[3]) and torch.equal(a[2], b[2])
    assert torch.equal(a[0].view(torch.int16), b[0].view(torch.int16)) and torch.equal(a[1].view(torch.int16), b[1].view(torch.int16))
    # and the clamped call is the dense call on the keys those pages hold
    Kp_h, Vp_h, tab = from_dev_bf16(Kp), from_dev_bf16(Vp), good.cpu().numpy()
    cu = w.cu_seqlens
    Kd = np.empty_like(K); Vd = np.empty_like(V)
    for s_, L in enumerate(w.seq_lens):
        for t in range(L):
            Kd[:, cu[s_] + t] = Kp_h[:, tab[s_, t // 64], t % 64]
            Vd[:, cu[s_] + t] = Vp_h[:, tab[s_, t // 64], t % 64]
    c = jq.evict(sh, Qd, to_dev_bf16(Kd), to_dev_bf16(Vd))
    torch.cuda.synchronize()
    assert torch.equal(a[3], c[3]) and torch.equal(a[2], c[2]) and torch.equal(a[0].view(torch.int16), c[0].view(torch.int16))


def test_evict_paged_very_long_sequence_takes_the_separate_gather():
    # beyond the selection's LDS bitmaps the kept rows are gathered by the stand-alone copy kernel, which
    # has to follow the block table as well
    torch = torch_()
    L, B = 660000, 300
    rng = np.random.default_rng(9)
    Q = rng.integers(0, 65536, (1, 1, 4, 2, 128)).astype(np.uint16) & np.uint16(0xBF7F)   # finite, modest magnitudes
    K = rng.integers(0, 65536, (1, L, 1, 128)).astype(np.uint16) & np.uint16(0xBF7F)
    V = rng.integers(0, 65536, (1, L, 1, 128)).astype(np.uint16)
    Kp, Vp, table = page_out(K, V, [L], 2048, seed=3)
    pages = jq.Pages(page_size=2048, n_pages=Kp.shape[1], block_table=torch.from_numpy(table).cuda())
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=4, h_q=2, h_kv=1, budgets=[B])
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, to_dev_bf16(Kp), to_dev_bf16(Vp))
    Ko1, Vo1, idx1, pooled1 = jq.evict(sh, Qd, to_dev_bf16(K), to_dev_bf16(V))
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled1) and torch.equal(idx, idx1)
    assert torch.equal(Ko.view(torch.int16), Ko1.view(torch.int16)) and torch.equal(Vo.view(torch.int16), Vo1.view(torch.int16))
    rk, rv = oracle.compact(K[0], V[0], np.ascontiguousarray(idx[0].cpu().numpy()))
    np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)
    np.testing.assert_array_equal(from_dev_bf16(Vo)[0], rv)


@pytest.mark.parametrize("out_page", [1, 16, 256])
def test_evict_paged_into_a_paged_pruned_cache(out_page):
    # the kept rows land in pages again: read back through the output table they are the dense pruned cache
    torch = torch_()
    w = make_workload(1, seq_lens=[1500, 700], budget=[200, 70], n_layers=2)
    Q, K, V, Kp, Vp, pages = paged_inputs(w, 64, seed=11)
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, Kp, Vp)                       # dense output
    per_seq = [(b + out_page - 1) // out_page for b in w.budgets]
    n_out = sum(per_seq) + 2
    order = np.random.default_rng(12).permutation(n_out)
    otab = np.full((2, max(per_seq)), -1, dtype=np.int32)
    nxt = 0
    for s in range(2):
        otab[s, :per_seq[s]] = order[nxt:nxt + per_seq[s]]; nxt += per_seq[s]
    out_pages = jq.Pages(page_size=out_page, n_pages=n_out, block_table=torch.from_numpy(otab).cuda())
    Kop, Vop, idx2, pooled2 = jq.evict_paged(sh, pages, Qd, Kp, Vp, out_pages=out_pages)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(pooled, pooled2)
    Ko_h, Vo_h, Kop_h, Vop_h = from_dev_bf16(Ko), from_dev_bf16(Vo), from_dev_bf16(Kop), from_dev_bf16(Vop)
    used = np.zeros((n_out, out_page), dtype=bool)
    cb = w.cu_budgets
    for s in range(2):
        for b in range(w.budgets[s]):
            pg, r = otab[s, b // out_page], b % out_page
            np.testing.assert_array_equal(Kop_h[:, pg, r], Ko_h[:, cb[s] + b])
            np.testing.assert_array_equal(Vop_h[:, pg, r], Vo_h[:, cb[s] + b])
            used[pg, r] = True
    assert not Kop_h[:, ~used].any() and not Vop_h[:, ~used].any()                      # nothing else was written


def test_sequences_that_share_prefix_pages():
    # prefix caching: two sequences whose block tables point at the same physical pages for their common prefix
    torch = torch_()
    ps, h_kv, h_q, n_q, d = 64, 2, 8, 16, 128
    rng = np.random.default_rng(13)
    from workloads import f32_to_bf16_bits
    shared = f32_to_bf16_bits(rng.standard_normal((1, 4 * ps, h_kv, d)).astype(np.float32))      # 4 pages both sequences use
    tails = [f32_to_bf16_bits(rng.standard_normal((1, n, h_kv, d)).astype(np.float32)) for n in (100, 200)]
    vsh = f32_to_bf16_bits(rng.standard_normal((1, 4 * ps, h_kv, d)).astype(np.float32))
    vtails = [f32_to_bf16_bits(rng.standard_normal((1, n, h_kv, d)).astype(np.float32)) for n in (100, 200)]
    seq_lens = [4 * ps + 100, 4 * ps + 200]
    K = np.concatenate([shared, tails[0], shared, tails[1]], axis=1)                            # the dense equivalent
    V = np.concatenate([vsh, vtails[0], vsh, vtails[1]], axis=1)
    Q = f32_to_bf16_bits(rng.standard_normal((1, 2, n_q, h_q, d)).astype(np.float32))
    # pool: pages 0..3 shared, then 2 pages for the first tail, 4 for the second
    n_pages = 4 + 2 + 4
    Kp = np.zeros((1, n_pages, ps, h_kv, d), dtype=np.uint16); Vp = np.zeros_like(Kp)
    Kp[:, :4] = shared.reshape(1, 4, ps, h_kv, d); Vp[:, :4] = vsh.reshape(1, 4, ps, h_kv, d)
    def fill(first, k, v):
        n = k.shape[1]
        for i in range((n + ps - 1) // ps):
            m = min(ps, n - i * ps)
            Kp[:, first + i, :m] = k[:, i * ps:i * ps + m]; Vp[:, first + i, :m] = v[:, i * ps:i * ps + m]
    fill(4, tails[0], vtails[0]); fill(6, tails[1], vtails[1])
    table = np.array([[0, 1, 2, 3, 4, 5, -1, -1], [0, 1, 2, 3, 6, 7, 8, 9]], dtype=np.int32)
    pages = jq.Pages(page_size=ps, n_pages=n_pages, block_table=torch.from_numpy(table).cuda())
    sh = jq.Shape(n_layers=1, seq_lens=seq_lens, n_q=n_q, h_q=h_q, h_kv=h_kv, budgets=[40, 70])
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, to_dev_bf16(Kp), to_dev_bf16(Vp))
    Ko1, Vo1, idx1, pooled1 = jq.evict(sh, Qd, to_dev_bf16(K), to_dev_bf16(V))
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled1) and torch.equal(idx, idx1)
    assert torch.equal(Ko.view(torch.int16), Ko1.view(torch.int16)) and torch.equal(Vo.view(torch.int16), Vo1.view(torch.int16))


def test_pages_at_the_top_of_a_pool_just_below_four_gib():
    # the score kernels address a layer's pool through one 32-bit offset: a sequence that lives in the LAST pages of
    # the largest pool allowed exercises offsets up to 2^32
    torch = torch_()
    ps, h_kv, h_q, n_q, d, L, B = 256, 8, 8, 4, 128, 40000, 512
    n_pages = (2 ** 32 - 1) // (ps * h_kv * d * 2)                      # 8191 pages
    assert n_pages * ps * h_kv * d * 2 < 2 ** 32
    rng = np.random.default_rng(14)
    from workloads import f32_to_bf16_bits
    Q = f32_to_bf16_bits(rng.standard_normal((1, 1, n_q, h_q, d)).astype(np.float32))
    K = f32_to_bf16_bits(rng.standard_normal((1, L, h_kv, d)).astype(np.float32))
    V = f32_to_bf16_bits(rng.standard_normal((1, L, h_kv, d)).astype(np.float32))
    n_used = (L + ps - 1) // ps
    table = (n_pages - 1 - rng.permutation(n_used)).astype(np.int32)[None, :]      # the top pages, shuffled
    Kp = torch.zeros((1, n_pages, ps, h_kv, d), dtype=torch.bfloat16, device="cuda")
    Vp = torch.zeros_like(Kp)
    Kd, Vd = to_dev_bf16(K), to_dev_bf16(V)
    for i in range(n_used):
        m = min(ps, L - i * ps)
        Kp[0, int(table[0, i]), :m] = Kd[0, i * ps:i * ps + m]
        Vp[0, int(table[0, i]), :m] = Vd[0, i * ps:i * ps + m]
    pages = jq.Pages(page_size=ps, n_pages=n_pages, block_table=torch.from_numpy(table).cuda())
    sh = jq.Shape(n_layers=1, seq_lens=[L], n_q=n_q, h_q=h_q, h_kv=h_kv, budgets=[B])
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, Kp, Vp)
    Ko1, Vo1, idx1, pooled1 = jq.evict(sh, Qd, Kd, Vd)
    torch.cuda.synchronize()
    assert torch.equal(pooled, pooled1) and torch.equal(idx, idx1)
    assert torch.equal(Ko.view(torch.int16), Ko1.view(torch.int16)) and torch.equal(Vo.view(torch.int16), Vo1.view(torch.int16))
    ref_p = oracle.pool(oracle.score(Q[0, 0], K[0]), 7)
    assert_scores_close(pooled[0].cpu().numpy(), ref_p, n_q / L, "pooled")
    rk, rv = oracle.compact(K[0], V[0], np.ascontiguousarray(idx[0].cpu().numpy()))
    np.testing.assert_array_equal(from_dev_bf16(Ko)[0], rk)


@pytest.mark.parametrize("where", ["own_first_pages", "other_sequences_pages", "free_pages"])
def test_evict_paged_inplace_writes_the_pruned_cache_into_the_same_pools(where):
    # The kept rows land on pages of the pools they are taken from: each sequence's own first pages (so the rest
    # can be freed), pages that another sequence of the call still reads, or spare pages.  Read back through the
    # output table they are the pruned cache of the ordinary paged call; pages that receive nothing are untouched.
    torch = torch_()
    print("paged in-place", where, flush=True)
    ps = 64
    w = make_workload(1, seq_lens=[1500, 700], budget=[200, 70], n_layers=2)
    Q, K, V = w.assemble()
    Kp_, Vp_, tab_ = page_out(K, V, w.seq_lens, ps, seed=21, spare_pages=8)
    pages = jq.Pages(page_size=ps, n_pages=Kp_.shape[1], block_table=torch.from_numpy(tab_).cuda())
    Kp, Vp = to_dev_bf16(Kp_), to_dev_bf16(Vp_)
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets)
    Qd = to_dev_bf16(Q)
    Ko, Vo, idx, pooled = jq.evict_paged(sh, pages, Qd, Kp, Vp)               # reference: dense pruned cache
    table = pages.block_table.cpu().numpy()
    n_out = [-(-b // ps) for b in w.budgets]                                  # pages each sequence's kept rows need
    used = set(int(x) for s_, L in enumerate(w.seq_lens) for x in table[s_, :-(-L // ps)])
    spare = [pg for pg in range(pages.n_pages) if pg not in used]
    out_table = np.zeros((2, max(n_out)), dtype=np.int32)
    if where == "own_first_pages":
        for s_ in range(2):
            out_table[s_, :n_out[s_]] = table[s_, :n_out[s_]]
    elif where == "other_sequences_pages":                                    # sequence 0 writes onto sequence 1's pages and vice versa
        out_table[0, :n_out[0]] = table[1, :n_out[0]]
        out_table[1, :n_out[1]] = table[0, 5:5 + n_out[1]]
    else:
        assert len(spare) >= sum(n_out)
        out_table[0, :n_out[0]] = spare[:n_out[0]]
        out_table[1, :n_out[1]] = spare[n_out[0]:n_out[0] + n_out[1]]
    out_pages = jq.Pages(page_size=ps, n_pages=pages.n_pages, block_table=torch.from_numpy(out_table).cuda())
    Kq, Vq = Kp.clone(), Vp.clone()
    _, _, idx2, pooled2 = jq.evict_paged_inplace(sh, pages, out_pages, Qd, Kq, Vq)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(pooled, pooled2)
    Kq_h, Vq_h, Kp_h = from_dev_bf16(Kq), from_dev_bf16(Vq), from_dev_bf16(Kp)
    Ko_h, Vo_h = from_dev_bf16(Ko), from_dev_bf16(Vo)
    cb = w.cu_budgets
    written = set()
    for s_ in range(2):
        for b in range(w.budgets[s_]):
            pg, r = int(out_table[s_, b // ps]), b % ps
            np.testing.assert_array_equal(Kq_h[:, pg, r], Ko_h[:, cb[s_] + b])
            np.testing.assert_array_equal(Vq_h[:, pg, r], Vo_h[:, cb[s_] + b])
            written.add((pg, r))
    for pg in range(pages.n_pages):                                           # every other row of the pools is as before
        for r in range(ps):
            if (pg, r) not in written:
                assert np.array_equal(Kq_h[:, pg, r], Kp_h[:, pg, r]), (pg, r)


def test_evict_paged_inplace_with_supplied_normalisers_and_forced_positions():
    # one pass over the pools (normalisers supplied), sinks and a local window always kept, per-layer budgets:
    # the same kept rows as the ordinary paged call, on the sequences' own first pages
    torch = torch_()
    ps = 32
    w = make_workload(1, seq_lens=[1100, 260], budget=[96, 40], n_layers=2)
    Q, K, V = w.assemble()
    Kp_, Vp_, tab_ = page_out(K, V, w.seq_lens, ps, seed=5, spare_pages=3)
    pages = jq.Pages(page_size=ps, n_pages=Kp_.shape[1], block_table=torch.from_numpy(tab_).cuda())
    Kp, Vp = to_dev_bf16(Kp_), to_dev_bf16(Vp_)
    lb = torch.tensor([[96, 40], [50, 17]], dtype=torch.int32, device="cuda")
    sh = jq.Shape(n_layers=2, seq_lens=w.seq_lens, n_q=w.n_q, h_q=w.h_q, h_kv=w.h_kv, pool_k=w.pool_k, budgets=w.budgets,
                  keep_first=4, keep_last=8, layer_budgets=lb)
    lse = torch.full((2, 2, w.n_q, w.h_q), 12.0, dtype=torch.float32, device="cuda")   # above every logit of this workload
    Qd = to_dev_bf16(Q)
    Ko = torch.zeros((2, sh.TB, w.h_kv, w.d), dtype=torch.bfloat16, device="cuda"); Vo = torch.zeros_like(Ko)
    idx = torch.full((2, w.h_kv, sh.TB), -1, dtype=torch.int32, device="cuda")
    _, _, _, pooled = jq.evict_paged(sh, pages, Qd, Kp, Vp, lse=lse, K_out=Ko, V_out=Vo, idx_out=idx)
    table = pages.block_table.cpu().numpy()
    n_out = [-(-b // ps) for b in w.budgets]
    out_table = np.zeros((2, max(n_out)), dtype=np.int32)
    for s_ in range(2):
        out_table[s_, :n_out[s_]] = table[s_, :n_out[s_]]
    out_pages = jq.Pages(page_size=ps, n_pages=pages.n_pages, block_table=torch.from_numpy(out_table).cuda())
    Kq, Vq = Kp.clone(), Vp.clone()
    idx2 = torch.full_like(idx, -1)
    _, _, _, pooled2 = jq.evict_paged_inplace(sh, pages, out_pages, Qd, Kq, Vq, lse=lse, idx_out=idx2)
    torch.cuda.synchronize()
    assert torch.equal(idx, idx2) and torch.equal(pooled, pooled2)
    Kq_h, Vq_h, Ko_h, Vo_h = from_dev_bf16(Kq), from_dev_bf16(Vq), from_dev_bf16(Ko), from_dev_bf16(Vo)
    idx_h, lb_h, cb = idx.cpu().numpy(), lb.cpu().numpy(), w.cu_budgets
    for layer in range(2):
        for s_ in range(2):
            B, L = int(lb_h[layer, s_]), w.seq_lens[s_]
            kept = idx_h[layer, :, cb[s_]:cb[s_] + B]
            assert (kept[:, :4] == np.arange(4)).all() and (kept[:, -8:] == np.arange(L - 8, L)).all()   # sinks and window
            assert (idx_h[layer, :, cb[s_] + B:cb[s_ + 1]] == -1).all()                                   # unused slots untouched
            for b in range(B):
                pg, r = int(out_table[s_, b // ps]), b % ps
                np.testing.assert_array_equal(Kq_h[layer, pg, r], Ko_h[layer, cb[s_] + b])
                np.testing.assert_array_equal(Vq_h[layer, pg, r], Vo_h[layer, cb[s_] + b])
