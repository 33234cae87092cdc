"""Pins for the oracle's pooling, top-B retention and pruned-cache gather
(Section 4.3; pooling as in the baselines paragraph of Section 5.1), and for the
hit-rate helper (Eq. 6)."""
import itertools

import numpy as np
import pytest

import oracle


# ---------------------------------------------------------------- pooling
@pytest.mark.parametrize("L", [1, 2, 3, 6, 7, 8, 40])
def test_pool_constant_input(L):
    c = 3.5
    j = np.arange(L)
    w = (np.minimum(j, 3) + np.minimum(L - 1 - j, 3) + 1) / 7.0
    np.testing.assert_allclose(oracle.pool(np.full(L, c), 7), c * w, rtol=1e-15)


def test_pool_constant_edges_are_4567():
    np.testing.assert_allclose(oracle.pool(np.full(20, 7.0), 7)[:5], [4, 5, 6, 7, 7], rtol=1e-15)
    np.testing.assert_allclose(oracle.pool(np.full(20, 7.0), 7)[-4:], [7, 6, 5, 4], rtol=1e-15)


@pytest.mark.parametrize("j", [0, 2, 10, 18, 19])
def test_pool_unit_impulse(j):
    L = 20
    x = np.zeros(L); x[j] = 1.0
    want = np.zeros(L); want[max(0, j - 3):min(L, j + 4)] = 1.0 / 7.0
    np.testing.assert_allclose(oracle.pool(x, 7), want, rtol=1e-15)


def test_pool_identity_linearity_and_weights():
    rng = np.random.default_rng(0)
    a, b = rng.random(57), rng.random(57)
    np.testing.assert_array_equal(oracle.pool(a, 1), a)
    np.testing.assert_allclose(oracle.pool(a + b, 7), oracle.pool(a, 7) + oracle.pool(b, 7), rtol=1e-14)
    j = np.arange(57)
    w = (np.minimum(j, 3) + np.minimum(56 - j, 3) + 1) / 7.0
    np.testing.assert_allclose(oracle.pool(a, 7).sum(), (w * a).sum(), rtol=1e-14)


@pytest.mark.parametrize("k", [3, 5, 7, 9])
def test_pool_matches_numpy_convolve(k):
    rng = np.random.default_rng(1)
    x = rng.random((3, 101))
    want = np.stack([np.convolve(r, np.ones(k) / k, mode="same") for r in x])
    np.testing.assert_allclose(oracle.pool(x, k), want, rtol=1e-13)


def test_pool_rejects_even_kernel():
    with pytest.raises(ValueError):
        oracle.pool(np.ones(8), 4)


# ---------------------------------------------------------------- top-B
def test_select_exhaustive_max_mass():
    rng = np.random.default_rng(2)
    for L in (5, 9, 12):
        x = rng.random(L)
        for B in range(1, L + 1):
            idx = oracle.select_topk(x, B)
            best = max(itertools.combinations(range(L), B), key=lambda c: sum(x[list(c)]))
            assert list(idx) == list(best)                                 # combinations are ascending tuples
            assert list(idx) == sorted(set(idx)) and idx.min() >= 0 and idx.max() < L


def test_select_special_cases():
    x = np.array([0.1, 0.9, 0.3, 0.9, 0.2])
    np.testing.assert_array_equal(oracle.select_topk(x, 1), [1])          # first argmax
    np.testing.assert_array_equal(oracle.select_topk(x, 2), [1, 3])
    np.testing.assert_array_equal(oracle.select_topk(x, 5), np.arange(5))  # B = L
    np.testing.assert_array_equal(oracle.select_topk(np.full(10, 0.5), 4), [0, 1, 2, 3])


def test_select_ties_prefer_lower_index():
    x = np.array([1.0, 2.0, 2.0, 2.0, 0.5, 2.0])
    np.testing.assert_array_equal(oracle.select_topk(x, 3), [1, 2, 3])
    np.testing.assert_array_equal(oracle.select_topk(x, 5), [0, 1, 2, 3, 5])


def test_select_matches_numpy_stable_sort():
    rng = np.random.default_rng(3)
    x = np.round(rng.random((4, 1000)), 2)                                # many exact ties
    for B in (1, 17, 500, 1000):
        got = oracle.select_topk(x, B)
        for g in range(4):
            order = np.lexsort((np.arange(1000), -x[g]))                  # score desc, index asc
            np.testing.assert_array_equal(got[g], np.sort(order[:B]))


def test_select_rejects_bad_budget():
    for B in (0, 6):
        with pytest.raises(ValueError):
            oracle.select_topk(np.ones(5), B)


# ---------------------------------------------------------------- top-B with forced positions
def test_select_keep_exhaustive():
    """Brute force: among all B-subsets that contain the forced positions, the kept set has the largest
    score mass over the free positions (random scores: no ties)."""
    rng = np.random.default_rng(21)
    for L in (6, 9, 11):
        x = rng.random(L)
        for kf, kl in ((0, 2), (1, 0), (2, 3), (1, 1)):
            forced = set(range(kf)) | set(range(L - kl, L))
            for B in range(kf + kl, L + 1):
                if B < 1:
                    continue
                idx = oracle.select_topk(x, B, kf, kl)
                cands = [c for c in itertools.combinations(range(L), B) if forced <= set(c)]
                best = max(cands, key=lambda c: sum(x[j] for j in c if j not in forced))
                assert list(idx) == list(best)


def test_select_keep_hand_cases():
    x = np.array([0.0, 0.9, 0.1, 0.8, 0.2, 0.7, 0.0, 0.0])
    np.testing.assert_array_equal(oracle.select_topk(x, 3, 1, 1), [0, 1, 7])       # sink + newest + best of the rest
    np.testing.assert_array_equal(oracle.select_topk(x, 4, 0, 2), [1, 3, 6, 7])    # window of two zeros is still kept
    np.testing.assert_array_equal(oracle.select_topk(x, 2, 1, 1), [0, 7])          # nothing left to compete for
    np.testing.assert_array_equal(oracle.select_topk(x, 8, 3, 3), np.arange(8))    # B = L
    # forced positions do not take part in the tie rule: of the free 0.5s the lowest positions win
    t = np.full(8, 0.5)
    np.testing.assert_array_equal(oracle.select_topk(t, 5, 1, 2), [0, 1, 2, 6, 7])
    # a forced position that would have been chosen anyway changes nothing
    np.testing.assert_array_equal(oracle.select_topk(x, 3, 0, 0), oracle.select_topk(x[:6], 3))
    np.testing.assert_array_equal(oracle.select_topk(x, 3, 2, 0), [0, 1, 3])


def test_select_keep_reduces_to_plain_selection_on_the_free_span():
    rng = np.random.default_rng(22)
    x = np.round(rng.random((3, 400)), 2)                                          # exact ties
    kf, kl, B = 4, 32, 100
    got = oracle.select_topk(x, B, kf, kl)
    inner = oracle.select_topk(np.ascontiguousarray(x[:, kf:400 - kl]), B - kf - kl) + kf
    for g in range(3):
        want = np.concatenate([np.arange(kf), inner[g], np.arange(400 - kl, 400)])
        np.testing.assert_array_equal(got[g], want)


def test_select_keep_rejects_more_forced_than_budget():
    with pytest.raises(ValueError):
        oracle.select_topk(np.ones(10), 4, 3, 2)
    with pytest.raises(ValueError):
        oracle.select_topk(np.ones(10), 4, -1, 2)


# ---------------------------------------------------------------- gather
def test_compact_is_a_gather():
    rng = np.random.default_rng(4)
    L, h_kv, d, B = 50, 3, 8, 7
    K = rng.integers(0, 65536, (L, h_kv, d)).astype(np.uint16)
    V = rng.integers(0, 65536, (L, h_kv, d)).astype(np.uint16)
    idx = np.stack([np.sort(rng.choice(L, B, replace=False)) for _ in range(h_kv)]).astype(np.int32)
    Ko, Vo = oracle.compact(K, V, idx)
    for g in range(h_kv):
        np.testing.assert_array_equal(Ko[:, g], np.take(K[:, g], idx[g], axis=0))
        np.testing.assert_array_equal(Vo[:, g], np.take(V[:, g], idx[g], axis=0))


def test_compact_full_budget_is_identity():
    rng = np.random.default_rng(5)
    K = rng.integers(0, 65536, (9, 2, 4)).astype(np.uint16)
    V = rng.integers(0, 65536, (9, 2, 4)).astype(np.uint16)
    idx = np.tile(np.arange(9, dtype=np.int32), (2, 1))
    Ko, Vo = oracle.compact(K, V, idx)
    np.testing.assert_array_equal(Ko, K)
    np.testing.assert_array_equal(Vo, V)


def test_compact_rejects_out_of_range_index():
    K = np.zeros((4, 1, 2), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.compact(K, K, np.array([[0, 4]], dtype=np.int32))


# ---------------------------------------------------------------- composition / hit rate
def test_evict_batch_equals_single_problems():
    from workloads import make_workload
    w = make_workload(1, seq_lens=[96, 40], budget=[16, 5], n_layers=2, plant="none")
    Q, K, V = w.assemble()
    out = oracle.evict_batch(Q, K, V, w.cu_seqlens, w.budgets, w.pool_k)
    cu, cb = w.cu_seqlens, w.cu_budgets
    for l in range(2):
        for s in range(2):
            one = oracle.evict(Q[l, s], K[l, cu[s]:cu[s + 1]], V[l, cu[s]:cu[s + 1]], w.budgets[s], w.pool_k)
            np.testing.assert_array_equal(out["idx"][l, :, cb[s]:cb[s + 1]], one["idx"])
            np.testing.assert_array_equal(out["K_out"][l, cb[s]:cb[s + 1]], one["K_out"])
            np.testing.assert_array_equal(out["pooled"][l, :, cu[s]:cu[s + 1]], one["pooled"])
    # ragged pooling must not bleed: first pooled value of sequence 1 only sees its own 4 taps
    np.testing.assert_allclose(out["pooled"][0, :, cu[1]], out["scores"][0, :, cu[1]:cu[1] + 4].sum(axis=1) / 7, rtol=1e-14)


def test_hit_rate():
    assert oracle.hit_rate([1, 2, 3, 4], [1, 2, 3, 4]) == 1.0
    assert oracle.hit_rate([1, 2, 9, 8], [1, 2, 3, 4]) == 0.5
    assert oracle.hit_rate([7], [1, 2]) == 0.0


# ---------------------------------------------------------------- Eq. 5 forward (training objective value)
def test_map_mse_closed_forms():
    L = 8
    a = np.full((1, L), 4.0)                       # 4 query rows, uniform map 1/L each -> averaged map 1/8
    assert oracle.map_mse(a, 4 * L, a, 4 * L)[0] == 0.0
    b = np.zeros((1, L)); b[0, 0] = 6.0            # 6 query rows, all mass on position 0 -> averaged map e_0
    # (1/8)[(1/8 - 1)^2 + 7 (1/8)^2] = (49 + 7) / 512
    np.testing.assert_allclose(oracle.map_mse(a, 4 * L, b, 6.0)[0], 56.0 / 512.0, rtol=1e-15)
    np.testing.assert_allclose(oracle.map_mse(b, 6.0, a, 4 * L)[0], 56.0 / 512.0, rtol=1e-15)   # symmetric
    # scaling both maps' row counts together with their scores changes nothing (maps are averages)
    np.testing.assert_allclose(oracle.map_mse(3 * a, 12 * L, 5 * b, 30.0)[0], 56.0 / 512.0, rtol=1e-15)


def test_map_mse_matches_numpy_on_real_maps_and_is_per_head():
    from workloads import f32_to_bf16_bits

    def rand_bits(rng, shape):
        return f32_to_bf16_bits(rng.standard_normal(shape).astype(np.float32))

    rng = np.random.default_rng(17)
    n, m, h_q, h_kv, d, L = 4, 9, 4, 2, 16, 50
    K = rand_bits(rng, (L, h_kv, d))
    Qs, Qr = rand_bits(rng, (n, h_q, d)), rand_bits(rng, (m, h_q, d))
    sa, sb = oracle.score(Qs, K), oracle.score(Qr, K)
    G = h_q // h_kv
    got = oracle.map_mse(sa, n * G, sb, m * G)
    want = ((sa / (n * G) - sb / (m * G)) ** 2).mean(axis=1)
    np.testing.assert_allclose(got, want, rtol=1e-13)
    assert abs(sa[0].sum() / (n * G) - 1.0) < 1e-12      # the averaged maps are probability vectors
    sb2 = sb.copy(); sb2[1] += 0.5                        # another head's map does not leak into head 0
    assert oracle.map_mse(sa, n * G, sb2, m * G)[0] == got[0]
    with pytest.raises(ValueError):
        oracle.map_mse(sa, 0.0, sb, 1.0)
