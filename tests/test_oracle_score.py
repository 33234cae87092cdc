"""Pins for the oracle's importance scores (Eq. 3 / Section 4.3 of the paper).

The paper prints no worked numeric example for this path, so the oracle is tied
to closed forms, invariants of the softmax, constructions whose answer is known
in advance, and independent brute force.  Each test is chosen so that one kind
of plausible slip (dropped scale, wrong sign, transposed operand, wrong GQA
mapping, missing max-subtraction, mean instead of sum) makes it fail.
"""
import math
import os

import numpy as np
import pytest

import oracle
from workloads import bf16_bits_to_f64, f32_to_bf16_bits


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def rand_bits(rng, shape, scale=1.0):
    return bits(rng.standard_normal(shape).astype(np.float32) * scale)


def test_hand_worked_three_keys(golden_dir):
    want = np.loadtxt(os.path.join(golden_dir, "softmax_three_keys.txt"))
    q = bits([[[2, 0, 0, 0]]])                                   # n_q=1, h_q=1, d=4  -> scale 1/2
    k = bits([[[1, 0, 0, 0]], [[0, 1, 0, 0]], [[-1, 0, 0, 0]]])  # L=3, h_kv=1
    got = oracle.score(q, k)
    assert got.shape == (1, 3)
    np.testing.assert_allclose(got[0], want, rtol=0, atol=1e-15)


def test_explicit_scale_overrides_default():
    # same logits (1,0,-1) reached with scale=1 and q=(1,0,0,0)
    q = bits([[[1, 0, 0, 0]]])
    k = bits([[[1, 0, 0, 0]], [[0, 1, 0, 0]], [[-1, 0, 0, 0]]])
    s = math.e + 1 + 1 / math.e
    np.testing.assert_allclose(oracle.score(q, k, scale=1.0)[0], [math.e / s, 1 / s, 1 / (math.e * s)], atol=1e-15)


@pytest.mark.parametrize("n_q,h_q,h_kv,d,L", [(3, 4, 2, 8, 37), (16, 8, 2, 128, 300), (5, 6, 6, 16, 64)])
def test_rows_sum_to_one(n_q, h_q, h_kv, d, L):
    rng = np.random.default_rng(1)
    Q, K = rand_bits(rng, (n_q, h_q, d)), rand_bits(rng, (L, h_kv, d))
    s = oracle.score(Q, K)
    G = h_q // h_kv
    np.testing.assert_allclose(s.sum(axis=1), n_q * G, rtol=1e-12)
    assert (s >= 0).all() and (s <= n_q * G).all()


def test_single_key_gets_everything():
    rng = np.random.default_rng(2)
    Q, K = rand_bits(rng, (4, 4, 8)), rand_bits(rng, (1, 2, 8))
    np.testing.assert_array_equal(oracle.score(Q, K), np.full((2, 1), 8.0))


def test_zero_queries_and_equal_keys_are_uniform():
    rng = np.random.default_rng(3)
    K = rand_bits(rng, (50, 2, 16))
    Q0 = np.zeros((3, 4, 16), dtype=np.uint16)
    np.testing.assert_allclose(oracle.score(Q0, K), 3 * 2 / 50, rtol=1e-14)
    Q = rand_bits(rng, (3, 4, 16))
    Keq = np.broadcast_to(rand_bits(rng, (1, 2, 16)), (50, 2, 16)).copy()
    np.testing.assert_allclose(oracle.score(Q, Keq), 3 * 2 / 50, rtol=1e-13)


def test_key_shift_invariance_with_large_shift():
    # adding one vector to every key changes each query's logits by a constant;
    # with a big shift this only survives if the maximum is subtracted before exp
    rng = np.random.default_rng(4)
    n_q, h_q, h_kv, d, L = 4, 2, 1, 8, 40
    Qf = rng.integers(-3, 4, (n_q, h_q, d)).astype(np.float32)
    Kf = rng.integers(-3, 4, (L, h_kv, d)).astype(np.float32)
    shift = np.full((1, 1, d), 96.0, dtype=np.float32)          # logits move by up to ~ +-800
    a = oracle.score(bits(Qf), bits(Kf))
    b = oracle.score(bits(Qf), bits(Kf + shift))                  # small ints + 96 are exact in bf16
    assert np.isfinite(b).all()
    np.testing.assert_allclose(a, b, rtol=1e-10)


def test_permutation_and_duplication_laws():
    rng = np.random.default_rng(5)
    n_q, h_q, h_kv, d, L = 5, 4, 2, 16, 33
    Q, K = rand_bits(rng, (n_q, h_q, d)), rand_bits(rng, (L, h_kv, d))
    base = oracle.score(Q, K)
    perm = rng.permutation(L)
    np.testing.assert_allclose(oracle.score(Q, K[perm]), base[:, perm], rtol=1e-12)
    np.testing.assert_allclose(oracle.score(Q[rng.permutation(n_q)], K), base, rtol=1e-12)
    Qs = Q.copy(); Qs[:, [0, 1]] = Q[:, [1, 0]]                  # swap two heads of KV group 0
    np.testing.assert_allclose(oracle.score(Qs, K), base, rtol=1e-12)
    np.testing.assert_allclose(oracle.score(np.concatenate([Q, Q]), K), 2 * base, rtol=1e-12)


def test_gqa_mapping_is_contiguous_groups():
    # h_q=4, h_kv=2: query heads {0,1} read KV head 0, {2,3} read KV head 1.
    # Only query head 1 is non-zero and KV head 0 has one aligned key; under an
    # interleaved mapping (h % h_kv) head 1 would read KV head 1 instead.
    d, L = 4, 6
    Q = np.zeros((1, 4, d), dtype=np.float32); Q[0, 1] = [4, 0, 0, 0]      # logit = 4*k0/2
    K = np.zeros((L, 2, d), dtype=np.float32)
    K[2, 0] = [1, 0, 0, 0]          # KV head 0: key 2 gets logit 2, others 0
    K[4, 1] = [1, 0, 0, 0]          # KV head 1: would light up key 4 if mapping were wrong
    s = oracle.score(bits(Q), bits(K))
    e2 = math.exp(2.0)
    want0 = np.full(L, 1.0 / L) + np.where(np.arange(L) == 2, e2, 1.0) / (e2 + L - 1)
    np.testing.assert_allclose(s[0], want0, rtol=1e-14)
    np.testing.assert_allclose(s[1], np.full(L, 2.0 / L), rtol=1e-14)


def test_operands_not_transposed():
    # distinct sizes everywhere and a key that matches exactly one query row
    d, L = 8, 5
    Q = np.zeros((2, 1, d), dtype=np.float32); Q[0, 0, 3] = 4.0; Q[1, 0, 5] = 4.0
    K = np.zeros((L, 1, d), dtype=np.float32); K[1, 0, 3] = 2.0; K[3, 0, 5] = -2.0
    sc = 1.0 / math.sqrt(d)
    a, b = math.exp(8 * sc), math.exp(-8 * sc)
    want = np.array([1.0, a, 1.0, 1.0, 1.0]) / (a + 4) + np.array([1.0, 1.0, 1.0, b, 1.0]) / (b + 4)
    np.testing.assert_allclose(oracle.score(bits(Q), bits(K))[0], want, rtol=1e-14)


def test_brute_force_without_max_subtraction():
    # independent naive loops (math.exp on raw logits, no stabilisation)
    rng = np.random.default_rng(6)
    n_q, h_q, h_kv, d, L = 3, 4, 2, 8, 11
    Q, K = rand_bits(rng, (n_q, h_q, d), 0.7), rand_bits(rng, (L, h_kv, d), 0.7)
    Qd, Kd = bf16_bits_to_f64(Q), bf16_bits_to_f64(K)
    G = h_q // h_kv
    want = [[0.0] * L for _ in range(h_kv)]
    for h in range(h_q):
        for i in range(n_q):
            e = []
            for j in range(L):
                dot = 0.0
                for c in range(d):
                    dot += Qd[i, h, c] * Kd[j, h // G, c]
                e.append(math.exp(dot / math.sqrt(d)))
            z = sum(e)
            for j in range(L):
                want[h // G][j] += e[j] / z
    np.testing.assert_allclose(oracle.score(Q, K), np.array(want), rtol=1e-12)


def test_matches_numpy_softmax_on_a_medium_case():
    rng = np.random.default_rng(7)
    n_q, h_q, h_kv, d, L = 16, 8, 2, 128, 517
    Q, K = rand_bits(rng, (n_q, h_q, d)), rand_bits(rng, (L, h_kv, d))
    Qd, Kd = bf16_bits_to_f64(Q), bf16_bits_to_f64(K)
    G = h_q // h_kv
    logits = np.einsum("ihc,jhc->hij", Qd, np.repeat(Kd, G, axis=1)) / math.sqrt(d)
    p = np.exp(logits - logits.max(axis=2, keepdims=True))
    p /= p.sum(axis=2, keepdims=True)
    want = p.sum(axis=1).reshape(h_kv, G, L).sum(axis=1)
    np.testing.assert_allclose(oracle.score(Q, K), want, rtol=1e-11)


def test_rejects_bad_shapes():
    Q = np.zeros((1, 3, 4), dtype=np.uint16); K = np.zeros((2, 2, 4), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.score(Q, K)                                       # 3 % 2 != 0


# ---------------------------------------------------------------- slice of a wider softmax (supplied lse)
def numpy_logits(Q, K):
    Qd, Kd = bf16_bits_to_f64(Q), bf16_bits_to_f64(K)
    G = Q.shape[1] // K.shape[1]
    return np.einsum("ihc,jhc->ihj", Qd, np.repeat(Kd, G, axis=1)) / math.sqrt(Q.shape[2])   # [n_q, h_q, L]


def test_score_lse_hand_worked_with_one_extra_key():
    # logits (1, 0, -1) over the prompt plus one soft-token key with logit 1/2 in the normaliser
    q = bits([[[2, 0, 0, 0]]])
    k = bits([[[1, 0, 0, 0]], [[0, 1, 0, 0]], [[-1, 0, 0, 0]]])
    z = math.e + 1 + 1 / math.e + math.exp(0.5)
    got = oracle.score_lse(q, k, np.array([[math.log(z)]]))
    np.testing.assert_allclose(got[0], [math.e / z, 1 / z, 1 / (math.e * z)], rtol=1e-15)


def test_score_lse_over_the_prompt_equals_score():
    rng = np.random.default_rng(8)
    Q, K = rand_bits(rng, (5, 4, 16)), rand_bits(rng, (77, 2, 16))
    s = numpy_logits(Q, K)
    m = s.max(axis=2)
    lse = m + np.log(np.exp(s - m[..., None]).sum(axis=2))        # [n_q, h_q], independent numpy logsumexp
    np.testing.assert_allclose(oracle.score_lse(Q, K, lse), oracle.score(Q, K), rtol=1e-12)


def test_score_lse_wider_domain_scales_each_row():
    # a causal soft-token tail adds mass to each row's normaliser: every row's contribution shrinks by
    # Z_prompt / Z_all, checked against numpy with explicit soft-token keys
    rng = np.random.default_rng(9)
    n_q, h_q, h_kv, d, L = 4, 4, 2, 8, 21
    Q, K, Ks = rand_bits(rng, (n_q, h_q, d)), rand_bits(rng, (L, h_kv, d)), rand_bits(rng, (n_q, h_kv, d))
    s, st = numpy_logits(Q, K), numpy_logits(Q, Ks)                # [n_q,h_q,L], [n_q,h_q,n_q]
    causal = np.tril(np.ones((n_q, n_q), dtype=bool))[:, None, :]  # soft token i sees soft keys 0..i
    z_all = np.exp(s).sum(axis=2) + np.where(causal, np.exp(st), 0.0).sum(axis=2)
    want = (np.exp(s) / z_all[..., None]).sum(axis=0).reshape(h_kv, h_q // h_kv, L).sum(axis=1)
    got = oracle.score_lse(Q, K, np.log(z_all))
    np.testing.assert_allclose(got, want, rtol=1e-12)
    assert (got.sum(axis=1) < n_q * (h_q // h_kv)).all()           # rows no longer sum to one


def test_score_lse_rejects_wrong_lse_shape():
    Q = np.zeros((2, 2, 4), dtype=np.uint16); K = np.zeros((3, 2, 4), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.score_lse(Q, K, np.zeros((2, 3)))


# ---------------------------------------------------------------- soft tokens' own keys in the softmax (causal tail)
def test_score_tail_hand_worked_powers_of_two(golden_dir):
    want = np.loadtxt(os.path.join(golden_dir, "softmax_with_soft_token_tail.txt"))
    q = bits([[[1.0]], [[1.0]]])                 # n_q=2, h_q=1, d=1
    k = bits([[[0.0]], [[1.0]]])                 # L=2
    kt = bits([[[2.0]], [[0.0]]])                # soft-token keys
    got = oracle.score_tail(q, k, kt, scale=math.log(2.0))
    np.testing.assert_allclose(got[0], want, rtol=1e-15)
    # dropping the diagonal (token not attending to itself) would give (1/3 + 1/7, 2/3 + 2/7); seeing the
    # future key from token 0 would give (1/8 + 1/8, 2/8 + 2/8): both are far from the stored values
    assert abs(got[0, 0] - (1 / 3 + 1 / 7)) > 0.1 and abs(got[0, 0] - 0.25) > 0.01


def test_score_tail_single_soft_token_is_plain_softmax_over_prompt_plus_itself():
    # with one soft token its row is the ordinary softmax over the L + 1 keys: the already pinned
    # jqo_score on the concatenated keys, prompt columns only
    rng = np.random.default_rng(21)
    Q, K, Kt = rand_bits(rng, (1, 4, 16)), rand_bits(rng, (50, 2, 16)), rand_bits(rng, (1, 2, 16))
    want = oracle.score(Q, np.concatenate([K, Kt], axis=0))[:, :50]
    np.testing.assert_allclose(oracle.score_tail(Q, K, Kt), want, rtol=1e-12)


def test_score_tail_matches_numpy_with_causal_mask_and_the_lse_variant():
    rng = np.random.default_rng(22)
    n_q, h_q, h_kv, d, L = 5, 6, 2, 8, 33
    Q, K, Kt = rand_bits(rng, (n_q, h_q, d), 1.5), rand_bits(rng, (L, h_kv, d)), rand_bits(rng, (n_q, h_kv, d), 2.0)
    s, st = numpy_logits(Q, K), numpy_logits(Q, Kt)
    causal = np.tril(np.ones((n_q, n_q), dtype=bool))[:, None, :]
    z_all = np.exp(s).sum(axis=2) + np.where(causal, np.exp(st), 0.0).sum(axis=2)
    want = (np.exp(s) / z_all[..., None]).sum(axis=0).reshape(h_kv, h_q // h_kv, L).sum(axis=1)
    got = oracle.score_tail(Q, K, Kt)
    np.testing.assert_allclose(got, want, rtol=1e-12)
    np.testing.assert_allclose(got, oracle.score_lse(Q, K, np.log(z_all)), rtol=1e-12)


def test_score_tail_is_causal_and_uses_the_right_kv_head():
    rng = np.random.default_rng(23)
    n_q, h_q, h_kv, d, L = 3, 4, 2, 8, 17
    Q, K, Kt = rand_bits(rng, (n_q, h_q, d)), rand_bits(rng, (L, h_kv, d)), rand_bits(rng, (n_q, h_kv, d))
    base = oracle.score_tail(Q, K, Kt)
    # the last soft token's key is seen by the last soft token only: with n_q = 1 rows nothing else changes
    Kt2 = Kt.copy(); Kt2[2] = bits(rng.standard_normal((h_kv, d)).astype(np.float32) * 3)
    first_two = oracle.score_tail(Q[:2], K, Kt[:2])
    np.testing.assert_allclose(oracle.score_tail(Q[:2], K, Kt2[:2]), first_two, rtol=0)
    changed = oracle.score_tail(Q, K, Kt2)
    last_old = base - first_two                    # contribution of soft token 2 alone (scores add over rows)
    last_new = changed - first_two
    assert not np.allclose(last_old, last_new)
    # soft-token keys of KV head 1 never touch the scores of KV head 0
    Kt3 = Kt.copy(); Kt3[:, 1] = bits(rng.standard_normal((n_q, d)).astype(np.float32) * 3)
    np.testing.assert_allclose(oracle.score_tail(Q, K, Kt3)[0], base[0], rtol=0)
    assert not np.allclose(oracle.score_tail(Q, K, Kt3)[1], base[1])


def test_score_tail_vanishing_tail_keys_give_the_prompt_only_scores():
    # soft-token keys pointing away from every query (logit about -|q|^2 * 40 * scale) carry no mass
    rng = np.random.default_rng(24)
    Q, K = rand_bits(rng, (2, 2, 16)), rand_bits(rng, (40, 2, 16))
    Qd = bf16_bits_to_f64(Q)
    Kt = bits((-40.0 * Qd.sum(axis=0)).astype(np.float32))       # [h_kv = h_q, d]: against both soft tokens' queries
    Kt = np.stack([Kt, Kt])
    logits = np.einsum("ihc,thc->iht", Qd, bf16_bits_to_f64(Kt)) / 4.0
    assert logits.max() < -50                                      # the construction did what it should
    np.testing.assert_allclose(oracle.score_tail(Q, K, Kt), oracle.score(Q, K), rtol=1e-12)


def test_score_tail_rejects_wrong_shape():
    Q = np.zeros((2, 2, 4), dtype=np.uint16); K = np.zeros((3, 2, 4), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.score_tail(Q, K, np.zeros((3, 2, 4), dtype=np.uint16))


# ---------------------------------------------------------------- the prompt's own last tokens as queries (observation window)
def test_score_window_hand_worked_powers_of_two(golden_dir):
    # the hand-worked tail case read as ONE key tensor: prompt keys (0, 1) followed by the window's keys (2, 0)
    want = np.loadtxt(os.path.join(golden_dir, "softmax_with_soft_token_tail.txt"))
    q = bits([[[1.0]], [[1.0]]])
    k = bits([[[0.0]], [[1.0]], [[2.0]], [[0.0]]])
    got = oracle.score_window(q, k, scale=math.log(2.0))
    np.testing.assert_allclose(got[0, :2], want, rtol=1e-15)
    np.testing.assert_array_equal(got[0, 2:], [0.0, 0.0])             # the window's own positions are not scored


def test_score_window_equals_the_tail_variant_on_the_split_keys():
    rng = np.random.default_rng(31)
    n_q, h_q, h_kv, d, L = 5, 6, 2, 8, 40
    Q, K = rand_bits(rng, (n_q, h_q, d), 1.5), rand_bits(rng, (L, h_kv, d))
    got = oracle.score_window(Q, K)
    np.testing.assert_allclose(got[:, :L - n_q], oracle.score_tail(Q, K[:L - n_q], K[L - n_q:]), rtol=1e-12)
    assert not got[:, L - n_q:].any()


def test_score_window_matches_numpy_with_a_causal_mask():
    rng = np.random.default_rng(32)
    n_q, h_q, h_kv, d, L = 4, 4, 2, 8, 21
    Q, K = rand_bits(rng, (n_q, h_q, d), 1.5), rand_bits(rng, (L, h_kv, d))
    s = numpy_logits(Q, K)                                            # [n_q, h_q, L]
    pos = np.arange(L)[None, None, :]
    visible = pos <= (L - n_q + np.arange(n_q))[:, None, None]
    e = np.where(visible, np.exp(s), 0.0)
    p = e / e.sum(axis=2, keepdims=True)
    want = p.sum(axis=0).reshape(h_kv, h_q // h_kv, L).sum(axis=1)
    want[:, L - n_q:] = 0.0
    np.testing.assert_allclose(oracle.score_window(Q, K), want, rtol=1e-12)


def test_score_window_single_query_is_the_plain_softmax_and_later_keys_stay_invisible():
    rng = np.random.default_rng(33)
    Q, K = rand_bits(rng, (1, 4, 16)), rand_bits(rng, (30, 2, 16))
    np.testing.assert_allclose(oracle.score_window(Q, K)[:, :29], oracle.score(Q, K)[:, :29], rtol=1e-12)
    # three window tokens: the first two rows never see the last key
    Q3 = rand_bits(rng, (3, 4, 16))
    base = oracle.score_window(Q3[:2], K[:29])                        # window = positions 27, 28
    K2 = K.copy(); K2[29] = bits(rng.standard_normal((2, 16)).astype(np.float32) * 4)
    a, b = oracle.score_window(Q3, K), oracle.score_window(Q3, K2)    # window = positions 27, 28, 29
    only_last_a = a[:, :27] - base[:, :27]
    only_last_b = b[:, :27] - base[:, :27]
    assert not np.allclose(only_last_a, only_last_b)                  # the last row does see its own key ...
    assert (only_last_a > 0).all() and (only_last_b > 0).all()        # ... and the first two rows are unchanged by it


def test_score_window_rejects_more_queries_than_keys():
    Q = np.zeros((5, 2, 4), dtype=np.uint16); K = np.zeros((3, 2, 4), dtype=np.uint16)
    with pytest.raises(ValueError):
        oracle.score_window(Q, K)
