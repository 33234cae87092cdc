"""Pins of the oracle's eviction step during decoding (`oracle.stream_step`).  The paper only names streaming
eviction in the decoding phase as future work (closing paragraph) and prints no example; the step is the Section 4.3
eviction applied to an already pruned cache plus a table of the rows' original positions, so it is pinned by a
hand-worked case, by its reduction to the prefill-time eviction, by the identity case, by an independent numpy
re-implementation run over several steps, and by the retention guarantees."""
import numpy as np

import oracle
from workloads import bf16_bits_to_f64, f32_to_bf16_bits


def bits(x):
    return f32_to_bf16_bits(np.asarray(x, dtype=np.float32))


def test_hand_worked_step_keeps_the_two_best_rows_and_their_positions():
    # one head, one query (sqrt 2, 0) at scale 1/sqrt 2: logits (1, 0, -1) over keys (1,0), (0,1), (-1,0) -- the softmax of
    # tests/golden/softmax_three_keys.txt: 0.665, 0.245, 0.090.  The rows came from tokens 10, 20, 30; with B = 2 the first
    # two stay.  (sqrt 2 is not a bf16 number, but any positive first coordinate gives the same ranking.)
    Q = bits([[[1.4140625, 0.0]]])                               # [n_q=1, h_q=1, d=2]
    K = bits([[[1.0, 0.0]], [[0.0, 1.0]], [[-1.0, 0.0]]])        # [3, 1, 2]
    V = bits([[[5.0, 6.0]], [[7.0, 8.0]], [[9.0, 10.0]]])
    r = oracle.stream_step(Q, K, V, np.array([[10, 20, 30]]), B=2)
    assert r["idx"].tolist() == [[0, 1]] and r["pos_out"].tolist() == [[10, 20]]
    assert np.array_equal(r["K_out"], K[:2]) and np.array_equal(r["V_out"], V[:2])
    r1 = oracle.stream_step(Q, K, V, np.array([[10, 20, 30]]), B=1, keep_last=1)     # the newest row is protected
    assert r1["pos_out"].tolist() == [[30]]


def test_first_step_on_an_unpruned_cache_is_the_prefill_eviction():
    rng = np.random.default_rng(5)
    Q = bits(rng.standard_normal((4, 4, 16))); K = bits(rng.standard_normal((50, 2, 16))); V = bits(rng.standard_normal((50, 2, 16)))
    pos = np.tile(np.arange(50), (2, 1))
    a = oracle.evict(Q, K, V, 12, 3)
    b = oracle.stream_step(Q, K, V, pos, 12, pool_k=3)
    assert np.array_equal(a["idx"], b["idx"]) and np.array_equal(b["pos_out"], b["idx"])
    assert np.array_equal(a["K_out"], b["K_out"]) and np.array_equal(a["V_out"], b["V_out"])


def test_keeping_every_row_changes_nothing():
    rng = np.random.default_rng(6)
    Q = bits(rng.standard_normal((3, 2, 8))); K = bits(rng.standard_normal((9, 2, 8))); V = bits(rng.standard_normal((9, 2, 8)))
    pos = np.stack([np.sort(rng.choice(100, 9, replace=False)) for _ in range(2)])
    r = oracle.stream_step(Q, K, V, pos, 9)
    assert np.array_equal(r["K_out"], K) and np.array_equal(r["V_out"], V) and np.array_equal(r["pos_out"], pos)


def numpy_step(Q, K, V, pos, B, keep_last, G):
    """The same step written independently with numpy (softmax, argsort)."""
    q, k = bf16_bits_to_f64(Q), bf16_bits_to_f64(K)
    rows, h_kv, d = k.shape
    Ko = np.empty((B, h_kv, d), dtype=np.uint16); Vo = np.empty_like(Ko); po = np.empty((h_kv, B), dtype=np.int64)
    for g in range(h_kv):
        logits = np.einsum("ihc,jc->ihj", q[:, g * G:(g + 1) * G], k[:, g]) / np.sqrt(d)
        p = np.exp(logits - logits.max(axis=2, keepdims=True))
        score = (p / p.sum(axis=2, keepdims=True)).sum(axis=(0, 1))
        forced = np.arange(rows - keep_last, rows)
        free = np.arange(rows - keep_last)
        order = free[np.lexsort((free, -score[free]))][:B - keep_last]
        keep = np.sort(np.concatenate([order, forced]))
        Ko[:, g], Vo[:, g], po[g] = K[keep, g], V[keep, g], pos[g, keep]
    return Ko, Vo, po


def test_several_steps_against_numpy():
    # prompt of 40 tokens, budget 12, eight decoded tokens between steps (always kept for one step), three steps
    rng = np.random.default_rng(7)
    h_kv, G, d, B, n_new = 2, 2, 16, 12, 4
    K = bits(rng.standard_normal((40, h_kv, d))); V = bits(rng.standard_normal((40, h_kv, d)))
    pos = np.tile(np.arange(40), (h_kv, 1))
    Kn, Vn, pn = K, V, pos
    next_tok = 40
    for step in range(3):
        Q = bits(rng.standard_normal((3, h_kv * G, d)))
        kl = 0 if step == 0 else n_new
        r = oracle.stream_step(Q, K, V, pos, B, keep_last=kl)
        Kn, Vn, pn = numpy_step(Q, Kn, Vn, pn, B, kl, G)
        assert np.array_equal(r["K_out"], Kn) and np.array_equal(r["V_out"], Vn) and np.array_equal(r["pos_out"], pn)
        assert (np.diff(r["pos_out"], axis=1) > 0).all()                       # rows stay in token order
        if step > 0:
            assert (r["pos_out"][:, -n_new:] == np.arange(next_tok - n_new, next_tok)).all()   # the newest tokens survive
        new_k = bits(rng.standard_normal((n_new, h_kv, d))); new_v = bits(rng.standard_normal((n_new, h_kv, d)))
        new_p = np.tile(np.arange(next_tok, next_tok + n_new), (h_kv, 1))
        next_tok += n_new
        K = np.concatenate([r["K_out"], new_k]); V = np.concatenate([r["V_out"], new_v]); pos = np.concatenate([r["pos_out"], new_p], axis=1)
        Kn, Vn, pn = K.copy(), V.copy(), pos.copy()
