"""The seeded input generators: determinism, shapes, bf16 rounding, planted structure."""
import numpy as np

import oracle
from workloads import CONFIGS, bf16_bits_to_f32, f32_to_bf16_bits, make_workload, page_out


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is exactly halfway between bf16 neighbours 1.0 and 1 + 2^-7 -> ties to even (1.0)
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20, 1.0 + 3 * 2.0 ** -8, -2.5, 0.0], dtype=np.float32)
    b = f32_to_bf16_bits(x)
    np.testing.assert_array_equal(bf16_bits_to_f32(b), np.array([1.0, 1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -6, -2.5, 0.0], dtype=np.float32))
    r = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    back = bf16_bits_to_f32(f32_to_bf16_bits(r))
    assert np.max(np.abs(back - r) / np.abs(r)) <= 2.0 ** -8


def test_deterministic_and_thread_independent():
    a = make_workload(2, seq_lens=[20000]); a.threads = 1
    b = make_workload(2, seq_lens=[20000]); b.threads = 4
    for x, y in zip(a.tensors(0, 0), b.tensors(0, 0)):
        np.testing.assert_array_equal(x, y)
    c = make_workload(2, seq_lens=[20000], seed=7)
    assert not np.array_equal(a.tensors(0, 0)[1], c.tensors(0, 0)[1])


def test_named_shapes():
    for cid, c in CONFIGS.items():
        w = make_workload(cid)
        assert w.h_q % w.h_kv == 0 and w.d == 128 and w.pool_k == 7
        assert len(w.budgets) == w.n_seq and all(1 <= b <= L for b, L in zip(w.budgets, w.seq_lens))
    w5 = make_workload(5)
    assert w5.n_seq == 16 and min(w5.seq_lens) >= 4096 and max(w5.seq_lens) <= 131072
    assert w5.budgets == [min(2048, L // 8) for L in w5.seq_lens]
    assert w5.cu_seqlens[-1] == sum(w5.seq_lens)
    assert make_workload(4).n_layers == 32 and make_workload(3).seq_lens == [131072]
    assert [make_workload(2, budget=b).budgets[0] for b in (128, 512, 2048)] == [128, 512, 2048]


def test_outlier_channels_are_scaled():
    w = make_workload(2, seq_lens=[4096])
    _, K, _ = w.tensors(0, 0)
    Kf = bf16_bits_to_f32(K)
    planted = np.zeros(4096, dtype=bool)
    for p in w.planted_positions(0, 0):
        planted[p] = True
    std = Kf[~planted].reshape(-1, 128).std(axis=0)
    out = np.zeros(128, dtype=bool); out[list(w.outlier_channels)] = True
    assert len(w.outlier_channels) == 4
    assert (std[out] > 7).all() and (std[~out] < 1.2).all()


def test_config1_planted_keys_are_recovered():
    w = make_workload(1)
    Q, K, V = w.tensors(0, 0)
    r = oracle.evict(Q, K, V, w.budgets[0], w.pool_k)
    for g, pos in enumerate(w.planted_positions(0, 0)):
        assert len(pos) == 20
        assert set(pos.tolist()) <= set(r["idx"][g].tolist())
        assert r["scores"][g][pos].mean() > 10 * r["scores"][g].mean()


def test_aligned_plants_are_heavy_hitters():
    # pooling spreads each isolated plant over 7 positions, so the budget is sized for 7 x 82
    w = make_workload(2, seq_lens=[4096], budget=1024)
    Q, K, V = w.tensors(0, 0)
    r = oracle.evict(Q, K, V, 1024, w.pool_k)
    for g, pos in enumerate(w.planted_positions(0, 0)):
        assert len(pos) == 82
        assert r["scores"][g][pos].mean() > 5 * r["scores"][g].mean()
        assert len(set(pos.tolist()) & set(r["idx"][g].tolist())) >= 0.9 * len(pos)


def test_spans_are_contiguous():
    w = make_workload(3, seq_lens=[8192])
    pos = w.planted_positions(0, 0)[0]
    assert len(pos) == 512
    runs = np.split(pos, np.where(np.diff(pos) != 1)[0] + 1)
    assert all(len(r) % 64 == 0 for r in runs)


def test_page_out_round_trip():
    rng = np.random.default_rng(5)
    seq_lens = [100, 7, 260]
    K = rng.integers(0, 60000, (2, sum(seq_lens), 3, 128)).astype(np.uint16)
    V = rng.integers(0, 60000, K.shape).astype(np.uint16)
    Kp, Vp, table = page_out(K, V, seq_lens, 64, seed=1)
    assert Kp.shape == (2, 2 + 1 + 5 + 3, 64, 3, 128) and table.shape == (3, 5)
    used = table[table >= 0]
    assert len(set(used.tolist())) == used.size == 8                      # every page belongs to one place only
    assert (table[1, 1:] == -1).all() and (table[0, 2:] == -1).all()
    tok = 0
    for s, L in enumerate(seq_lens):
        for t in range(L):
            np.testing.assert_array_equal(Kp[:, table[s, t // 64], t % 64], K[:, tok + t])
            np.testing.assert_array_equal(Vp[:, table[s, t // 64], t % 64], V[:, tok + t])
        tok += L
    assert (Kp[:, table[1, 0], 7:] == 0x7FC0).all()                       # rows past a sequence's end are poisoned
    a = page_out(K, V, seq_lens, 64, seed=1)[2]
    b = page_out(K, V, seq_lens, 64, seed=2)[2]
    assert np.array_equal(a, table) and not np.array_equal(b, table)
