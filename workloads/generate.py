"""Seeded generators for the five benchmark workloads.

Every tensor is drawn as fp32 N(0,1) from numpy's PCG64 with a SeedSequence
keyed by (layer, sequence, tensor, chunk), rounded to bf16 (round to nearest
even) and handed out as raw uint16 bit patterns, so that every consumer sees
identical bits whatever it does with them afterwards.  Chunked keys make the
result independent of how many worker threads fill a tensor.

Value structure (stand-ins for the paper's long-context workloads, whose data
and trained soft tokens are not available):

* "subset"  : a few positions whose key, for each KV head, is 3 x the mean of a
              random subset of that head's query vectors plus N(0, 0.1^2).
* "aligned" : a fraction of positions per KV head whose key is
              2.5 * sqrt(d) * qbar / |qbar| + N(0, 0.1^2), qbar = mean of the
              query vectors of the head's GQA group.
* "spans"   : same key as "aligned" but on 8 contiguous spans of 64 tokens,
              shared by all KV heads.

Keys of the 8B/7B-shaped workloads also carry 4 outlier channels scaled x8.
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

BASE_SEED = 250900
_CHUNK_TOKENS = 8192
_T_Q, _T_K, _T_V, _T_PLANT, _T_NOISE = 0, 1, 2, 3, 4


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round finite fp32 values to bf16 (nearest even); returns uint16 bits."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + bias) >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


CONFIGS = {
    1: dict(name="tiny_L2048", n_layers=1, seq_lens=[2048], h_q=8, h_kv=2, d=128, n_q=16,
            budget=256, pool_k=7, plant="subset", outliers=False),
    2: dict(name="llama31_8b_layer_L32768", n_layers=1, seq_lens=[32768], h_q=32, h_kv=8, d=128,
            n_q=32, budget=512, pool_k=7, plant="aligned", density=0.02, outliers=True),
    3: dict(name="mistral_7b_layer_L131072", n_layers=1, seq_lens=[131072], h_q=32, h_kv=8, d=128,
            n_q=32, budget=2048, pool_k=7, plant="spans", outliers=True),
    4: dict(name="llama31_8b_32layers_L65536", n_layers=32, seq_lens=[65536], h_q=32, h_kv=8, d=128,
            n_q=32, budget=1024, pool_k=7, plant="aligned", density=0.02, outliers=True),
    5: dict(name="ragged_16seq", n_layers=1, seq_lens="ragged16", h_q=32, h_kv=8, d=128, n_q=32,
            budget="min(2048,L/8)", pool_k=7, plant="aligned", density="ragged", outliers=True),
}


def _rng(seed: int, *key: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(entropy=seed, spawn_key=tuple(key))))


def _normal_bf16(seed: int, key: tuple, rows: int, row_elems: int, pool: ThreadPoolExecutor | None) -> np.ndarray:
    """rows x row_elems N(0,1) values as bf16 bits, filled chunk by chunk."""
    out = np.empty((rows, row_elems), dtype=np.uint16)
    starts = list(range(0, rows, _CHUNK_TOKENS))

    def fill(ci_start):
        ci, start = ci_start
        stop = min(rows, start + _CHUNK_TOKENS)
        x = _rng(seed, *key, ci).standard_normal((stop - start, row_elems), dtype=np.float32)
        out[start:stop] = f32_to_bf16_bits(x)

    jobs = list(enumerate(starts))
    if pool is None or len(jobs) == 1:
        for j in jobs:
            fill(j)
    else:
        list(pool.map(fill, jobs))
    return out


@dataclass
class Workload:
    config_id: int
    name: str
    n_layers: int
    seq_lens: list
    budgets: list
    n_q: int
    h_q: int
    h_kv: int
    d: int
    pool_k: int
    plant: str
    seed: int
    outliers: bool = False
    densities: list = field(default_factory=list)
    outlier_channels: tuple = ()
    threads: int = 0

    # ---- shape helpers -------------------------------------------------
    @property
    def n_seq(self) -> int:
        return len(self.seq_lens)

    @property
    def group(self) -> int:
        return self.h_q // self.h_kv

    @property
    def cu_seqlens(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.seq_lens)]).astype(np.int32)

    @property
    def cu_budgets(self) -> np.ndarray:
        return np.concatenate([[0], np.cumsum(self.budgets)]).astype(np.int32)

    @property
    def total_tokens(self) -> int:
        return int(sum(self.seq_lens))

    @property
    def total_budget(self) -> int:
        return int(sum(self.budgets))

    # ---- generation ----------------------------------------------------
    def _pool(self):
        n = self.threads or min(16, os.cpu_count() or 1)
        return ThreadPoolExecutor(max_workers=n) if n > 1 else None

    def planted_positions(self, layer: int, seq: int) -> list:
        """Planted heavy-hitter positions per KV head (sorted int64 arrays)."""
        L = self.seq_lens[seq]
        r = _rng(self.seed, layer, seq, _T_PLANT)
        if self.plant == "none":
            return [np.zeros(0, dtype=np.int64) for _ in range(self.h_kv)]
        if self.plant == "subset":
            n = min(20, L)
            pos = np.sort(r.choice(L, size=n, replace=False))
            return [pos.astype(np.int64) for _ in range(self.h_kv)]
        if self.plant == "spans":
            n_span, span = 8, 64
            if L < 2 * n_span * span:
                n_span, span = max(1, L // 256), min(64, max(1, L // 8))
            slots = r.choice(L // span, size=n_span, replace=False)
            pos = np.sort(np.concatenate([np.arange(s * span, s * span + span) for s in slots]))
            pos = pos[pos < L]
            return [pos.astype(np.int64) for _ in range(self.h_kv)]
        if self.plant == "aligned":
            dens = self.densities[seq]
            n = max(1, int(round(dens * L)))
            return [np.sort(r.choice(L, size=n, replace=False)).astype(np.int64) for _ in range(self.h_kv)]
        raise ValueError(self.plant)

    def tensors(self, layer: int, seq: int):
        """(Q, K, V) bf16 bit patterns for one (layer, sequence).

        Q [n_q, h_q, d], K and V [L, h_kv, d], all uint16, C-contiguous.
        """
        L, d, G = self.seq_lens[seq], self.d, self.group
        pool = self._pool()
        try:
            Q = _normal_bf16(self.seed, (layer, seq, _T_Q), self.n_q, self.h_q * d, None).reshape(self.n_q, self.h_q, d)
            K = _normal_bf16(self.seed, (layer, seq, _T_K), L, self.h_kv * d, pool).reshape(L, self.h_kv, d)
            V = _normal_bf16(self.seed, (layer, seq, _T_V), L, self.h_kv * d, pool).reshape(L, self.h_kv, d)
        finally:
            if pool is not None:
                pool.shutdown()
        if self.outliers:
            for c in self.outlier_channels:
                # x8 is exact in bf16 (exponent bump), so no re-rounding is needed
                K[:, :, c] = f32_to_bf16_bits(bf16_bits_to_f32(K[:, :, c]) * np.float32(8.0))
        planted = self.planted_positions(layer, seq)
        rp = _rng(self.seed, layer, seq, _T_NOISE)
        Qf = bf16_bits_to_f32(Q)  # [n_q, h_q, d]
        for g in range(self.h_kv):
            pos = planted[g]
            if pos.size == 0:
                continue
            qg = Qf[:, g * G:(g + 1) * G, :].reshape(-1, d)  # the group's n_q*G query vectors
            noise = rp.standard_normal((pos.size, d), dtype=np.float32) * np.float32(0.1)
            if self.plant == "subset":
                rows = np.empty((pos.size, d), dtype=np.float32)
                for t in range(pos.size):
                    m = int(rp.integers(1, 9))
                    sub = rp.choice(qg.shape[0], size=min(m, qg.shape[0]), replace=False)
                    rows[t] = np.float32(3.0) * qg[sub].mean(axis=0)
                rows += noise
            else:
                qbar = qg.mean(axis=0)
                nrm = float(np.linalg.norm(qbar))
                unit = qbar / np.float32(nrm if nrm > 0 else 1.0)
                rows = np.float32(2.5 * np.sqrt(d)) * unit[None, :] + noise
            K[pos, g, :] = f32_to_bf16_bits(rows)
        return Q, K, V

    def assemble(self, layers=None):
        """Whole-call tensors: Q [nl, n_seq, n_q, h_q, d], K/V [nl, T, h_kv, d] (uint16)."""
        layers = list(range(self.n_layers)) if layers is None else list(layers)
        T = self.total_tokens
        Q = np.empty((len(layers), self.n_seq, self.n_q, self.h_q, self.d), dtype=np.uint16)
        K = np.empty((len(layers), T, self.h_kv, self.d), dtype=np.uint16)
        V = np.empty_like(K)
        cu = self.cu_seqlens
        for li, layer in enumerate(layers):
            for s in range(self.n_seq):
                q, k, v = self.tensors(layer, s)
                Q[li, s] = q
                K[li, cu[s]:cu[s + 1]] = k
                V[li, cu[s]:cu[s + 1]] = v
        return Q, K, V


def make_workload(config_id: int, *, budget=None, seq_lens=None, n_layers=None, seed=None, **over) -> Workload:
    """Build one of the five named workloads; keyword arguments shrink or vary it."""
    c = dict(CONFIGS[config_id])
    c.update(over)
    seed = BASE_SEED + config_id if seed is None else int(seed)
    aux = _rng(seed, 9999)
    if seq_lens is None:
        seq_lens = c["seq_lens"]
        if isinstance(seq_lens, str):  # "ragged16"
            seq_lens = [int(x) for x in aux.integers(4096, 131072 + 1, size=16)]
    seq_lens = [int(x) for x in seq_lens]
    if c.get("density") == "ragged":
        dens = [float(x) for x in aux.uniform(0.005, 0.05, size=len(seq_lens))]
    else:
        dens = [float(c.get("density", 0.0))] * len(seq_lens)
    b = c["budget"] if budget is None else budget
    if isinstance(b, str):  # "min(2048,L/8)"
        budgets = [max(1, min(2048, L // 8)) for L in seq_lens]
    elif isinstance(b, (list, tuple)):
        budgets = [int(x) for x in b]
    else:
        budgets = [min(int(b), L) for L in seq_lens]
    out_ch = tuple(int(x) for x in np.sort(_rng(seed, 9998).choice(c["d"], size=4, replace=False))) if c["outliers"] else ()
    return Workload(
        config_id=config_id, name=c["name"], n_layers=int(c["n_layers"] if n_layers is None else n_layers),
        seq_lens=seq_lens, budgets=budgets, n_q=int(c["n_q"]), h_q=int(c["h_q"]), h_kv=int(c["h_kv"]),
        d=int(c["d"]), pool_k=int(c["pool_k"]), plant=c["plant"], seed=seed, outliers=bool(c["outliers"]),
        densities=dens, outlier_channels=out_ch,
    )


def page_out(K: np.ndarray, V: np.ndarray, seq_lens, page_size: int, seed: int = 0, spare_pages: int = 3):
    """Lay dense K/V [nl, T, h_kv, d] (uint16) out as a paged cache.

    Returns (K_pool, V_pool, block_table): pools [nl, n_pages, page_size, h_kv, d], block_table int32
    [n_seq, max_pages].  Pages are handed out in a seeded random order, the same for every layer; page
    rows past a sequence's end, and `spare_pages` pages that belong to no sequence, hold bf16 NaN patterns
    (a consumer that reads them shows it); table entries past a sequence's last page are -1.
    """
    nl, T, h_kv, d = K.shape
    seq_lens = [int(x) for x in seq_lens]
    assert sum(seq_lens) == T
    per_seq = [(L + page_size - 1) // page_size for L in seq_lens]
    n_pages = sum(per_seq) + int(spare_pages)
    order = np.random.default_rng([BASE_SEED, 77, int(seed)]).permutation(n_pages)
    table = np.full((len(seq_lens), max(per_seq)), -1, dtype=np.int32)
    Kp = np.full((nl, n_pages, page_size, h_kv, d), 0x7FC0, dtype=np.uint16)
    Vp = np.full_like(Kp, 0x7FC0)
    nxt, tok = 0, 0
    for s, L in enumerate(seq_lens):
        for i in range(per_seq[s]):
            pg = int(order[nxt]); nxt += 1
            table[s, i] = pg
            n = min(page_size, L - i * page_size)
            Kp[:, pg, :n] = K[:, tok + i * page_size: tok + i * page_size + n]
            Vp[:, pg, :n] = V[:, tok + i * page_size: tok + i * page_size + n]
        tok += L
    return Kp, Vp, table
