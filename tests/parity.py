"""Helpers shared by the GPU parity tests: tensor marshalling and the parity rules.

Tolerances (stated by the benchmark spec, made operational here):
  * scores: |gpu - oracle| <= 2e-3 * |oracle| + floor, floor = 1e-6 * (n_q * G / L)
    (one millionth of the uniform score, for entries that underflow towards 0);
  * kept sets: identical whenever the oracle's pooled scores leave a relative gap
    > 1e-3 at the top-B boundary; otherwise everything clearly above the boundary
    must be kept, nothing clearly below may be, and the kept oracle-score mass must
    agree to 1e-4;
  * compacted K/V: bit-exact gather of the GPU's own indices.
"""
import numpy as np

SCORE_RTOL = 2e-3
GAP_RTOL = 1e-3
MASS_RTOL = 1e-4


def to_dev_bf16(u16: np.ndarray):
    import torch
    return torch.from_numpy(np.ascontiguousarray(u16).view(np.int16)).cuda().view(torch.bfloat16)


def from_dev_bf16(t) -> np.ndarray:
    import torch
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def assert_scores_close(gpu: np.ndarray, ref: np.ndarray, uniform: float, what=""):
    gpu = np.asarray(gpu, dtype=np.float64)
    err = np.abs(gpu - ref)
    bound = SCORE_RTOL * np.abs(ref) + 1e-6 * uniform
    bad = err > bound
    assert not bad.any(), "%s: %d of %d scores off; worst rel err %.3e" % (
        what, int(bad.sum()), bad.size, float((err / np.maximum(np.abs(ref), 1e-300)).max()))
    return float((err / np.maximum(np.abs(ref), 1e-6 * uniform)).max())


def assert_kept_set_ok(pooled_ref: np.ndarray, idx_ref: np.ndarray, idx_gpu: np.ndarray, what=""):
    """One (layer, sequence, head): pooled_ref [L] float64, idx_* [B] ascending int."""
    L, B = pooled_ref.shape[0], idx_ref.shape[0]
    idx_gpu = np.asarray(idx_gpu, dtype=np.int64)
    assert idx_gpu.shape == (B,), what
    assert (np.diff(idx_gpu) > 0).all() and idx_gpu.min() >= 0 and idx_gpu.max() < L, what + ": not ascending/in range"
    if B == L or np.array_equal(idx_gpu, idx_ref):
        return "identical"
    srt = np.sort(pooled_ref)[::-1]
    tau, tau_next = srt[B - 1], srt[B]
    gap = (tau - tau_next) / tau if tau > 0 else 0.0
    assert gap <= GAP_RTOL, "%s: kept sets differ although the boundary gap is %.3e" % (what, gap)
    kept = np.zeros(L, dtype=bool); kept[idx_gpu] = True
    must = pooled_ref > tau * (1 + GAP_RTOL)
    never = pooled_ref < tau * (1 - GAP_RTOL)
    assert kept[must].all(), what + ": a clearly-above-threshold position was dropped"
    assert not kept[never].any(), what + ": a clearly-below-threshold position was kept"
    m_gpu, m_ref = pooled_ref[idx_gpu].sum(), pooled_ref[idx_ref].sum()
    assert abs(m_gpu - m_ref) <= MASS_RTOL * m_ref, what + ": kept mass differs by %.3e" % (abs(m_gpu - m_ref) / m_ref)
    return "contested"


def assert_kept_set_ok_keep(pooled_ref, idx_ref, idx_gpu, keep_first, keep_last, what=""):
    """The same check when the first keep_first / last keep_last positions are kept unconditionally:
    they must all be present, and the rest is judged as a selection among the other positions."""
    L, B = pooled_ref.shape[0], idx_ref.shape[0]
    idx_gpu = np.asarray(idx_gpu, dtype=np.int64)
    assert idx_gpu.shape == (B,), what
    forced = np.concatenate([np.arange(keep_first), np.arange(L - keep_last, L)])
    assert np.isin(forced, idx_gpu).all(), what + ": an always-kept position is missing"
    assert np.isin(forced, idx_ref).all(), what
    if B == forced.size:
        assert (np.diff(idx_gpu) > 0).all(), what
        return "forced only"
    free = lambda idx: np.asarray([j - keep_first for j in idx if keep_first <= j < L - keep_last], dtype=np.int64)
    return assert_kept_set_ok(pooled_ref[keep_first:L - keep_last], free(idx_ref), free(idx_gpu), what)
