"""Comparison helpers for the GPU parity tests (HIP path vs. CPU oracle)."""
from __future__ import annotations

import numpy as np

TIE_REL = 1e-6     # documented tie band: |score - cut| <= TIE_REL * max(|cut|, 1e-3)
TOL_OUT = {"f32": 1e-4, "bf16": 2e-2}   # max-abs tolerance of attention outputs
TOL_SCORE = 1e-6   # float32-accumulated cosine-like scores in [-1, 1] vs. the float64 oracle
TOL_QBAR = 5e-7


def two_pass_scores(w) -> bool:
    """Whether quoka_select_keys (and so quoka_chunk_attn) takes its two-pass route for this workload: bf16 caches
    longer than 32768 positions (include/quoka.h).  `scores` then holds exact values near the cut only."""
    return w.dtype == "bf16" and w.t_max > 32768


def check_two_pass_scores(got, want, qbar, budget, what=""):
    """Scores left by the two-pass stage for one KV head.  got, want: [T] (GPU float32, oracle float64); qbar: the
    head's [N', d] float32 Q-bar.  Every score is within the proven bound of the provisional pass,
    max_r ||qbar_r - bf16(qbar_r)||_2 + 4e-6, and the scores that decide the selection -- every key within 2^-11 of
    the cut, the margin the interface states -- meet the bar of the exact scorer."""
    from gen.workloads import bf16_round
    T = want.shape[0]
    if T == 0:
        return
    q = np.asarray(qbar, dtype=np.float32)
    delta = q.astype(np.float64) - bf16_round(q).astype(np.float64)
    eps = float(np.sqrt((delta * delta).sum(axis=1)).max()) + 4e-6
    err = np.abs(np.asarray(got, dtype=np.float64) - want)
    assert err.max() <= eps, f"{what}: provisional score off by {err.max()} > bound {eps}"
    Bp = max(0, min(int(budget), T))
    if 0 < Bp < T:
        cut = np.sort(want)[T - Bp]
        near = np.abs(want - cut) <= 2.0 ** -11 - 1e-5
        assert near.sum() >= 1
        assert err[near].max() <= TOL_SCORE, f"{what}: score near the cut off by {err[near].max()}"


def tie_band(cut: float) -> float:
    return TIE_REL * max(abs(cut), 1e-3)


def check_topk_set(gpu_idx, oracle_scores, budget, what=""):
    """gpu_idx: 1-D ascending positions selected on the GPU.  oracle_scores: float64 [T].

    The set must have the right size, be strictly ascending and in range, and may differ from the
    oracle's (stable sort, ties to lower index) only on elements whose oracle score lies inside the
    tie band around the cut score.  Returns the number of tie-band substitutions.
    """
    T = oracle_scores.shape[0]
    Bp = max(0, min(int(budget), T))
    g = np.asarray(gpu_idx, dtype=np.int64)
    assert g.shape == (Bp,), f"{what}: count {g.shape} != {Bp}"
    if Bp == 0:
        return 0
    assert g.min() >= 0 and g.max() < T, f"{what}: index out of range"
    assert np.all(np.diff(g) > 0), f"{what}: indices not strictly ascending"
    order = np.argsort(-oracle_scores, kind="stable")
    want = np.sort(order[:Bp])
    if np.array_equal(g, want):
        return 0
    cut = oracle_scores[order[Bp - 1]]
    band = tie_band(cut)
    only_g = np.setdiff1d(g, want)
    only_o = np.setdiff1d(want, g)
    assert only_g.size == only_o.size
    bad = [int(i) for i in np.concatenate([only_g, only_o]) if abs(oracle_scores[i] - cut) > band]
    assert not bad, (f"{what}: {len(bad)} selected/dropped keys differ from the oracle outside the tie band "
                     f"(cut {cut:.9g}, band {band:.3g}): first {bad[:5]}, scores {oracle_scores[bad[:5]]}")
    return int(only_g.size)


def check_query_ranking(gpu_qidx, oracle_cos, n_keep, what=""):
    """gpu_qidx: retained positions of one head in rank order.  Must equal the oracle's stable ascending
    ranking except for swaps among cosines that tie within the band."""
    C = oracle_cos.shape[0]
    g = np.asarray(gpu_qidx, dtype=np.int64)
    assert g.shape == (n_keep,), f"{what}: shape {g.shape}"
    if n_keep == C:
        assert np.array_equal(g, np.arange(C)), f"{what}: identity order expected"
        return 0
    want = np.argsort(oracle_cos, kind="stable")[:n_keep]
    if np.array_equal(g, want):
        return 0
    assert len(set(g.tolist())) == n_keep and g.min() >= 0 and g.max() < C, f"{what}: invalid positions"
    diff = np.nonzero(g != want)[0]
    for r in diff:
        a, b = oracle_cos[g[r]], oracle_cos[want[r]]
        assert abs(a - b) <= tie_band(b), f"{what}: rank {r}: got pos {g[r]} (cos {a}) want {want[r]} (cos {b})"
    return int(diff.size)


def max_abs(a, b) -> float:
    return float(np.max(np.abs(np.asarray(a, dtype=np.float64) - np.asarray(b, dtype=np.float64)))) if a.size else 0.0
