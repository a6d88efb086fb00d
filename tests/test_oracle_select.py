"""Pins for the oracle's query sub-selection (Alg. 1 first block; Sec. 3.1; Theorem 1)."""
import math

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st
from scipy.spatial.distance import cosine as scipy_cosine_distance

import gen
from oracle import quoka_oracle as O


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_cosine_matches_library_routine():
    Q = _rand(0, 3, 17, 8) + 0.7
    s = O.cos_to_mean(Q)
    for h in range(3):
        m = np.mean(Q[h], axis=0)
        for i in range(17):
            assert s[h, i] == pytest.approx(1.0 - scipy_cosine_distance(Q[h, i], m), abs=1e-12)


def test_cosine_closed_form_planar_angles():
    # Two queries at angles +a and -a from the x axis: their mean lies on the x axis, so both cosines are cos(a);
    # a third copy of the mean direction has cosine 1.
    a = 0.3
    Q = np.zeros((1, 2, 4))
    Q[0, 0, :2] = [math.cos(a), math.sin(a)]
    Q[0, 1, :2] = [math.cos(a), -math.sin(a)]
    s = O.cos_to_mean(Q)
    assert s[0, 0] == pytest.approx(math.cos(a), abs=1e-14)
    assert s[0, 1] == pytest.approx(math.cos(a), abs=1e-14)
    # unequal lengths: q0 = 3*(cos a, sin a), q1 = (1, 0): mean = ((3cos a+1)/2, 3 sin a/2)
    Q[0, 0, :2] = [3 * math.cos(a), 3 * math.sin(a)]
    Q[0, 1, :2] = [1.0, 0.0]
    s = O.cos_to_mean(Q)
    ang_mean = math.atan2(3 * math.sin(a), 3 * math.cos(a) + 1)
    assert s[0, 0] == pytest.approx(math.cos(a - ang_mean), abs=1e-14)
    assert s[0, 1] == pytest.approx(math.cos(ang_mean), abs=1e-14)


def test_mean_is_per_head_over_tokens():
    Q = _rand(1, 4, 9, 5)
    M = O.mean_query(Q)
    assert M.shape == (4, 5)
    for h in range(4):
        for c in range(5):
            assert M[h, c] == pytest.approx(sum(Q[h, i, c] for i in range(9)) / 9, abs=1e-14)


def test_cosine_invariant_to_positive_rescaling_of_one_query_direction():
    # Scaling ALL queries by a > 0 scales the mean too and leaves every cosine unchanged.
    Q = _rand(2, 2, 11, 6) + 0.5
    assert np.allclose(O.cos_to_mean(Q), O.cos_to_mean(3.7 * Q), atol=1e-13)
    # and negating all queries leaves them unchanged as well (both q and M flip)
    assert np.allclose(O.cos_to_mean(Q), O.cos_to_mean(-Q), atol=1e-13)


def test_selection_equals_exhaustive_sort_lowest_cosine_first():
    Q = _rand(3, 3, 40, 8) + 1.0
    s = O.cos_to_mean(Q)
    idx = O.select_queries(Q, 7)
    assert idx.shape == (3, 7)
    for h in range(3):
        ranked = sorted(range(40), key=lambda i: (s[h, i], i))   # smallest cosine first
        assert idx[h].tolist() == ranked[:7]
        # every retained query has cosine <= every dropped one
        dropped = set(range(40)) - set(idx[h].tolist())
        assert max(s[h, i] for i in idx[h]) <= min(s[h, i] for i in dropped)


def test_selection_ties_go_to_lower_index():
    q = _rand(4, 1, 1, 6)
    Q = np.repeat(q, 10, axis=1)           # all queries identical: every cosine ties (=1)
    assert O.select_queries(Q, 4)[0].tolist() == [0, 1, 2, 3]


def test_no_subselection_when_chunk_not_longer_than_n_retain():
    Q = _rand(5, 2, 6, 4)
    for n in (6, 7, 100):
        idx = O.select_queries(Q, n)
        assert idx.tolist() == [list(range(6))] * 2


def test_zero_queries_do_not_divide_by_zero():
    Q = np.zeros((1, 5, 4))
    assert np.all(O.cos_to_mean(Q) == 0.0)
    assert O.select_queries(Q, 2)[0].tolist() == [0, 1]


def test_planted_outliers_of_config1_are_the_retained_queries():
    w = gen.make_workload("c1")
    idx = O.select_queries(w.Q[0], w.n_retain)
    assert sorted(idx[0].tolist()) == w.notes["outlier_queries_head0"]
    # head 1 has no planted outliers: its selection is still the 16 lowest cosines
    s = O.cos_to_mean(w.Q[0])
    assert set(idx[1].tolist()) == set(np.argsort(s[1], kind="stable")[:16].tolist())


@settings(max_examples=200, deadline=None)
@given(st.integers(0, 2**31 - 1), st.integers(2, 12))
def test_theorem1_inequality_holds_for_arbitrary_vectors(seed, d):
    # For any M, q, k: cos(M, q) <= 1 + a*b - a^2/2 - b^2/2 with a = cos(M, k), b = cos(k, q)
    # (what the proof of Theorem 1 establishes: orthonormal expansion + Young's inequality).
    r = np.random.default_rng(seed)
    M, q, k = r.standard_normal((3, d))

    def cs(x, y):
        return float(x @ y / (np.linalg.norm(x) * np.linalg.norm(y)))

    a, b = cs(M, k), cs(k, q)
    # route cos(M, q) through the oracle: a two-query chunk [q, 2M - q] has mean exactly M
    Q = np.stack([q, 2 * M - q])[None]
    c = O.cos_to_mean(Q)[0, 0]
    assert c == pytest.approx(cs(M, q), abs=1e-10)
    assert c <= 1 + a * b - 0.5 * a * a - 0.5 * b * b + 1e-10


# ---- uniform query sampling (the query-sampling baseline of Sec. 4) -----------------------------------------
def test_uniform_rule_is_an_even_stride_independent_of_the_data():
    # C a multiple of N_Q: exactly every (C / N_Q)-th position, starting at 0
    Q = _rand(7, 3, 32, 4)
    idx = O.select_queries(Q, 8, rule="uniform")
    assert idx.tolist() == [[0, 4, 8, 12, 16, 20, 24, 28]] * 3
    # the sample does not look at the values
    assert np.array_equal(idx, O.select_queries(-5.0 * Q[::-1], 8, rule="uniform"))


@pytest.mark.parametrize("C,n", [(10, 3), (11, 4), (97, 16), (1024, 64), (129, 128)])
def test_uniform_rule_ragged_stride_properties(C, n):
    # positions strictly increase, start at 0, stay inside the chunk, and consecutive gaps are floor or ceil of C/n
    idx = O.select_queries(np.ones((1, C, 2)), n, rule="uniform")[0]
    assert idx[0] == 0 and idx[-1] < C and len(idx) == n
    gaps = np.diff(idx)
    assert gaps.min() >= C // n >= 1 and gaps.max() <= -(-C // n)
    # sample r is the last integer point not beyond r*C/n (integer form of the inequality, no rounding involved)
    for r in range(n):
        assert int(idx[r]) * n <= r * C < (int(idx[r]) + 1) * n


def test_uniform_rule_keeps_everything_for_short_chunks():
    assert O.select_queries(_rand(8, 2, 5, 3), 5, rule="uniform").tolist() == [[0, 1, 2, 3, 4]] * 2


def test_uniform_rule_feeds_the_same_scoring_as_an_explicit_index_list():
    Q, K = _rand(9, 4, 24, 8), _rand(10, 2, 40, 8)
    q_idx, scores, k_idx = O.quoka_select(Q, K, 6, 10, query_rule="uniform")
    assert q_idx.tolist() == [[0, 4, 8, 12, 16, 20]] * 4
    # brute force: group mean of cosines with the strided queries, max over them
    for kv in range(2):
        for t in range(40):
            best = -np.inf
            for r in range(6):
                c = 0.0
                for j in range(2):
                    qv = Q[2 * kv + j, 4 * r]
                    c += 1.0 - scipy_cosine_distance(qv, K[kv, t])
                best = max(best, c / 2)
            assert abs(scores[kv, t] - best) < 1e-12
    assert np.array_equal(k_idx, O.topk_keys(scores, 10))
