"""Pins for the oracle's key scoring and top-B selection (Alg. 1 second block; Sec. 3.2-3.3)."""
import numpy as np
import pytest
from scipy.spatial.distance import cdist

import gen
from oracle import quoka_oracle as O
from tests.bf16_round import round_to_bf16


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def test_group_of_one_is_max_of_library_cosines():
    # n_q == n_kv: S-hat[t] = max_r cos(q_r, k_t), brute-forced with scipy's cosine distance.
    Q = _rand(0, 2, 12, 6) + 0.4
    K = _rand(1, 2, 30, 6)
    q_idx = O.select_queries(Q, 5)
    S = O.key_scores(Q, q_idx, K, n_kv=2)
    for kv in range(2):
        cosm = 1.0 - cdist(Q[kv][q_idx[kv]], K[kv], metric="cosine")     # [5, 30]
        for t in range(30):
            assert S[kv, t] == pytest.approx(max(cosm[r, t] for r in range(5)), abs=1e-12)


def test_preaggregation_identity_of_section_3_3():
    # mean over the group of per-head cosines == (mean of unit queries) . (unit key)
    Q = _rand(2, 8, 20, 16) + 0.3
    K = _rand(3, 2, 50, 16)
    q_idx = O.select_queries(Q, 6)
    post = O.key_scores(Q, q_idx, K, n_kv=2)
    qbar = O.group_mean_queries(Q, q_idx, n_kv=2)
    pre = O.key_scores_preagg(qbar, K)
    assert qbar.shape == (2, 6, 16)
    assert np.max(np.abs(post - pre)) < 1e-12


def test_group_mean_pairs_queries_by_rank_and_uses_contiguous_groups():
    # 4 q-heads, 2 KV heads: head h belongs to KV head h // 2; row r averages the r-th RANKED query of each head.
    Q = _rand(4, 4, 9, 5) + 0.2
    q_idx = O.select_queries(Q, 3)
    qbar = O.group_mean_queries(Q, q_idx, n_kv=2)
    for kv in range(2):
        for r in range(3):
            a = Q[2 * kv, q_idx[2 * kv, r]]
            b = Q[2 * kv + 1, q_idx[2 * kv + 1, r]]
            want = 0.5 * (a / np.linalg.norm(a) + b / np.linalg.norm(b))
            assert np.allclose(qbar[kv, r], want, atol=1e-14)


def test_scores_bounded_and_invariant_to_key_and_query_scale():
    Q = _rand(5, 4, 16, 8) + 0.5
    K = _rand(6, 2, 40, 8)
    q_idx = O.select_queries(Q, 4)
    S = O.key_scores(Q, q_idx, K, 2)
    assert np.all(np.abs(S) <= 1.0 + 1e-12)
    scale = np.random.default_rng(7).uniform(0.1, 9.0, size=(2, 40, 1))
    assert np.allclose(O.key_scores(Q, q_idx, K * scale, 2), S, atol=1e-12)
    # per-query positive rescaling does not change any cosine (same retained set passed in)
    qs = np.random.default_rng(8).uniform(0.2, 5.0, size=(4, 16, 1))
    assert np.allclose(O.key_scores(Q * qs, q_idx, K, 2), S, atol=1e-12)


def test_max_not_mean_over_queries():
    # One retained query is exactly parallel to key 3; every other (query, key) pair is orthogonal.
    d = 8
    Q = np.zeros((1, 3, d))
    Q[0, 0, 0] = 1.0
    Q[0, 1, 1] = 2.0
    Q[0, 2, 2] = 0.5
    K = np.zeros((1, 5, d))
    K[0, :, 7] = 1.0           # orthogonal to all queries
    K[0, 3] = 0.0
    K[0, 3, 1] = 4.0           # parallel to query 1
    S = O.key_scores(Q, np.array([[0, 1, 2]]), K, 1)
    assert S[0].tolist() == [0.0, 0.0, 0.0, 1.0, 0.0]


def test_zero_key_scores_zero():
    Q = _rand(9, 1, 4, 4)
    K = _rand(10, 1, 3, 4)
    K[0, 1] = 0.0
    S = O.key_scores(Q, O.select_queries(Q, 4), K, 1)
    assert S[0, 1] == 0.0


def test_topk_equals_exhaustive_sort():
    s = _rand(11, 3, 200)
    idx = O.topk_keys(s, 17)
    assert idx.shape == (3, 17)
    for kv in range(3):
        ranked = sorted(range(200), key=lambda t: (-s[kv, t], t))
        assert idx[kv].tolist() == sorted(ranked[:17])
        assert np.all(np.diff(idx[kv]) > 0)
        rest = set(range(200)) - set(idx[kv].tolist())
        assert min(s[kv, t] for t in idx[kv]) >= max(s[kv, t] for t in rest)


def test_topk_ties_lower_index_and_full_budget():
    s = np.array([[1.0, 2.0, 2.0, 2.0, 0.5, 2.0]])
    assert O.topk_keys(s, 2)[0].tolist() == [1, 2]
    assert O.topk_keys(s, 4)[0].tolist() == [1, 2, 3, 5]
    assert O.topk_keys(s, 6)[0].tolist() == [0, 1, 2, 3, 4, 5]
    assert O.topk_keys(s, 99)[0].tolist() == [0, 1, 2, 3, 4, 5]
    assert O.topk_keys(s, 0).shape == (1, 0)
    assert O.topk_keys(np.zeros((2, 0)), 5).shape == (2, 0)


def test_topk_is_equivariant_under_permutation_of_cache_positions():
    r = np.random.default_rng(12)
    s = r.standard_normal((1, 64))        # distinct scores almost surely
    perm = r.permutation(64)
    a = set(O.topk_keys(s, 9)[0].tolist())
    b = set(O.topk_keys(s[:, perm], 9)[0].tolist())
    assert {int(perm[j]) for j in b} == a


def test_planted_heavy_keys_of_config1_are_selected():
    w = gen.make_workload("c1")
    q_idx, scores, k_idx = O.quoka_select(w.Q[0], w.K[0], w.n_retain, w.budgets[0])
    assert k_idx.shape == (1, 128)
    assert set(w.notes["heavy_key_pos"]) <= set(k_idx[0].tolist())
    # each heavy key is parallel to one retained query of head 0 and the other head of the group is
    # independent noise, so its group-mean score sits near 0.5 -- far above the bulk of the cache
    heavy = scores[0, w.notes["heavy_key_pos"]]
    assert np.all(heavy > 0.35)
    assert np.quantile(scores[0], 0.99) < 0.35


# ---- ablation scorers (Sec. 3.2: dot product instead of cosine; Sec. 3.3: mean instead of max over queries) ----
def _brute_scores(Q, q_idx, K, n_kv, normalise, reduce):
    """Element-by-element Python loops over the definition."""
    n_q, g, T = Q.shape[0], Q.shape[0] // n_kv, K.shape[1]
    out = np.zeros((n_kv, T))
    for kv in range(n_kv):
        for t in range(T):
            k = K[kv, t].astype(np.float64)
            if normalise:
                k = k / max(np.linalg.norm(k), 1e-8)
            per_query = []
            for r in range(q_idx.shape[1]):
                acc = 0.0
                for j in range(g):
                    q = Q[kv * g + j, q_idx[kv * g + j, r]].astype(np.float64)
                    if normalise:
                        q = q / max(np.linalg.norm(q), 1e-8)
                    acc += float(np.dot(q, k))
                per_query.append(acc / g)
            out[kv, t] = max(per_query) if reduce == "max" else sum(per_query) / len(per_query)
    return out


@pytest.mark.parametrize("similarity,reduce", [("dot", "max"), ("cosine", "mean"), ("dot", "mean")])
def test_ablation_scorers_match_brute_force_and_preaggregation(similarity, reduce):
    rng = np.random.default_rng(77)
    n_q, n_kv, C, T, d = 4, 2, 12, 9, 8
    Q = rng.normal(size=(n_q, C, d)) * rng.uniform(0.2, 5.0, size=(n_q, C, 1))   # norms vary: dot != cosine
    K = rng.normal(size=(n_kv, T, d)) * rng.uniform(0.2, 5.0, size=(n_kv, T, 1))
    q_idx = O.select_queries(Q, 5)
    want = _brute_scores(Q, q_idx, K, n_kv, similarity == "cosine", reduce)
    got = O.key_scores(Q, q_idx, K, n_kv, similarity, reduce)
    assert np.allclose(got, want, rtol=0, atol=1e-12)
    qbar = O.group_mean_queries(Q, q_idx, n_kv, similarity)
    assert np.allclose(O.key_scores_preagg(qbar, K, similarity, reduce), want, rtol=0, atol=1e-12)
    # the variants really differ from the method's scorer on these inputs
    assert np.abs(got - O.key_scores(Q, q_idx, K, n_kv)).max() > 1e-3


def test_ablation_scorers_degenerate_cases():
    rng = np.random.default_rng(78)
    Q = O.unit(rng.normal(size=(2, 6, 8)))
    K = O.unit(rng.normal(size=(1, 7, 8)))
    q_idx = O.select_queries(Q, 6)
    # unit-norm inputs: dot product and cosine coincide
    assert np.allclose(O.key_scores(Q, q_idx, K, 1, "dot"), O.key_scores(Q, q_idx, K, 1), atol=1e-12)
    # the mean over queries never exceeds the max, and equals it for a single retained query
    assert np.all(O.key_scores(Q, q_idx, K, 1, reduce="mean") <= O.key_scores(Q, q_idx, K, 1) + 1e-15)
    one = O.select_queries(Q[:, :1], 4)
    assert np.allclose(O.key_scores(Q[:, :1], one, K, 1, reduce="mean"), O.key_scores(Q[:, :1], one, K, 1), atol=1e-15)


# ---- reduced-precision scorer (Q-bar in bfloat16; the cheaper product named as future work in Sec. 6) ------------
def test_round_to_bf16_hand_values_and_ties_to_even():
    one = 1.0
    ulp = 2.0 ** -7                      # spacing of bfloat16 in [1, 2)
    cases = [
        (one, one),
        (one + ulp, one + ulp),          # representable
        (one + ulp / 2, one),            # tie -> even mantissa (1.0)
        (one + 3 * ulp / 2, one + 2 * ulp),   # tie -> even mantissa (1 + 2 ulp)
        (one + 0.49 * ulp, one),
        (one + 0.51 * ulp, one + ulp),
        (-(one + 0.51 * ulp), -(one + ulp)),
        (2.0 - ulp / 4, 2.0),            # rounds up into the next binade
        (3.0e-5, None), (0.0, 0.0),
    ]
    for x, want in cases:
        got = float(round_to_bf16(np.array([x]))[0])
        if want is None:
            assert abs(got - x) <= abs(x) * 2.0 ** -9
        else:
            assert got == want, (x, got, want)


def test_round_to_bf16_matches_the_library_conversion():
    import torch
    x = np.random.default_rng(3).standard_normal(4000).astype(np.float32) * np.float32(0.37)
    x[:8] = [1.00390625, 1.01171875, -1.00390625, 0.333251953125, 65280.0, 1e-20, -3.0, 0.1]
    want = torch.from_numpy(x).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(round_to_bf16(x), want)


def test_reduced_precision_scores_are_the_exact_scores_of_the_rounded_queries():
    rng = np.random.default_rng(4)
    qbar = rng.standard_normal((2, 5, 16)) * 0.2
    K = rng.standard_normal((2, 30, 16))
    got = O.key_scores_preagg(round_to_bf16(qbar), K)
    # brute force with the library's rounding: cosine-style scores, max over queries
    import torch
    qr = torch.from_numpy(qbar.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    for kv in range(2):
        for t in range(30):
            k = K[kv, t] / np.linalg.norm(K[kv, t])
            assert abs(got[kv, t] - max(float(qr[kv, r] @ k) for r in range(5))) < 1e-12
    # bf16-exact queries: the option changes nothing
    assert np.array_equal(round_to_bf16(qr), qr)
    # and it stays within the rounding bound of the exact scores: |dq| <= 2^-9 |q| elementwise, |k-hat| = 1
    exact = O.key_scores_preagg(qbar, K)
    bound = 2.0 ** -9 * np.abs(qbar).sum(axis=2).max()
    assert np.abs(got - exact).max() <= bound
