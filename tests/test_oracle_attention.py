"""Pins for the oracle's attention (Eq. 1-3, Alg. 2): library routine, closed forms, invariants."""
import math

import numpy as np
import pytest
import torch

from oracle import quoka_oracle as O


def _rand(seed, *shape):
    return np.random.default_rng(seed).standard_normal(shape)


def _sdpa(q, k, v, mask=None, causal=False):
    t = lambda x: torch.from_numpy(np.ascontiguousarray(x)).double()
    m = None if mask is None else torch.from_numpy(mask)
    return torch.nn.functional.scaled_dot_product_attention(t(q), t(k), t(v), attn_mask=m, is_causal=causal).numpy()


def test_empty_cache_is_textbook_causal_attention():
    n_q, n_kv, C, d = 4, 2, 11, 8
    Q, Kc, Vc = _rand(0, n_q, C, d), _rand(1, n_kv, C, d), _rand(2, n_kv, C, d)
    K = np.zeros((n_kv, 0, d))
    out = O.dense_attn(Q, K, K, Kc, Vc)
    for h in range(n_q):
        ref = _sdpa(Q[h], Kc[h // 2], Vc[h // 2], causal=True)
        assert np.max(np.abs(out[h] - ref)) < 1e-12


def test_dense_chunk_attention_matches_library_with_explicit_mask():
    n_q, n_kv, T, C, d = 4, 2, 23, 7, 16
    Q, K, V = _rand(3, n_q, C, d), _rand(4, n_kv, T, d), _rand(5, n_kv, T, d)
    Kc, Vc = _rand(6, n_kv, C, d), _rand(7, n_kv, C, d)
    out = O.dense_attn(Q, K, V, Kc, Vc)
    allow = np.ones((C, T + C), dtype=bool)
    allow[:, T:] = np.tril(np.ones((C, C), dtype=bool))     # diagonal visible
    for h in range(n_q):
        kv = h // 2
        ref = _sdpa(Q[h], np.concatenate([K[kv], Kc[kv]]), np.concatenate([V[kv], Vc[kv]]), mask=allow)
        assert np.max(np.abs(out[h] - ref)) < 1e-12


def test_chunked_dense_prefill_equals_full_causal_attention():
    # Eq. 2 applied chunk after chunk == Eq. 1 on the whole sequence; includes a ragged last chunk.
    n_q, n_kv, L, d = 2, 1, 29, 8
    Q, K, V = _rand(8, n_q, L, d), _rand(9, n_kv, L, d), _rand(10, n_kv, L, d)
    out = O.chunked_prefill(Q, K, V, chunk=8, budget=None)
    for h in range(n_q):
        ref = _sdpa(Q[h], K[0], V[0], causal=True)
        assert np.max(np.abs(out[h] - ref)) < 1e-12


def test_full_budget_reproduces_dense_attention():
    n_q, n_kv, T, C, d = 4, 2, 37, 9, 8
    Q, K, V = _rand(11, n_q, C, d) + 0.3, _rand(12, n_kv, T, d), _rand(13, n_kv, T, d)
    Kc, Vc = _rand(14, n_kv, C, d), _rand(15, n_kv, C, d)
    dense = O.dense_attn(Q, K, V, Kc, Vc)
    for budget in (T, T + 5):
        out, k_idx = O.quoka_chunk_attn(Q, K, V, Kc, Vc, n_retain=4, budget=budget)
        assert all(k.tolist() == list(range(T)) for k in k_idx)
        assert np.array_equal(out, dense)


def test_attention_uses_unnormalised_keys_and_all_queries():
    # Scaling one selected key changes the output (so attention is not run on unit keys), and every
    # chunk query gets an output row even when only 2 queries are retained for scoring.
    n_q, n_kv, T, C, d = 2, 1, 12, 6, 4
    Q, K, V = _rand(16, n_q, C, d), _rand(17, n_kv, T, d), _rand(18, n_kv, T, d)
    Kc, Vc = _rand(19, n_kv, C, d), _rand(20, n_kv, C, d)
    out, k_idx = O.quoka_chunk_attn(Q, K, V, Kc, Vc, n_retain=2, budget=5)
    assert out.shape == (n_q, C, d) and k_idx.shape == (1, 5)
    K2 = K.copy()
    K2[0, k_idx[0][0]] *= 3.0                       # same direction => same selection
    out2, k_idx2 = O.quoka_chunk_attn(Q, K2, V, Kc, Vc, n_retain=2, budget=5)
    assert np.array_equal(k_idx, k_idx2)
    assert np.max(np.abs(out - out2)) > 1e-3


def test_uniform_logits_give_prefix_means():
    # All keys zero => every visible key gets the same weight: row i is the mean of the selected past
    # values and chunk values 0..i (diagonal included, later chunk tokens excluded).
    n_kv, T, C, d = 1, 10, 5, 4
    Q = _rand(21, 2, C, d)
    K, Kc = np.zeros((n_kv, T, d)), np.zeros((n_kv, C, d))
    V, Vc = _rand(22, n_kv, T, d), _rand(23, n_kv, C, d)
    sel = [np.array([1, 4, 7])]
    out = O.sparse_attn(Q, K, V, sel, Kc, Vc)
    for i in range(C):
        want = (V[0][[1, 4, 7]].sum(0) + Vc[0][: i + 1].sum(0)) / (3 + i + 1)
        assert np.allclose(out[0, i], want, atol=1e-14) and np.allclose(out[1, i], want, atol=1e-14)


def test_two_key_closed_form_fixes_the_softmax_scale():
    # One past key k = sqrt(d) * e0 and the chunk's own key 0: row 0 has logits (a, 0) for q = a * e0,
    # so the weight on the past value is the logistic function of a -- only true with the 1/sqrt(d) scale.
    d, a = 16, 1.7
    Q = np.zeros((1, 1, d)); Q[0, 0, 0] = a
    K = np.zeros((1, 1, d)); K[0, 0, 0] = math.sqrt(d)
    V = np.zeros((1, 1, d)); V[0, 0, 0] = 1.0
    Kc = np.zeros((1, 1, d)); Vc = np.zeros((1, 1, d)); Vc[0, 0, 1] = 1.0
    out, lse = O.sparse_attn(Q, K, V, [np.array([0])], Kc, Vc, return_lse=True)
    p = 1.0 / (1.0 + math.exp(-a))
    assert out[0, 0, 0] == pytest.approx(p, abs=1e-14)
    assert out[0, 0, 1] == pytest.approx(1 - p, abs=1e-14)
    assert lse[0, 0] == pytest.approx(math.log(math.exp(a) + 1.0), abs=1e-14)


def test_rows_sum_to_one_and_outputs_stay_in_value_hull():
    n_q, n_kv, T, C, d = 4, 2, 50, 13, 8
    Q, K, V = 3 * _rand(24, n_q, C, d), _rand(25, n_kv, T, d), _rand(26, n_kv, T, d)
    Kc, Vc = _rand(27, n_kv, C, d), _rand(28, n_kv, C, d)
    sel = [np.arange(0, T, 3), np.arange(1, T, 5)]
    ones = O.sparse_attn(Q, K, np.ones_like(V), sel, Kc, np.ones_like(Vc))
    assert np.max(np.abs(ones - 1.0)) < 1e-13
    out = O.sparse_attn(Q, K, V, sel, Kc, Vc)
    for h in range(n_q):
        kv = h // 2
        for i in range(C):
            vis = np.concatenate([V[kv][sel[kv]], Vc[kv][: i + 1]])
            assert np.all(out[h, i] <= vis.max(0) + 1e-12) and np.all(out[h, i] >= vis.min(0) - 1e-12)


def test_one_hot_values_recover_the_probability_rows():
    # With V = identity the output row IS the softmax row; compare with scipy's softmax of the masked logits.
    from scipy.special import softmax
    T, C = 6, 4
    d = T + C
    Q, K, Kc = _rand(29, 1, C, d), _rand(30, 1, T, d), _rand(31, 1, C, d)
    eye = np.eye(d)
    out = O.dense_attn(Q, K, eye[None, :T], Kc, eye[None, T:])
    logits = Q[0] @ np.concatenate([K[0], Kc[0]]).T / math.sqrt(d)
    for i in range(C):
        vis = T + i + 1
        assert np.allclose(out[0, i, :vis], softmax(logits[i, :vis]), atol=1e-14)
        assert np.all(out[0, i, vis:] == 0.0)


def test_order_of_selected_keys_does_not_matter():
    n_q, n_kv, T, C, d = 2, 1, 20, 5, 8
    Q, K, V = _rand(32, n_q, C, d), _rand(33, n_kv, T, d), _rand(34, n_kv, T, d)
    Kc, Vc = _rand(35, n_kv, C, d), _rand(36, n_kv, C, d)
    a = O.sparse_attn(Q, K, V, [np.array([2, 5, 11, 17])], Kc, Vc)
    b = O.sparse_attn(Q, K, V, [np.array([17, 2, 11, 5])], Kc, Vc)
    assert np.max(np.abs(a - b)) < 1e-13


def test_quoka_prefill_with_huge_budget_equals_full_causal():
    n_q, n_kv, L, d = 4, 2, 40, 8
    Q, K, V = _rand(37, n_q, L, d) + 0.2, _rand(38, n_kv, L, d), _rand(39, n_kv, L, d)
    sparse_all = O.chunked_prefill(Q, K, V, chunk=8, n_retain=3, budget=10**6)
    dense = O.chunked_prefill(Q, K, V, chunk=8, budget=None)
    assert np.array_equal(sparse_all, dense)
    # and a small budget really changes the result (the selection is doing something)
    sparse = O.chunked_prefill(Q, K, V, chunk=8, n_retain=3, budget=4)
    assert np.max(np.abs(sparse - dense)) > 1e-3
    # first chunk has no past: identical regardless of budget
    assert np.array_equal(sparse[:, :8], dense[:, :8])


def test_row_and_head_sampling_matches_the_full_result():
    n_q, n_kv, T, C, d = 4, 2, 30, 12, 8
    Q, K, V = _rand(40, n_q, C, d), _rand(41, n_kv, T, d), _rand(42, n_kv, T, d)
    Kc, Vc = _rand(43, n_kv, C, d), _rand(44, n_kv, C, d)
    sel = [np.arange(0, T, 2), np.arange(1, T, 3)]
    full, lse = O.sparse_attn(Q, K, V, sel, Kc, Vc, return_lse=True)
    rows, heads = [0, 5, 11], [1, 2]
    part, lse_p = O.sparse_attn(Q, K, V, sel, Kc, Vc, return_lse=True, rows=rows, heads=heads)
    assert np.allclose(part, full[heads][:, rows], atol=1e-15)
    assert np.allclose(lse_p, lse[heads][:, rows], atol=1e-15)
