"""GPU parity of the multi-chunk prefill driver (Alg. 2's loop) against the oracle."""
import numpy as np
import pytest
import torch

import gen
from oracle import quoka_oracle as O
from tests import parity as P

pytestmark = pytest.mark.gpu


def _prompt(seed, n_q, n_kv, d, L):
    """A whole prompt as one 'chunk' of the seeded generator: Q [1, n_q, L, d], K / V [1, n_kv, L, d] (bf16-exact)."""
    w = gen.make_custom(dtype="bf16", n_q=n_q, n_kv=n_kv, d=d, chunk=L, n_retain=1, kv_lens=[0], budgets=[0],
                        batch=1, seed=seed)
    return w.Q[0], w.Kc[0], w.Vc[0]


def _full_causal(Q, K, V):
    """Plain causal attention over the whole prompt in float64: the definition dense chunked prefill must reach."""
    n_q, L, d = Q.shape
    g = n_q // K.shape[0]
    out = np.empty((n_q, L, d))
    mask = np.tril(np.ones((L, L), dtype=bool))
    for h in range(n_q):
        s = (Q[h].astype(np.float64) @ K[h // g].astype(np.float64).T) / np.sqrt(d)
        s = np.where(mask, s, -np.inf)
        p = np.exp(s - s.max(axis=1, keepdims=True))
        out[h] = (p / p.sum(axis=1, keepdims=True)) @ V[h // g].astype(np.float64)
    return out


def _to_dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to("cuda:0")[None]


@pytest.mark.parametrize("L,chunk", [(640, 128), (700, 192), (96, 128), (130, 128), (1027, 256)])  # the last two end in a decode-sized chunk
def test_dense_chunked_prefill_is_full_causal_attention(L, chunk):
    import paper_2602_08722_amd as pk
    pk.load_library()
    Q, K, V = _prompt(31, 8, 2, 128, L)
    pb = pk.PrefillBuffers(_to_dev(Q), _to_dev(K), _to_dev(V), chunk, n_retain=16, budget=0)
    out = pb.run(sparse=False)
    torch.cuda.synchronize()
    got = out[0].float().cpu().numpy()
    assert P.max_abs(got, _full_causal(Q, K, V)) <= P.TOL_OUT["bf16"]


@pytest.mark.parametrize("L,chunk,n_retain,budget", [(768, 128, 16, 96), (700, 192, 32, 64), (1027, 256, 16, 200)])
def test_sparse_chunked_prefill_matches_oracle(L, chunk, n_retain, budget):
    import paper_2602_08722_amd as pk
    pk.load_library()
    Q, K, V = _prompt(32, 8, 2, 128, L)
    pb = pk.PrefillBuffers(_to_dev(Q), _to_dev(K), _to_dev(V), chunk, n_retain=n_retain, budget=budget)
    out = pb.run(sparse=True)
    torch.cuda.synchronize()
    got = out[0].float().cpu().numpy()
    want = O.chunked_prefill(Q, K, V, chunk, n_retain=n_retain, budget=budget)
    assert P.max_abs(got, want) <= P.TOL_OUT["bf16"]
    # the scratch buffers hold the last chunk's selection: it must be the oracle's for that chunk
    s = (L - 1) // chunk * chunk
    _, _, k_idx = O.quoka_select(Q[:, s:], K[:, :s], n_retain, budget)
    cnt = pb.k_cnt[0].cpu().numpy()
    got_idx = pb.k_idx[0].cpu().numpy()
    scores = O.key_scores(Q[:, s:], O.select_queries(Q[:, s:], n_retain), K[:, :s], K.shape[0])
    for kv in range(K.shape[0]):
        assert cnt[kv] == min(budget, s)
        P.check_topk_set(got_idx[kv, :cnt[kv]], scores[kv], min(budget, s), what=f"last chunk kv{kv}")
