"""quoka_select_keys (scoring + top-B as one stage; Alg. 1 S = Qbar K^T, max, topk) against the oracle and against the
two separate calls.  On long bf16 caches the stage scores every key with one bf16 term first and re-scores only the
keys near the cut exactly; its index lists must still be the top-B of the exact scores."""
import numpy as np
import pytest
import torch

import gen
from oracle import quoka_oracle as O
from tests import parity as P

pytestmark = pytest.mark.gpu


def _pk():
    import paper_2602_08722_amd as pk
    pk.load_library()
    return pk


def _buffers(pk, w, t=None):
    t = gen.to_torch(w, "cuda:0") if t is None else t
    mb = min(max(w.budgets), w.t_max)
    return pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain, max_budget=mb)


def _staged(buf):
    buf.select_queries()
    buf.scores.fill_(float("nan"))
    buf.k_idx.fill_(-1)
    buf.score_keys()
    buf.topk_keys()
    torch.cuda.synchronize()
    return buf.scores.clone(), buf.k_idx.clone(), buf.k_cnt.clone()


def _fused(buf, dirty=0x5A):
    buf.select_queries()
    buf.scores.fill_(float("nan"))
    buf.k_idx.fill_(-1)
    buf.k_cnt.fill_(-1)
    buf.workspace.fill_(dirty)       # the stage clears what it needs itself
    buf.select_queries()             # (its workspace region was just overwritten; Q-bar is an input of the stage)
    buf.select_keys()
    torch.cuda.synchronize()
    return buf.scores.clone(), buf.k_idx.clone(), buf.k_cnt.clone()


def _compare(pk, w, t=None, oracle=True):
    buf = _buffers(pk, w, t)
    sc_s, idx_s, cnt_s = _staged(buf)
    sc_f, idx_f, cnt_f = _fused(buf)
    assert torch.equal(cnt_f, cnt_s)
    qbar = gen.from_torch(buf.qbar)
    q_idx = gen.from_torch(buf.q_idx)
    n_exact = n_all = 0
    for b in range(w.batch):
        T, n = w.kv_lens[b], int(cnt_s[b, 0])
        assert n == min(w.budgets[b], T, buf.shape.max_budget)
        # the same index lists, bit for bit, as the two separate calls
        assert torch.equal(idx_f[b, :, :n], idx_s[b, :, :n]), f"sequence {b}: index lists differ from the staged calls"
        if T == 0:
            continue
        got, exact = sc_f[b, :, :T], sc_s[b, :, :T]
        assert not torch.isnan(got).any()
        same = got.view(torch.int32) == exact.view(torch.int32)
        n_exact += int(same.sum())
        n_all += same.numel()
        if oracle:
            want = O.key_scores(w.Q[b], q_idx[b], w.K[b][:, :T], w.n_kv)
            for kv in range(w.n_kv):
                if P.two_pass_scores(w):
                    P.check_two_pass_scores(got[kv].cpu().numpy(), want[kv], qbar[b, kv], w.budgets[b],
                                            what=f"b{b} kv{kv}")
                else:
                    assert P.max_abs(got[kv].cpu().numpy(), want[kv]) <= P.TOL_SCORE
                P.check_topk_set(idx_f[b, kv, :n].cpu().numpy(), want[kv], w.budgets[b], what=f"b{b} kv{kv}")
    return n_exact, n_all


CASES = [
    # just past the single-block limit; budgets on both sides of the tile size; N_Q variants 4 / 2 / 1 query blocks
    dict(n_q=8, n_kv=2, d=128, chunk=256, n_retain=128, kv_lens=[33000], budgets=[4000]),
    dict(n_q=8, n_kv=2, d=128, chunk=256, n_retain=64, kv_lens=[40000], budgets=[1]),
    dict(n_q=4, n_kv=2, d=128, chunk=64, n_retain=20, kv_lens=[36111], budgets=[36110]),
    dict(n_q=4, n_kv=4, d=64, chunk=96, n_retain=40, kv_lens=[50001], budgets=[7777]),
    dict(n_q=4, n_kv=1, d=64, chunk=200, n_retain=128, kv_lens=[34000], budgets=[3000]),
    # ragged batch: an empty cache, one shorter than a tile, a full-budget one and a budget beyond the cache
    dict(n_q=8, n_kv=2, d=128, chunk=128, n_retain=32, kv_lens=[45000, 0, 1500, 33333, 70000],
         budgets=[5000, 10, 150, 33333, 99999], batch=5),
    # one head per group (Q-bar rows are single unit queries), decode-sized chunk (identity selection)
    dict(n_q=2, n_kv=2, d=128, chunk=4, n_retain=16, kv_lens=[65537], budgets=[8000]),
    # short caches go through the stage too (it is then the two separate launches)
    dict(n_q=8, n_kv=2, d=128, chunk=100, n_retain=16, kv_lens=[3000, 32768], budgets=[300, 4000], batch=2),
]


@pytest.mark.parametrize("case", CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_select_keys_matches_the_oracle_and_the_staged_calls(case):
    pk = _pk()
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(dtype="bf16", batch=batch, seed=31, **case)
    n_exact, n_all = _compare(pk, w)
    if P.two_pass_scores(w):
        assert n_exact < 0.7 * n_all, (n_exact, n_all)   # the cheaper pass really ran: most keys keep their provisional score
    else:
        assert n_exact == n_all                          # short caches: the stage is the two separate launches


def test_select_keys_with_planted_exact_ties_and_repeated_keys():
    """Equal exact scores go to the lower position, also when they straddle the cut and sit in different tiles: rows
    of the cache are repeated (identical keys score identically in both passes) so that the cut falls inside a group
    of equal scores."""
    pk = _pk()
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=128, n_retain=64, kv_lens=[40000], budgets=[500],
                        seed=32)
    # find a key that ranks near the budget, then copy it to many positions spread over the cache
    q_idx = O.select_queries(w.Q[0], w.n_retain)
    sc = O.key_scores(w.Q[0], q_idx, w.K[0], w.n_kv)
    for kv in range(w.n_kv):
        order = np.argsort(-sc[kv], kind="stable")
        src = order[480]
        dst = np.arange(17, 40000, 1301)       # 31 copies: more than the 20 places left below rank 480
        w.K[0, kv, dst] = w.K[0, kv, src]
    _compare(pk, w)


def test_select_keys_when_every_key_is_a_candidate():
    """A cache of identical keys: every score ties, the band is the whole cache, and the first B positions win."""
    pk = _pk()
    w = gen.make_custom(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=64, n_retain=32, kv_lens=[33500], budgets=[1000],
                        seed=33)
    w.K[0, :, :] = w.K[0, :, :1]
    buf = _buffers(pk, w)
    _, idx_f, cnt_f = _fused(buf)
    assert cnt_f.tolist() == [[1000, 1000]]
    assert torch.equal(idx_f[0, :, :1000].cpu(), torch.arange(1000, dtype=torch.int32).expand(2, 1000))
    _compare(pk, w, oracle=False)


@pytest.mark.parametrize("name,kw", [("c4", {}), ("c5", dict(n_retain=128, budget_frac=0.12))])
def test_select_keys_full_size(name, kw):
    pk = _pk()
    w = gen.make_workload(name, **kw)
    n_exact, n_all = _compare(pk, w, oracle=(name == "c4"))
    assert n_exact < 0.5 * n_all


def test_select_keys_token_major_cache():
    """Strided (token-major) caches give the same lists as their head-major copies."""
    pk = _pk()
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=4, d=128, chunk=64, n_retain=32, kv_lens=[40000], budgets=[3000],
                        seed=34)
    t = gen.to_torch(w, "cuda:0")
    tm = dict(t)
    for k in ("k", "v"):
        tm[k] = t[k].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    a, b = _buffers(pk, w, t), _buffers(pk, w, tm)
    ra, rb = _fused(a), _fused(b)
    for x, y in zip(ra, rb):
        assert torch.equal(x.view(torch.int32), y.view(torch.int32))
