"""Stage-wise GPU parity: each HIP stage is fed the ORACLE's upstream output and compared with the oracle."""
import ctypes

import numpy as np
import pytest
import torch

import gen
from oracle import quoka_oracle as O
from tests.bf16_round import round_to_bf16
from tests import parity as P

pytestmark = pytest.mark.gpu


def _pk():
    import paper_2602_08722_amd as pk
    pk.load_library()
    return pk


def _buffers(w, max_budget=None, score_flags=0):
    pk = _pk()
    t = gen.to_torch(w, "cuda:0")
    mb = max_budget if max_budget is not None else min(max(w.budgets), w.t_max)
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain, max_budget=mb,
                          score_flags=score_flags)
    return buf


SELECT_CASES = [
    dict(dtype="f32", n_q=2, n_kv=1, d=64, chunk=128, n_retain=16),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=200, n_retain=64),     # ragged tile
    dict(dtype="bf16", n_q=8, n_kv=2, d=64, chunk=77, n_retain=33),
    dict(dtype="f32", n_q=4, n_kv=4, d=128, chunk=513, n_retain=128),
    dict(dtype="bf16", n_q=4, n_kv=1, d=128, chunk=24, n_retain=32),      # C <= N_Q: identity
    dict(dtype="bf16", n_q=2, n_kv=2, d=128, chunk=1, n_retain=16),       # single query (decode-like)
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=2048, n_retain=128, batch=2),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=2500, n_retain=100),                 # multi-block path
    dict(dtype="f32", n_q=2, n_kv=1, d=64, chunk=3000, n_retain=7),
    dict(dtype="bf16", n_q=16, n_kv=1, d=64, chunk=300, n_retain=128),                  # group of 16
    dict(dtype="bf16", n_q=2, n_kv=1, d=128, chunk=8192, n_retain=128),                 # largest chunk, largest N_Q
    dict(dtype="bf16", n_q=2, n_kv=2, d=128, chunk=5000, n_retain=1),                   # a single retained query
    dict(dtype="bf16", n_q=2, n_kv=2, d=128, chunk=700, n_retain=3),
    # batches of short chunks (at least 128 heads): mean, cosines and selection of a head in one block
    dict(dtype="bf16", n_q=32, n_kv=8, d=64, chunk=200, n_retain=48, batch=4),
    dict(dtype="f32", n_q=64, n_kv=16, d=128, chunk=300, n_retain=17, batch=2),
    dict(dtype="bf16", n_q=32, n_kv=4, d=128, chunk=512, n_retain=128, batch=4),
]


@pytest.mark.parametrize("case", SELECT_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_select_queries(case):
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, kv_lens=[64] * batch, budgets=[8] * batch, seed=11, **case)
    buf = _buffers(w)
    buf.select_queries()
    torch.cuda.synchronize()
    q_idx = gen.from_torch(buf.q_idx)
    qbar = gen.from_torch(buf.qbar)
    n_keep = min(w.n_retain, w.chunk)
    for b in range(w.batch):
        cos = O.cos_to_mean(w.Q[b])
        for h in range(w.n_q):
            P.check_query_ranking(q_idx[b, h], cos[h], n_keep, what=f"b{b} h{h}")
        # Q-bar from the GPU's own ranking (equal to the oracle's unless a documented tie swapped rows)
        want = O.group_mean_queries(w.Q[b], q_idx[b], w.n_kv)
        assert P.max_abs(qbar[b], want) <= P.TOL_QBAR


@pytest.mark.parametrize("case", [
    dict(n_q=4, n_kv=2, d=128, chunk=300, n_retain=64),                      # one block per head
    dict(n_q=4, n_kv=2, d=128, chunk=2600, n_retain=100),                    # several blocks per head
    dict(n_q=32, n_kv=8, d=64, chunk=256, n_retain=48, batch=4),             # batched: one block does a whole head
], ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_select_queries_with_repeated_zero_and_rescaled_rows(case):
    """Rows of the chunk repeated many times (equal cosines bit for bit: the lower position must win wherever the cut
    falls inside such a group), rows scaled by powers of two from 2^-6 to 2^6 (the cosine of a row does not depend on
    its length, the mean query does) and zero rows (cosine 0 by definition).  N(0,1) inputs have none of these."""
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(dtype="bf16", batch=batch, kv_lens=[64] * batch, budgets=[8] * batch, seed=18, **case)
    rng = np.random.default_rng(7)
    C = w.chunk
    groups = []
    for b in range(w.batch):
        w.Q[b] *= np.exp2(rng.integers(-6, 7, size=(w.n_q, C)).astype(np.float64))[:, :, None]
        src = rng.choice(C, size=3, replace=False)
        members = [np.sort(rng.choice(C, size=max(w.n_retain // 2, 2), replace=False)) for _ in src]
        for s0, m in zip(src, members):
            w.Q[b][:, m] = w.Q[b][:, s0:s0 + 1]
        w.Q[b][:, rng.choice(C, size=5, replace=False)] = 0.0
        # groups of identical rows as they ended up (later writes may have overwritten earlier ones), per head
        per_head = []
        for h in range(w.n_q):
            seen = {}
            for i in range(C):
                seen.setdefault(w.Q[b][h, i].tobytes(), []).append(i)
            per_head.append([g for g in seen.values() if len(g) > 1])
        groups.append(per_head)
    buf = _buffers(w)
    buf.select_queries()
    torch.cuda.synchronize()
    q_idx = gen.from_torch(buf.q_idx)
    qbar = gen.from_torch(buf.qbar)
    n_keep = min(w.n_retain, C)
    for b in range(w.batch):
        cos = O.cos_to_mean(w.Q[b])
        for h in range(w.n_q):
            P.check_query_ranking(q_idx[b, h], cos[h], n_keep, what=f"b{b} h{h}")
            chosen = set(int(i) for i in q_idx[b, h, :n_keep])
            for g in groups[b][h]:
                picked = [i in chosen for i in g]
                assert picked == sorted(picked, reverse=True), f"b{b} h{h}: a later copy was preferred to an earlier one"
        want = O.group_mean_queries(w.Q[b], q_idx[b], w.n_kv)
        assert P.max_abs(qbar[b], want) <= P.TOL_QBAR * max(1.0, float(np.abs(want).max()))


SCORE_CASES = [
    dict(dtype="f32", n_q=2, n_kv=1, d=64, chunk=128, n_retain=16, kv_lens=[1000]),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=256, n_retain=64, kv_lens=[1500]),          # ragged tail tile
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=256, n_retain=128, kv_lens=[4096 + 37]),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=256, n_retain=20, kv_lens=[700]),           # one partly padded block
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=256, n_retain=96, kv_lens=[700]),           # 3 blocks -> padded 4th
    dict(dtype="bf16", n_q=4, n_kv=4, d=64, chunk=64, n_retain=40, kv_lens=[900]),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=64, n_retain=32, kv_lens=[300, 0, 1029], batch=3),
    dict(dtype="f32", n_q=4, n_kv=2, d=128, chunk=64, n_retain=32, kv_lens=[300, 5], batch=2),
    dict(dtype="bf16", n_q=2, n_kv=1, d=128, chunk=8, n_retain=16, kv_lens=[40000]),            # several tiles per block
]


@pytest.mark.parametrize("case", SCORE_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_score_keys(case):
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, budgets=[8] * batch, seed=12, **case)
    buf = _buffers(w)
    # feed the oracle's Q-bar (rounded to float32, which is what the interface carries)
    qbar_o = np.stack([O.group_mean_queries(w.Q[b], O.select_queries(w.Q[b], w.n_retain), w.n_kv)
                       for b in range(w.batch)]).astype(np.float32)
    buf.qbar.copy_(torch.from_numpy(qbar_o))
    buf.scores.fill_(float("nan"))
    buf.score_keys()
    torch.cuda.synchronize()
    sc = gen.from_torch(buf.scores)
    worst = 0.0
    for b in range(w.batch):
        T = w.kv_lens[b]
        want = O.key_scores_preagg(qbar_o[b].astype(np.float64), w.K[b][:, :T])
        got = sc[b, :, :T]
        assert not np.isnan(got).any()
        worst = max(worst, P.max_abs(got, want))
    assert worst <= P.TOL_SCORE, f"max |score - oracle| = {worst}"


@pytest.mark.parametrize("kv_len", [3000, 40000], ids=["exact-scorer", "two-pass-stage"])
def test_scores_with_zero_keys_and_keys_of_very_different_norms(kv_len):
    """Cosine scores do not depend on the length of a key (Sec. 3.2) and a zero key scores zero: keys scaled by powers
    of two from 2^-6 to 2^6 (exact in bf16), some keys and one retained query set to zero.  N(0,1) inputs have norms
    within a few per cent of each other and never a zero."""
    pk = _pk()
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=96, n_retain=32, kv_lens=[kv_len],
                        budgets=[kv_len // 8], seed=17)
    T = kv_len
    rng = np.random.default_rng(5)
    w.K[0][:, :T] *= np.exp2(rng.integers(-6, 7, size=(w.n_kv, T)).astype(np.float64))[:, :, None]
    zero_at = rng.choice(T, size=40, replace=False)
    w.K[0][:, zero_at] = 0.0
    w.Q[0][3, 11] = 0.0                       # a zero query: cosine 0 to the mean, neither smallest nor largest
    buf = _buffers(w)
    buf.select_queries()
    buf.scores.fill_(float("nan"))
    buf.k_idx.fill_(-1)
    buf.select_keys()
    torch.cuda.synchronize()
    q_idx = gen.from_torch(buf.q_idx)
    qbar = gen.from_torch(buf.qbar)
    sc = gen.from_torch(buf.scores)[0, :, :T]
    idx = gen.from_torch(buf.k_idx)[0]
    n = int(gen.from_torch(buf.k_cnt)[0, 0])
    assert n == w.budgets[0]
    want = O.key_scores(w.Q[0], q_idx[0], w.K[0][:, :T], w.n_kv)
    assert not np.isnan(sc).any()
    assert np.all(sc[:, zero_at] == 0.0) and np.all(want[:, zero_at] == 0.0)
    for kv in range(w.n_kv):
        if P.two_pass_scores(w):
            P.check_two_pass_scores(sc[kv], want[kv], qbar[0, kv], w.budgets[0], what=f"kv{kv}")
        else:
            assert P.max_abs(sc[kv], want[kv]) <= P.TOL_SCORE
        P.check_topk_set(idx[kv, :n], want[kv], w.budgets[0], what=f"kv{kv}")


ABLATION_CASES = [
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=256, n_retain=64, kv_lens=[1500]),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=256, n_retain=100, kv_lens=[4096 + 37]),   # padded query block
    dict(dtype="bf16", n_q=4, n_kv=4, d=64, chunk=64, n_retain=40, kv_lens=[900]),
    dict(dtype="f32", n_q=4, n_kv=2, d=128, chunk=64, n_retain=32, kv_lens=[300, 5], batch=2),
]


@pytest.mark.parametrize("flags", [1, 2, 3], ids=["dot", "mean", "dot+mean"])
@pytest.mark.parametrize("case", ABLATION_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_ablation_scorers(case, flags):
    """Sec. 3.2-3.3 ablations: dot product instead of cosine (bit 0), mean instead of max over queries (bit 1).
    Q-bar and the scores are checked against the oracle's variants; the query sub-selection must not change."""
    pk = _pk()
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, budgets=[8] * batch, seed=14, **case)
    t = gen.to_torch(w, "cuda:0")
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain,
                          max_budget=min(8, w.t_max), score_flags=flags)
    similarity = "dot" if flags & 1 else "cosine"
    reduce = "mean" if flags & 2 else "max"
    buf.select_queries()
    buf.scores.fill_(float("nan"))
    buf.score_keys()
    torch.cuda.synchronize()
    q_idx = gen.from_torch(buf.q_idx)
    qbar = gen.from_torch(buf.qbar)
    sc = gen.from_torch(buf.scores)
    n_keep = min(w.n_retain, w.chunk)
    for b in range(w.batch):
        cos = O.cos_to_mean(w.Q[b])
        for h in range(w.n_q):
            P.check_query_ranking(q_idx[b, h], cos[h], n_keep, what=f"b{b} h{h}")
        want_qbar = O.group_mean_queries(w.Q[b], q_idx[b], w.n_kv, similarity)
        scale_q = max(1.0, float(np.abs(want_qbar).max()))
        assert P.max_abs(qbar[b], want_qbar) <= P.TOL_QBAR * scale_q
        T = w.kv_lens[b]
        want = O.key_scores_preagg(qbar[b].astype(np.float64), w.K[b][:, :T], similarity, reduce)
        got = sc[b, :, :T]
        assert not np.isnan(got).any()
        # dot products are not bounded by 1: the float32 accumulation error scales with the magnitudes involved
        scale = max(1.0, float(np.abs(want).max())) if T > 0 else 1.0
        assert P.max_abs(got, want) <= P.TOL_SCORE * scale * (4.0 if flags & 1 else 1.0)
        # and the whole chain against the literal post-hoc form
        lit = O.key_scores(w.Q[b], q_idx[b], w.K[b][:, :T], w.n_kv, similarity, reduce)
        assert P.max_abs(got, lit) <= 4e-6 * scale * (4.0 if flags & 1 else 1.0)


@pytest.mark.parametrize("flags", [8, 9, 10], ids=["qbar-bf16", "qbar-bf16+dot", "qbar-bf16+mean"])
@pytest.mark.parametrize("case", ABLATION_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_reduced_precision_scorer(case, flags):
    """Cheaper Qbar K^T (the paper's conclusion names it as future work): Qbar rounded to bfloat16 before the
    product.  Q-bar itself is unchanged (float32); the scores must be the exact scores of the rounded Q-bar, and the
    selected keys the top-B of those scores."""
    pk = _pk()
    case = dict(case)
    batch = case.pop("batch", 1)
    budgets = [max(1, t // 6) for t in case["kv_lens"]]
    w = gen.make_custom(batch=batch, budgets=budgets, seed=16, **case)
    t = gen.to_torch(w, "cuda:0")
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain,
                          score_flags=flags)
    similarity = "dot" if flags & 1 else "cosine"
    reduce = "mean" if flags & 2 else "max"
    buf.select_queries()
    buf.scores.fill_(float("nan"))
    buf.score_keys()
    buf.topk_keys()
    torch.cuda.synchronize()
    q_idx, qbar, sc = gen.from_torch(buf.q_idx), gen.from_torch(buf.qbar), gen.from_torch(buf.scores)
    k_idx, k_cnt = gen.from_torch(buf.k_idx), gen.from_torch(buf.k_cnt)
    for b in range(w.batch):
        T, B = w.kv_lens[b], w.budgets[b]
        want_qbar = O.group_mean_queries(w.Q[b], q_idx[b], w.n_kv, similarity)
        assert P.max_abs(qbar[b], want_qbar) <= P.TOL_QBAR * max(1.0, float(np.abs(want_qbar).max()))
        want = O.key_scores_preagg(round_to_bf16(qbar[b]), w.K[b][:, :T], similarity, reduce)
        got = sc[b, :, :T]
        assert not np.isnan(got).any()
        scale = max(1.0, float(np.abs(want).max())) if T > 0 else 1.0
        assert P.max_abs(got, want) <= P.TOL_SCORE * scale * (4.0 if flags & 1 else 1.0)
        # not the exact scorer in disguise: the rounding is visible
        exact = O.key_scores_preagg(qbar[b].astype(np.float64), w.K[b][:, :T], similarity, reduce)
        # (with one head per group and dot products Q-bar is a bf16 query itself: nothing to round)
        if T > 64 and not (flags & 1 and w.n_q == w.n_kv and w.dtype == "bf16"):
            assert P.max_abs(want, exact) > 20 * P.TOL_SCORE * scale
        for kv in range(w.n_kv):
            n = int(k_cnt[b, kv])
            assert n == min(B, T)
            P.check_topk_set(k_idx[b, kv, :n], want[kv], B, what=f"b{b} kv{kv}")


@pytest.mark.parametrize("flags", [4, 7], ids=["uniform", "uniform+dot+mean"])
@pytest.mark.parametrize("case", ABLATION_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_uniform_query_sampling(case, flags):
    """The query-sampling baseline of Sec. 4 (queries sampled uniformly): q_idx is the even stride, bit-exact, and
    everything downstream (Q-bar, scores, selected keys, attention output) follows the oracle run with that rule."""
    pk = _pk()
    case = dict(case)
    batch = case.pop("batch", 1)
    budgets = [max(1, t // 5) for t in case["kv_lens"]]
    w = gen.make_custom(batch=batch, budgets=budgets, seed=15, **case)
    t = gen.to_torch(w, "cuda:0")
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain,
                          score_flags=flags)
    similarity = "dot" if flags & 1 else "cosine"
    reduce = "mean" if flags & 2 else "max"
    buf.q_idx.fill_(-1)
    buf.chunk_attn()
    torch.cuda.synchronize()
    q_idx, qbar, sc = gen.from_torch(buf.q_idx), gen.from_torch(buf.qbar), gen.from_torch(buf.scores)
    k_idx, k_cnt, out = gen.from_torch(buf.k_idx), gen.from_torch(buf.k_cnt), gen.from_torch(buf.out)
    tol_out = P.TOL_OUT[w.dtype]
    for b in range(w.batch):
        T, B = w.kv_lens[b], w.budgets[b]
        want_idx, want_sc, _ = O.quoka_select(w.Q[b], w.K[b][:, :T], w.n_retain, B, similarity, reduce, "uniform")
        assert np.array_equal(q_idx[b], want_idx)
        assert P.max_abs(qbar[b], O.group_mean_queries(w.Q[b], want_idx, w.n_kv, similarity)) <= \
            P.TOL_QBAR * max(1.0, float(np.abs(w.Q[b]).max()) if flags & 1 else 1.0)
        scale = max(1.0, float(np.abs(want_sc).max()))
        assert P.max_abs(sc[b, :, :T], want_sc) <= 4e-6 * scale * (4.0 if flags & 1 else 1.0)
        sel = []
        for kv in range(w.n_kv):
            n = int(k_cnt[b, kv])
            assert n == min(B, T)
            P.check_topk_set(k_idx[b, kv, :n], want_sc[kv], B, what=f"b{b} kv{kv}")
            sel.append(k_idx[b, kv, :n])
        want_out = O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], np.stack(sel), w.Kc[b], w.Vc[b])
        assert P.max_abs(out[b], want_out) <= tol_out


def _scores_for_topk(rng, n_kv, T, kind):
    if kind == "normal":
        return rng.standard_normal((n_kv, T)).astype(np.float32) * 0.2
    if kind == "ties":          # heavy ties: only 17 distinct values
        return (rng.integers(0, 17, size=(n_kv, T)).astype(np.float32) - 8) / 16
    if kind == "const":
        return np.full((n_kv, T), 0.25, dtype=np.float32)
    if kind == "narrow":        # all scores inside one float exponent, differing in the low mantissa bits
        base = np.float32(0.3)
        ulp = np.spacing(base)
        return (base + ulp * rng.integers(0, 64, size=(n_kv, T))).astype(np.float32)
    if kind == "signed":        # positive, negative and zero scores
        s = rng.standard_normal((n_kv, T)).astype(np.float32)
        s[:, ::7] = 0.0
        return s
    raise ValueError(kind)


TOPK_CASES = [
    # (T list, budgets, T_max, kind)
    ([1000], [100], 1000, "normal"),
    ([1000], [100], 1000, "ties"),
    ([1000], [999], 1000, "signed"),
    ([777], [1], 1024, "normal"),
    ([8192], [983], 8192, "normal"),
    ([16384], [4000], 16384, "ties"),
    ([500, 0, 1000], [50, 10, 2000], 1000, "normal"),       # empty sequence, budget > T
    ([300], [0], 300, "normal"),                            # zero budget
    ([64], [64], 64, "const"),
    ([5000], [1234], 5000, "const"),
    ([5000], [1234], 5000, "narrow"),
    ([40000], [4800], 40000, "normal"),                     # multi-block path
    ([40000], [4800], 40000, "ties"),
    ([40000], [39999], 40000, "signed"),
    ([70001], [12345], 70001, "narrow"),
    ([20000, 33000, 0, 17000], [2000, 33000, 5, 1], 33000, "normal"),
    ([131072], [8192], 131072, "normal"),
    ([131072], [8192], 131072, "const"),
    ([16384], [16383], 16384, "normal"),                    # budget T-1
    ([16385], [1], 16385, "signed"),
    ([32768], [7000], 32768, "normal"),                     # largest single-block size
    ([32768, 20000], [33, 19999], 32768, "ties"),
    ([32769], [100], 32769, "ties"),                        # smallest multi-block size
    ([65000, 40000], [33, 39999], 65536, "ties"),
    ([1], [1], 1, "normal"),
    ([3, 1, 2], [2, 5, 1], 3, "ties"),
]


@pytest.mark.parametrize("case", TOPK_CASES, ids=lambda c: f"T{c[0]}-B{c[1]}-{c[3]}")
def test_topk_keys_bit_exact(case):
    pk = _pk()
    Ts, budgets, t_max, kind = case
    b, n_kv = len(Ts), 3
    rng = np.random.default_rng(13)
    scores = np.stack([_scores_for_topk(rng, n_kv, t_max, kind) for _ in range(b)])
    # this stage reads no Q/K/V: describe the problem by hand instead of allocating a cache
    dev = "cuda:0"
    mb = min(max(budgets), t_max)
    shape = pk.QuokaShape()
    shape.batch, shape.n_q_heads, shape.n_kv_heads, shape.head_dim = b, n_kv, n_kv, 64
    shape.chunk_len, shape.max_kv_len, shape.n_retain, shape.max_budget = 8, t_max, 4, mb
    shape.dtype = pk.QUOKA_BF16
    for name, tok in (("q_stride", 8), ("kv_stride", t_max), ("ck_stride", 8), ("o_stride", 8)):
        setattr(shape, name, (ctypes.c_int64 * 3)(n_kv * tok * 64, tok * 64, 64))
    ws = torch.empty(pk.quoka_workspace_bytes(shape), dtype=torch.uint8, device=dev)
    sc = torch.from_numpy(scores).to(dev)
    k_idx = torch.full((b, n_kv, max(mb, 1)), -7, dtype=torch.int32, device=dev)
    k_cnt = torch.full((b, n_kv), -7, dtype=torch.int32, device=dev)
    kv_lens = torch.tensor(Ts, dtype=torch.int32, device=dev)
    bud = torch.tensor(budgets, dtype=torch.int32, device=dev)
    for rep in range(2):   # second call reuses the workspace: it must be re-initialised by the library
        pk.quoka_topk_keys(shape, sc, kv_lens, bud, k_idx, k_cnt, ws)
        torch.cuda.synchronize()
        gi, gc = gen.from_torch(k_idx), gen.from_torch(k_cnt)
        for bi in range(b):
            want = O.topk_keys(scores[bi][:, :Ts[bi]].astype(np.float64), budgets[bi])
            for kv in range(n_kv):
                n = want.shape[1]
                assert gc[bi, kv] == n
                assert np.array_equal(gi[bi, kv, :n], want[kv]), f"rep{rep} b{bi} kv{kv}"


ATTN_CASES = [
    dict(dtype="f32", n_q=2, n_kv=1, d=64, chunk=128, kv_lens=[1024], budgets=[128]),
    dict(dtype="f32", n_q=4, n_kv=2, d=128, chunk=37, kv_lens=[100], budgets=[13]),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=128, kv_lens=[1000], budgets=[200]),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=100, kv_lens=[500], budgets=[65]),       # ragged rows and tiles
    dict(dtype="bf16", n_q=4, n_kv=4, d=128, chunk=96, kv_lens=[300], budgets=[64]),        # group of 1
    dict(dtype="bf16", n_q=4, n_kv=2, d=64, chunk=70, kv_lens=[300], budgets=[33]),         # head_dim 64, group of 2
    dict(dtype="bf16", n_q=16, n_kv=2, d=128, chunk=64, kv_lens=[256], budgets=[128]),      # group of 8
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=64, kv_lens=[0], budgets=[16]),          # empty cache
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=1, kv_lens=[200], budgets=[50]),         # single query
    # decode-sized chunks (g * C <= 32): split-KV kernel
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=1, kv_lens=[5000], budgets=[1300]),      # several splits and tiles
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=8, kv_lens=[3000], budgets=[700]),       # 32 rows, causal chunk rows
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=5, kv_lens=[1, 0, 131], budgets=[1, 4, 128], batch=3),
    dict(dtype="bf16", n_q=4, n_kv=4, d=64, chunk=32, kv_lens=[2000], budgets=[257]),       # group of 1, head_dim 64
    dict(dtype="bf16", n_q=32, n_kv=2, d=128, chunk=2, kv_lens=[777], budgets=[100]),       # group of 16
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=9, kv_lens=[300], budgets=[64]),         # 36 rows: prefill kernel
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=80, kv_lens=[150, 0, 64], budgets=[40, 9, 64], batch=3),
    dict(dtype="f32", n_q=4, n_kv=2, d=64, chunk=20, kv_lens=[90, 0], budgets=[30, 5], batch=2),
    # ragged batches: the kernel takes the sequences longest first (up to 64 of them; beyond that in batch order)
    dict(dtype="bf16", n_q=2, n_kv=1, d=64, chunk=40, kv_lens=[(37 * i) % 211 for i in range(64)],
         budgets=[(37 * i) % 211 // 3 + 1 for i in range(64)], batch=64),
    dict(dtype="bf16", n_q=2, n_kv=1, d=64, chunk=40, kv_lens=[(53 * i) % 173 for i in range(70)],
         budgets=[(53 * i) % 173 // 2 + 1 for i in range(70)], batch=70),
]


def _attn_id(c):
    return "-".join(f"{k}{v}" if len(str(v)) < 40 else f"{k}[{len(v)} values]" for k, v in c.items())


# every case as it is, and the bf16 ones again with the softmax scale applied in float32
ATTN_PARAMS = [pytest.param(c, False, id=_attn_id(c)) for c in ATTN_CASES] + \
              [pytest.param(c, True, id=_attn_id(c) + "-scale-f32") for c in ATTN_CASES if c["dtype"] == "bf16"]


@pytest.mark.parametrize("case,scale_f32", ATTN_PARAMS)
def test_sparse_and_dense_attention(case, scale_f32):
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, n_retain=8, seed=14, **case)
    buf = _buffers(w, score_flags=_pk().QUOKA_ATTN_SCALE_F32 if scale_f32 else 0)
    tol = P.TOL_OUT[w.dtype]
    # sparse: feed the oracle's index sets
    k_idx_o = []
    mb = buf.shape.max_budget
    idx_host = np.zeros((w.batch, w.n_kv, max(mb, 1)), dtype=np.int32)
    cnt_host = np.zeros((w.batch, w.n_kv), dtype=np.int32)
    for b in range(w.batch):
        T = w.kv_lens[b]
        _, _, ki = O.quoka_select(w.Q[b], w.K[b][:, :T], w.n_retain, w.budgets[b])
        k_idx_o.append(ki)
        idx_host[b, :, :ki.shape[1]] = ki
        cnt_host[b] = ki.shape[1]
    buf.k_idx.copy_(torch.from_numpy(idx_host))
    buf.k_cnt.copy_(torch.from_numpy(cnt_host))
    buf.out.fill_(float("nan"))
    buf.lse.fill_(float("nan"))
    buf.sparse_attn()
    torch.cuda.synchronize()
    out, lse = gen.from_torch(buf.out), gen.from_torch(buf.lse)
    for b in range(w.batch):
        T = w.kv_lens[b]
        want, want_lse = O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], k_idx_o[b], w.Kc[b], w.Vc[b], True)
        assert P.max_abs(out[b], want) <= tol, f"sparse b{b}: {P.max_abs(out[b], want)}"
        assert P.max_abs(lse[b], want_lse) <= (1e-4 if w.dtype == "f32" else 2e-2)
    # dense baseline
    buf.out.fill_(float("nan"))
    buf.dense_attn()
    torch.cuda.synchronize()
    out = gen.from_torch(buf.out)
    for b in range(w.batch):
        T = w.kv_lens[b]
        want = O.dense_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], w.Kc[b], w.Vc[b])
        assert P.max_abs(out[b], want) <= tol, f"dense b{b}: {P.max_abs(out[b], want)}"


@pytest.mark.parametrize("order", ["growing", "shrinking"])
@pytest.mark.parametrize("chunk,kv_len", [(160, 1500), (1024, 300), (8, 1500)],
                         ids=["prefill-kernel", "prefill-kernel-key-split", "decode-kernel"])
def test_attention_with_logits_that_span_many_octaves(order, chunk, kv_len):
    """Keys scaled by powers of two along the cache (exact in bf16), so that the largest logit keeps growing from tile
    to tile (the reference point of the online softmax moves again and again, with accumulator rescaling each time) or
    is met first and everything after it underflows against it.  Random N(0,1) inputs never do either.  With
    QUOKA_ATTN_SCALE_F32 the usual bar holds up to 32 times the size of unit-variance inputs; without it the bf16
    prefill kernel rounds Q a second time, and the documented, looser bound is checked at 8 times."""
    pk = _pk()
    for flags, n_oct, tol in ((pk.QUOKA_ATTN_SCALE_F32, 6, P.TOL_OUT["bf16"]), (0, 4, 8e-2)):
        w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=chunk, kv_lens=[kv_len], budgets=[kv_len // 3],
                            n_retain=8, seed=16)
        T = kv_len
        octave = (np.arange(T) * n_oct // T).astype(np.float64)        # 0 .. n_oct - 1
        if order == "shrinking":
            octave = octave[::-1].copy()
        w.K[0][:, :T] *= np.exp2(octave)[None, :, None]
        w.Kc[0] *= 2.0                                                 # the chunk's own keys sit inside the range
        _, _, ki = O.quoka_select(w.Q[0], w.K[0], w.n_retain, w.budgets[0])
        want_s, want_lse = O.sparse_attn(w.Q[0], w.K[0], w.V[0], ki, w.Kc[0], w.Vc[0], True)
        want_d = O.dense_attn(w.Q[0], w.K[0], w.V[0], w.Kc[0], w.Vc[0])
        buf = _buffers(w, score_flags=flags)
        idx_host = np.zeros((1, w.n_kv, buf.shape.max_budget), dtype=np.int32)
        idx_host[0, :, :ki.shape[1]] = ki
        buf.k_idx.copy_(torch.from_numpy(idx_host))
        buf.k_cnt.fill_(ki.shape[1])
        buf.out.fill_(float("nan"))
        buf.lse.fill_(float("nan"))
        buf.sparse_attn()
        torch.cuda.synchronize()
        assert P.max_abs(gen.from_torch(buf.out)[0], want_s) <= tol, (flags, P.max_abs(gen.from_torch(buf.out)[0], want_s))
        # log-sum-exp values reach into the tens and hundreds here: relative bar
        lse = gen.from_torch(buf.lse)[0]
        assert np.max(np.abs(lse - want_lse) / (1.0 + np.abs(want_lse))) <= 2e-2
        buf.out.fill_(float("nan"))
        buf.dense_attn()
        torch.cuda.synchronize()
        assert P.max_abs(gen.from_torch(buf.out)[0], want_d) <= tol, (flags, P.max_abs(gen.from_torch(buf.out)[0], want_d))


def test_sparse_attention_accepts_unsorted_indices_and_strided_views():
    pk = _pk()
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=64, kv_lens=[400], budgets=[96], n_retain=8, seed=15)
    t = gen.to_torch(w)
    # K/V cache stored token-major ([b, T, n_kv, d]) and viewed as [b, n_kv, T, d]: non-trivial strides
    k_tm = t["k"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    v_tm = t["v"].permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3)
    buf = pk.ChunkBuffers(t["q"], k_tm, v_tm, t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain)
    rng = np.random.default_rng(0)
    idx = np.stack([rng.permutation(400)[:96] for _ in range(2)])[None].astype(np.int32)   # unsorted
    buf.k_idx.copy_(torch.from_numpy(idx))
    buf.k_cnt.fill_(96)
    buf.sparse_attn()
    torch.cuda.synchronize()
    want = O.sparse_attn(w.Q[0], w.K[0], w.V[0], idx[0], w.Kc[0], w.Vc[0])
    assert P.max_abs(gen.from_torch(buf.out)[0], want) <= P.TOL_OUT["bf16"]


@pytest.mark.parametrize("d", [64, 128])
def test_scoring_topk_and_attention_at_the_longest_cache(d):
    """max_kv_len at its limit (2^24 - 1 tokens; with 128 dims a head's rows end 256 bytes short of 4 GiB): 32-bit row
    offsets, tile counts and histogram counts at their largest.  The cache is drawn on the device from a seeded
    generator (2 or 4 GiB; the host generator would need minutes); scores are checked against the oracle on sampled
    positions including both ends, the index set against the oracle's top-B of the very scores the kernel read, and
    the attention output (values = keys) against the oracle run on the gathered rows."""
    pk = _pk()
    dev = "cuda:0"
    T, C, B = (1 << 24) - 1, 40, 4099
    g = torch.Generator(device=dev).manual_seed(2024)
    k = torch.randn((1, 1, T, d), device=dev, generator=g).to(torch.bfloat16)
    q = torch.randn((1, 2, C, d), device=dev, generator=g).to(torch.bfloat16)
    kc = torch.randn((1, 1, C, d), device=dev, generator=g).to(torch.bfloat16)
    buf = pk.ChunkBuffers(q, k, k, kc, kc, [T], [B], n_retain=C)     # C <= N_Q: every query is kept
    buf.scores.fill_(float("nan"))
    buf.select_queries()
    buf.score_keys()
    buf.topk_keys()
    torch.cuda.synchronize()
    assert int(buf.k_cnt[0, 0]) == B
    Q = q[0].float().cpu().numpy().astype(np.float64)
    qbar = O.group_mean_queries(Q, O.select_queries(Q, C), 1)
    rng = np.random.default_rng(7)
    pos = np.unique(np.concatenate([np.arange(300), np.arange(T - 300, T), rng.integers(0, T, size=4000)]))
    pos_t = torch.from_numpy(pos).to(dev)
    Ks = k[0, :, pos_t].float().cpu().numpy().astype(np.float64)
    want = O.key_scores_preagg(qbar, Ks)
    got = buf.scores[0, :, pos_t].cpu().numpy()
    assert not np.isnan(got).any()
    assert P.max_abs(got, want) <= P.TOL_SCORE
    sc = buf.scores[0, :, :T].cpu().numpy()
    assert not np.isnan(sc).any()
    want_idx = O.topk_keys(sc.astype(np.float64), B)
    assert np.array_equal(buf.k_idx[0, :, :B].cpu().numpy(), want_idx)
    # the one-stage selection (provisional scores, exact re-scoring near the cut) must give the same list bit for bit;
    # at this length a scoring block works through more than 255 steps of one head (its 16-bit histogram counters are
    # flushed on the way) and the candidate list runs to thousands of entries over 8192 tiles
    staged_idx = buf.k_idx.clone()
    buf.k_idx.fill_(-1)
    buf.scores.fill_(float("nan"))
    buf.select_keys()
    torch.cuda.synchronize()
    assert int(buf.k_cnt[0, 0]) == B
    assert torch.equal(buf.k_idx[0, :, :B], staged_idx[0, :, :B])
    got2 = buf.scores[0, :, pos_t].cpu().numpy()
    qb32 = gen.from_torch(buf.qbar)[0, 0]
    delta = qb32.astype(np.float64) - gen.workloads.bf16_round(qb32).astype(np.float64)
    assert np.abs(got2 - want).max() <= float(np.sqrt((delta * delta).sum(axis=1)).max()) + 4e-6
    cut = np.sort(sc[0])[T - B]
    near = np.abs(want[0] - cut) <= 2.0 ** -11 - 1e-5
    if near.any():
        assert np.abs(got2[0][near] - want[0][near]).max() <= P.TOL_SCORE
    # attention over rows gathered from all over the cache: the oracle gets the gathered rows as its whole cache
    buf.out.fill_(float("nan"))
    buf.sparse_attn()
    torch.cuda.synchronize()
    idx_t = torch.from_numpy(want_idx[0]).to(dev)
    Kg = k[0, :, idx_t].float().cpu().numpy().astype(np.float64)
    Kc = kc[0].float().cpu().numpy().astype(np.float64)
    want_out = O.sparse_attn(Q, Kg, Kg, np.arange(B)[None], Kc, Kc)
    assert P.max_abs(gen.from_torch(buf.out)[0], want_out) <= P.TOL_OUT["bf16"]
