"""End-to-end GPU parity: the four sparse stages back to back (quoka_chunk_attn) against the oracle,
at small sizes in full and at the full workload sizes on sampled rows."""
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


def _run(w, max_budget=None):
    pk = _pk()
    t = gen.to_torch(w, "cuda:0")
    mb = max_budget if max_budget is not None else min(max(w.budgets), w.t_max)
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain, max_budget=mb)
    buf.out.fill_(float("nan"))
    buf.chunk_attn()
    torch.cuda.synchronize()
    return buf


def _check_selection(w, buf, b):
    """Checks q_idx, scores and k_idx of sequence b against the oracle; returns the GPU's index lists."""
    T = w.kv_lens[b]
    n_keep = min(w.n_retain, w.chunk)
    q_idx = gen.from_torch(buf.q_idx[b])
    cos = O.cos_to_mean(w.Q[b])
    swaps = sum(P.check_query_ranking(q_idx[h], cos[h], n_keep, what=f"b{b} h{h}") for h in range(w.n_q))
    # scores against the oracle evaluated on the GPU's own retained queries (identical unless a tie swapped)
    want_scores = O.key_scores(w.Q[b], q_idx, w.K[b][:, :T], w.n_kv)
    got_scores = gen.from_torch(buf.scores[b])[:, :T]
    if P.two_pass_scores(w):
        # long bf16 caches: exact scores near the cut, provisional ones (within their proven bound) elsewhere; the
        # index sets below are held to the same bar as everywhere else
        qbar = gen.from_torch(buf.qbar[b])
        for kv in range(w.n_kv):
            P.check_two_pass_scores(got_scores[kv], want_scores[kv], qbar[kv], w.budgets[b], what=f"b{b} kv{kv}")
    else:
        assert P.max_abs(got_scores, want_scores) <= P.TOL_SCORE
    cnt = gen.from_torch(buf.k_cnt[b])
    k_idx = gen.from_torch(buf.k_idx[b])
    subs = 0
    sel = []
    for kv in range(w.n_kv):
        n = int(cnt[kv])
        assert n == min(w.budgets[b], T)
        subs += P.check_topk_set(k_idx[kv, :n], want_scores[kv], w.budgets[b], what=f"b{b} kv{kv}")
        sel.append(k_idx[kv, :n])
    return sel, swaps, subs


def test_config1_end_to_end_fp32():
    w = gen.make_workload("c1")
    buf = _run(w)
    sel, swaps, subs = _check_selection(w, buf, 0)
    assert swaps == 0 and subs == 0            # no ties in this seeded case: the sets are bit-exact
    q_idx_o, _, k_idx_o = O.quoka_select(w.Q[0], w.K[0], w.n_retain, w.budgets[0])
    assert np.array_equal(gen.from_torch(buf.q_idx[0]), q_idx_o)
    assert np.array_equal(np.stack(sel), k_idx_o)
    assert set(w.notes["heavy_key_pos"]) <= set(sel[0].tolist())
    want, want_lse = O.sparse_attn(w.Q[0], w.K[0], w.V[0], k_idx_o, w.Kc[0], w.Vc[0], return_lse=True)
    assert P.max_abs(gen.from_torch(buf.out[0]), want) <= P.TOL_OUT["f32"]
    assert P.max_abs(gen.from_torch(buf.lse[0]), want_lse) <= 1e-4


E2E_CASES = [
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=192, n_retain=48, kv_lens=[3000], budgets=[360]),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=100, n_retain=16, kv_lens=[777, 0, 2049, 130],
         budgets=[93, 10, 245, 400], batch=4),
    dict(dtype="bf16", n_q=4, n_kv=4, d=64, chunk=65, n_retain=65, kv_lens=[1000], budgets=[250]),
    dict(dtype="f32", n_q=4, n_kv=2, d=128, chunk=48, n_retain=8, kv_lens=[500, 33], budgets=[60, 20], batch=2),
    dict(dtype="bf16", n_q=16, n_kv=2, d=128, chunk=130, n_retain=128, kv_lens=[20000], budgets=[2400]),
    # decode-sized chunks: every query is retained (C <= N_Q), attention runs on the split-KV kernel
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=1, n_retain=16, kv_lens=[4000], budgets=[480]),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=4, n_retain=16, kv_lens=[2500, 0, 37], budgets=[300, 5, 37], batch=3),
]


@pytest.mark.parametrize("case", E2E_CASES, ids=lambda c: "-".join(f"{k}{v}" for k, v in c.items()))
def test_chunk_attn_end_to_end(case):
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, seed=21, **case)
    buf = _run(w)
    out = gen.from_torch(buf.out)
    for b in range(w.batch):
        T = w.kv_lens[b]
        sel, _, _ = _check_selection(w, buf, b)
        want = O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], sel, w.Kc[b], w.Vc[b])
        assert P.max_abs(out[b], want) <= P.TOL_OUT[w.dtype], f"b{b}: {P.max_abs(out[b], want)}"


def test_full_budget_reproduces_dense_and_runs_are_deterministic():
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=96, n_retain=16, kv_lens=[600, 300],
                        budgets=[600, 9999], batch=2, seed=22)
    buf = _run(w, max_budget=600)
    sparse_out = buf.out.clone()
    cnt = gen.from_torch(buf.k_cnt)
    assert cnt.tolist() == [[600, 600], [300, 300]]
    for b, T in enumerate(w.kv_lens):
        assert np.array_equal(gen.from_torch(buf.k_idx[b])[:, :T], np.tile(np.arange(T), (2, 1)))
    dense_out = torch.empty_like(buf.out)
    buf.dense_attn(out=dense_out)
    torch.cuda.synchronize()
    # same kernel, same key order, same arithmetic: identical bits
    assert torch.equal(sparse_out.view(torch.int16), dense_out.view(torch.int16))
    want = np.stack([O.dense_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], w.Kc[b], w.Vc[b])
                     for b, T in enumerate(w.kv_lens)])
    assert P.max_abs(gen.from_torch(dense_out), want) <= P.TOL_OUT["bf16"]
    # determinism: a second run gives identical indices and output bits
    k_idx1, q_idx1 = buf.k_idx.clone(), buf.q_idx.clone()
    buf.chunk_attn()
    torch.cuda.synchronize()
    assert torch.equal(buf.q_idx, q_idx1)
    for b, T in enumerate(w.kv_lens):
        assert torch.equal(buf.k_idx[b, :, :T], k_idx1[b, :, :T])
    assert torch.equal(buf.out.view(torch.int16), sparse_out.view(torch.int16))


def _sample_rows(C, n, seed):
    rng = np.random.default_rng(seed)
    fixed = {0, 31, 32, 63, 64, C - 1, C - 33 if C > 33 else 0}
    rows = set(int(r) for r in fixed if 0 <= r < C)
    while len(rows) < min(n, C):
        rows.add(int(rng.integers(0, C)))
    return sorted(rows)


def _full_size_check(w, n_rows, dense_heads, dense_rows):
    buf = _run(w)
    out = gen.from_torch(buf.out)
    total_subs = 0
    for b in range(w.batch):
        T = w.kv_lens[b]
        sel, swaps, subs = _check_selection(w, buf, b)
        total_subs += subs
        rows = _sample_rows(w.chunk, n_rows, seed=100 + b)
        want = O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], sel, w.Kc[b], w.Vc[b], rows=rows)
        err = P.max_abs(out[b][:, rows], want)
        assert err <= P.TOL_OUT[w.dtype], f"sparse b{b}: {err}"
    if not dense_heads:
        return total_subs
    # dense baseline on a few heads / rows
    dense_out = torch.empty_like(buf.out)
    buf.dense_attn(out=dense_out)
    torch.cuda.synchronize()
    dout = gen.from_torch(dense_out)
    for b in range(w.batch):
        T = w.kv_lens[b]
        rows = _sample_rows(w.chunk, dense_rows, seed=200 + b)
        want = O.dense_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], w.Kc[b], w.Vc[b], rows=rows, heads=dense_heads)
        err = P.max_abs(dout[b][dense_heads][:, rows], want)
        assert err <= P.TOL_OUT[w.dtype], f"dense b{b}: {err}"
    return total_subs


def test_config2_full_size():
    w = gen.make_workload("c2")
    _full_size_check(w, n_rows=128, dense_heads=[0, 13, 31], dense_rows=48)


def test_config3_full_size():
    w = gen.make_workload("c3")
    _full_size_check(w, n_rows=64, dense_heads=[5, 30], dense_rows=24)


def test_config4_full_size():
    w = gen.make_workload("c4")
    _full_size_check(w, n_rows=48, dense_heads=[17], dense_rows=16)


def test_launch_of_several_rounds_with_ragged_row_blocks():
    """Enough row blocks for more than two blocks per compute unit: the attention kernel then groups neighbouring row
    blocks and takes the longest causal ranges first.  188 row blocks per KV head do not fill the last block, one
    sequence has an empty cache and one a budget equal to its cache."""
    w = gen.make_custom(dtype="bf16", n_q=32, n_kv=8, d=64, chunk=1500, n_retain=64, kv_lens=[900, 0, 333],
                        budgets=[100, 10, 333], batch=3, seed=88)
    _full_size_check(w, n_rows=40, dense_heads=[3, 30], dense_rows=24)


def test_largest_chunk_largest_group():
    """The stated limits together: 8192 chunk tokens, 16 q-heads per KV head, 128 retained queries."""
    w = gen.make_custom(dtype="bf16", n_q=16, n_kv=1, d=64, chunk=8192, n_retain=128, kv_lens=[5000], budgets=[600],
                        seed=89)
    _full_size_check(w, n_rows=40, dense_heads=[0, 15], dense_rows=16)


@pytest.mark.parametrize("frac", [0.04, 0.12, 0.25])
@pytest.mark.parametrize("n_retain", [32, 64, 128])
def test_config5_ragged_batch(n_retain, frac):
    """All nine (N_Q, budget) points of the mixed-length batch: the three N_Q values take three variants of the scoring
    kernel and the budgets fall on both sides of the single-block / multi-block top-k boundary.  Selection stages are
    checked in full, attention on sampled rows; the dense baseline (the same for all points) on the diagonal only."""
    w = gen.make_workload("c5", n_retain=n_retain, budget_frac=frac)
    diag = (n_retain, frac) in ((32, 0.04), (64, 0.12), (128, 0.25))
    _full_size_check(w, n_rows=24, dense_heads=[9] if diag else [], dense_rows=8)


def test_config5_full_budget_is_the_dense_baseline():
    """Budget 100 % on the mixed-length batch (the last point of the speed-up curve): every cache position is selected,
    in order, so the sparse path runs the dense kernel's arithmetic on the same key order -- identical output bits --
    and both agree with the oracle's dense attention."""
    w = gen.make_workload("c5", n_retain=64, budget_frac=1.0)
    assert w.budgets == w.kv_lens
    buf = _run(w)
    cnt = gen.from_torch(buf.k_cnt)
    for b, T in enumerate(w.kv_lens):
        assert cnt[b].tolist() == [T] * w.n_kv
        assert torch.equal(buf.k_idx[b, :, :T], torch.arange(T, dtype=torch.int32, device="cuda:0").expand(w.n_kv, T))
    sparse_out = buf.out.clone()
    dense_out = torch.empty_like(buf.out)
    buf.dense_attn(out=dense_out)
    torch.cuda.synchronize()
    assert torch.equal(sparse_out.view(torch.int16), dense_out.view(torch.int16))
    out = gen.from_torch(sparse_out)
    for b, T in enumerate(w.kv_lens):
        rows = _sample_rows(w.chunk, 8, seed=300 + b)
        heads = [b % w.n_q, (5 * b + 17) % w.n_q]
        want = O.dense_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], w.Kc[b], w.Vc[b], rows=rows, heads=heads)
        err = P.max_abs(out[b][heads][:, rows], want)
        assert err <= P.TOL_OUT["bf16"], f"b{b}: {err}"


@pytest.mark.parametrize("case", [
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=200, n_retain=32, kv_lens=[1500, 700], budgets=[180, 90], batch=2),
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=3, n_retain=16, kv_lens=[2100], budgets=[260]),      # decode path
    dict(dtype="bf16", n_q=4, n_kv=4, d=64, chunk=96, n_retain=16, kv_lens=[40000], budgets=[512]),     # multi-block top-k
    dict(dtype="f32", n_q=4, n_kv=2, d=64, chunk=64, n_retain=16, kv_lens=[300], budgets=[40]),
], ids=["prefill", "decode", "long", "f32"])
def test_token_major_layout_gives_the_same_result(case):
    """Caches are often stored token-major ([b, tokens, heads, d]).  The ABI takes strides, so such tensors are passed
    as they are; every stage must produce exactly what it produces for the head-major copy of the same values."""
    import paper_2602_08722_amd as pk
    pk.load_library()
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, seed=23, **case)
    t = gen.to_torch(w, "cuda:0")
    tm = {k: v.permute(0, 2, 1, 3).contiguous().permute(0, 2, 1, 3) for k, v in t.items() if k in ("q", "k", "v", "kc", "vc")}
    assert tm["k"].stride() != t["k"].stride() or w.n_kv == 1
    a = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain)
    b = pk.ChunkBuffers(tm["q"], tm["k"], tm["v"], tm["kc"], tm["vc"], w.kv_lens, w.budgets, w.n_retain)
    assert b.out.stride() == tm["q"].stride()          # the output takes the layout of Q
    for buf in (a, b):
        buf.out.zero_()
        buf.chunk_attn()
    torch.cuda.synchronize()
    assert torch.equal(a.q_idx, b.q_idx)
    assert torch.equal(a.qbar, b.qbar)
    assert torch.equal(a.k_cnt, b.k_cnt)
    for bi in range(w.batch):
        n = int(a.k_cnt[bi, 0])
        assert torch.equal(a.k_idx[bi, :, :n], b.k_idx[bi, :, :n])
        T = w.kv_lens[bi]
        assert torch.equal(a.scores[bi, :, :T], b.scores[bi, :, :T])
    assert torch.equal(a.out, b.out)
    a.dense_attn()
    b.dense_attn()
    torch.cuda.synchronize()
    assert torch.equal(a.out, b.out)


def _random_case(rnd, it):
    """A small random problem: odd head counts, ragged sizes around the tile edges, empty and tiny caches."""
    dtype = rnd.choice(["bf16", "bf16", "bf16", "f32"])
    d = rnd.choice([64, 128])
    n_kv = rnd.choice([1, 2, 3, 4])
    g = rnd.choice([1, 2, 4, 8, 16]) if dtype == "bf16" else rnd.choice([1, 2])
    batch = rnd.choice([1, 1, 2, 3])
    chunk = rnd.choice([1, 2, 7, 16, 33, 64, 100, 129, 200, 257, 300])
    n_retain = rnd.choice([1, 5, 16, 31, 32, 33, 64, 100, 128])
    kv_lens = [rnd.choice([0, 1, 17, 63, 64, 65, 127, 128, 129, 500, 1000, 2049, 4097, 33000]) for _ in range(batch)]
    budgets = [max(1, rnd.choice([1, t // 10 + 1, t // 3 + 1, t, t + 5])) for t in kv_lens]
    if dtype == "f32":   # the float32 kernels are plain: keep their cases small
        chunk = min(chunk, 100)
        kv_lens = [min(t, 600) for t in kv_lens]
        budgets = [min(b, 700) for b in budgets]
    return dict(dtype=dtype, n_q=n_kv * g, n_kv=n_kv, d=d, chunk=chunk, n_retain=n_retain, kv_lens=kv_lens,
                budgets=budgets, batch=batch, seed=2000 + it)


@pytest.mark.parametrize("sweep", [0, 1, 2])
def test_random_small_shapes(sweep):
    """Seeded sweep over shapes nobody would pick by hand; every stage and both attention paths against the oracle."""
    import random
    rnd = random.Random(100 + sweep)
    for it in range(10):
        case = _random_case(rnd, 10 * sweep + it)
        w = gen.make_custom(**case)
        buf = _run(w)
        out = gen.from_torch(buf.out)
        for b in range(w.batch):
            sel, _, _ = _check_selection(w, buf, b)
            T = w.kv_lens[b]
            idx = np.stack(sel) if len(sel[0]) > 0 else np.zeros((w.n_kv, 0), dtype=np.int64)
            want = O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], idx, w.Kc[b], w.Vc[b])
            assert P.max_abs(out[b], want) <= P.TOL_OUT[w.dtype], f"{case} b{b}"
        buf.out.fill_(float("nan"))
        buf.dense_attn()
        torch.cuda.synchronize()
        out = gen.from_torch(buf.out)
        for b in range(w.batch):
            T = w.kv_lens[b]
            want = O.dense_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], w.Kc[b], w.Vc[b])
            assert P.max_abs(out[b], want) <= P.TOL_OUT[w.dtype], f"dense {case} b{b}"


@pytest.mark.parametrize("case", [
    dict(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=64, n_retain=32, kv_lens=[40000, 35000], budgets=[4000, 100], batch=2),
    dict(dtype="bf16", n_q=4, n_kv=2, d=128, chunk=96, n_retain=16, kv_lens=[3000], budgets=[300]),
    dict(dtype="f32", n_q=2, n_kv=1, d=64, chunk=32, n_retain=8, kv_lens=[33000], budgets=[64]),
], ids=["multi-block-topk", "single-block-topk", "f32-multi-block"])
def test_fused_call_equals_the_stage_calls_on_a_dirty_workspace(case):
    """quoka_chunk_attn shares work between stages (the scoring launch clears the top-k histograms).  With the
    workspace filled with garbage before each run, it must give exactly what the four stage calls give."""
    pk = _pk()
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(batch=batch, seed=51, **case)
    t = gen.to_torch(w, "cuda:0")
    res = []
    for fused in (False, True, True):
        buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain)
        buf.workspace.fill_(0xA5)
        buf.k_idx.fill_(-1)
        buf.out.zero_()
        if fused:
            buf.chunk_attn()
        else:
            buf.select_queries()
            buf.score_keys()
            buf.topk_keys()
            buf.sparse_attn()
        torch.cuda.synchronize()
        res.append((buf.q_idx.clone(), buf.qbar.clone(), buf.k_cnt.clone(), buf.k_idx.clone(), buf.out.clone()))
    for other in res[1:]:
        for a, b in zip(res[0], other):
            assert torch.equal(a.view(torch.uint8) if a.dtype == torch.bfloat16 else a,
                               b.view(torch.uint8) if b.dtype == torch.bfloat16 else b)
