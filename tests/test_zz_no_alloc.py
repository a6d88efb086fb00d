"""quoka_topk_keys_noalloc (library-owned scratch array instead of a caller workspace) against quoka_topk_keys.

Two calls in a row through the C ABI, the second on a smaller problem, so that the second call finds the first one's
contents in the array: both must give exactly what the workspace-taking entry point gives.  Integer work: bit-exact.
"""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu


def _pk():
    import paper_2602_08722_amd as pk
    pk.load_library()
    return pk


def _problem(pk, batch, n_kv, t_max, kv_lens, budgets, seed):
    dev = "cuda:0"
    g = torch.Generator(device="cpu").manual_seed(seed)
    scores = (torch.randn(batch, n_kv, t_max, generator=g) * 0.05).to(dev)
    # planted ties around the cut and a constant stretch: the tie rule (lower position first) is exercised too
    scores[:, :, 1000:1400] = 0.0625
    scores[:, :, ::977] = scores[:, :, 5:6]
    # the top-k reads neither queries nor the cache: the shape is filled in by hand (contiguous strides), no tensors
    max_budget = min(max(budgets), t_max)
    shape = pk.QuokaShape()
    shape.batch, shape.n_q_heads, shape.n_kv_heads, shape.head_dim = batch, n_kv, n_kv, 64
    shape.chunk_len, shape.max_kv_len, shape.n_retain, shape.max_budget = 8, t_max, 8, max_budget
    shape.dtype, shape.score_flags = pk.QUOKA_BF16, 0
    for name, tokens in (("q_stride", 8), ("kv_stride", t_max), ("ck_stride", 8), ("o_stride", 8)):
        getattr(shape, name)[:] = [n_kv * tokens * 64, tokens * 64, 64]
    lens = torch.tensor(kv_lens, dtype=torch.int32, device=dev)
    buds = torch.tensor(budgets, dtype=torch.int32, device=dev)
    return shape, scores, lens, buds, max_budget


def _run_both(pk, batch, n_kv, t_max, kv_lens, budgets, seed):
    dev = "cuda:0"
    shape, scores, lens, buds, mb = _problem(pk, batch, n_kv, t_max, kv_lens, budgets, seed)
    ws = torch.full((pk.quoka_workspace_bytes(shape),), 0x5A, dtype=torch.uint8, device=dev)
    ref_idx = torch.full((batch, n_kv, mb), -1, dtype=torch.int32, device=dev)
    ref_cnt = torch.full((batch, n_kv), -1, dtype=torch.int32, device=dev)
    pk.quoka_topk_keys(shape, scores, lens, buds, ref_idx, ref_cnt, ws)
    got_idx = torch.full_like(ref_idx, -1)
    got_cnt = torch.full_like(ref_cnt, -1)
    pk.quoka_topk_keys_noalloc(shape, scores, lens, buds, got_idx, got_cnt)
    torch.cuda.synchronize()
    assert torch.equal(got_cnt, ref_cnt)
    for b in range(batch):
        n = int(ref_cnt[b, 0])
        assert n == min(budgets[b], kv_lens[b], mb)
        assert torch.equal(got_idx[b, :, :n], ref_idx[b, :, :n]), f"sequence {b}"
    # and the reference itself is the stable top-B (ties to the lower position), ascending
    sc = scores.cpu().numpy()
    for b in range(batch):
        T, n = kv_lens[b], int(ref_cnt[b, 0])
        for kv in range(n_kv):
            want = np.sort(np.argsort(-sc[b, kv, :T], kind="stable")[:n])
            assert np.array_equal(got_idx[b, kv, :n].cpu().numpy(), want)


def test_noalloc_topk_matches_the_workspace_entry_point_twice_in_a_row():
    pk = _pk()
    # both problems take the multi-block path (more than 32768 positions), the one that uses the scratch array
    _run_both(pk, batch=2, n_kv=4, t_max=100_000, kv_lens=[100_000, 41_234], budgets=[9_000, 50_000], seed=1)
    _run_both(pk, batch=1, n_kv=2, t_max=40_000, kv_lens=[39_999], budgets=[1_234], seed=2)
    # a short cache (single-block path, no scratch use) still goes through the same entry point
    _run_both(pk, batch=3, n_kv=2, t_max=3_000, kv_lens=[3_000, 0, 17], budgets=[100, 5, 40], seed=3)


def test_noalloc_topk_rejects_what_the_array_cannot_hold():
    pk = _pk()
    # 1200 KV-head slices need 1200 * (6152 + 2 * 17) * 4 bytes = 28 MiB of histograms and counts: more than the array
    shape, scores, lens, buds, mb = _problem(pk, batch=150, n_kv=8, t_max=33_000, kv_lens=[33_000] * 150,
                                             budgets=[64] * 150, seed=4)
    idx = torch.empty((150, 8, mb), dtype=torch.int32, device="cuda:0")
    cnt = torch.empty((150, 8), dtype=torch.int32, device="cuda:0")
    with pytest.raises(pk.QuokaError) as e:
        pk.quoka_topk_keys_noalloc(shape, scores, lens, buds, idx, cnt)
    assert e.value.status == 3   # QUOKA_EWORKSPACE
