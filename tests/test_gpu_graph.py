"""The library's entry points under HIP graph capture: they allocate nothing, clear nothing with memset nodes and never
synchronise, so a caller may record them once and replay them.  Each replay (on fresh input values, with ordinary eager
work and synchronisations between the replays) must reproduce the eager result bit for bit."""
import numpy as np
import pytest
import torch

import gen

pytestmark = pytest.mark.gpu


def _eager_noise(dev):
    # unrelated eager work between replays (allocations, a reduction, a sync), as a real program would have
    x = torch.randn(1 << 16, device=dev)
    y = (x * 2 + 1).sum()
    torch.cuda.synchronize()
    return float(y)


@pytest.mark.parametrize("case", [
    dict(n_q=8, n_kv=2, d=128, chunk=256, n_retain=64, kv_lens=[3000], budgets=[360]),          # single-block top-k
    dict(n_q=8, n_kv=2, d=128, chunk=128, n_retain=32, kv_lens=[40000, 33000], budgets=[4000, 10], batch=2),  # multi-block top-k
    dict(n_q=8, n_kv=2, d=128, chunk=4, n_retain=16, kv_lens=[5000], budgets=[600]),             # decode-sized chunk
], ids=["small", "multiblock-topk", "decode"])
def test_chunk_attn_replays_from_a_graph(case):
    import paper_2602_08722_amd as pk
    pk.load_library()
    case = dict(case)
    batch = case.pop("batch", 1)
    w = gen.make_custom(dtype="bf16", batch=batch, seed=41, **case)
    t = gen.to_torch(w, "cuda:0")
    buf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        buf.chunk_attn()          # first call outside the capture (module load, lazy initialisation)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        buf.chunk_attn()
    torch.cuda.synchronize()
    gen_t = torch.Generator(device="cuda:0").manual_seed(5)
    for rep in range(3):
        # new query values in the same buffers: the graph must read what is there at replay time
        buf.q.copy_(torch.randn(buf.q.shape, device="cuda:0", generator=gen_t).to(buf.q.dtype))
        buf.out.zero_()
        buf.k_idx.fill_(-1)
        graph.replay()
        torch.cuda.synchronize()
        got_out, got_idx, got_cnt = buf.out.clone(), buf.k_idx.clone(), buf.k_cnt.clone()
        _eager_noise("cuda:0")
        buf.out.zero_()
        buf.k_idx.fill_(-1)
        buf.chunk_attn()
        torch.cuda.synchronize()
        assert torch.equal(got_cnt, buf.k_cnt), f"replay {rep}"
        assert torch.equal(got_idx, buf.k_idx), f"replay {rep}"
        assert torch.equal(got_out.view(torch.int16), buf.out.view(torch.int16)), f"replay {rep}"


def test_whole_prefill_replays_from_a_graph():
    """Alg. 2's loop (here 5 chunks, the last one short) recorded as one graph."""
    import paper_2602_08722_amd as pk
    pk.load_library()
    L, chunk = 1100, 256
    w = gen.make_custom(dtype="bf16", n_q=8, n_kv=2, d=128, chunk=L, n_retain=1, kv_lens=[0], budgets=[0], batch=1,
                        seed=42)
    dev = "cuda:0"
    to = lambda x: torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16).to(dev)
    q, k, v = to(w.Q), to(w.Kc), to(w.Vc)
    pb = pk.PrefillBuffers(q, k, v, chunk, n_retain=32, budget=150)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        pb.run(sparse=True)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        pb.run(sparse=True)
    torch.cuda.synchronize()
    gen_t = torch.Generator(device=dev).manual_seed(6)
    for rep in range(3):
        pb.k.copy_(torch.randn(pb.k.shape, device=dev, generator=gen_t).to(pb.k.dtype))
        pb.out.zero_()
        graph.replay()
        torch.cuda.synchronize()
        got = pb.out.clone()
        _eager_noise(dev)
        pb.out.zero_()
        pb.run(sparse=True)
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), pb.out.view(torch.int16)), f"replay {rep}"
