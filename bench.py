#!/usr/bin/env python3
"""Benchmark of libquoka's per-chunk sparse attention path on one MI355X.

One "step" = one pass of the whole hot path over one chunk: quoka_select_queries -> quoka_score_keys ->
quoka_topk_keys -> quoka_sparse_attn, inputs resident in HBM.  The default workload is config c2
(Llama-3-8B-shaped layer, 8192 cached tokens, chunk 1024, 64 retained queries, 12 % key budget).

Prints ONE JSON line: whole-path microseconds per chunk (`value`), the in-repo dense HIP baseline and the
speedup over it, per-stage times, a roofline object for the dominant kernel, and the CPU oracle timed on
the host cores as a reference baseline.

K/V caches are rotated over enough distinct copies (> 512 MiB in total) that the 256 MB last-level cache
cannot serve them: "HBM" numbers are HBM numbers.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the dominant kernel, from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE passes over
# `bench.py --profile-stage sparse_attn`, scaled by the same counters' reading for a 1 GiB device copy
# (profiles/hbm_traffic_c2.txt, hbm_traffic_c3_c5.txt, hbm_traffic_c4.txt: KiB read + KiB written).  None where it has not been
# measured.
MEASURED_TRAFFIC_BYTES = {"c2": (16449 + 8320) * 1024, "c3": (40596 + 16640) * 1024, "c4": (127638 + 33281) * 1024,
                          "c5": (244391 + 33280) * 1024}

HBM_PEAK_GBS = 8000.0
MFMA_BF16_PEAK_TFLOPS = 2500.0
FP32_VALU_PEAK_TFLOPS = 157.3


def _parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="c2", choices=["c1", "c2", "c3", "c4", "c5"])
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--rotate-mib", type=int, default=640, help="total MiB of distinct K/V copies to rotate over")
    ap.add_argument("--prefill-sweep", default=None, metavar="L1,L2,...",
                    help="instead of the chunk benchmark: whole-prompt chunked prefill (quoka_prefill_attn, one layer "
                         "of the c2 shape, chunk 1024, N_Q 64, budget 12 %% of the cache) at these prompt lengths, "
                         "sparse against dense; prints one JSON object")
    ap.add_argument("--budget-sweep", action="store_true",
                    help="instead of the chunk benchmark: the mixed-length batch c5 at N_Q in {32, 64, 128} x budget "
                         "in {4, 12, 25} %% of each sequence's cache, each against the dense kernel on the same batch "
                         "(the speed-up curve); prints one JSON object")
    ap.add_argument("--profile-stage", default=None,
                    choices=["select_queries", "score_keys", "topk_keys", "sparse_attn", "dense_attn", "copy"],
                    help="run only this stage --steps times (for rocprofv3 counter passes) and print a short JSON; "
                         "'copy' runs a plain device copy of known size, used to calibrate the HBM byte counters")
    return ap.parse_args()


def _algorithmic(w):
    """Algorithmic bytes / flops per chunk for each stage (what the method must move or compute)."""
    es = 2 if w.dtype == "bf16" else 4
    n_keep = min(w.n_retain, w.chunk)
    g = {"select_bytes": 0, "score_bytes": 0, "score_flops": 0, "topk_bytes": 0, "sparse_flops": 0, "dense_flops": 0,
         "sparse_bytes": 0}
    for T, B in zip(w.kv_lens, w.budgets):
        Bp = min(B, T)
        g["select_bytes"] += w.n_q * w.chunk * w.d * es + w.n_kv * n_keep * w.d * 4 + w.n_q * n_keep * 4
        g["score_bytes"] += w.n_kv * T * w.d * es + w.n_kv * T * 4
        g["score_flops"] += 2 * w.n_kv * n_keep * T * w.d
        g["topk_bytes"] += w.n_kv * T * 4 + w.n_kv * Bp * 4
        g["sparse_flops"] += 4 * w.d * w.n_q * w.chunk * (Bp + (w.chunk + 1) / 2)
        g["dense_flops"] += 4 * w.d * w.n_q * w.chunk * (T + (w.chunk + 1) / 2)
        g["sparse_bytes"] += 2 * w.n_q * w.chunk * w.d * es + 2 * w.n_kv * (Bp + w.chunk) * w.d * es
    return g


def _cpu_baseline(w):
    """The oracle as it stands, timed on the host cores on a bounded sample of the same workload."""
    import numpy as np
    from oracle import quoka_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        cores = os.cpu_count() or 1
    b = 0
    T = w.kv_lens[b]
    target_s = 10.0   # CPU work to spend on the sample

    def select():
        t0 = time.perf_counter()
        out = O.quoka_select(w.Q[b], w.K[b][:, :T], w.n_retain, w.budgets[b])
        return time.perf_counter() - t0, out

    def attend(k_idx, rows):
        t0 = time.perf_counter()
        O.sparse_attn(w.Q[b], w.K[b][:, :T], w.V[b][:, :T], k_idx, w.Kc[b], w.Vc[b], rows=rows)
        return time.perf_counter() - t0

    sel_s, (_, _, k_idx) = select()
    probe_rows = np.linspace(0, w.chunk - 1, min(w.chunk, 32)).astype(np.int64).tolist()
    per_row = attend(k_idx, probe_rows) / len(probe_rows)
    n_rows = int(min(w.chunk, max(32, (target_s - sel_s) / max(per_row, 1e-9))))
    rows = np.linspace(0, w.chunk - 1, n_rows).astype(np.int64).tolist()
    attn_s = attend(k_idx, rows)
    if n_rows < w.chunk and sel_s + attn_s < target_s / 2:   # the probe over-estimated the cost per row: one larger sample
        n_rows = int(min(w.chunk, n_rows * (target_s - sel_s) / max(attn_s, 1e-9)))
        rows = np.linspace(0, w.chunk - 1, n_rows).astype(np.int64).tolist()
        attn_s = attend(k_idx, rows)
    reps = 1
    if n_rows == w.chunk and sel_s + attn_s < target_s / 2:   # the whole chunk is cheap: repeat it
        reps = int(min(50, target_s / (sel_s + attn_s)))
        sel_t, attn_t = [sel_s], [attn_s]
        for _ in range(reps - 1):
            sel_t.append(select()[0])
            attn_t.append(attend(k_idx, rows))
        sel_s, attn_s = sum(sel_t) / reps, sum(attn_t) / reps
    total = (sel_s + attn_s * (w.chunk / n_rows)) * (w.batch if w.batch > 1 else 1)
    return {"value": total * 1e6, "unit": "us/chunk", "cores": int(cores), "kind": "oracle",
            "sample": (f"sequence 0 of {w.batch}: selection stages in full ({sel_s:.2f} s); attention on {n_rows} of "
                       f"{w.chunk} query rows x all heads ({attn_s:.2f} s)"
                       + (", scaled to all rows" if n_rows < w.chunk else "")
                       + (f"; mean of {reps} repetitions" if reps > 1 else "")
                       + ("; scaled by the batch size" if w.batch > 1 else ""))}


def _prefill_sweep(args, torch, pk, dev):
    """Whole-prompt attention time of one layer against the prompt length (the shape of the paper's
    speedup-versus-length plots, on synthetic activations)."""
    n_q, n_kv, d, chunk, n_retain = 32, 8, 128, 1024, 64
    rows = []
    for L in [int(x) for x in args.prefill_sweep.split(",")]:
        g = torch.Generator(device=dev).manual_seed(L)
        q = torch.randn(1, n_q, L, d, device=dev, generator=g).bfloat16()
        k = torch.randn(1, n_kv, L, d, device=dev, generator=g).bfloat16()
        v = torch.randn(1, n_kv, L, d, device=dev, generator=g).bfloat16()
        pb = pk.PrefillBuffers(q, k, v, chunk, n_retain, budget=lambda t: int(0.12 * t))
        res = {}
        for name, sparse in (("sparse", True), ("dense", False)):
            pb.run(sparse=sparse)
            torch.cuda.synchronize()
            reps = max(1, min(10, (1 << 17) // L))
            t0 = time.perf_counter()
            for _ in range(reps):
                pb.run(sparse=sparse)
            torch.cuda.synchronize()
            res[name] = (time.perf_counter() - t0) * 1e3 / reps
        rows.append({"prompt_len": L, "sparse_ms": res["sparse"], "dense_ms": res["dense"],
                     "speedup": res["dense"] / res["sparse"]})
        del pb, q, k, v
    print(json.dumps({"mode": "prefill_sweep", "layer": f"n_q={n_q} n_kv={n_kv} d={d} chunk={chunk} N_Q={n_retain} "
                      "budget=12% of the cache", "data": "synthetic", "rows": rows}))


def _budget_sweep(args, torch, gen, pk, dev):
    """Speed-up over the dense kernel against the key budget and the number of retained queries, on the batch of eight
    mixed-length sequences (workload c5).  The batch's data does not depend on the two knobs, so it is generated once."""
    w = gen.make_workload("c5")
    t = gen.to_torch(w, dev)
    K, W = max(10, args.steps // 4), max(3, args.warmup // 4)

    def timed(f):
        for _ in range(W):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(K):
            f()
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e6 / K

    dense = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain)
    dense_us = timed(dense.dense_attn)
    rows = []
    for n_retain in (32, 64, 128):
        for frac in (0.04, 0.12, 0.25):
            budgets = [int(frac * x) for x in w.kv_lens]
            bf = pk.ChunkBuffers(t["q"], t["k"], t["v"], t["kc"], t["vc"], w.kv_lens, budgets, n_retain)
            us = timed(bf.chunk_attn)
            rows.append({"n_retain": n_retain, "budget_frac": frac, "sparse_us": us, "speedup_vs_dense": dense_us / us})
            del bf
    print(json.dumps({"mode": "budget_sweep", "workload": f"c5: b={w.batch} n_q={w.n_q} n_kv={w.n_kv} d={w.d} "
                      f"T={w.kv_lens} C={w.chunk}", "data": "synthetic", "steps": K, "warmup": W,
                      "dense_us": dense_us, "rows": rows}))


def main():
    args = _parse()
    if args.gpus != 1:
        print("bench.py: this build is single-GPU by design (one MI355X per box); run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import gen
    import paper_2602_08722_amd as pk

    pk.load_library()
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    dev = "cuda:0"
    if args.prefill_sweep:
        _prefill_sweep(args, torch, pk, dev)
        return
    if args.budget_sweep:
        _budget_sweep(args, torch, gen, pk, dev)
        return
    w = gen.make_workload(args.workload)
    t = gen.to_torch(w, dev)
    es = 2 if w.dtype == "bf16" else 4
    copy_bytes = 2 * t["k"].numel() * es
    n_copies = max(1, -(-args.rotate_mib * (1 << 20) // copy_bytes))
    n_copies = min(n_copies, 64)
    bufs = []
    for i in range(n_copies):
        k = t["k"] if i == 0 else t["k"].clone()
        v = t["v"] if i == 0 else t["v"].clone()
        bufs.append(pk.ChunkBuffers(t["q"], k, v, t["kc"], t["vc"], w.kv_lens, w.budgets, w.n_retain))

    def step(i):
        bufs[i % n_copies].chunk_attn()

    def dense_step(i):
        bufs[i % n_copies].dense_attn()

    K, W = args.steps, args.warmup
    if args.profile_stage is not None:
        if args.profile_stage == "copy":
            n = 256 << 20   # 1 GiB of float32 read + 1 GiB written per copy
            src = torch.ones(n, dtype=torch.float32, device=dev)
            dst = torch.empty_like(src)
            for _ in range(K):
                dst.copy_(src)
            torch.cuda.synchronize()
            print(json.dumps({"profile_stage": "copy", "steps": K, "bytes_read_per_step": 4 * n,
                              "bytes_written_per_step": 4 * n}))
            return
        for i in range(n_copies):   # every buffer set gets valid intermediates
            step(i)
        torch.cuda.synchronize()
        for i in range(K):
            getattr(bufs[i % n_copies], args.profile_stage)()
        torch.cuda.synchronize()
        print(json.dumps({"profile_stage": args.profile_stage, "steps": K, "workload": w.name,
                          "algorithmic": _algorithmic(w)}))
        return
    for i in range(W):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(K):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / K

    # dense baseline, same protocol (fewer steps: it is several times slower)
    Kd = max(5, K // 5)
    for i in range(max(2, W // 5)):
        dense_step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(Kd):
        dense_step(i)
    torch.cuda.synchronize()
    dense_ms = (time.perf_counter() - t0) * 1e3 / Kd

    # second pass of the same K steps with HIP events around every stage (kept out of the headline timing,
    # since the event records themselves cost a few microseconds per step)
    stage_names = ["select_queries", "score_keys", "topk_keys", "sparse_attn"]
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(5)] for _ in range(K)]
    for i in range(K):
        bf = bufs[i % n_copies]
        ev[i][0].record()
        bf.select_queries()
        ev[i][1].record()
        bf.score_keys()
        ev[i][2].record()
        bf.topk_keys()
        ev[i][3].record()
        bf.sparse_attn()
        ev[i][4].record()
    torch.cuda.synchronize()
    stage_samples = {n: np.array([ev[i][j].elapsed_time(ev[i][j + 1]) for i in range(K)]) * 1e3
                     for j, n in enumerate(stage_names)}
    stage_us = {n: float(np.mean(x)) for n, x in stage_samples.items()}
    stage_pct = {n: [float(np.percentile(x, q)) for q in (10, 50, 90)] for n, x in stage_samples.items()}
    # average launch duration of the dominant kernel: K launches back to back between one pair of events
    # (a per-launch event pair would add its own few microseconds to a ~50 us kernel)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(K):
        bufs[i % n_copies].sparse_attn()
    e1.record()
    torch.cuda.synchronize()
    attn_kernel_us = e0.elapsed_time(e1) * 1e3 / K
    evd = [[torch.cuda.Event(enable_timing=True) for _ in range(2)] for _ in range(Kd)]
    for i in range(Kd):
        evd[i][0].record()
        dense_step(i)
        evd[i][1].record()
    torch.cuda.synchronize()
    dense_kernel_us = float(np.mean([a.elapsed_time(b) for a, b in evd])) * 1e3

    # measured-achievable memory rate beside the vendor peak: a plain device copy of 1 GiB (read + write)
    src = torch.ones(256 << 20, dtype=torch.float32, device=dev)
    dst = torch.empty_like(src)
    dst.copy_(src)
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(5):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    copy_gbs = 5 * 2 * src.numel() * 4 / (c0.elapsed_time(c1) * 1e-3) / 1e9
    del src, dst

    alg = _algorithmic(w)
    attn_us = attn_kernel_us
    sel_us = stage_us["score_keys"] + stage_us["topk_keys"]
    attn_tflops = alg["sparse_flops"] / (attn_us * 1e-6) / 1e12
    if w.dtype == "bf16":
        roofline = {"kernel": "attn_bf16 (quoka_sparse_attn)", "bound": "mfma", "achieved": attn_tflops,
                    "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / MFMA_BF16_PEAK_TFLOPS,
                    "traffic": MEASURED_TRAFFIC_BYTES.get(w.name), "algorithmic_bytes": alg["sparse_bytes"],
                    "algorithmic_flops": alg["sparse_flops"], "kernel_us": attn_us}
    else:
        roofline = {"kernel": "attn_f32 (quoka_sparse_attn)", "bound": "alu", "achieved": attn_tflops,
                    "peak": FP32_VALU_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": attn_tflops / FP32_VALU_PEAK_TFLOPS,
                    "traffic": None}
    score_gbs = alg["score_bytes"] / (stage_us["score_keys"] * 1e-6) / 1e9
    seltopk_gbs = (alg["score_bytes"] + alg["topk_bytes"]) / (sel_us * 1e-6) / 1e9
    dense_tflops = alg["dense_flops"] / (dense_kernel_us * 1e-6) / 1e12

    out = {
        "metric": "chunk_prefill_attention_us_per_chunk",
        "value": ms_per_step * 1e3,
        "unit": "us/chunk",
        "n_gpus": 1,
        "steps": K,
        "warmup": W,
        "ms_per_step": ms_per_step,
        "higher_is_better": False,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": w.dtype,
        "data": "synthetic",
        "config": {"workload": f"{w.name}: b={w.batch} n_q={w.n_q} n_kv={w.n_kv} d={w.d} T={w.kv_lens} C={w.chunk} "
                               f"N_Q={w.n_retain} B={w.budgets}",
                   "kv_copies_rotated": n_copies},
        "dense_us_per_chunk": dense_ms * 1e3,
        "speedup_vs_dense": dense_ms / ms_per_step,
        "stages_us": stage_us,
        "stages_us_p10_p50_p90": stage_pct,
        "dense_kernel_us": dense_kernel_us,
        "dense_mfma_frac": dense_tflops / MFMA_BF16_PEAK_TFLOPS if w.dtype == "bf16" else None,
        "score_keys_hbm_frac": score_gbs / HBM_PEAK_GBS,
        "score_topk_hbm_frac": seltopk_gbs / HBM_PEAK_GBS,
        "device_copy_gbs": copy_gbs,
        "score_keys_frac_of_device_copy": score_gbs / copy_gbs,
        "roofline": roofline,
        "paper_context": "paper reports up to 5x attention speedup on NVIDIA A100 and ~7x on Intel Xeon (other hardware)",
    }
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = _cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
