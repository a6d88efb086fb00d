#!/usr/bin/env python3
"""Turns rocprofv3 CSV output of bench.py runs into the short text summaries kept under profiles/.

    python3 profile_summary.py trace <workload> <rocprofv3 output dir> <bench.py stdout file>
    python3 profile_summary.py traffic <workload> <dir holding one rocprofv3 output dir per pass>
    python3 profile_summary.py counters <title> <kernel substring> <rocprofv3 output dir> [<dir> ...]

Each mode prints the summary to stdout, with the commands that produce its input.  The traffic summary carries
machine-readable lines (`TRAFFIC <stage> read_bytes=<n> write_bytes=<n>`) that bench.py reads back as
`roofline.traffic`, so the figure in a bench line always names the profile it came from.
"""
from __future__ import annotations

import collections
import csv
import glob
import json
import os
import re
import sys


def _find(d, pattern):
    hits = sorted(glob.glob(os.path.join(d, "**", pattern), recursive=True))
    if not hits:
        raise SystemExit(f"no {pattern} under {d}")
    return hits[0]


def _short(name):
    name = re.sub(r"\(.*", "", name).replace("void quoka::", "").replace("quoka::", "")
    return name.strip()


def _is_ours(name):
    return "quoka::" in name


def trace(workload, out_dir, bench_log):
    rows = list(csv.DictReader(open(_find(out_dir, "*kernel_trace.csv"))))
    dur = collections.defaultdict(list)
    for r in rows:
        if _is_ours(r["Kernel_Name"]):
            dur[_short(r["Kernel_Name"])].append((int(r["End_Timestamp"]) - int(r["Start_Timestamp"])) / 1e3)
    total = sum(sum(v) for v in dur.values())
    line = [l for l in open(bench_log) if l.startswith('{"metric"')][-1]
    j = json.loads(line)
    out = [f"# rocprofv3 kernel trace of bench.py, workload {workload}", "",
           "Command (run from /tmp with TMPDIR=/tmp, repository root = $R):",
           f"    rocprofv3 --kernel-trace --stats --output-format csv -d <out> -o kt -- python3 $R/bench.py --workload "
           f"{workload} --no-configs --no-cpu-baseline --steps {j['steps']} --warmup {j['warmup']} > <log>",
           f"    python3 $R/profile_summary.py trace {workload} <out> <log>", "",
           "Per-kernel durations over the whole run (warm-up, timed whole-path steps, dense baseline steps, the",
           "per-stage and back-to-back passes).  attn_bf16 serves the sparse path and the dense baseline: its launches are",
           "split below by duration.", "",
           f"{'kernel':54s} {'calls':>6s} {'avg_us':>9s} {'min_us':>9s} {'max_us':>9s} {'share%':>7s}"]
    for n, v in sorted(dur.items(), key=lambda kv: -sum(kv[1])):
        out.append(f"{n[:54]:54s} {len(v):6d} {sum(v) / len(v):9.2f} {min(v):9.2f} {max(v):9.2f} {100 * sum(v) / total:7.2f}")
    att = [v for n, v in dur.items() if n.startswith("attn_bf16")]
    if att:
        a = sorted(x for v in att for x in v)
        thr = (a[0] + a[-1]) / 2
        sp, de = [x for x in a if x < thr], [x for x in a if x >= thr]
        flops, dflops = j["roofline"]["algorithmic_flops"], None
        out += ["", f"attn_bf16 sparse launches: n={len(sp)} avg {sum(sp) / len(sp):.2f} us  ->  "
                    f"{flops / (sum(sp) / len(sp) * 1e-6) / 1e12 / 2500 * 100:.1f} % of 2.5 PFLOP/s "
                    f"({flops / 1e9:.1f} GF algorithmic)",
                f"attn_bf16 dense launches:  n={len(de)} avg {sum(de) / len(de):.2f} us"]
    sel = {n: sum(v) / len(v) for n, v in dur.items()}
    chain = [n for n in sel if n.startswith(("score_stream", "sel_band", "sel_emit", "score_bf16", "topk_"))]
    if chain:
        out += ["", "key scoring + top-B kernels (average launch durations): " +
                ", ".join(f"{n.split('<')[0]} {sel[n]:.1f}" for n in sorted(chain))]
        st = j["roofline_score_topk"]
        out += [f"algorithmic bytes of scoring + top-B: {st['algorithmic_bytes']} "
                f"({st['algorithmic_bytes'] / 2**20:.1f} MiB); bench.py timed the stage at {st['kernel_us']:.1f} us "
                f"-> {st['frac'] * 100:.1f} % of 8 TB/s"]
    keep = {k: j[k] for k in ("value", "unit", "dense_us_per_chunk", "speedup_vs_dense", "stages_us", "kernels_us")}
    out += ["", "bench.py line of the same run (under the profiler):", "    " + json.dumps(keep),
            "    roofline: " + json.dumps(j["roofline"]),
            "    roofline_score_topk: " + json.dumps(j["roofline_score_topk"]),
            "    probes: " + json.dumps(j["probes"])]
    print("\n".join(out))


def _pmc(out_dir):
    agg = collections.defaultdict(lambda: collections.defaultdict(list))
    for r in csv.DictReader(open(_find(out_dir, "*counter_collection.csv"))):
        agg[r["Kernel_Name"]][r["Counter_Name"]].append(float(r["Counter_Value"]))
    return agg


def _mean_tail(v, n=4):
    v = v[-n:]
    return sum(v) / len(v)


STAGE_KERNELS = {   # stage -> substrings of the kernels it launches
    "sparse_attn": ("attn_bf16", "attn_decode", "attn_f32"),
    "dense_attn": ("attn_bf16", "attn_decode", "attn_f32"),
    "select_keys": ("score_stream", "sel_", "score_bf16", "score_f32", "topk_"),
    "select_queries": ("sq_",),
}


def traffic(workload, base):
    """base/<stage>_<COUNTER>/ hold the rocprofv3 output of one pass each; base/copy_<COUNTER>/ the calibration."""
    cal = {}
    for c in ("FETCH_SIZE", "WRITE_SIZE"):
        a = _pmc(os.path.join(base, f"copy_{c}"))
        vals = [v[c] for k, v in a.items() if c in v and ("copy" in k.lower() or "elementwise" in k.lower())]
        cal[c] = _mean_tail(max(vals, key=len), 8)
    kib = 1048576.0   # the calibration copy reads 1 GiB and writes 1 GiB
    sf, sw = kib / cal["FETCH_SIZE"], kib / cal["WRITE_SIZE"]
    out = [f"# HBM traffic per launch (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE), workload {workload}", "",
           "Commands (one counter per run; run from /tmp with TMPDIR=/tmp, repository root = $R):",
           f"    rocprofv3 --pmc <FETCH_SIZE|WRITE_SIZE> --output-format csv -d <base>/<stage>_<counter> -o p -- python3 "
           f"$R/bench.py --workload {workload} --steps 6 --profile-stage <stage>",
           "    calibration: the same two runs with  --workload c1 --steps 10 --profile-stage copy  (1 GiB float32 device "
           "copy) into <base>/copy_<counter>",
           f"    python3 $R/profile_summary.py traffic {workload} <base>", "",
           f"Calibration: the copy kernel reads 1048576 KiB and writes 1048576 KiB; the counters read FETCH_SIZE = "
           f"{cal['FETCH_SIZE']:.1f}, WRITE_SIZE = {cal['WRITE_SIZE']:.1f}",
           f"  => FETCH_SIZE x {sf:.3f} and WRITE_SIZE x {sw:.3f} give KiB.", "",
           f"{'stage / kernel':52s} {'FETCH raw':>11s} {'WRITE raw':>11s} {'read MiB':>9s} {'write MiB':>9s}"]
    totals = {}
    for stage, pats in STAGE_KERNELS.items():
        fd, wd = os.path.join(base, f"{stage}_FETCH_SIZE"), os.path.join(base, f"{stage}_WRITE_SIZE")
        if not (os.path.isdir(fd) and os.path.isdir(wd)):
            continue
        fa, wa = _pmc(fd), _pmc(wd)
        rd_tot = wr_tot = 0.0
        for k in fa:
            if not (_is_ours(k) and any(p in k for p in pats)) or k not in wa:
                continue
            f, w = _mean_tail(fa[k]["FETCH_SIZE"]), _mean_tail(wa[k]["WRITE_SIZE"])
            rd, wr = f * sf / 1024, w * sw / 1024
            rd_tot += rd
            wr_tot += wr
            out.append(f"{(stage + ' / ' + _short(k))[:52]:52s} {f:11.1f} {w:11.1f} {rd:9.2f} {wr:9.2f}")
        totals[stage] = (rd_tot, wr_tot)
    out.append("")
    out.append("Per stage (sum over its kernels, one launch of each), as bench.py reads them back:")
    for stage, (rd, wr) in totals.items():
        out.append(f"TRAFFIC {stage} read_bytes={int(rd * 2**20)} write_bytes={int(wr * 2**20)}")
    out += ["", "WRITE_SIZE also counts write-backs of lines that an earlier kernel left dirty in L2, so small write figures",
            "are not attributable to one kernel."]
    print("\n".join(out))


def counters(title, kernel_sub, dirs):
    vals = {}
    launches = None
    for d in dirs:
        for k, v in _pmc(d).items():
            if kernel_sub in k:
                for c, x in v.items():
                    vals[c] = _mean_tail(x)
                    launches = len(x)
    out = [f"# {title}", "", f"Mean per launch of the kernels whose name contains '{kernel_sub}' (last 4 of {launches} "
           f"launches per pass).  Commands (one rocprofv3 --pmc pass per directory; from /tmp with TMPDIR=/tmp):"]
    for d in dirs:
        cmd = os.path.join(d, "command.txt")
        out.append("    " + (open(cmd).read().strip() if os.path.exists(cmd) else f"<pass in {os.path.basename(d)}>"))
    out.append(f"    python3 $R/profile_summary.py counters '{title}' {kernel_sub} <dir> ...")
    out.append("")
    for c in sorted(vals):
        out.append(f"    {c:30s} {vals[c]:.5g}")
    g = vals.get
    out.append("")
    if g("SQ_VALU_MFMA_BUSY_CYCLES") and g("GRBM_GUI_ACTIVE"):
        util = g("SQ_VALU_MFMA_BUSY_CYCLES") / (g("GRBM_GUI_ACTIVE") / 8 * 1024)
        out.append(f"matrix-core utilisation = SQ_VALU_MFMA_BUSY_CYCLES / (GRBM_GUI_ACTIVE / 8 XCDs x 1024 matrix cores) "
                   f"= {100 * util:.1f} % of the cycles at the clock the kernel ran at")
    if g("SQ_VALU_MFMA_BUSY_CYCLES") and g("SQ_INSTS_MFMA"):
        out.append(f"SQ_VALU_MFMA_BUSY_CYCLES / SQ_INSTS_MFMA = {g('SQ_VALU_MFMA_BUSY_CYCLES') / g('SQ_INSTS_MFMA'):.1f} "
                   f"matrix-core cycles per MFMA")
    if g("SQ_WAIT_ANY") and g("SQ_WAVE_CYCLES"):
        out.append(f"SQ_WAIT_ANY / SQ_WAVE_CYCLES = {g('SQ_WAIT_ANY') / g('SQ_WAVE_CYCLES'):.3f}")
    if g("SQ_LDS_BANK_CONFLICT") is not None and g("SQ_LDS_IDX_ACTIVE"):
        out.append(f"SQ_LDS_BANK_CONFLICT / SQ_LDS_IDX_ACTIVE = {g('SQ_LDS_BANK_CONFLICT') / g('SQ_LDS_IDX_ACTIVE'):.4f}")
    if g("FETCH_SIZE"):
        out.append(f"FETCH_SIZE (raw, units of the traffic summary's calibration) = {g('FETCH_SIZE'):.1f}")
    print("\n".join(out))


def main():
    if len(sys.argv) < 2:
        raise SystemExit(__doc__)
    mode = sys.argv[1]
    if mode == "trace" and len(sys.argv) == 5:
        trace(sys.argv[2], sys.argv[3], sys.argv[4])
    elif mode == "traffic" and len(sys.argv) == 4:
        traffic(sys.argv[2], sys.argv[3])
    elif mode == "counters" and len(sys.argv) >= 5:
        counters(sys.argv[2], sys.argv[3], sys.argv[4:])
    else:
        raise SystemExit(__doc__)


if __name__ == "__main__":
    main()
