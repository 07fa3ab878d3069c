#!/usr/bin/env python3
"""Scoring function f(x) in the paper's sense (section 3.1): a vector with one entry per benchmark
configuration, equal to the measured TFLOPS when the kernel's output is numerically correct against the
reference and to 0 otherwise; candidates are compared by the geometric mean, measured as the mean and
standard deviation of 10 runs (section 4.1), and a candidate is only "committed" when it is correct and at
least as good as the best so far (section 3.2).  Here the candidate is the built library, the reference is
the FP64 oracle on a stratified sample of rows, and the lineage is a JSON-lines file.

    python tests/score_f.py [--grid baseline|paper|tiny] [--runs 10] [--launches 20] [--lineage FILE]
"""
import argparse
import json
import math
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import oracle                                          # noqa: E402
import paper_2603_24517_amd as A                       # noqa: E402
from paper_2603_24517_amd import workloads as W        # noqa: E402

O_MAX_ABS, O_MEAN_ABS, LSE_REL = 2e-2, 2e-3, 1e-3


def score_one(w, runs, launches, nrows):
    dev = torch.device("cuda:0")
    q, k, v = W.make_qkv(w)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    o = torch.full_like(qd, float("nan"))
    lse = torch.full((w.B, w.Hq, w.Sq), float("nan"), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    def launch():
        rc = A.attn_fwd(qd, kd, vd, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, w.causal, w.scale, stream.cuda_stream)
        if rc != 0:
            raise A.AttnError(rc)

    launch()
    torch.cuda.synchronize()
    rows = W.sample_rows(w, nrows)
    o_ref, lse_ref = oracle.attn_ref_rows(q, k, v, rows, w.causal, w.scale)
    b, h, i = rows[:, 0], rows[:, 1], rows[:, 2]
    og = o[b, i, h].double().cpu().numpy()
    lg = lse[b, h, i].double().cpu().numpy()
    err = np.abs(og - o_ref)
    fin = np.isfinite(lse_ref)
    dl = np.abs(lg[fin] - lse_ref[fin]) / np.maximum(1.0, np.abs(lse_ref[fin]))
    correct = bool(not np.isnan(og).any() and np.array_equal(np.isfinite(lg), fin)
                   and err.max() <= O_MAX_ABS and err.mean() <= O_MEAN_ABS and (dl.size == 0 or dl.max() <= LSE_REL))
    tf = []
    for _ in range(5):
        launch()
    for _ in range(runs):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(launches):
            launch()
        e1.record(stream)
        torch.cuda.synchronize()
        tf.append(w.flops / (e0.elapsed_time(e1) / launches * 1e-3) * 1e-12)
    mean, std = float(np.mean(tf)), float(np.std(tf))
    return {"workload": w.name, "correct": correct, "f": mean if correct else 0.0, "tflops_mean": mean,
            "tflops_std": std, "o_max_abs": float(err.max()), "o_mean_abs": float(err.mean()),
            "lse_rel_max": float(dl.max()) if dl.size else 0.0, "rows_checked": int(len(rows))}


def geomean(xs):
    return 0.0 if any(x <= 0 for x in xs) else math.exp(sum(math.log(x) for x in xs) / len(xs))


def record_in_lineage(path, rec):
    """Append rec to the lineage file and decide, as section 3.2 has it, whether it is committed: only if
    every configuration is correct and its geometric mean is at least the best committed one on the
    same grid.  Returns (committed, best so far)."""
    best = 0.0
    if os.path.exists(path):
        for line in open(path):
            prev = json.loads(line)
            if prev.get("committed") and prev.get("grid") == rec["grid"]:
                best = max(best, prev["geomean"])
    rec["committed"] = bool(rec["all_correct"] and rec["geomean"] >= best)
    with open(path, "a") as f:
        f.write(json.dumps(rec) + "\n")
    return rec["committed"], best


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--grid", default="baseline", choices=["baseline", "paper", "tiny"])
    ap.add_argument("--runs", type=int, default=10)
    ap.add_argument("--launches", type=int, default=20)
    ap.add_argument("--rows", type=int, default=1024)
    ap.add_argument("--lineage", default=None, help="JSON-lines file holding one record per scored candidate")
    ap.add_argument("--label", default="candidate")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("score_f.py needs a GPU")
    if args.grid == "baseline":
        ws = list(W.WORKLOADS.values())
    elif args.grid == "paper":
        ws = list(W.PAPER_GRID.values())
    else:
        ws = [W.WORKLOADS[W.SMALL], W.custom("tiny_gqa_c", 2, 8, 2, 384, 384, causal=True, seed=5)]
    res = []
    for w in ws:
        r = score_one(w, args.runs, args.launches, args.rows)
        res.append(r)
        print(f"{r['workload']:34s} correct={r['correct']!s:5s} f={r['f']:8.1f} TFLOPS  "
              f"(mean {r['tflops_mean']:.1f} +- {r['tflops_std']:.1f}; O max {r['o_max_abs']:.2e} mean {r['o_mean_abs']:.2e}; "
              f"LSE {r['lse_rel_max']:.1e})", flush=True)
    g = geomean([r["f"] for r in res])
    rec = {"label": args.label, "time": time.time(), "grid": args.grid, "geomean": g,
           "all_correct": all(r["correct"] for r in res), "scores": res}
    verdict = "n/a (no lineage file)"
    if args.lineage:
        committed, best = record_in_lineage(args.lineage, rec)
        verdict = f"{'COMMIT' if committed else 'REJECT'} (best so far {best:.1f})"
    print(f"geomean f = {g:.1f} TFLOPS over {len(res)} configurations; all correct: {rec['all_correct']}; {verdict}")
    print(json.dumps({"geomean": g, "all_correct": rec["all_correct"], "n": len(res)}))


if __name__ == "__main__":
    main()
