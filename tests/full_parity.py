"""Every-row parity of one benchmark workload: O and LSE of the HIP path against the FP64 oracle.

The parity tests check the large workloads on a stratified sample of rows; this script checks ALL
rows (or one contiguous part of them, so that a long workload can be split over several runs), in
the launch configuration bench.py times.  It prints a progress line per chunk and one JSON line at
the end, and exits non-zero if a bar is missed.

    python tests/full_parity.py --workload cfg2_mha_nc_b8_h16_s4096 [--part 0/3] [--out result.json]
"""
import argparse
import json
import os
import sys
import time

import numpy as np

sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))

import gpu_util as U                                    # noqa: E402
import oracle                                           # noqa: E402
from paper_2603_24517_amd import workloads as W         # noqa: E402


def check_every_row(name, part=0, nparts=1, chunk=8192, log=print):
    """Run workload `name` on the GPU and compare rows [part/nparts slice] of O and LSE with the oracle.

    Returns the error figures and `pass`; raises only on NaN or a differing -inf pattern."""
    w = {**W.WORKLOADS, **W.PAPER_GRID}[name]
    assert 0 <= part < nparts
    t0 = time.monotonic()
    q, k, v = W.make_qkv(w)
    o_gpu, lse_gpu = U.run_gpu(q, k, v, w.causal, w.scale)
    qd, kd, vd = (x.double().numpy() for x in (q, k, v))
    del q, k, v
    total = w.B * w.Hq * w.Sq
    lo, hi = total * part // nparts, total * (part + 1) // nparts
    log(f"{w.name}: rows {lo}..{hi} of {total}, oracle threads {oracle.threads()}, "
        f"set-up {time.monotonic() - t0:.1f} s")

    max_abs, sum_abs, n_el, lse_max, lse_ratio, n_inf = 0.0, 0.0, 0, 0.0, 0.0, 0
    t1 = time.monotonic()
    for c0 in range(lo, hi, chunk):
        idx = np.arange(c0, min(c0 + chunk, hi), dtype=np.int64)
        b, rem = np.divmod(idx, w.Hq * w.Sq)
        h, i = np.divmod(rem, w.Sq)
        rows = np.stack([b, h, i], axis=1).astype(np.int32)
        o_ref, lse_ref = oracle.attn_ref_rows(qd, kd, vd, rows, w.causal, w.scale)
        og, lg = o_gpu[b, i, h], lse_gpu[b, h, i]
        assert not np.isnan(og).any() and not np.isnan(lg).any(), "NaN in the HIP path's output"
        err = np.abs(og - o_ref)
        max_abs = max(max_abs, float(err.max()))
        sum_abs += float(err.sum())
        n_el += err.size
        fin = np.isfinite(lse_ref)
        assert np.array_equal(np.isfinite(lg), fin), "-inf pattern of LSE differs"
        n_inf += int((~fin).sum())
        if fin.any():
            dl = np.abs(lg[fin] - lse_ref[fin])
            lse_max = max(lse_max, float(dl.max()))
            lse_ratio = max(lse_ratio, float((dl / (U.LSE_REL * np.maximum(1.0, np.abs(lse_ref[fin])))).max()))
        done = idx[-1] + 1 - lo
        log(f"  {done}/{hi - lo} rows, {time.monotonic() - t1:.0f} s, max_abs {max_abs:.3e}, "
            f"mean_abs {sum_abs / n_el:.3e}, lse {lse_max:.3e}")

    res = dict(workload=w.name, part=f"{part}/{nparts}", rows=hi - lo, rows_total=total, max_abs=max_abs,
               mean_abs=sum_abs / max(n_el, 1), lse_max_abs=lse_max, lse_worst_ratio=lse_ratio,
               rows_without_keys=n_inf, oracle_seconds=round(time.monotonic() - t1, 1),
               bars=dict(max_abs=U.O_MAX_ABS, mean_abs=U.O_MEAN_ABS, lse_rel=U.LSE_REL))
    res["pass"] = bool(max_abs <= U.O_MAX_ABS and res["mean_abs"] <= U.O_MEAN_ABS and lse_ratio <= 1.0)
    ceiling = U.CEILINGS.get(w.name)
    if ceiling is not None:             # the regression ceiling of the workload, where it has one
        res["ceiling"] = dict(max_abs=ceiling[0], mean_abs=ceiling[1])
        res["pass"] = bool(res["pass"] and max_abs <= ceiling[0] and res["mean_abs"] <= ceiling[1])
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--workload", required=True)
    ap.add_argument("--part", default="0/1", help="k/n: the k-th of n contiguous slices of the (b, h, i) rows")
    ap.add_argument("--chunk", type=int, default=8192)
    ap.add_argument("--out", default=None)
    a = ap.parse_args()
    part, nparts = (int(x) for x in a.part.split("/"))
    res = check_every_row(a.workload, part, nparts, a.chunk, log=lambda m: print(m, flush=True))
    line = json.dumps(res)
    print(line, flush=True)
    if a.out:
        with open(a.out, "a") as f:
            f.write(line + "\n")
    return 0 if res["pass"] else 1


if __name__ == "__main__":
    sys.exit(main())
