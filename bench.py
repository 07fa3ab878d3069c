#!/usr/bin/env python3
"""Benchmark of the fused attention forward on one MI355X.

A "step" is one pass of the whole hot path (one attn_fwd launch) over one batch of seeded
synthetic input that is already resident in HBM.  Metric: forward TFLOPS counted as
4*B*Hq*Sq*Skv*D (halved for causal), and the fraction of the dense BF16 MFMA peak.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--all]

Prints ONE JSON line (with --all: one line per workload, the headline workload last).
"""
import argparse
import json
import os
import sys
import time

import numpy as np
import torch

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import paper_2603_24517_amd as A                       # noqa: E402
from paper_2603_24517_amd import workloads as W        # noqa: E402

PEAK_BF16_TFLOPS = 2516.6      # MI355X dense BF16 MFMA: 256 CU x 4 SIMD x 1024 FLOP/clk x 2.4 GHz
METRIC = "attention fwd TFLOPS (BF16, D=128) and % of MI355X dense BF16 MFMA peak"


def mfma_probe():
    """What the matrix pipe sustains on this board, and at which shader clock (context for `frac`).

    A bare loop of v_mfma_f32_32x32x16_bf16 on register operands at 1, 2 and 4 wavefronts per SIMD, for
    all-zero and for N(0,1) BF16 operands; then, at the attention kernel's 2 wavefronts per SIMD and with
    N(0,1) operands, the same loop with the work that accompanies every MFMA in the attention kernel added
    step by step: the softmax's vector instructions, the LDS read of one operand, the tile requests.  The
    last of these is the ceiling of THIS instruction mix with a matrix pipe that never waits."""
    from paper_2603_24517_amd import probe as P
    dev = torch.device("cuda:0")
    stream = torch.cuda.current_stream()
    sink = torch.zeros(1, dtype=torch.float32, device=dev)
    clocks = torch.zeros(4, dtype=torch.int64, device=dev)
    g = torch.Generator().manual_seed(7)
    # 4 MiB of N(0,1) BF16 for the tile requests: like the attention kernel's K/V tiles, mostly served by L2
    tiles = torch.randn(1 << 21, generator=g).to(torch.bfloat16).to(dev)
    data = {"zeros": torch.zeros(12, 64, 8), "normal_0_1": torch.randn(12, 64, 8, generator=g)}

    def run(ops, mode, waves):
        iters = 4000 // waves
        for _ in range(2):
            rc = P.attn_probe_mfma(ops, tiles, tiles.numel() * 2, sink, clocks, mode, waves, iters, stream.cuda_stream)
            if rc != 0:
                raise RuntimeError(f"attn_probe_mfma failed ({rc})")
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(stream)
        for _ in range(5):
            P.attn_probe_mfma(ops, tiles, tiles.numel() * 2, sink, clocks, mode, waves, iters, stream.cuda_stream)
        e1.record(stream)
        torch.cuda.synchronize()
        c = clocks.cpu().numpy()
        cycles, ticks = int(c[1] - c[0]), int(c[3] - c[2])
        return {"tflops": P.probe_flops(waves, iters) * 5 / (e0.elapsed_time(e1) * 1e-3) * 1e-12,
                "clock_ghz": 0.1 * cycles / ticks, "cycles_per_mfma_per_simd": cycles / (32.0 * iters * waves)}

    out = {"unit": "TFLOP/s", "what": "v_mfma_f32_32x32x16_bf16 loop, register operands, 256 workgroups; "
                                      "wN = N wavefronts per SIMD; clock = shader cycle counter / 100 MHz counter in the launch"}
    for name, ops in data.items():
        ops = ops.to(torch.bfloat16).to(dev)
        out[name] = {f"w{w}": run(ops, 0, w) for w in (1, 2, 4)}
        if name == "normal_0_1":
            out[name]["w2_valu"] = run(ops, P.PROBE_VALU, 2)
            out[name]["w2_valu_lds"] = run(ops, P.PROBE_VALU | P.PROBE_LDS, 2)
            out[name]["w2_valu_lds_dma"] = run(ops, P.PROBE_VALU | P.PROBE_LDS | P.PROBE_DMA, 2)
    out["ceiling"] = dict(out["normal_0_1"]["w2_valu_lds_dma"],
                          what="N(0,1) operands, 2 wavefronts per SIMD, every MFMA accompanied by the attention kernel's "
                               "vector instructions per score, LDS operand read and share of the tile requests; "
                               "matrix pipe never idle")
    return out


def kernel_name(w, compute_units):
    """Which of the library's two kernels a launch of this workload runs (the rule of include/attn.h: the
    split-key kernel when the 256-row work items would occupy at most a quarter of the compute units)."""
    g = w.Hq // w.Hkv
    pack = 8 if g % 8 == 0 else 4 if g % 4 == 0 else 2 if g % 2 == 0 else 1
    items = w.B * w.Hkv * (g // pack) * -(-w.Sq // (256 // pack))
    return "attn_fwd_split_kernel" if items * 4 <= compute_units else "attn_fwd_kernel"


def kernel_clock(w, qd, kd, vd, o, lse, launches=40):
    """Shader clock and cycle count of the attention kernel on this workload: the build of the shipped kernel
    with clock stamps (variants/libattn_clocks.so), launched back to back like the timed run (the stamps are
    those of the last launch, when the board has settled at the clock this load allows)."""
    from paper_2603_24517_amd import probe as P
    stream = torch.cuda.current_stream()
    for _ in range(launches):
        rc = P.variant_attn_fwd("clocks", qd, kd, vd, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, w.causal, w.scale,
                                stream.cuda_stream)
        if rc != 0:
            raise A.AttnError(rc)
    return P.clocks_read()


def item_phases(w, qd, kd, vd, o, lse, launches=10):
    """One wavefront's cycles through the phases of a work item (variants/libattn_phases.so: set-up, first score
    blocks, first softmax, iterations by kind, epilogue), for the first and the last wavefront of the first
    workgroup; None where the split-key kernel runs or a workgroup has fewer than two items."""
    from paper_2603_24517_amd import probe as P
    stream = torch.cuda.current_stream()
    for _ in range(launches):
        rc = P.variant_attn_fwd("phases", qd, kd, vd, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, w.causal, w.scale,
                                stream.cuda_stream)
        if rc != 0:
            raise A.AttnError(rc)
    return P.phases_read()


TRAFFIC_FILE = "profiles/attn_fwd_kernel_hbm_traffic.md"


def traffic_from_profiles(name):
    """(HBM bytes per launch, where the figure comes from) out of the committed counter summary: it is a
    rocprofv3 --pmc measurement made beforehand, not a measurement of this run.  (None, None) if absent."""
    import re
    path = os.path.join(ROOT, TRAFFIC_FILE)
    if not os.path.exists(path):
        return None, None
    text = open(path).read()
    m = re.search(r"traffic_bytes_per_launch\[%s\]\s*=\s*(\d+)" % re.escape(name), text)
    c = re.search(r"kernel source at commit\s+`?([0-9a-f]{7,40})", text, flags=re.I)
    return (int(m.group(1)), f"{TRAFFIC_FILE}@{c.group(1) if c else 'unknown'}") if m else (None, None)


def cpu_baseline(w, q, k, v, o_gpu, lse_gpu, budget_s=12.0):
    """Time the FP64 oracle (as it stands) on a bounded row sample and check the GPU output on it.

    The stratified sample is worked through in chunks of growing size until about budget_s seconds of
    oracle time have been spent (or the sample is exhausted); the first, small chunk only warms up the
    oracle's threads and is not timed."""
    import oracle
    rows_all = W.sample_rows(w, 393216)
    rows_all = rows_all[np.random.default_rng(w.seed).permutation(len(rows_all))]   # any prefix is a stratified sample
    qd, kd, vd = q.double().numpy(), k.double().numpy(), v.double().numpy()
    oracle.attn_ref_rows(qd, kd, vd, rows_all[:64], w.causal, w.scale)
    done, chunk, dt = 0, 1024, 0.0
    o_parts, l_parts, r_parts = [], [], []
    while done < len(rows_all) and dt < budget_s:
        rows = rows_all[done:done + chunk]
        rows = rows[np.lexsort((rows[:, 2], rows[:, 1], rows[:, 0]))]    # rows of one head side by side, as a full run has them
        r_parts.append(rows)
        t0 = time.perf_counter()
        o_ref, lse_ref = oracle.attn_ref_rows(qd, kd, vd, rows, w.causal, w.scale)
        dt += time.perf_counter() - t0
        o_parts.append(o_ref)
        l_parts.append(lse_ref)
        done += len(rows)
        chunk *= 2
    rows = np.concatenate(r_parts)
    o_ref, lse_ref = np.concatenate(o_parts), np.concatenate(l_parts)
    i = rows[:, 2].astype(np.int64)
    nvalid = np.minimum(w.Skv, i + 1 + w.Skv - w.Sq) if w.causal else np.full_like(i, w.Skv)
    flops = 4.0 * float(nvalid.clip(min=0).sum()) * w.D          # work the oracle really did
    b, h = rows[:, 0], rows[:, 1]
    og = o_gpu[b, i, h].double().cpu().numpy()
    lg = lse_gpu[b, h, i].double().cpu().numpy()
    err = np.abs(og - o_ref)
    dl = np.abs(lg - lse_ref) / np.maximum(1.0, np.abs(lse_ref))
    base = {"value": flops / dt * 1e-12, "unit": "TFLOPS", "cores": oracle.threads(), "kind": "oracle",
            "sample": f"{len(rows)} stratified query rows of {w.name}, every valid key, FP64, {dt:.1f} s"}
    parity = {"rows": int(len(rows)), "o_max_abs": float(err.max()), "o_mean_abs": float(err.mean()),
              "lse_rel_max": float(dl.max()),
              "pass": bool(err.max() <= 2e-2 and err.mean() <= 2e-3 and dl.max() <= 1e-3)}
    return base, parity


def run_workload(name, steps, warmup, with_cpu, repeats=1, variant=None):
    """`variant`: time that variant build of the kernel (paper_2603_24517_amd/variants/) instead of the
    shipped library; the line then carries "variant" and is not a benchmark result of the product."""
    w = W.WORKLOADS[name]
    dev = torch.device("cuda:0")
    q, k, v = W.make_qkv(w)
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    o = torch.empty_like(qd)
    lse = torch.empty((w.B, w.Hq, w.Sq), dtype=torch.float32, device=dev)
    stream = torch.cuda.current_stream()

    entry = A.attn_fwd
    if variant is not None:
        from paper_2603_24517_amd import probe as PV
        entry = lambda *a: PV.variant_attn_fwd(variant, *a)     # noqa: E731

    def step():
        rc = entry(qd, kd, vd, o, lse, w.B, w.Hq, w.Hkv, w.Sq, w.Skv, w.D, w.causal, w.scale,
                   stream.cuda_stream)
        if rc != 0:
            raise A.AttnError(rc)

    for _ in range(warmup):
        step()
    torch.cuda.synchronize()
    wall, dev_ms = [], []
    for _ in range(repeats):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        e0.record(stream)              # HIP events on the very stream the kernel is launched on
        for _ in range(steps):
            step()
        e1.record(stream)
        torch.cuda.synchronize()
        wall.append((time.perf_counter() - t0) * 1e3 / steps)
        dev_ms.append(e0.elapsed_time(e1) / steps)
    ms = float(np.mean(wall))
    kms = float(np.mean(dev_ms))
    tflops = w.flops / (ms * 1e-3) * 1e-12
    ktflops = w.flops / (kms * 1e-3) * 1e-12
    traffic, traffic_source = traffic_from_profiles(w.name)
    from paper_2603_24517_amd import probe as P
    rc, cus, khz = P.attn_probe_device_info()
    out = {
        "metric": METRIC, "value": tflops, "unit": "TFLOPS", "n_gpus": 1, "steps": steps, "warmup": warmup,
        "ms_per_step": ms, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "pct_of_peak": 100.0 * tflops / PEAK_BF16_TFLOPS,
        "config": {"workload": w.name, "B": w.B, "Hq": w.Hq, "Hkv": w.Hkv, "Sq": w.Sq, "Skv": w.Skv, "D": w.D,
                   "causal": w.causal, "q_mul": w.q_mul, "v_dist": w.v_dist, "seed": w.seed,
                   "flops_per_step": w.flops},
        "roofline": {"bound": "mfma", "achieved": ktflops, "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s",
                     "frac": ktflops / PEAK_BF16_TFLOPS, "traffic": traffic, "traffic_source": traffic_source,
                     "kernel": kernel_name(w, cus), "kernel_ms": kms,
                     "algorithmic_bytes": w.algorithmic_bytes},
    }
    out["device"] = {"name": torch.cuda.get_device_properties(0).name, "compute_units": cus if rc == 0 else None,
                     "max_clock_mhz": khz / 1e3 if rc == 0 else None,
                     "peak_note": "2516.6 = 256 CU x 4 SIMD x 1024 FLOP/clk x 2.4 GHz"}
    if variant is not None:
        out["variant"] = variant
    if repeats > 1:
        out["ms_std"] = float(np.std(dev_ms))
    if with_cpu:
        out["cpu_baseline"], out["parity"] = cpu_baseline(w, q, k, v, o, lse)
        out["roofline"].update(kernel_clock(w, qd, kd, vd, o, lse))
        if out["roofline"]["kernel"] == "attn_fwd_kernel":
            out["roofline"]["item_phases_cycles"] = item_phases(w, qd, kd, vd, o, lse)
        out["mfma_probe"] = mfma_probe()
        ceiling = out["mfma_probe"]["ceiling"]["tflops"]
        out["roofline"]["frac_of_probe_ceiling"] = ktflops / ceiling
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default=W.HEADLINE, choices=sorted(W.WORKLOADS))
    ap.add_argument("--all", action="store_true", help="every workload, 10 repeats of --steps each")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing leg")
    ap.add_argument("--variant", default=None,
                    help="time a variant build of the kernel instead of the shipped one (implies --no-cpu)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="run a plain 1 GiB device copy instead (reference for the FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on exactly one GPU (no collectives, no sharding); use --gpus 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible; there is no CPU path")
    A.load()
    if args.copy_calibration:
        n = 1 << 30
        src = torch.full((n,), 3, dtype=torch.uint8, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"copy_bytes_read": n, "copy_bytes_written": n, "launches": 3}))
        return
    if args.all:
        names = [n for n in W.WORKLOADS if n != W.HEADLINE] + [W.HEADLINE]
        for n in names:
            steps = max(3, min(args.steps, 30))
            print(json.dumps(run_workload(n, steps, min(args.warmup, 10), not args.no_cpu, repeats=10)), flush=True)
    else:
        print(json.dumps(run_workload(args.workload, args.steps, args.warmup, not args.no_cpu and args.variant is None,
                                      variant=args.variant)), flush=True)


if __name__ == "__main__":
    main()
