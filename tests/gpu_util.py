"""Helpers shared by the GPU parity tests: run the HIP path, run the oracle, compare to the stated bars."""
import numpy as np
import torch

import oracle
import paper_2603_24517_amd as A
from paper_2603_24517_amd import workloads as W

O_MAX_ABS = 2e-2       # tolerance on BF16 O against the unrounded FP64 oracle
O_MEAN_ABS = 2e-3
LSE_REL = 1e-3         # |dLSE| <= LSE_REL * max(1, |LSE_ref|)


def run_gpu(q, k, v, causal, scale, stream=None):
    """q, k, v: CPU BF16 tensors [B,S,H,D].  Returns (O float64 numpy, LSE float64 numpy) from the HIP path."""
    dev = torch.device("cuda:0")
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    B, Sq, Hq, D = q.shape
    _, Skv, Hkv, _ = k.shape
    o = torch.full_like(qd, float("nan"))
    lse = torch.full((B, Hq, Sq), float("nan"), dtype=torch.float32, device=dev)
    st = torch.cuda.current_stream().cuda_stream if stream is None else stream
    rc = A.attn_fwd(qd, kd, vd, o, lse, B, Hq, Hkv, Sq, Skv, D, causal, scale, st)
    assert rc == 0, A.attn_strerror(rc)
    torch.cuda.synchronize()
    return o.cpu().double().numpy(), lse.cpu().double().numpy()


def compare(o_gpu, lse_gpu, o_ref, lse_ref, what=""):
    """Gate O and LSE; returns the error figures."""
    assert not np.isnan(o_gpu).any(), f"{what}: NaN in O"
    assert not np.isnan(lse_gpu).any(), f"{what}: NaN in LSE"
    err = np.abs(o_gpu - o_ref)
    fin = np.isfinite(lse_ref)
    assert np.array_equal(np.isfinite(lse_gpu), fin), f"{what}: -inf pattern of LSE differs"
    if (~fin).any():
        assert np.all(lse_gpu[~fin] == -np.inf)
    dl = np.abs(lse_gpu[fin] - lse_ref[fin])
    bar = LSE_REL * np.maximum(1.0, np.abs(lse_ref[fin]))
    res = dict(max_abs=float(err.max()), mean_abs=float(err.mean()),
               lse_max=float(dl.max()) if dl.size else 0.0,
               lse_worst_ratio=float((dl / bar).max()) if dl.size else 0.0)
    assert res["max_abs"] <= O_MAX_ABS, f"{what}: O max-abs {res['max_abs']:.3e}"
    assert res["mean_abs"] <= O_MEAN_ABS, f"{what}: O mean-abs {res['mean_abs']:.3e}"
    assert res["lse_worst_ratio"] <= 1.0, f"{what}: LSE error {res['lse_max']:.3e}"
    return res


def check_full(q, k, v, causal, scale, what=""):
    o_ref, lse_ref = oracle.attn_ref(q, k, v, causal, scale)
    o, lse = run_gpu(q, k, v, causal, scale)
    return compare(o, lse, o_ref, lse_ref, what)


def check_rows(q, k, v, rows, causal, scale, what=""):
    o_ref, lse_ref = oracle.attn_ref_rows(q, k, v, rows, causal, scale)
    o, lse = run_gpu(q, k, v, causal, scale)
    b, h, i = rows[:, 0], rows[:, 1], rows[:, 2]
    return compare(o[b, i, h], lse[b, h, i], o_ref, lse_ref, what)


def rand_qkv(B, Hq, Hkv, Sq, Skv, seed, q_mul=1.0, D=128):
    w = W.custom("adhoc", B, Hq, Hkv, Sq, Skv, D=D, seed=seed, q_mul=q_mul)
    return W.make_qkv(w)
