"""ctypes front end of the C oracle (attn_oracle.c).  TEST INFRASTRUCTURE ONLY.

The arithmetic lives in attn_oracle.c (naive FP64 attention with an explicit
full-row softmax, paper section 2.2).  This file only builds that file with
gcc, widens the inputs to float64 (exact for BF16/FP32 inputs) and marshals
pointers.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(_HERE, "attn_oracle.c")
SO = os.path.join(_HERE, "libattn_oracle.so")


def compile_c(src, so):
    subprocess.run(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                    "-o", so, src, "-lm"], check=True)
    return so


def build(force=False):
    """Compile attn_oracle.c into libattn_oracle.so next to it."""
    if (not force and os.path.exists(SO)
            and os.path.getmtime(SO) >= os.path.getmtime(SRC)):
        return SO
    return compile_c(SRC, SO)


def _f64(x):
    """Any array-like / torch tensor -> contiguous float64 numpy (exact widening)."""
    if hasattr(x, "detach"):  # torch tensor, possibly bfloat16
        x = x.detach().cpu().double().numpy()
    return np.ascontiguousarray(np.asarray(x, dtype=np.float64))


def _ptr(a):
    return a.ctypes.data_as(ctypes.POINTER(ctypes.c_double))


def _dims(q, k, v):
    if q.ndim != 4 or k.ndim != 4 or v.ndim != 4:
        raise ValueError("q, k, v must be [B, S, H, D]")
    B, Sq, Hq, D = q.shape
    Bk, Skv, Hkv, Dk = k.shape
    if (Bk, Dk) != (B, D) or v.shape != k.shape:
        raise ValueError("inconsistent shapes")
    return B, Hq, Hkv, Sq, Skv, D


class Oracle:
    """One loaded oracle shared object (the tests also load deliberately broken builds)."""

    def __init__(self, so_path):
        lib = ctypes.CDLL(so_path)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        ci = ctypes.c_int
        lib.attn_ref_f64.argtypes = [dp, dp, dp, dp, dp, ci, ci, ci, ci, ci, ci, ci, ctypes.c_double]
        lib.attn_ref_f64.restype = ci
        lib.attn_ref_rows_f64.argtypes = [dp, dp, dp, ip, ctypes.c_long, dp, dp,
                                          ci, ci, ci, ci, ci, ci, ci, ctypes.c_double]
        lib.attn_ref_rows_f64.restype = ci
        lib.attn_ref_probs_f64.argtypes = [dp, dp, ci, ci, ci, dp, ci, ci, ci, ci, ci, ci, ci, ctypes.c_double]
        lib.attn_ref_probs_f64.restype = ci
        lib.attn_ref_threads.restype = ci
        self.lib = lib

    def threads(self):
        return int(self.lib.attn_ref_threads())

    def attn_ref(self, q, k, v, causal, scale):
        """All rows.  q [B,Sq,Hq,D]; k, v [B,Skv,Hkv,D] -> (O [B,Sq,Hq,D], LSE [B,Hq,Sq]), float64."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        B, Hq, Hkv, Sq, Skv, D = _dims(q, k, v)
        o = np.empty((B, Sq, Hq, D), dtype=np.float64)
        lse = np.empty((B, Hq, Sq), dtype=np.float64)
        rc = self.lib.attn_ref_f64(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                                   B, Hq, Hkv, Sq, Skv, D, int(bool(causal)), float(scale))
        if rc != 0:
            raise RuntimeError(f"attn_ref_f64 failed: {rc}")
        return o, lse

    def attn_ref_rows(self, q, k, v, rows, causal, scale):
        """Only the rows listed as (b, h, i) triples -> (O_rows [n,D], LSE_rows [n]), float64."""
        q, k, v = _f64(q), _f64(k), _f64(v)
        B, Hq, Hkv, Sq, Skv, D = _dims(q, k, v)
        rows = np.ascontiguousarray(np.asarray(rows, dtype=np.int32).reshape(-1, 3))
        n = rows.shape[0]
        o = np.empty((n, D), dtype=np.float64)
        lse = np.empty((n,), dtype=np.float64)
        rc = self.lib.attn_ref_rows_f64(_ptr(q), _ptr(k), _ptr(v),
                                        rows.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)), n,
                                        _ptr(o), _ptr(lse),
                                        B, Hq, Hkv, Sq, Skv, D, int(bool(causal)), float(scale))
        if rc != 0:
            raise RuntimeError(f"attn_ref_rows_f64 failed: {rc}")
        return o, lse

    def attn_ref_probs(self, q, k, b, h, i, causal, scale):
        """Softmax weights p_j / l of one row (zeros where masked), float64 [Skv]."""
        q, k = _f64(q), _f64(k)
        B, Sq, Hq, D = q.shape
        _, Skv, Hkv, _ = k.shape
        p = np.empty((Skv,), dtype=np.float64)
        rc = self.lib.attn_ref_probs_f64(_ptr(q), _ptr(k), int(b), int(h), int(i), _ptr(p),
                                         B, Hq, Hkv, Sq, Skv, D, int(bool(causal)), float(scale))
        if rc != 0:
            raise RuntimeError(f"attn_ref_probs_f64 failed: {rc}")
        return p


_default = None


def default():
    global _default
    if _default is None:
        _default = Oracle(build())
    return _default


def threads():
    return default().threads()


def attn_ref(q, k, v, causal, scale):
    return default().attn_ref(q, k, v, causal, scale)


def attn_ref_rows(q, k, v, rows, causal, scale):
    return default().attn_ref_rows(q, k, v, rows, causal, scale)


def attn_ref_probs(q, k, b, h, i, causal, scale):
    return default().attn_ref_probs(q, k, b, h, i, causal, scale)
