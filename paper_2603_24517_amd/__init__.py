"""MI355X-native fused attention forward: thin Python binding over the C ABI of include/attn.h.

Argument marshalling only: every step of the computation runs in the HIP
kernels of csrc/attn_fwd.hip.  There is no CPU or PyTorch fallback; if the
shared library has not been built, importing the entry points fails loudly.
"""
import ctypes
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libattn_mi355x.so")

ATTN_OK = 0
ATTN_E_NULL = -1
ATTN_E_SHAPE = -2
ATTN_E_UNSUPPORTED = -3
ATTN_E_ALIGN = -4
ATTN_E_SCALE = -5
ATTN_E_LAUNCH = -6

_lib = None


class AttnError(RuntimeError):
    def __init__(self, code):
        self.code = code
        super().__init__(f"attn_fwd failed ({code}): {attn_strerror(code)}")


def open_library(path):
    """ctypes handle of a build of the attention library, with the argument types of include/attn.h set."""
    if not os.path.exists(path):
        raise ImportError(
            f"{path} is missing: build it with `python -m paper_2603_24517_amd.build [--all]` "
            "(there is no fallback path)")
    lib = ctypes.CDLL(path)
    vp, ci = ctypes.c_void_p, ctypes.c_int
    lib.attn_fwd.argtypes = [vp, vp, vp, vp, vp, ci, ci, ci, ci, ci, ci, ci, ctypes.c_float, vp]
    lib.attn_fwd.restype = ci
    lib.attn_strerror.argtypes = [ci]
    lib.attn_strerror.restype = ctypes.c_char_p
    lib.attn_version.argtypes = []
    lib.attn_version.restype = ci
    return lib


def load():
    """Load the built library (never builds, never falls back)."""
    global _lib
    if _lib is None:
        _lib = open_library(LIB_PATH)
    return _lib


def _ptr(x):
    if x is None:
        return None
    if hasattr(x, "data_ptr"):
        return x.data_ptr()
    return int(x)


def attn_fwd(q, k, v, o, lse, B, Hq, Hkv, Sq, Skv, D, causal, scale, stream=None):
    """C-ABI call attn_fwd(...).  Tensors (anything with .data_ptr()) or raw device addresses.

    Returns the library's status code (0 = ok); enqueues on `stream` (a raw hipStream_t
    handle, e.g. torch.cuda.current_stream().cuda_stream; None = default stream).
    """
    return load().attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse),
                           int(B), int(Hq), int(Hkv), int(Sq), int(Skv), int(D),
                           int(bool(causal)), float(scale), stream)


def attn_strerror(code):
    return load().attn_strerror(int(code)).decode()


def attn_version():
    return int(load().attn_version())


def attention(q, k, v, causal=False, scale=None):
    """Allocate O and LSE with torch on q's device and run attn_fwd on torch's current stream.

    q [B,Sq,Hq,D], k/v [B,Skv,Hkv,D], BF16, contiguous, on a ROCm device.
    Returns (O BF16 [B,Sq,Hq,D], LSE FP32 [B,Hq,Sq]).
    """
    import torch
    if not (q.is_cuda and k.is_cuda and v.is_cuda):
        raise ValueError("attention() needs device tensors; there is no CPU path")
    for t in (q, k, v):
        if t.dtype != torch.bfloat16 or not t.is_contiguous() or t.dim() != 4:
            raise ValueError("q, k, v must be contiguous 4-d BF16 tensors [B, S, H, D]")
    B, Sq, Hq, D = q.shape
    Bk, Skv, Hkv, Dk = k.shape
    if (Bk, Dk) != (B, D) or v.shape != k.shape:
        raise ValueError("inconsistent q/k/v shapes")
    if scale is None:
        scale = D ** -0.5
    o = torch.empty_like(q)
    lse = torch.empty((B, Hq, Sq), dtype=torch.float32, device=q.device)
    with torch.cuda.device(q.device):
        rc = attn_fwd(q, k, v, o, lse, B, Hq, Hkv, Sq, Skv, D, causal, scale,
                      torch.cuda.current_stream().cuda_stream)
    if rc != ATTN_OK:
        raise AttnError(rc)
    return o, lse
