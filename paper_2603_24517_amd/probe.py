"""Bindings of the measurement-aid library (include/attn_probe.h) and of the variant builds of the
attention kernel.  Used by bench.py and by the tests of the variants; the product path (`attention`,
`attn_fwd` of the package) loads none of this."""
import ctypes
import os

from . import open_library
from .build import PROBE_LIB, VARIANTS, variant_path

PROBE_VALU, PROBE_LDS, PROBE_DMA = 1, 2, 4
PROBE_BLOCKS = 256
FLOP_PER_MFMA = 32768

_probe = None
_variants = {}


def load_probe():
    global _probe
    if _probe is None:
        if not os.path.exists(PROBE_LIB):
            raise ImportError(f"{PROBE_LIB} is missing: build it with `python -m paper_2603_24517_amd.build --all`")
        lib = ctypes.CDLL(PROBE_LIB)
        vp, ci = ctypes.c_void_p, ctypes.c_int
        lib.attn_probe_mfma.argtypes = [vp, vp, ctypes.c_size_t, vp, vp, ci, ci, ci, vp]
        lib.attn_probe_mfma.restype = ci
        lib.attn_probe_device_info.argtypes = [ctypes.POINTER(ci), ctypes.POINTER(ci)]
        lib.attn_probe_device_info.restype = ci
        _probe = lib
    return _probe


def _ptr(x):
    if x is None:
        return None
    return x.data_ptr() if hasattr(x, "data_ptr") else int(x)


def attn_probe_mfma(operands, tiles, tiles_bytes, sink, clocks, mode, waves_per_simd, iters, stream=None):
    """C-ABI call attn_probe_mfma(...), see include/attn_probe.h.  Returns the status code."""
    return load_probe().attn_probe_mfma(_ptr(operands), _ptr(tiles), int(tiles_bytes), _ptr(sink), _ptr(clocks),
                                        int(mode), int(waves_per_simd), int(iters), stream)


def probe_flops(waves_per_simd, iters):
    return PROBE_BLOCKS * 4 * waves_per_simd * iters * 32 * FLOP_PER_MFMA


def attn_probe_device_info():
    """(status code, compute units, peak shader clock in kHz) of the current device."""
    cus, khz = ctypes.c_int(0), ctypes.c_int(0)
    rc = load_probe().attn_probe_device_info(ctypes.byref(cus), ctypes.byref(khz))
    return int(rc), cus.value, khz.value


def load_variant(name):
    """ctypes handle of one variant build of the attention library (same C ABI as the shipped one)."""
    if name not in VARIANTS:
        raise KeyError(f"unknown variant {name!r}; known: {sorted(VARIANTS)}")
    if name not in _variants:
        lib = open_library(variant_path(name))
        if name in ("clocks", "phases"):
            lib.attn_clocks_read.argtypes = [ctypes.POINTER(ctypes.c_ulonglong)]
            lib.attn_clocks_read.restype = ctypes.c_int
        if name == "phases":
            lib.attn_phases_read.argtypes = [ctypes.POINTER(ctypes.c_ulonglong)]
            lib.attn_phases_read.restype = ctypes.c_int
        _variants[name] = lib
    return _variants[name]


def variant_attn_fwd(name, q, k, v, o, lse, B, Hq, Hkv, Sq, Skv, D, causal, scale, stream=None):
    """attn_fwd of the variant build `name`; same arguments and return value as the package's attn_fwd."""
    return load_variant(name).attn_fwd(_ptr(q), _ptr(k), _ptr(v), _ptr(o), _ptr(lse), int(B), int(Hq), int(Hkv),
                                       int(Sq), int(Skv), int(D), int(bool(causal)), float(scale), stream)


def clocks_read():
    """Stamps of the last launch of the `clocks` variant, as a dict: cycles and clock of the first workgroup,
    and (256-row kernel, a workgroup with at least three items) the cycles per key-block iteration of its
    third item and the cycles between the loops of its second and third item.  Waits for the device."""
    out = (ctypes.c_ulonglong * 10)()
    rc = load_variant("clocks").attn_clocks_read(out)
    if rc != 0:
        raise RuntimeError(f"attn_clocks_read failed ({rc})")
    cycles, ticks = out[1] - out[0], out[3] - out[2]
    res = {"cycles_first_workgroup": int(cycles), "clock_ghz": (0.1 * cycles / ticks) if ticks else None}
    s2, e2, n2, s3, e3, n3 = (int(out[i]) for i in range(4, 10))
    if out[0] <= s2 < e2 <= s3 < e3 <= out[1] and n3 > 0:     # stamps of this launch, in order
        res["cycles_per_iteration"] = (e3 - s3) / n3
        res["cycles_between_items"] = s3 - e2
        res["iterations_per_item"] = n3
    return res


PHASES = ("setup", "first_two_score_blocks", "first_softmax", "barrier_and_first_requests", "fast_iterations",
          "fast_iterations_n", "other_iterations", "other_iterations_n", "last_iteration", "wait_for_loads", "epilogue",
          "item")


def phases_read():
    """Cycle sums per phase of the second work item of the first workgroup in the last launch of the `phases`
    variant: {"first_wavefront": {phase: cycles}, "last_wavefront": {...}}, or None if that workgroup had fewer
    than two items (or took the split-key kernel).  Waits for the device."""
    out = (ctypes.c_ulonglong * 24)()
    rc = load_variant("phases").attn_phases_read(out)
    if rc != 0:
        raise RuntimeError(f"attn_phases_read failed ({rc})")
    res = {}
    for w, name in enumerate(("first_wavefront", "last_wavefront")):
        v = [int(out[12 * w + k]) for k in range(12)]
        if v[11] == 0 or sum(v[k] for k in (0, 1, 2, 3, 4, 6, 8, 9, 10)) != v[11]:     # nothing written, or torn
            return None
        res[name] = dict(zip(PHASES, v))
    return res
