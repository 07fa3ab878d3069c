"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol
include/attn.h declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

import paper_2603_24517_amd as A

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols(header):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(attn_[a-z_0-9]+)\s*\(", text)))


def _exported_symbols(path):
    """The attn_* functions a shared object defines (dynamic symbol table, via nm)."""
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", path], check=True, capture_output=True, text=True).stdout
    return sorted({ln.split()[-1] for ln in out.splitlines() if ln.split()[-1].startswith("attn_")})


def test_header_symbols_exported():
    syms = _declared_symbols("attn.h")
    assert syms == ["attn_fwd", "attn_strerror", "attn_version"]
    lib = ctypes.CDLL(A.LIB_PATH)
    for s in syms:
        assert hasattr(lib, s), f"{s} declared in include/attn.h but not exported"
    # and the attention library exports nothing beyond its header
    assert _exported_symbols(A.LIB_PATH) == syms


def test_probe_header_symbols_exported():
    from paper_2603_24517_amd import build as B
    syms = _declared_symbols("attn_probe.h")
    assert syms == ["attn_clocks_read", "attn_phases_read", "attn_probe_device_info", "attn_probe_mfma"]
    assert _exported_symbols(B.PROBE_LIB) == ["attn_probe_device_info", "attn_probe_mfma"]
    # every variant build keeps the C ABI of include/attn.h; the clocks and phases builds add their readers
    for name in B.VARIANTS:
        want = ["attn_fwd", "attn_strerror", "attn_version"]
        if name in ("clocks", "phases"):
            want = ["attn_clocks_read"] + want
        if name == "phases":
            want = ["attn_phases_read"] + want
        assert _exported_symbols(B.variant_path(name)) == sorted(want), name


def test_version_and_strerror():
    assert A.attn_version() >= 1000
    for code in range(0, -8, -1):
        assert isinstance(A.attn_strerror(code), str) and A.attn_strerror(code)
    assert "unknown" in A.attn_strerror(-99)


GOOD = dict(q=4096, k=8192, v=12288, o=16384, lse=20480, B=1, Hq=4, Hkv=2, Sq=8, Skv=8, D=128,
            causal=0, scale=0.1)


def _call(**kw):
    a = dict(GOOD); a.update(kw)
    return A.attn_fwd(a["q"], a["k"], a["v"], a["o"], a["lse"], a["B"], a["Hq"], a["Hkv"],
                      a["Sq"], a["Skv"], a["D"], a["causal"], a["scale"], None)


@pytest.mark.parametrize("kw,code", [
    (dict(q=None), A.ATTN_E_NULL), (dict(k=None), A.ATTN_E_NULL), (dict(v=None), A.ATTN_E_NULL),
    (dict(o=None), A.ATTN_E_NULL), (dict(lse=None), A.ATTN_E_NULL),
    (dict(B=0), A.ATTN_E_SHAPE), (dict(Hq=0), A.ATTN_E_SHAPE), (dict(Hkv=-1), A.ATTN_E_SHAPE),
    (dict(Sq=0), A.ATTN_E_SHAPE), (dict(Skv=0), A.ATTN_E_SHAPE), (dict(D=0), A.ATTN_E_SHAPE),
    (dict(Hq=5, Hkv=2), A.ATTN_E_SHAPE),
    (dict(D=64), A.ATTN_E_UNSUPPORTED), (dict(D=256), A.ATTN_E_UNSUPPORTED),
    (dict(Sq=2**31 - 200, Skv=1), A.ATTN_E_UNSUPPORTED),
    (dict(B=2**20, Hq=2**10, Hkv=2**10, Sq=2**12), A.ATTN_E_UNSUPPORTED),
    (dict(Hq=65536, Hkv=2), A.ATTN_E_UNSUPPORTED), (dict(Hq=65536, Hkv=65536), A.ATTN_E_UNSUPPORTED),
    (dict(q=4096 + 8), A.ATTN_E_ALIGN), (dict(o=16384 + 2), A.ATTN_E_ALIGN), (dict(lse=20480 + 2), A.ATTN_E_ALIGN),
    (dict(scale=float("nan")), A.ATTN_E_SCALE), (dict(scale=float("inf")), A.ATTN_E_SCALE),
    (dict(scale=float("-inf")), A.ATTN_E_SCALE),
])
def test_bad_arguments_rejected_on_host(kw, code):
    # none of these calls may reach the device: the pointers are fake addresses
    assert _call(**kw) == code


def test_no_cpu_fallback():
    import torch
    x = torch.zeros(1, 8, 2, 128, dtype=torch.bfloat16)
    with pytest.raises(ValueError):
        A.attention(x, x, x)


@pytest.mark.parametrize("kw", [
    dict(operands=None), dict(sink=None), dict(clocks=None), dict(operands=4096 + 4), dict(clocks=12288 + 4),
    dict(iters=0), dict(iters=(1 << 20) + 1), dict(waves=3), dict(waves=0), dict(mode=8), dict(mode=-1),
    dict(mode=4, tiles=None), dict(mode=4, tiles=1 << 20, tiles_bytes=3 << 20), dict(mode=4, tiles=1 << 20, tiles_bytes=1 << 19),
    dict(mode=5, tiles=(1 << 20) + 8, tiles_bytes=1 << 20),
])
def test_probe_bad_arguments_rejected_on_host(kw):
    from paper_2603_24517_amd import probe as P
    a = dict(operands=4096, tiles=None, tiles_bytes=0, sink=8192, clocks=12288, mode=0, waves=2, iters=10)
    a.update(kw)
    rc = P.attn_probe_mfma(a["operands"], a["tiles"], a["tiles_bytes"], a["sink"], a["clocks"], a["mode"],
                           a["waves"], a["iters"])
    assert rc == -1          # ATTN_PROBE_E_ARG: no launch was attempted with these fake addresses


def test_device_info_without_a_device_reports_an_error():
    import torch
    from paper_2603_24517_amd import probe as P
    rc, cus, khz = P.attn_probe_device_info()
    if torch.cuda.is_available():
        assert rc == 0 and cus > 0 and khz > 0
    else:
        assert rc == -2      # ATTN_PROBE_E_LAUNCH


def test_row_sampler_terminates_and_is_stratified():
    from paper_2603_24517_amd import workloads as W
    small = W.WORKLOADS[W.SMALL]
    every = W.sample_rows(small, 10 ** 6)                      # more rows asked for than exist: all of them, once
    assert every.shape == (small.B * small.Hq * small.Sq, 3)
    w = W.WORKLOADS[W.HEADLINE]
    rows = W.sample_rows(w, 4096)
    assert len({tuple(r) for r in rows.tolist()}) == len(rows) >= 4096
    assert {(b, h) for b, h, _ in rows.tolist()} == {(b, h) for b in range(w.B) for h in range(w.Hq)}
    assert {0, w.Sq - 1} <= set(rows[:, 2].tolist())
    assert (W.sample_rows(w, 4096) == rows).all()               # seeded
