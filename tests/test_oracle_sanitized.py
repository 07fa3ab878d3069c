"""The oracle's C code under AddressSanitizer and UndefinedBehaviorSanitizer (host code only, no GPU):
every pin must pass on an instrumented build without a report.  Runs in a child process, because the
sanitizer runtime has to be loaded before the interpreter starts."""
import os
import subprocess
import sys

import pytest

import oracle

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))

CHILD = r"""
import sys
sys.path.insert(0, {root!r}); sys.path.insert(0, {tests!r})
import oracle, pins
orc = oracle.Oracle({so!r})
for pin in pins.ALL_PINS:
    pin(orc)
print("pins passed:", len(pins.ALL_PINS))
"""


def _runtime(name):
    path = subprocess.run(["gcc", f"-print-file-name={name}"], check=True, capture_output=True, text=True).stdout.strip()
    return path if os.path.isabs(path) and os.path.exists(path) else None


def test_pins_pass_on_an_asan_ubsan_build(tmp_path):
    asan = _runtime("libasan.so")
    if asan is None:
        pytest.skip("gcc has no libasan.so here")
    so = str(tmp_path / "libattn_oracle_san.so")
    subprocess.run(["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=undefined", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                    "-o", so, oracle.SRC, "-lm"], check=True)
    env = dict(os.environ)
    # the sanitizer runtime goes in front of whatever is preloaded already
    env["LD_PRELOAD"] = asan + (":" + env["LD_PRELOAD"] if env.get("LD_PRELOAD") else "")
    # leak checking would report the interpreter's own allocations at exit
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0:abort_on_error=0:exitcode=97"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:exitcode=98"
    env["OMP_NUM_THREADS"] = "4"
    code = CHILD.format(root=ROOT, tests=os.path.join(ROOT, "tests"), so=so)
    r = subprocess.run([sys.executable, "-c", code], env=env, capture_output=True, text=True, timeout=600)
    assert r.returncode == 0, r.stdout[-2000:] + r.stderr[-4000:]
    assert "pins passed" in r.stdout
    assert "ERROR: AddressSanitizer" not in r.stderr and "runtime error" not in r.stderr, r.stderr[-4000:]
