"""bench.py prints ONE strictly valid JSON line that carries the fields its readers depend on."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _reject(name):
    raise ValueError(f"non-finite constant {name} in the benchmark line")


@pytest.mark.parametrize("workload", ["cfg1_mha_nc_b1_h4_s512", "cfg2_mha_nc_b8_h16_s4096"])
def test_bench_line_is_valid_json_with_the_contract_fields(workload):
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--workload", workload, "--steps", "5", "--warmup", "2"],
                       capture_output=True, text=True, timeout=600, cwd=ROOT)
    assert r.returncode == 0, r.stderr[-2000:]
    lines = [ln for ln in r.stdout.splitlines() if ln.strip()]
    assert len(lines) == 1, r.stdout[-2000:]
    d = json.loads(lines[0], parse_constant=_reject)          # NaN / Infinity are not JSON
    for key in ("metric", "value", "unit", "n_gpus", "steps", "warmup", "ms_per_step", "higher_is_better", "scaling",
                "vs_baseline", "dtype", "data", "config", "roofline", "cpu_baseline"):
        assert key in d, key
    assert d["n_gpus"] == 1 and d["steps"] == 5 and d["warmup"] == 2 and d["dtype"] == "bf16" and d["vs_baseline"] is None
    assert d["config"]["workload"] == workload
    rl = d["roofline"]
    assert rl["bound"] == "mfma" and rl["peak"] == 2516.6 and rl["unit"] == "TFLOP/s"
    assert abs(rl["frac"] - rl["achieved"] / rl["peak"]) < 1e-9 and 0 < rl["frac"] < 1
    assert rl["kernel"] == ("attn_fwd_split_kernel" if workload.startswith("cfg1") else "attn_fwd_kernel")
    cb = d["cpu_baseline"]
    assert cb["kind"] == "oracle" and cb["cores"] >= 1 and cb["value"] > 0 and cb["sample"]
    assert d["parity"]["pass"] is True
    assert d["mfma_probe"]["ceiling"]["tflops"] > 0


def test_bench_refuses_more_than_one_gpu():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=300, cwd=ROOT)
    assert r.returncode != 0 and "one GPU" in (r.stderr + r.stdout)
