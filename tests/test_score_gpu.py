"""The scoring function f(x) (paper section 3.1) on a tiny grid: correct kernel -> positive scores, commit rule."""
import json
import os
import subprocess
import sys

import pytest

pytestmark = pytest.mark.gpu
HERE = os.path.dirname(os.path.abspath(__file__))


def test_score_tiny_grid(tmp_path):
    lineage = tmp_path / "lineage.jsonl"
    for label in ("first", "second"):
        out = subprocess.run([sys.executable, os.path.join(HERE, "score_f.py"), "--grid", "tiny", "--runs", "2",
                              "--launches", "3", "--rows", "128", "--lineage", str(lineage), "--label", label],
                             capture_output=True, text=True, timeout=300)
        assert out.returncode == 0, out.stderr[-2000:]
        last = json.loads(out.stdout.strip().splitlines()[-1])
        assert last["all_correct"] and last["geomean"] > 0 and last["n"] == 2
    recs = [json.loads(x) for x in open(lineage)]
    assert len(recs) == 2 and recs[0]["committed"] is True
    assert all(s["f"] == s["tflops_mean"] for r in recs for s in r["scores"])
