"""The scoring function's bookkeeping (paper sections 3.1, 3.2), without a GPU: the geometric mean with its
correctness gate, and the commit rule of the lineage file."""
import json
import math

import score_f as S


def test_geomean_is_zero_as_soon_as_one_configuration_scores_zero():
    assert math.isclose(S.geomean([100.0, 400.0]), 200.0)
    assert math.isclose(S.geomean([2.0, 4.0, 8.0]), 4.0)
    assert S.geomean([1200.0, 0.0, 1100.0]) == 0.0          # an incorrect configuration scores 0 and sinks the candidate


def _rec(label, g, ok=True, grid="paper"):
    return {"label": label, "grid": grid, "geomean": g, "all_correct": ok, "scores": []}


def test_commit_only_if_correct_and_at_least_as_good(tmp_path):
    path = str(tmp_path / "lineage.jsonl")
    assert S.record_in_lineage(path, _rec("v1", 1000.0)) == (True, 0.0)
    assert S.record_in_lineage(path, _rec("slower", 900.0)) == (False, 1000.0)
    assert S.record_in_lineage(path, _rec("faster but wrong", 1500.0, ok=False)) == (False, 1000.0)
    assert S.record_in_lineage(path, _rec("v2", 1100.0)) == (True, 1000.0)
    assert S.record_in_lineage(path, _rec("equal", 1100.0)) == (True, 1100.0)
    assert S.record_in_lineage(path, _rec("other grid", 10.0, grid="tiny")) == (True, 0.0)   # grids do not compete
    recs = [json.loads(l) for l in open(path)]
    assert [r["committed"] for r in recs] == [True, False, False, True, True, True]
    # a rejected candidate never becomes the bar
    assert S.record_in_lineage(path, _rec("after", 1050.0)) == (False, 1100.0)
