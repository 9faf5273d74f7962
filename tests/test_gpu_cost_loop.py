"""The measure -> fit -> select loop runs end to end on the device (small sizes)."""
import math

import pytest

pytestmark = pytest.mark.gpu


def test_cost_loop_small():
    from paper_2604_09731_amd import cost_loop
    rows = cost_loop.main(["--batches", "2", "--prefix", "512", "--sizes", "1", "4", "8", "16", "32", "--reps", "5"])
    assert len(rows) == 1
    r = rows[0]
    assert len(r["us"]) == 5 and all(v > 0 for v in r["us"])
    assert all(math.isfinite(r[k]) and r[k] > 0 for k in ("gamma", "delta", "rho", "c_T_us"))
    lo, med, hi = r["tree_nodes_min_median_max"]
    assert 1 <= lo <= med <= hi <= 64
