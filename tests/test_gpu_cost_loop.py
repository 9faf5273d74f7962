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
    # the fixed policy keeps its 59 draft nodes whatever they cost; the rule's modelled speedup is never the smaller one
    # by much (alpha < 1 makes it conservative), and both policies' trees were really run through the kernel
    assert r["baseline_nodes"] == 60 and r["smart_us"] > 0 and r["baseline_us"] > 0
    assert r["smart_measured_R"] > 0 and r["baseline_measured_R"] > 0


def test_cost_loop_with_an_extra_cost_from_the_caller_and_a_draft_leg():
    """The caller's per-token extra (a whole layer's dense products in bench.py --cost-loop --with-dense; a plain
    linear stand-in here), a 32-layer target and a one-layer drafter: lambda is fitted and positive, the tables come
    from the library, and the rule is run with the exact difference and with the differentiated marginal cost."""
    from paper_2604_09731_amd import cost_loop
    rows = cost_loop.main(["--batches", "4", "--prefix", "256", "--sizes", "1", "4", "16", "32", "--reps", "3",
                           "--target-layers", "32", "--draft-layers", "1"], extra_us=lambda tokens: 0.05 * tokens)
    r = rows[0]
    assert r["extra"] and r["target_layers"] == 32 and r["draft_layers"] == 1
    assert len(r["us"]) == 4 and all(v > 0 for v in r["us"]) and r["us"][-1] > r["us"][0]
    assert r["lam"] > 0 and math.isfinite(r["lam"])
    lo, med, hi = r["tree_nodes_min_median_max"]
    dlo, dmed, dhi = r["derivative_tree_nodes_min_median_max"]
    assert 1 <= lo <= med <= hi <= 64 and 1 <= dlo <= dmed <= dhi <= 64
    if r["rho"] >= 1.0:
        assert dmed >= med      # the derivative understates the next node's cost of a convex model
    else:
        assert dmed == 1        # a concave fit has an infinite derivative where nothing is drafted yet: root only
    assert r["smart_measured_R"] > 0 and r["baseline_measured_R"] > 0


def test_cost_loop_over_product_forests():
    """Candidate forests of a drafter with independent positions (Cartesian product, cut at 1024 candidates)."""
    from paper_2604_09731_amd import cost_loop
    rows = cost_loop.main(["--batches", "2", "--prefix", "256", "--sizes", "1", "4", "16", "32", "--reps", "3",
                           "--forest", "product"])
    r = rows[0]
    assert r["forest"] == "product" and r["baseline_nodes"] == 60
    lo, med, hi = r["tree_nodes_min_median_max"]
    assert 1 <= lo <= med <= hi <= 64 and r["smart_measured_R"] > 0 and r["baseline_measured_R"] > 0
