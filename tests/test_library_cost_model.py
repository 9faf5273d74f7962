"""The library's cost-model tables and fits against the oracle (host only)."""
import ctypes
import math

import numpy as np
import pytest

from oracle import cost_model as CM
from paper_2604_09731_amd import binding as B


@pytest.mark.parametrize("params", [(0.02, 1.5, 0.002, 1.2, 4.0, 32.0, 64), (0.0, 3.0, 1e-5, 2.0, 1.0, 1.0, 128),
                                    (0.3, 0.7, 0.05, 0.5, 2.5, 8.0, 20)])
def test_tables_match_the_oracle(params):
    lam, gamma, delta, rho, c_T, tpn, n_max = params
    cost, dcost = B.smart_cost_tables(lam, gamma, delta, rho, c_T, tpn, n_max)
    r_cost, r_dcost = CM.cost_tables(lam, gamma, delta, rho, c_T, tpn, n_max)
    assert np.allclose(cost, r_cost, rtol=1e-12, atol=0)
    assert math.isinf(dcost[0]) == math.isinf(r_dcost[0])
    assert np.allclose(dcost[1:], r_dcost[1:], rtol=1e-12, atol=0)


def _curve(x, g, d, r):
    return np.array([CM.spec_cost(v, 0.0, g, d, r) for v in x])


@pytest.mark.parametrize("seed", range(6))
def test_fit_reaches_the_oracle_minimum(seed):
    """Different search, same least-squares problem: the library's residual is not worse than the
    oracle's (beyond rounding) and the two fitted curves agree at and between the samples.
    The parameters themselves are compared only where the data identify them."""
    rng = np.random.default_rng(seed)
    x = np.sort(rng.choice(np.arange(8, 2048), size=5 + seed % 3, replace=False)).astype(np.float64)
    gamma, rho = 10 ** rng.uniform(-1, 1.5), rng.uniform(0.6, 2.0)
    delta = math.exp(rng.uniform(math.log(0.05), math.log(8.0))) / x.max() ** rho   # exponent at the largest sample: 0.05 .. 8
    noise = 0.0 if seed % 2 == 0 else 0.02
    t_verify = _curve(x, gamma, delta, rho) * (1 + rng.normal(0, noise, len(x)))
    t_draft = 0.05 * x * (1 + rng.normal(0, noise, len(x)))
    fit = B.smart_fit_cost_models(x, t_draft, t_verify)
    assert fit["lambda"] == pytest.approx(CM.fit_linear(x, t_draft), rel=1e-12)
    g, d, r, sse = CM.fit_exp(x, t_verify)
    scale = float((t_verify * t_verify).sum())
    assert fit["sse"] <= sse + 1e-9 * scale
    dense = np.linspace(x.min(), x.max(), 200)
    lib_curve, ref_curve = _curve(dense, fit["gamma"], fit["delta"], fit["rho"]), _curve(dense, g, d, r)
    assert np.abs(lib_curve - ref_curve).max() <= 2e-3 * ref_curve.max()
    if noise == 0.0:
        assert np.abs(_curve(x, fit["gamma"], fit["delta"], fit["rho"]) - t_verify).max() <= 1e-5 * t_verify.max()
        if delta * x.max() ** rho > 0.5:
            assert fit["rho"] == pytest.approx(rho, rel=5e-3)


def test_cost_model_argument_checks():
    lib = B._lib()
    buf = (ctypes.c_double * 16)()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert lib.smart_cost_tables(0.1, 1.0, 0.01, 1.0, 0.0, 1.0, 4, p, p) == B.SMART_EINVAL      # c_T
    assert lib.smart_cost_tables(0.1, 1.0, 0.01, 0.0, 1.0, 1.0, 4, p, p) == B.SMART_EINVAL      # rho
    assert lib.smart_cost_tables(0.1, 1.0, 0.01, 1.0, 1.0, 1.0, 4, None, p) == B.SMART_EINVAL
    assert lib.smart_cost_tables(0.1, 1.0, 0.01, 1.0, 1.0, 1.0, 4, p, None) == B.SMART_OK
    x = (ctypes.c_double * 3)(1.0, 2.0, 3.0)
    bad = (ctypes.c_double * 3)(1.0, -2.0, 3.0)
    px, pbad = ctypes.cast(x, ctypes.c_void_p), ctypes.cast(bad, ctypes.c_void_p)
    o = [ctypes.byref(ctypes.c_double()) for _ in range(5)]
    assert lib.smart_fit_cost_models(3, px, None, None, *o) == B.SMART_EINVAL
    assert lib.smart_fit_cost_models(2, px, None, px, *o) == B.SMART_EINVAL                       # three parameters
    assert lib.smart_fit_cost_models(3, pbad, None, px, *o) == B.SMART_EINVAL
    assert lib.smart_fit_cost_models(3, px, px, None, None, o[1], o[2], o[3], o[4]) == B.SMART_EINVAL
    assert lib.smart_fit_cost_models(3, px, px, px, *o) == B.SMART_OK


def test_fitted_tables_drive_the_selection_rule():
    """End of the loop on the host: timings -> fit -> tables -> smart_select_tree.  A steeper
    verification cost (a larger batch putting more tokens per node into the pass) must not grow
    the trees (Sec. 1: large batches favour shallower trees), and the library's trees equal the
    oracle's on the same fitted tables."""
    from oracle import selection as OS
    from paper_2604_09731_amd import workloads as W
    x = np.array([64.0, 256.0, 512.0, 1024.0, 2048.0])
    t_verify = _curve(x, 40.0, 4e-4, 1.25)                 # a convex latency curve, in microseconds
    t_draft = 0.01 * x
    fit = B.smart_fit_cost_models(x, t_draft, t_verify)
    w = W.WORKLOADS["cfg3a"].scaled(batch=4)
    forest = W.make_forest(w)
    c_T = 30.0                                              # one plain decoding step of the target, same unit
    sizes = []
    for batch in (1, 8, 32, 128):
        cost, dcost = B.smart_cost_tables(fit["lambda"], fit["gamma"], fit["delta"], fit["rho"], c_T, batch, w.budget)
        cost = cost + 1.0                                   # the step's fixed cost (one target pass) in units of c_T
        got = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost, dcost,
                                  alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
        ref = OS.select_batch(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, list(cost),
                              list(dcost), alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
        assert got["cu_nodes"].tolist() == np.cumsum([0] + [len(t.parent) for t in ref]).tolist()
        assert got["parent"].tolist() == [p for t in ref for p in t.parent]
        sizes.append(int(got["cu_nodes"][-1]))
    assert all(a >= b for a, b in zip(sizes, sizes[1:])) and sizes[0] > sizes[-1]


@pytest.mark.parametrize("params", [(0.02, 0.0, 1.5, 0.002, 1.2, 4.0, 4.0, 32.0, 1, 64), (0.1, 0.3, 3.0, 1e-5, 2.0, 0.7, 1.0, 1.0, 0, 128),
                                    (0.3, 0.0, 0.7, 0.05, 0.5, 2.5, 2.5, 8.0, 2, 20)])
def test_biased_tables_match_the_oracle(params):
    lam, beta, gamma, delta, rho, eta, c_T, tpn, undrafted, n_max = params
    cost, dcost = B.smart_cost_tables_biased(lam, beta, gamma, delta, rho, eta, c_T, tpn, undrafted, n_max)
    r_cost, r_dcost = CM.cost_tables_biased(lam, beta, gamma, delta, rho, eta, c_T, tpn, undrafted, n_max)
    assert np.allclose(cost, r_cost, rtol=1e-12, atol=0)
    inf = np.isinf(r_dcost)
    assert np.array_equal(np.isinf(dcost), inf)
    assert np.allclose(dcost[~inf], np.array(r_dcost)[~inf], rtol=1e-12, atol=0)
    lib = B._lib()
    buf = (ctypes.c_double * (n_max + 2))()
    p = ctypes.cast(buf, ctypes.c_void_p)
    assert lib.smart_cost_tables_biased(lam, -1.0, gamma, delta, rho, eta, c_T, tpn, undrafted, n_max, p, None) == B.SMART_EINVAL
    assert lib.smart_cost_tables_biased(lam, beta, gamma, delta, rho, float("inf"), c_T, tpn, undrafted, n_max, p, None) == B.SMART_EINVAL
    assert lib.smart_cost_tables_biased(lam, beta, gamma, delta, rho, eta, c_T, tpn, -1, n_max, p, None) == B.SMART_EINVAL


def test_draft_and_verify_legs_with_both_marginal_costs():
    """The whole loop of Sec. 3.1 / 3.2 on the host with BOTH cost legs: a linear draft cost (Eq. "linear_model",
    lambda fitted) and a power-exponential verification cost (Eq. "exp_model") measured as extra time over the plain
    step, tables built by the library alone, and the rule run once with the exact finite difference and once with
    the differentiated marginal cost of Eq. "marginal_cost".  Library against the oracle in every leg: the fitted
    lambda, the tables, and the trees, L and R of both runs."""
    from oracle import selection as OS
    from paper_2604_09731_amd import workloads as W
    batch = 32
    n_nodes = np.array([4.0, 8.0, 16.0, 32.0, 64.0])
    x = batch * (n_nodes - 1.0)                              # drafted tokens (the root is not drafted)
    c_T = 80.0
    extra_verify = _curve(x, 25.0, 6e-4, 1.15)              # verification time over the plain step, microseconds
    extra_draft = 0.004 * x                                 # the draft model's time for those tokens
    fit = B.smart_fit_cost_models(x, extra_draft, extra_verify)
    assert fit["lambda"] == pytest.approx(CM.fit_linear(x, extra_draft), rel=1e-12)
    w = W.WORKLOADS["cfg3a"].scaled(batch=6)
    forest = W.make_forest(w)
    cost, dcost = B.smart_cost_tables_biased(fit["lambda"], 0.0, fit["gamma"], fit["delta"], fit["rho"], c_T, c_T, batch, 1, w.budget)
    r_cost, r_dcost = CM.cost_tables_biased(fit["lambda"], 0.0, fit["gamma"], fit["delta"], fit["rho"], c_T, c_T, batch, 1, w.budget)
    assert cost[1] == 1.0 and np.allclose(cost, r_cost, rtol=1e-12, atol=0)
    sizes = {}
    for name, marginal, r_marginal in (("difference", None, None), ("derivative", dcost, list(r_dcost))):
        got = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost, marginal,
                                  alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
        ref = OS.select_batch(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, list(r_cost),
                              r_marginal, alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
        assert got["cu_nodes"].tolist() == np.cumsum([0] + [len(t.parent) for t in ref]).tolist()
        assert got["parent"].tolist() == [p for t in ref for p in t.parent]
        assert np.allclose(got["L"], [t.L for t in ref], rtol=0, atol=0) and np.allclose(got["R"], [t.R for t in ref], rtol=1e-15)
        sizes[name] = np.diff(got["cu_nodes"])
    # the derivative at n nodes is below the step to n + 1 nodes of a convex cost, so it can only let more nodes in
    assert (sizes["derivative"] >= sizes["difference"]).all()
    # the draft leg matters: without it the trees are at least as large
    cost_nd, _ = B.smart_cost_tables_biased(0.0, 0.0, fit["gamma"], fit["delta"], fit["rho"], c_T, c_T, batch, 1, w.budget)
    no_draft = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost_nd, None,
                                   alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
    assert (np.diff(no_draft["cu_nodes"]) >= sizes["difference"]).all()
