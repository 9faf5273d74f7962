"""Pins of the cost-model oracle: closed forms, derivative identities, exact recovery."""
import math

import numpy as np
import pytest

from oracle import cost_model as CM


def test_cost_and_marginal_closed_forms():
    # rho = 1: C(x) = lam x + gamma (e^{delta x} - 1), dC = lam + gamma delta e^{delta x}
    lam, gamma, delta = 0.25, 3.0, 0.01
    for x in (0.0, 1.0, 17.0, 300.0):
        assert CM.spec_cost(x, lam, gamma, delta, 1.0) == pytest.approx(lam * x + gamma * (math.exp(delta * x) - 1), rel=1e-13)
        assert CM.spec_marginal(x, lam, gamma, delta, 1.0) == pytest.approx(lam + gamma * delta * math.exp(delta * x), rel=1e-13)
    # through the origin (both biases are zero in the paper)
    assert CM.spec_cost(0.0, 1.0, 2.0, 3.0, 0.7) == 0.0
    # small exponents: the model is gamma delta x^rho to first order
    assert CM.spec_cost(2.0, 0.0, 5.0, 1e-9, 1.5) == pytest.approx(5.0 * 1e-9 * 2.0 ** 1.5, rel=1e-8)


@pytest.mark.parametrize("rho", [0.6, 1.0, 1.7])
def test_marginal_is_the_derivative(rho):
    lam, gamma, delta = 0.1, 2.0, 0.003
    for x in (3.0, 40.0, 200.0):
        h = 1e-5 * x
        num = (CM.spec_cost(x + h, lam, gamma, delta, rho) - CM.spec_cost(x - h, lam, gamma, delta, rho)) / (2 * h)
        assert CM.spec_marginal(x, lam, gamma, delta, rho) == pytest.approx(num, rel=1e-6)


def test_tables_units_batch_scaling_and_edges():
    lam, gamma, delta, rho, c_T = 0.02, 1.5, 0.002, 1.2, 4.0
    cost, dcost = CM.cost_tables(lam, gamma, delta, rho, c_T, 32.0, 10)
    assert len(cost) == 12 and len(dcost) == 11 and cost[0] == 0.0
    # a tree of n nodes in a batch of 32 puts 32 n tokens into the pass; costs are in units of c_T
    assert cost[3] == pytest.approx(CM.spec_cost(96.0, lam, gamma, delta, rho) / c_T, rel=1e-14)
    # per-node marginal = 32 x per-token derivative; it sits between the neighbouring finite differences (convex model)
    for n in range(1, 10):
        assert cost[n] - cost[n - 1] < dcost[n] < cost[n + 1] - cost[n]
    # rho < 1: the derivative at zero tokens is infinite, and finite from the root on
    _, d2 = CM.cost_tables(lam, gamma, delta, 0.5, c_T, 1.0, 3)
    assert math.isinf(d2[0]) and all(math.isfinite(v) for v in d2[1:])


def test_linear_fit_is_the_normal_equation():
    rng = np.random.default_rng(0)
    x = np.array([8.0, 16.0, 32.0, 64.0, 128.0])
    t = 0.37 * x + rng.normal(0, 0.5, 5)
    lam = CM.fit_linear(x, t)
    ref = np.linalg.lstsq(x[:, None], t, rcond=None)[0][0]
    assert lam == pytest.approx(ref, rel=1e-12)
    assert CM.fit_linear(x, 0.37 * x) == pytest.approx(0.37, rel=1e-14)


@pytest.mark.parametrize("gamma,delta,rho", [(2.0, 0.004, 1.3), (0.5, 0.02, 0.9), (10.0, 1e-4, 1.8)])
def test_exp_fit_recovers_noiseless_data(gamma, delta, rho):
    """Five points, as the paper profiles; data made from the model itself must be
    reproduced (residual ~ 0) and, where the exponent is large enough for the three
    parameters to be identifiable, recovered."""
    x = np.array([16.0, 64.0, 128.0, 256.0, 512.0])
    t = np.array([CM.spec_cost(v, 0.0, gamma, delta, rho) for v in x])
    g, d, r, sse = CM.fit_exp(x, t)
    pred = np.array([CM.spec_cost(v, 0.0, g, d, r) for v in x])
    assert np.abs(pred - t).max() <= 1e-6 * t.max()
    if delta * x.max() ** rho > 0.5:
        assert r == pytest.approx(rho, rel=1e-3) and d == pytest.approx(delta, rel=2e-2) and g == pytest.approx(gamma, rel=2e-2)


def test_exp_fit_beats_every_grid_point_on_noisy_data():
    rng = np.random.default_rng(3)
    x = np.array([32.0, 64.0, 128.0, 256.0, 512.0, 1024.0])
    t = np.array([CM.spec_cost(v, 0.0, 3.0, 0.002, 1.1) for v in x]) * (1 + rng.normal(0, 0.03, len(x)))
    g, d, r, sse = CM.fit_exp(x, t)
    resid = np.array([CM.spec_cost(v, 0.0, g, d, r) for v in x]) - t
    assert float((resid * resid).sum()) == pytest.approx(sse, rel=1e-9)
    xm = x.max()
    for rho in np.linspace(0.1, 3.9, 39):
        for s in np.exp(np.linspace(math.log(1e-5), math.log(30.0), 60)):
            grid_sse, _ = CM._reduced(x, t, s / xm ** rho, rho)
            assert sse <= grid_sse * (1 + 1e-9)


def test_biased_tables_closed_forms_and_reductions():
    """The tables with the bias terms of Eqs. "linear_model" / "exp_model" kept and the root left out of the
    drafted tokens: pinned to hand-evaluated closed forms (rho = 1), to the unbiased tables they reduce to,
    and to the shift by one node."""
    lam, gamma, delta, c_T, b = 0.25, 3.0, 0.01, 2.0, 4.0
    cost, dcost = CM.cost_tables_biased(lam, 0.5, gamma, delta, 1.0, 2.0, c_T, b, 1, 6)
    assert len(cost) == 8 and len(dcost) == 7
    # n = 0 and n = 1 (only the root): no drafted token, the biases alone
    assert cost[0] == pytest.approx((0.5 + 2.0) / c_T, rel=1e-15) and cost[1] == cost[0]
    # n = 4: x = 4 (4 - 1) = 12 drafted tokens
    assert cost[4] == pytest.approx((0.25 * 12 + 0.5 + 3.0 * (math.exp(0.12) - 1.0) + 2.0) / c_T, rel=1e-14)
    assert dcost[4] == pytest.approx(b * (0.25 + 3.0 * 0.01 * math.exp(0.12)) / c_T, rel=1e-14)
    # zero biases, every node drafted: the unbiased tables
    c0, d0 = CM.cost_tables(lam, gamma, delta, 1.3, c_T, b, 9)
    c1, d1 = CM.cost_tables_biased(lam, 0.0, gamma, delta, 1.3, 0.0, c_T, b, 0, 9)
    assert c0 == c1 and d0 == d1
    # leaving the root out shifts the unbiased tables by one node and adds the constant
    c2, d2 = CM.cost_tables_biased(lam, 0.0, gamma, delta, 1.3, c_T, c_T, b, 1, 8)
    assert all(c2[n] == pytest.approx(1.0 + c0[n - 1], rel=1e-14) for n in range(1, 10))
    assert all(d2[n] == pytest.approx(d0[n - 1], rel=1e-14) for n in range(1, 9))
    # a plain step costs exactly one unit when eta = c_T: R(root only) = 1
    assert c2[1] == 1.0
    # rho < 1: infinite marginal cost where nothing is drafted yet
    _, d3 = CM.cost_tables_biased(lam, 0.0, gamma, delta, 0.5, c_T, c_T, b, 1, 3)
    assert math.isinf(d3[0]) and math.isinf(d3[1]) and all(math.isfinite(v) for v in d3[2:])
