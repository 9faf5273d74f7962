"""CPU oracle: the paper's device cost models.  TEST INFRASTRUCTURE ONLY.

Sec. 3.1 ("Cost Modeling") models the draft cost of a tree of x drafted tokens
as a line through the origin (Eq. "linear_model", beta = 0) and the
verification cost as a power-exponential through the origin (Eq. "exp_model",
eta = 0):

    C_draft(x)  = lambda * x
    C_verify(x) = gamma * (exp(delta * x**rho) - 1)

with parameters fitted for each device from a handful of timed forward passes.  Sec. 3.2 then
takes the marginal cost of one more node as the derivative of their sum
(Eq. "marginal_cost"):

    dC(x) = lambda + gamma * delta * rho * x**(rho - 1) * exp(delta * x**rho)

The paper does not say how the fit is computed; a least-squares fit is taken
here (minimum of the summed squared residuals), and this file finds it the slow
way: gamma in closed form for every (delta, rho) of a dense grid, then a
simplex polish of the best grid points.
"""
from __future__ import annotations

import math

import numpy as np


def spec_cost(x, lam, gamma, delta, rho):
    """C_draft(x) + C_verify(x), Eqs. "linear_model" + "exp_model" with zero biases."""
    return lam * x + gamma * math.expm1(delta * x ** rho)


def spec_marginal(x, lam, gamma, delta, rho):
    """Eq. "marginal_cost": d/dx of spec_cost."""
    return lam + gamma * delta * rho * x ** (rho - 1.0) * math.exp(delta * x ** rho)


def cost_tables(lam, gamma, delta, rho, c_T, tokens_per_node, n_max):
    """The tables smart_select_tree takes, in units of c_T (Eq. "definition"):
    cost[n] for n = 0 .. n_max + 1 and dcost[n] for n = 0 .. n_max, for trees of n
    nodes that put x = tokens_per_node * n tokens into the forward pass
    (tokens_per_node = batch size when a batch verifies together and every
    sequence assumes the same tree size).  dcost is per NODE: tokens_per_node
    times the per-token derivative.  dcost[0] is +inf for rho < 1 (never used:
    a tree has at least its root)."""
    cost = [spec_cost(tokens_per_node * n, lam, gamma, delta, rho) / c_T for n in range(n_max + 2)]
    dcost = []
    for n in range(n_max + 1):
        x = tokens_per_node * n
        if x == 0.0 and rho < 1.0:
            dcost.append(math.inf)
        else:
            dcost.append(tokens_per_node * spec_marginal(x, lam, gamma, delta, rho) / c_T)
    return cost, dcost


def cost_tables_biased(lam, beta, gamma, delta, rho, eta, c_T, tokens_per_node, undrafted_nodes, n_max):
    """The same tables with the bias terms of Eqs. "linear_model" and "exp_model" kept (the paper
    sets both to zero when it fits whole forward passes; a cost that is measured as the extra time
    over a plain decoding step needs them: eta = c_T, beta = 0) and with the nodes that are not
    drafted (the root, which every verification step carries anyway) left out of the token count:

        x(n)     = tokens_per_node * max(n - undrafted_nodes, 0)
        cost[n]  = (lambda x + beta + gamma (exp(delta x**rho) - 1) + eta) / c_T
        dcost[n] = tokens_per_node * (lambda + gamma delta rho x**(rho-1) exp(delta x**rho)) / c_T

    (dcost at x = 0 with rho < 1: +inf.)"""
    def x_of(n):
        return tokens_per_node * max(n - undrafted_nodes, 0)
    cost = [(spec_cost(x_of(n), lam, gamma, delta, rho) + beta + eta) / c_T for n in range(n_max + 2)]
    dcost = []
    for n in range(n_max + 1):
        x = x_of(n)
        if x == 0.0 and rho < 1.0:
            dcost.append(math.inf)
        else:
            dcost.append(tokens_per_node * spec_marginal(x, lam, gamma, delta, rho) / c_T)
    return cost, dcost


def fit_linear(x, t):
    """Least squares for t ~ lambda * x (a line through the origin)."""
    x = np.asarray(x, np.float64)
    t = np.asarray(t, np.float64)
    return float((x * t).sum() / (x * x).sum())


def _reduced(x, t, delta, rho):
    """For fixed (delta, rho) the best gamma is linear least squares; returns (sse, gamma)."""
    f = np.expm1(delta * x ** rho)
    ff = float((f * f).sum())
    if not np.isfinite(ff) or ff <= 0.0:
        return math.inf, 0.0
    gamma = float((f * t).sum() / ff)
    r = gamma * f - t
    return float((r * r).sum()), gamma


def fit_exp(x, t, rho_range=(0.05, 4.0), exponent_range=(1e-6, 40.0)):
    """Least-squares fit of t ~ gamma * (exp(delta * x**rho) - 1).

    The search runs over rho and over s = delta * max(x)**rho, the exponent at the
    largest sample (so the grid is scale-free).  Returns (gamma, delta, rho, sse)."""
    from scipy.optimize import minimize
    x = np.asarray(x, np.float64)
    t = np.asarray(t, np.float64)
    xm = float(x.max())
    rhos = np.linspace(rho_range[0], rho_range[1], 160)
    ss = np.exp(np.linspace(math.log(exponent_range[0]), math.log(exponent_range[1]), 240))
    grid = []
    for rho in rhos:
        for s in ss:
            sse, _ = _reduced(x, t, s / xm ** rho, rho)
            grid.append((sse, rho, s))
    grid.sort()
    best = None
    for sse0, rho0, s0 in grid[:8]:
        def obj(p):
            rho, ls = p
            if not (rho_range[0] <= rho <= rho_range[1]):
                return 1e300
            s = math.exp(ls)
            if not (exponent_range[0] <= s <= exponent_range[1]):
                return 1e300
            return _reduced(x, t, s / xm ** rho, rho)[0]
        res = minimize(obj, [rho0, math.log(s0)], method="Nelder-Mead",
                       options={"xatol": 1e-10, "fatol": 1e-18, "maxiter": 4000})
        cand = (min(res.fun, sse0), res.x[0], math.exp(res.x[1])) if res.fun <= sse0 else (sse0, rho0, s0)
        if best is None or cand[0] < best[0]:
            best = cand
    sse, rho, s = best
    delta = s / xm ** rho
    _, gamma = _reduced(x, t, delta, rho)
    return gamma, delta, rho, sse
