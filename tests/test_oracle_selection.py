"""Pins for the selection oracle (CPU only).

The paper gives no worked numeric example of Algorithm 1, so the oracle is
pinned to (i) exhaustive search of Eq. "optimization" on tiny forests, where
the node-by-node rule with alpha = 1, exact marginals and a convex cost is
provably optimal, (ii) the acceptance-length identity below Eq. "cum_prob",
checked by enumerating every verification outcome through the accept walk,
(iii) the decision rule Eq. "decision_rule" re-evaluated on the finished
tree, and (iv) the termination conditions and monotonic trends of Sec. 3.2.
"""
import itertools

import numpy as np
import pytest

from oracle import pack_accept as PA
from oracle import selection as S
from paper_2604_09731_amd import workloads as W


def tiny_forest(seed, k=2, d=3):
    rng = np.random.default_rng(seed)
    parent, prob, depth = [-1], [1.0], [0]
    i = 0
    while i < len(parent):
        if depth[i] < d:
            p = rng.dirichlet(np.ones(k + 1))[:k]       # leaves mass for "other token"
            for j in np.argsort(-p):
                parent.append(i)
                prob.append(float(p[j]))
                depth.append(depth[i] + 1)
        i += 1
    token = list(range(100, 100 + len(parent)))
    return parent, prob, token


COSTS = {
    "linear": lambda n: 1.0 + 0.05 * n,
    "knee": lambda n: 1.0 + 0.01 * n + 0.2 * max(0, n - 5),
    "powexp": lambda n: 0.3 * n * 0.02 + 1.0 + 2.0 * (np.exp(0.002 * n ** 1.7) - 1.0),
}


@pytest.mark.parametrize("cost_name", list(COSTS))
@pytest.mark.parametrize("seed", range(12))
def test_best_first_alpha1_matches_exhaustive_search(cost_name, seed):
    parent, prob, token = tiny_forest(seed)            # 14 non-root candidates
    cost = [float(COSTS[cost_name](n)) for n in range(len(parent) + 2)]
    t = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=3, budget=len(parent))
    R_star, best_sets = S.brute_force_best(parent, prob, cost, max_depth=3, budget=len(parent))
    assert abs(t.R - R_star) <= 1e-12 * R_star
    assert tuple(sorted(t.cand_index)) in best_sets
    # and the expected acceptance the greedy reports is the plain sum over chosen nodes
    P, _ = S.path_prob_and_depth(parent, prob)
    assert abs(t.L - sum(P[u] for u in t.cand_index)) < 1e-12


@pytest.mark.parametrize("seed", range(6))
def test_budget_and_depth_constrained_optimum(seed):
    parent, prob, token = tiny_forest(seed)
    cost = [1.0 + 0.01 * n for n in range(len(parent) + 2)]
    for budget, depth in [(1, 3), (4, 3), (6, 2), (15, 1)]:
        t = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=depth, budget=budget)
        R_star, _ = S.brute_force_best(parent, prob, cost, max_depth=depth, budget=budget)
        assert len(t) <= budget
        _, dep = S.path_prob_and_depth(parent, prob)
        assert all(dep[u] <= depth for u in t.cand_index)
        assert abs(t.R - R_star) <= 1e-12 * R_star


def _expected_emitted_tokens_by_enumeration(node_parent, node_cond_prob, node_token):
    """Every node's verification outcome is independent: the target continues
    with child c with probability p(c), or with a token no child carries.
    Enumerate the product space, run the accept walk, average emitted tokens."""
    n = len(node_parent)
    kids = [[] for _ in range(n)]
    for j in range(1, n):
        kids[node_parent[j]].append(j)
    options = []
    for i in range(n):
        opts = [(node_token[c], node_cond_prob[c]) for c in kids[i]]
        opts.append((-7, 1.0 - sum(p for _, p in opts)))
        options.append(opts)
    total = 0.0
    for combo in itertools.product(*options):
        pr = 1.0
        for _, p in combo:
            pr *= p
        if pr == 0.0:
            continue
        target_next = [tok for tok, _ in combo]
        alen, _, _ = PA.accept([0, n], node_parent, node_token, target_next, max_depth=n)
        total += pr * (alen[0] + 1)
    return total


@pytest.mark.parametrize("seed", range(5))
def test_L_is_the_expected_number_of_emitted_tokens(seed):
    parent, prob, token = tiny_forest(seed, k=2, d=2)   # 6 candidates
    cost = [1.0 + 0.02 * n for n in range(len(parent) + 2)]
    t = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=2, budget=6)
    assert len(t) >= 3
    cond = [prob[u] for u in t.cand_index]
    expect = _expected_emitted_tokens_by_enumeration(t.parent, cond, t.token)
    assert abs(t.L - expect) < 1e-12


def test_rule_holds_for_every_kept_node_and_fails_at_the_stop():
    w = W.WORKLOADS["cfg2"].scaled(batch=3)
    f = W.make_forest(w)
    cost = W.cost_table(w)
    for alpha in (1.0, 0.8, 0.5):
        for b in range(w.batch):
            lo, hi = f.cand_cu[b], f.cand_cu[b + 1]
            par, pr = f.cand_parent[lo:hi].tolist(), f.cand_prob[lo:hi].tolist()
            t = S.select_tree(par, pr, f.cand_token[lo:hi], cost, alpha=alpha,
                              max_depth=w.max_depth, budget=w.budget)
            P, dep = S.path_prob_and_depth(par, pr)
            L = 1.0
            for n in range(1, len(t)):
                u = t.cand_index[n]
                dC = cost[n + 1] - cost[n]
                assert alpha * P[u] / dC > L / cost[n]           # Eq. "decision_rule"
                if alpha == 1.0:                                  # exact: reward strictly rises
                    assert (L + P[u]) / cost[n + 1] > L / cost[n]
                L += P[u]
            # stop: the best remaining frontier candidate fails the rule (or budget/none left)
            chosen = set(t.cand_index)
            frontier = [u for u in range(1, len(par)) if u not in chosen and par[u] in chosen
                        and dep[u] <= w.max_depth]
            if frontier and len(t) < w.budget:
                u = max(frontier, key=lambda x: (P[x], -x))
                n = len(t)
                assert not (alpha * P[u] / (cost[n + 1] - cost[n]) > t.L / cost[n])
            # node ids are a topological order and path probabilities are products
            for i in range(1, len(t)):
                assert 0 <= t.parent[i] < i
                assert t.pathprob[i] == t.pathprob[t.parent[i]] * pr[t.cand_index[i]]


def test_trends_alpha_scale_flat_and_steep_costs():
    w = W.WORKLOADS["cfg2"].scaled(batch=2)
    f = W.make_forest(w)
    cost = W.cost_table(w)
    lo, hi = f.cand_cu[0], f.cand_cu[1]
    par, pr, tok = f.cand_parent[lo:hi].tolist(), f.cand_prob[lo:hi].tolist(), f.cand_token[lo:hi]
    prev = None
    for alpha in (0.4, 0.6, 0.8, 1.0):            # smaller alpha prunes more, nested trees
        t = S.select_tree(par, pr, tok, cost, alpha=alpha, max_depth=8, budget=128)
        if prev is not None:
            assert prev == t.cand_index[:len(prev)]
        prev = list(t.cand_index)
    t1 = S.select_tree(par, pr, tok, cost, alpha=0.8, max_depth=8, budget=128)
    t2 = S.select_tree(par, pr, tok, cost * 4.0, alpha=0.8, max_depth=8, budget=128)
    assert t1.cand_index == t2.cand_index and abs(t1.R - 4.0 * t2.R) < 1e-12   # scale invariance
    flat = W.cost_table(w, name="flat")
    t3 = S.select_tree(par, pr, tok, flat, alpha=0.8, max_depth=8, budget=20)
    P, _ = S.path_prob_and_depth(par, pr)
    top = sorted(range(len(par)), key=lambda u: (-P[u], u))[:20]
    assert len(t3) == 20 and t3.cand_index == top       # fills the budget in P order
    steep = np.array([1.0 + 10.0 * n for n in range(130)])
    assert len(S.select_tree(par, pr, tok, steep, alpha=0.8, max_depth=8, budget=128)) == 1
    # larger batches shrink the trees (cost of the batch-wide token count has a knee)
    w3 = W.WORKLOADS["cfg3a"]
    sizes = []
    for batch in (1, 8, 32):
        wb = w3.scaled(batch=batch)
        sizes.append(len(S.select_tree(par, pr, tok, W.cost_table(wb), alpha=0.8, max_depth=8, budget=64)))
    assert sizes[0] >= sizes[1] >= sizes[2] and sizes[0] > sizes[2]


def test_derivative_marginal_table_is_used_when_given():
    parent, prob, token = tiny_forest(3)
    lam, gam, delta, rho = 0.01, 1.0, 0.01, 1.5          # Eqs. "linear_model", "exp_model"
    cost = [lam * n + gam * (np.exp(delta * n ** rho) - 1.0) + 1.0 for n in range(len(parent) + 2)]
    dcost = [lam + gam * delta * rho * max(n, 1) ** (rho - 1) * np.exp(delta * n ** rho)
             for n in range(len(parent) + 1)]              # Eq. "marginal_cost"
    t_fd = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=3, budget=15)
    t_d = S.select_tree(parent, prob, token, cost, dcost, alpha=1.0, max_depth=3, budget=15)
    # the derivative under-estimates the finite difference of a convex cost: never a smaller tree
    assert len(t_d) >= len(t_fd)
    assert t_d.cand_index[:len(t_fd)] == t_fd.cand_index
    huge = [1e9] * len(dcost)
    assert len(S.select_tree(parent, prob, token, cost, huge, alpha=1.0, max_depth=3, budget=15)) == 1


@pytest.mark.parametrize("dilution", [S.DILUTION_NONE, S.DILUTION_PATH_MEAN])
@pytest.mark.parametrize("seed", range(6))
def test_layerwise_schedule_frozen_terms_termination_and_bound(seed, dilution):
    parent, prob, token = tiny_forest(seed)
    cost = [1.0 + 0.03 * n for n in range(len(parent) + 2)]
    P, dep = S.path_prob_and_depth(parent, prob)
    for budget in (15, 6, 1):
        t = S.select_tree(parent, prob, token, cost, alpha=0.9, max_depth=3, budget=budget,
                          schedule=S.LAYERWISE, dilution=dilution)
        assert 1 <= len(t) <= budget                     # Eq. "optimization": |S| <= B
        R_star, _ = S.brute_force_best(parent, prob, cost, max_depth=3, budget=budget, dilution=dilution)
        assert t.R <= R_star * (1 + 1e-12)               # greedy is not globally optimal
        # replay layer by layer: every kept node passed the rule against its layer's frozen terms
        ids = t.cand_index
        layer_of = [dep[u] for u in ids]
        assert layer_of == sorted(layer_of)
        for layer in range(1, max(layer_of) + 1 if len(ids) > 1 else 1):
            prev_nodes = [i for i in range(len(ids)) if layer_of[i] < layer]
            n = len(prev_nodes)
            if dilution == S.DILUTION_NONE:
                L, paths = sum(t.pathprob[i] for i in prev_nodes), 1
            else:
                L, paths = S.path_mean_L([t.parent[i] for i in prev_nodes],
                                         [t.pathprob[i] for i in prev_nodes])
            for i in range(len(ids)):
                if layer_of[i] == layer:
                    ben = P[ids[i]] / paths
                    assert 0.9 * ben / (cost[n + 1] - cost[n]) > L / cost[n] * (1 - 1e-12)
                    assert layer_of[t.parent[i]] == layer - 1


def test_path_mean_L_matches_the_printed_formula_on_a_hand_tree():
    # root(1.0) -> a(0.5) -> c(0.25); root -> b(0.25).  Paths: root-a-c, root-b.
    # Eq. "expected_acc_length": ((1 + .5 + .25) + (1 + .25)) / 2 = 1.5
    L, paths = S.path_mean_L([-1, 0, 0, 1], [1.0, 0.5, 0.25, 0.25])
    assert paths == 2 and L == 1.5
    assert S.path_mean_L([-1], [1.0]) == (1.0, 1)


def test_relabelled_forest_selects_the_same_set():
    w = W.WORKLOADS["cfg4"].scaled(batch=1)
    f = W.make_forest(w)
    par, pr, tok = f.cand_parent.tolist(), f.cand_prob.tolist(), f.cand_token.tolist()
    C = len(par)
    rng = np.random.default_rng(0)
    placed, order = set(), []
    while len(order) < C:
        ready = [i for i in range(C) if i not in placed and (par[i] < 0 or par[i] in placed)]
        pick = 0 if not order else int(rng.choice(ready))
        placed.add(pick)
        order.append(pick)
    new_of_old = {o: i for i, o in enumerate(order)}
    par2 = [-1 if par[o] < 0 else new_of_old[par[o]] for o in order]
    pr2 = [pr[o] for o in order]
    tok2 = [tok[o] for o in order]
    cost = W.cost_table(w)
    t1 = S.select_tree(par, pr, tok, cost, alpha=0.8, max_depth=6, budget=96)
    t2 = S.select_tree(par2, pr2, tok2, cost, alpha=0.8, max_depth=6, budget=96)
    assert sorted(t1.cand_index) == sorted(order[i] for i in t2.cand_index)


def _hand_worked():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "selection_hand_worked.json")) as f:
        return json.load(f)


def test_hand_worked_example_oracle():
    """Decisions, node order, L and R of a forest worked by hand from the paper's equations
    (tests/golden/selection_hand_worked.json, all numbers dyadic: exact in binary64)."""
    g = _hand_worked()
    fo = g["forest"]
    P, _ = S.path_prob_and_depth(fo["parent"], fo["prob"])
    assert P == fo["path_prob"]
    cost = [1.0 + n / 8.0 for n in range(9)]
    for case in g["cases"]:
        t = S.select_tree(fo["parent"], fo["prob"], fo["token"], cost, alpha=case["alpha"], max_depth=g["max_depth"],
                          budget=g["budget"], schedule=getattr(S, case["schedule"]),
                          dilution=getattr(S, "DILUTION_" + case["dilution"]))
        assert t.cand_index == case["cand_index"], case["name"]
        assert t.parent == case["parent"], case["name"]
        assert t.token == [fo["token"][i] for i in case["cand_index"]]
        assert t.L == case["L"] and t.R == case["R"], case["name"]


# ---------------------------------------------------------------------------
# Algorithm 1 one layer at a time
# ---------------------------------------------------------------------------
def _stepwise(parent, prob, token, cost, dcost=None, alpha=0.8, max_depth=8, budget=64, dilution=S.DILUTION_NONE):
    from tests.helpers import drive_layers
    st = S.LayerState(token[0], cost)
    cand = drive_layers(parent, max_depth, lambda ids, par_nodes: S.select_layer(
        st, par_nodes, [prob[u] for u in ids], [token[u] for u in ids], cost, dcost, alpha=alpha,
        budget=budget, dilution=dilution))
    return st, cand


def test_hand_worked_example_layer_at_a_time():
    """The layer-wise cases of the hand-worked forest, fed one layer at a time."""
    g = _hand_worked()
    fo = g["forest"]
    cost = [1.0 + n / 8.0 for n in range(9)]
    seen = 0
    for case in g["cases"]:
        if case["schedule"] != "LAYERWISE":
            continue
        seen += 1
        st, cand = _stepwise(fo["parent"], fo["prob"], fo["token"], cost, alpha=case["alpha"],
                             max_depth=g["max_depth"], budget=g["budget"],
                             dilution=getattr(S, "DILUTION_" + case["dilution"]))
        assert cand == case["cand_index"] and st.parent == case["parent"], case["name"]
        assert st.token == [fo["token"][i] for i in case["cand_index"]]
        assert st.L == case["L"] and st.R == case["R"], case["name"]
    assert seen >= 1


@pytest.mark.parametrize("dilution", [S.DILUTION_NONE, S.DILUTION_PATH_MEAN])
@pytest.mark.parametrize("seed", range(8))
def test_layer_at_a_time_equals_the_whole_forest_schedule(seed, dilution):
    """Algorithm 1 looks at one layer per iteration, so running it on a forest known in advance
    and on layers that arrive one by one must give the same tree, bit for bit, also when the
    budget cuts a layer and when the depth cap ends the loop."""
    parent, prob, token = tiny_forest(seed, k=3, d=4)
    cost = [1.0 + 0.01 * n + 0.002 * n * n for n in range(130)]
    dcost = [0.01 + 0.004 * n for n in range(129)] if seed % 2 else None
    for budget, max_depth in ((128, 4), (9, 4), (4, 4), (1, 4), (40, 2)):
        t = S.select_tree(parent, prob, token, cost, dcost, alpha=0.9, max_depth=max_depth, budget=budget,
                          schedule=S.LAYERWISE, dilution=dilution)
        st, cand = _stepwise(parent, prob, token, cost, dcost, alpha=0.9, max_depth=max_depth, budget=budget,
                             dilution=dilution)
        assert cand == t.cand_index and st.parent == t.parent and st.token == t.token
        assert st.pathprob == t.pathprob and st.L == t.L and st.R == t.R


def test_one_layer_against_exact_rational_arithmetic():
    """One layer on dyadic inputs, decided again in exact fractions: the kept set is
    {c : alpha P(c) / dC > L / cost[n]}, cut to the room the budget leaves by largest P."""
    from fractions import Fraction as F
    cost = [1.0 + n / 8.0 for n in range(12)]
    st = S.LayerState(7, cost)
    out = S.select_layer(st, [0, 0, 0, 0], [0.5, 0.25, 0.125, 0.0625], [1, 2, 3, 4], cost, alpha=0.5, budget=8)
    # threshold L / cost[1] = 1 / 1.125 = 8/9; alpha p / 0.125 = 4 p: 2, 1, 0.5, 0.25
    assert out == [1, 2, -1, -1] and st.L == 1.75 and st.layer_begin == 1 and len(st) == 3
    cands = [(1, 0.5), (1, 0.5), (2, 0.75), (2, 0.25), (1, 0.125)]
    P = [F(st.pathprob[p]) * F(q) for p, q in cands]
    thr = F(st.L) / F(cost[3])
    passing = [c for c in range(5) if F(1) * P[c] / (F(cost[4]) - F(cost[3])) > thr]
    assert passing == [0, 1, 2]                                        # 2, 2, 1.5 > 14/11 > 0.5, 0.5
    room = 2
    expect = sorted(sorted(passing, key=lambda c: (-P[c], c))[:room])
    out = S.select_layer(st, [p for p, _ in cands], [q for _, q in cands], [5, 6, 7, 8, 9], cost, alpha=1.0,
                         budget=len(st) + room)
    assert [c for c in range(5) if out[c] >= 0] == expect == [0, 1]     # P = 0.1875 goes, the tie at 0.25 stays
    assert [out[c] for c in expect] == [3, 4] and st.layer_begin == 3
    # a full tree accepts nothing more and has no active layer left
    out = S.select_layer(st, [3], [1.0], [1], cost, alpha=1.0, budget=len(st))
    assert out == [-1] and st.layer_begin == len(st) == 5
    with pytest.raises(ValueError):
        S.select_layer(st, [3], [1.0], [1], cost, budget=8)            # node 3 is not in the newest layer


# ---------------------------------------------------------------------------
# The likelihood-maximising baseline policy
# ---------------------------------------------------------------------------
def _baseline_hand_worked():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "baseline_hand_worked.json")) as f:
        return json.load(f)


def test_baseline_policy_hand_worked_example_oracle():
    g = _baseline_hand_worked()
    fo = g["forest"]
    P, _ = S.path_prob_and_depth(fo["parent"], fo["prob"])
    assert P == fo["path_prob"]
    cost = [1.0 + n / 8.0 for n in range(70)]
    for case in g["cases"]:
        t = S.baseline_tree(fo["parent"], fo["prob"], fo["token"], cost, k=case["k"],
                            max_depth=case.get("max_depth", g["max_depth"]), g=case["g"])
        assert t.cand_index == case["cand_index"] and t.parent == case["parent"], case["name"]
        assert t.token == [fo["token"][i] for i in case["cand_index"]]
        assert t.L == case["L"] and t.R == case["R"], case["name"]


@pytest.mark.parametrize("seed", range(6))
def test_baseline_policy_properties(seed):
    parent, prob, token = tiny_forest(seed, k=3, d=4)
    P, dep = S.path_prob_and_depth(parent, prob)
    cost = [1.0 + 0.05 * n for n in range(len(parent) + 2)]
    C = len(parent)
    # expanding everything and keeping everything returns the whole forest down to the depth cap
    t = S.baseline_tree(parent, prob, token, cost, k=C, max_depth=3, g=C)
    assert sorted(t.cand_index) == [u for u in range(C) if dep[u] <= 3]
    for k, g in ((2, 5), (3, 9), (1, 4), (2, 100)):
        t = S.baseline_tree(parent, prob, token, cost, k=k, max_depth=4, g=g)
        kept = set(t.cand_index)
        assert all(parent[u] in kept for u in kept if u)                       # a tree
        # what the expansion phase generates, by a recursion of its own: a node is generated iff its parent
        # is the root or was among its layer's k best generated nodes
        gen_by_layer, expanded = {}, {0}
        for layer in range(1, 5):
            gen = [u for u in range(1, C) if dep[u] == layer and parent[u] in expanded]
            gen_by_layer[layer] = gen
            expanded = set(sorted(gen, key=lambda u: (-P[u], u))[:k])
        generated = [u for gen in gen_by_layer.values() for u in gen]
        assert kept - {0} <= set(generated) and len(kept) - 1 == min(g, len(generated))
        # nothing left out is better than anything kept
        worst_kept = min((P[u], -u) for u in kept - {0})
        assert all((P[u], -u) < worst_kept for u in generated if u not in kept)
        assert abs(t.L - sum(P[u] for u in kept)) < 1e-12 and t.R == t.L / cost[len(kept)]
        dl = [dep[u] for u in t.cand_index]
        assert dl == sorted(dl)                                                # numbered layer by layer


def test_smart_never_loses_to_the_baseline_in_modelled_speedup_when_the_rule_is_optimal():
    """With alpha = 1, exact marginals and a convex cost the node-by-node rule maximises R over all
    parent-closed subsets (pinned above by exhaustive search), so no tree the baseline policy keeps can
    have a larger modelled speedup."""
    for seed in range(8):
        parent, prob, token = tiny_forest(seed, k=3, d=4)
        cost = [1.0 + 0.02 * n + 0.004 * n * n for n in range(len(parent) + 2)]
        smart = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=4, budget=len(parent))
        for k, g in ((2, 8), (3, 20), (3, 60)):
            base = S.baseline_tree(parent, prob, token, cost, k=k, max_depth=4, g=g)
            assert smart.R >= base.R * (1 - 1e-12)


# ---------------------------------------------------------------------------
# Cartesian-product candidate forest (drafter with independent positions)
# ---------------------------------------------------------------------------
def _product_hand_worked():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "product_forest_hand_worked.json")) as f:
        return json.load(f)


def test_product_forest_hand_worked_example_oracle():
    g = _product_hand_worked()
    for cap in range(1, 8):
        parent, prob, token, P = S.product_forest(g["pos_prob"], g["pos_token"], cap)
        assert parent == g["parent"][:cap] and prob == g["prob"][:cap] and token == g["token"][:cap]
        assert P == g["P"][:cap]
    t = g["tie_case"]
    parent, _prob, _token, _P = S.product_forest(t["pos_prob"], [[1, 2], [3, 4]], 7)
    assert parent == t["parent"]


def _dyadic_positions(rng, d, k):
    """Probabilities that are multiples of 1/64: every product of up to five of them is exact in binary64."""
    return [[float(v) / 64.0 for v in rng.integers(1, 33, size=k)] for _ in range(d)]


@pytest.mark.parametrize("seed", range(6))
def test_product_forest_against_closed_forms_and_direct_enumeration(seed):
    rng = np.random.default_rng(seed)
    d, k = int(rng.integers(1, 5)), int(rng.integers(1, 5))
    pp = _dyadic_positions(rng, d, k)
    tok = [[100 * l + j for j in range(k)] for l in range(d)]
    total = sum(k ** l for l in range(d + 1))
    parent, prob, token, P = S.product_forest(pp, tok, total + 5)
    assert len(parent) == total                                               # the whole product, nothing twice
    depth = [0] * total
    for u in range(1, total):
        assert 0 <= parent[u] < u
        depth[u] = depth[parent[u]] + 1
        assert P[u] == P[parent[u]] * prob[u]
    # mass of a layer = product of the positions' masses (every factor and product is exact here)
    for l in range(d + 1):
        want = 1.0
        for i in range(l):
            want *= sum(pp[i])
        assert abs(sum(P[u] for u in range(total) if depth[u] == l) - want) < 1e-12
    # every index sequence occurs once, with the token and probability of its last position
    seqs = {}
    for u in range(total):
        s, v = [], u
        while v:
            s.append(v)
            v = parent[v]
        path = tuple(int(round(token[x] % 100)) for x in reversed(s))
        assert all(token[x] // 100 == i for i, x in enumerate(reversed(s)))
        seqs[path] = u
    assert len(seqs) == total
    direct = {path: float(np.prod([pp[i][j] for i, j in enumerate(path)])) for l in range(d + 1)
              for path in itertools.product(range(k), repeat=l)}
    assert all(P[seqs[path]] == direct[path] for path in direct)              # dyadic: no rounding either way
    # a smaller cap keeps exactly the head of the full list, and nothing left out beats anything kept
    for cap in (1, 2, total // 2 + 1, total - 1):
        if cap < 1:
            continue
        p2, q2, t2, P2 = S.product_forest(pp, tok, cap)
        assert (p2, q2, t2, P2) == (parent[:cap], prob[:cap], token[:cap], P[:cap])
    assert all(P[u] >= P[u + 1] for u in range(total - 1))
    order = sorted(direct.items(), key=lambda e: (-e[1], len(e[0]), e[0]))
    assert [seqs[path] for path, _ in order] == list(range(total))


def test_product_forest_special_cases():
    # one candidate per position: a chain of running products
    parent, prob, token, P = S.product_forest([[0.5], [0.25], [0.5]], [[7], [8], [9]], 10)
    assert parent == [-1, 0, 1, 2] and token == [-1, 7, 8, 9] and P == [1.0, 0.5, 0.125, 0.0625]
    # one position: the candidates in order of probability
    parent, prob, token, P = S.product_forest([[0.1, 0.4, 0.2, 0.3]], [[0, 1, 2, 3]], 10)
    assert parent == [-1, 0, 0, 0, 0] and token == [-1, 1, 3, 2, 0] and prob[1:] == [0.4, 0.3, 0.2, 0.1]
    # the rule on such a forest with a flat cost and a budget takes the head of the list: best-first
    # selection only ever looks at the most probable remaining candidate
    rng = np.random.default_rng(3)
    pp = _dyadic_positions(rng, 3, 3)
    parent, prob, token, P = S.product_forest(pp, [[1, 2, 3]] * 3, 40)
    cost = [1.0 + 1e-9 * n for n in range(42)]
    t = S.select_tree(parent, prob, token, cost, alpha=1.0, max_depth=3, budget=12)
    if len(set(P[:13])) == 13:                                               # no ties at the cut
        assert t.cand_index == list(range(12))
