"""CPU oracle: SMART draft-tree selection.  TEST INFRASTRUCTURE ONLY.

Follows the paper's Sec. 3.2 ("Speedup-Maximizing Draft Tree") in its own
notation.  Plain Python floats (IEEE binary64), one operation per statement
where rounding order matters, no fused multiply-add.

Quantities (costs are in units of c_T, which cancels from both sides of the
decision rule, Eq. "decision_rule"):

  P(u)      cumulative path probability, Eq. "cum_prob": P(root) = 1,
            P(u) = P(parent(u)) * p(u)
  n = |S|   number of selected nodes, root included
  cost[n]   C_spec(n) = C_draft + C_verify of an n-node tree (Eq. "definition")
  dC(n)     marginal cost of the (n+1)-th node: dcost[n] if a table is given
            (the differentiated form, Eq. "marginal_cost"), else the exact
            finite difference cost[n+1] - cost[n]
  L         expected accepted tokens of S.  dilution NONE: sum_{u in S} P(u)
            (the identity behind Eq. "expected_acc_length": expected number of
            consecutively accepted tokens = sum of prefix acceptance
            probabilities).  dilution PATH_MEAN: Eq. "expected_acc_length"
            literally, the mean over root-to-leaf paths of the summed P along
            the path (root counted in every path).
  rule      keep u  iff  alpha * dL(u) / dC(n)  >  L / cost[n]   (strict),
            dL(u) = P(u)               (NONE)
                  = P(u) / |paths|     (PATH_MEAN, Eq. "marginal_benefit")

Schedules:
  BEST_FIRST  node-by-node: always test the not-yet-selected candidate with the
              largest P whose parent is selected (ties: smaller candidate
              index); stop at the first failed test or when |S| = budget.
  LAYERWISE   Algorithm 1 as printed: per layer the global terms are frozen,
              every child of the previous layer's survivors is tested against
              them, survivors beyond the budget are dropped lowest-P first
              (Eq. "optimization" requires |S| <= B).
"""
from __future__ import annotations

BEST_FIRST, LAYERWISE = 0, 1
DILUTION_NONE, DILUTION_PATH_MEAN = 0, 1


def path_prob_and_depth(cand_parent, cand_prob):
    """Eq. "cum_prob" over a candidate forest given in topological order."""
    C = len(cand_parent)
    P = [0.0] * C
    depth = [0] * C
    if C == 0:
        raise ValueError("a sequence needs at least its root candidate")
    if cand_parent[0] != -1:
        raise ValueError("candidate 0 must be the root")
    P[0] = 1.0
    for u in range(1, C):
        par = cand_parent[u]
        if not (0 <= par < u):
            raise ValueError("candidate parents must precede their children")
        P[u] = P[par] * float(cand_prob[u])
        depth[u] = depth[par] + 1
    return P, depth


def path_mean_L(node_parent, node_P):
    """Eq. "expected_acc_length": mean over root-to-leaf paths; leaves taken in
    increasing node id, each path summed from the root down."""
    n = len(node_parent)
    has_child = [False] * n
    for i in range(1, n):
        has_child[node_parent[i]] = True
    total = 0.0
    leaves = 0
    for leaf in range(n):
        if has_child[leaf]:
            continue
        path = []
        v = leaf
        while v >= 0:
            path.append(v)
            v = node_parent[v]
        acc = 0.0
        for v in reversed(path):
            acc = acc + node_P[v]
        total = total + acc
        leaves += 1
    return total / leaves, leaves


def _marginal_cost(cost, dcost, n):
    if dcost is not None:
        return float(dcost[n])
    return float(cost[n + 1]) - float(cost[n])


def _rule(alpha, benefit, dC, L, cost_n):
    lhs = alpha * benefit
    lhs = lhs / dC
    rhs = L / cost_n
    return lhs > rhs


class SelectedTree:
    __slots__ = ("parent", "token", "cand_index", "pathprob", "L", "R")

    def __init__(self):
        self.parent, self.token, self.cand_index, self.pathprob = [], [], [], []
        self.L = 0.0
        self.R = 0.0

    def __len__(self):
        return len(self.parent)


def select_tree(cand_parent, cand_prob, cand_token, cost, dcost=None, alpha=0.8,
                max_depth=8, budget=64, schedule=BEST_FIRST, dilution=DILUTION_NONE):
    """One sequence.  Returns a SelectedTree whose node ids are a topological
    order (selection rank for BEST_FIRST; layer, then candidate index, for
    LAYERWISE)."""
    if budget < 1:
        raise ValueError("budget must admit the root")
    P, depth = path_prob_and_depth(cand_parent, cand_prob)
    C = len(cand_parent)
    out = SelectedTree()
    node_of = {0: 0}
    out.parent.append(-1)
    out.token.append(int(cand_token[0]))
    out.cand_index.append(0)
    out.pathprob.append(1.0)
    L_sum = 1.0  # running sum_{u in S} P(u), in selection order

    def current_L():
        if dilution == DILUTION_NONE:
            return L_sum, 1
        return path_mean_L(out.parent, out.pathprob)

    def append(u):
        nonlocal L_sum
        node_of[u] = len(out.parent)
        out.parent.append(node_of[cand_parent[u]])
        out.token.append(int(cand_token[u]))
        out.cand_index.append(u)
        out.pathprob.append(P[u])
        L_sum = L_sum + P[u]

    if schedule == BEST_FIRST:
        # Sorting by (P descending, index ascending) lists candidates exactly in
        # the order a best-first frontier would pop them: a child never has a
        # larger P than its parent and always a larger index.
        order = sorted((u for u in range(1, C) if depth[u] <= max_depth),
                       key=lambda u: (-P[u], u))
        for u in order:
            n = len(out)
            if n >= budget:
                break
            L, paths = current_L()
            benefit = P[u] if dilution == DILUTION_NONE else P[u] / paths
            if not _rule(alpha, benefit, _marginal_cost(cost, dcost, n), L, float(cost[n])):
                break
            append(u)
    elif schedule == LAYERWISE:
        children = [[] for _ in range(C)]
        for u in range(1, C):
            children[cand_parent[u]].append(u)
        active = [0]
        for _layer in range(1, max_depth + 1):
            n = len(out)
            if n >= budget:
                break
            L, paths = current_L()
            dC = _marginal_cost(cost, dcost, n)
            cost_n = float(cost[n])
            survivors = []
            for a in active:
                for u in children[a]:
                    benefit = P[u] if dilution == DILUTION_NONE else P[u] / paths
                    if _rule(alpha, benefit, dC, L, cost_n):
                        survivors.append(u)
            room = budget - n
            if len(survivors) > room:
                survivors = sorted(survivors, key=lambda u: (-P[u], u))[:room]
            survivors.sort()
            if not survivors:
                break
            for u in survivors:
                append(u)
            active = survivors
    else:
        raise ValueError("unknown schedule")

    L, _ = current_L()
    out.L = L
    out.R = L / float(cost[len(out)])
    return out


def select_batch(cand_cu, cand_parent, cand_prob, cand_token, cost, dcost=None, **kw):
    """Batched form over a CSR candidate forest; ``cost`` / ``dcost`` are one
    table shared by all sequences."""
    trees = []
    for b in range(len(cand_cu) - 1):
        lo, hi = int(cand_cu[b]), int(cand_cu[b + 1])
        trees.append(select_tree(list(cand_parent[lo:hi]), list(cand_prob[lo:hi]),
                                 list(cand_token[lo:hi]), cost, dcost, **kw))
    return trees


def reward(node_parent, node_P, cost, dilution=DILUTION_NONE):
    """R(S) of Eq. "definition" for an explicit node set (c_T = 1)."""
    if dilution == DILUTION_NONE:
        L = 0.0
        for p in node_P:
            L = L + p
    else:
        L, _ = path_mean_L(node_parent, node_P)
    return L / float(cost[len(node_parent)]), L


def brute_force_best(cand_parent, cand_prob, cost, max_depth=8, budget=64,
                     dilution=DILUTION_NONE):
    """Exhaustive search of Eq. "optimization": every parent-closed subset that
    contains the root (feasible for <= ~16 non-root candidates).  Returns
    (R*, list of optimal candidate-index tuples)."""
    P, depth = path_prob_and_depth(cand_parent, cand_prob)
    C = len(cand_parent)
    if C - 1 > 20:
        raise ValueError("brute force is for tiny forests only")
    best_R = None
    best_sets = []
    for bits in range(1 << (C - 1)):
        members = [0] + [u for u in range(1, C) if (bits >> (u - 1)) & 1]
        if len(members) > budget:
            continue
        mset = set(members)
        ok = True
        for u in members[1:]:
            if cand_parent[u] not in mset or depth[u] > max_depth:
                ok = False
                break
        if not ok:
            continue
        idx = {u: i for i, u in enumerate(members)}
        node_parent = [-1] + [idx[cand_parent[u]] for u in members[1:]]
        node_P = [P[u] for u in members]
        R, _ = reward(node_parent, node_P, cost, dilution)
        if best_R is None or R > best_R:
            best_R, best_sets = R, [tuple(members)]
        elif R == best_R:
            best_sets.append(tuple(members))
    return best_R, best_sets


# ---------------------------------------------------------------------------
# Algorithm 1 one layer at a time (a live draft model proposes the children of
# the previous layer's survivors, the rule prunes them, and only the survivors
# are expanded next).
# ---------------------------------------------------------------------------
class LayerState:
    """The tree built so far.  Nodes of the newest layer (the active set
    A_{l-1} of Sec. 3.2 "Sequential Decision Formulation") are
    ``layer_begin .. len(parent) - 1``."""
    __slots__ = ("parent", "token", "pathprob", "layer_begin", "L_sum", "L", "R")

    def __init__(self, root_token, cost):
        self.parent = [-1]
        self.token = [int(root_token)]
        self.pathprob = [1.0]
        self.layer_begin = 0
        self.L_sum = 1.0
        self.L = 1.0
        self.R = 1.0 / float(cost[1])

    def __len__(self):
        return len(self.parent)


def select_layer(state, cand_parent_node, cand_prob, cand_token, cost, dcost=None, alpha=0.8,
                 budget=64, dilution=DILUTION_NONE):
    """One iteration of Algorithm 1's loop over layers.

    ``cand_parent_node[c]`` is the tree node (of the newest layer) that
    candidate c extends, ``cand_prob[c]`` its conditional draft probability.
    The terms L, n, #paths are those of the tree before this layer (frozen);
    every candidate is tested against them; if more survive than the budget
    leaves room for, the lowest-P ones are dropped (ties: larger index first);
    survivors are appended in candidate order and become the next active set.
    Returns, per candidate, its new node id or -1.  ``state.L`` and ``state.R``
    are refreshed.
    """
    n = len(state)
    C = len(cand_parent_node)
    out_node = [-1] * C
    P = [0.0] * C
    for c in range(C):
        par = int(cand_parent_node[c])
        if not (state.layer_begin <= par < n):
            raise ValueError("a candidate must extend a node of the newest layer")
        pr = float(cand_prob[c])
        if not (0.0 <= pr <= 1.0):
            raise ValueError("probabilities lie in [0, 1]")
        P[c] = state.pathprob[par] * pr
    survivors = []
    if n < budget:
        if dilution == DILUTION_NONE:
            L, paths = state.L_sum, 1
        else:
            L, paths = path_mean_L(state.parent, state.pathprob)
        dC = _marginal_cost(cost, dcost, n)
        cost_n = float(cost[n])
        for c in range(C):
            benefit = P[c] if dilution == DILUTION_NONE else P[c] / paths
            if _rule(alpha, benefit, dC, L, cost_n):
                survivors.append(c)
        room = budget - n
        if len(survivors) > room:
            survivors = sorted(survivors, key=lambda c: (-P[c], c))[:room]
        survivors.sort()
    state.layer_begin = n
    for c in survivors:
        out_node[c] = len(state.parent)
        state.parent.append(int(cand_parent_node[c]))
        state.token.append(int(cand_token[c]))
        state.pathprob.append(P[c])
        state.L_sum = state.L_sum + P[c]
    if dilution == DILUTION_NONE:
        state.L = state.L_sum
    else:
        state.L, _ = path_mean_L(state.parent, state.pathprob)
    state.R = state.L / float(cost[len(state)])
    return out_node


# ---------------------------------------------------------------------------
# The likelihood-maximising policy SMART is compared with (Sec. 3.1, first
# paragraph; Fig. "method-comparison" (a), (b)).
# ---------------------------------------------------------------------------
def baseline_tree(cand_parent, cand_prob, cand_token, cost, k=10, max_depth=6, g=60):
    """Expansion phase: layer by layer, the k candidates of the layer with the
    largest cumulative probability P are expanded (their children, as the
    candidate forest lists them, form the next layer); the first layer is the
    root's children.  Rerank phase: every candidate generated in layers
    1 .. max_depth is ranked by P and the best g are kept (ties anywhere:
    smaller candidate index first; the root is kept besides).  Nodes are numbered
    by layer, then candidate index.  L = sum of P over the kept nodes, R = L /
    cost[n] as for the other policies (dilution NONE)."""
    P, depth = path_prob_and_depth(cand_parent, cand_prob)
    C = len(cand_parent)
    children = [[] for _ in range(C)]
    for u in range(1, C):
        children[cand_parent[u]].append(u)
    generated = []
    expanded = [0]
    for _layer in range(1, max_depth + 1):
        layer = [u for e in expanded for u in children[e]]
        if not layer:
            break
        generated += layer
        expanded = sorted(layer, key=lambda u: (-P[u], u))[:k]
    kept = sorted(generated, key=lambda u: (-P[u], u))[:g]
    kept = [0] + sorted(kept, key=lambda u: (depth[u], u))
    out = SelectedTree()
    node_of = {}
    L = 0.0
    for u in kept:
        node_of[u] = len(out.parent)
        out.parent.append(-1 if u == 0 else node_of[cand_parent[u]])
        out.token.append(int(cand_token[u]))
        out.cand_index.append(u)
        out.pathprob.append(P[u])
        L = L + P[u]
    out.L = L
    out.R = L / float(cost[len(out)])
    return out


# ---------------------------------------------------------------------------
# Candidate forest of a drafter whose positions are independent (Appendix
# "Additional Experimental Results": the block-diffusion drafter proposes top-k
# candidates per position in one pass; the tree is the Cartesian product of the
# positions' candidates, kept to the most probable nodes).
# ---------------------------------------------------------------------------
def product_forest(pos_prob, pos_token, cap):
    """pos_prob[l][j], pos_token[l][j]: probability and token of candidate j at
    position l (l = 0 .. d-1, j = 0 .. k-1), the same whatever came before.
    Every sequence (j_1, .., j_l), l <= d, is a node at depth l whose parent is
    (j_1, .., j_{l-1}); its conditional probability is pos_prob[l-1][j_l], so
    P = product along the path, multiplied root to leaf.  Kept: the `cap` nodes
    with the largest P, the root among them (ties: smaller depth, then the
    lexicographically smaller sequence), listed in that order -- a parent
    precedes its children because P(child) <= P(parent) and it is shallower.
    Returns (cand_parent, cand_prob, cand_token, P) in candidate-forest form
    (root first, parent = -1, probability 1.0, token -1)."""
    d = len(pos_prob)
    nodes = [((), 1.0)]
    layer = [((), 1.0)]
    for l in range(d):
        nxt = []
        for path, P in layer:
            for j in range(len(pos_prob[l])):
                nxt.append((path + (j,), P * float(pos_prob[l][j])))
        nodes += nxt
        layer = nxt
    nodes.sort(key=lambda e: (-e[1], len(e[0]), e[0]))
    nodes = nodes[:max(int(cap), 1)]
    index = {path: i for i, (path, _P) in enumerate(nodes)}
    cand_parent, cand_prob, cand_token, cum = [], [], [], []
    for path, P in nodes:
        if not path:
            cand_parent.append(-1)
            cand_prob.append(1.0)
            cand_token.append(-1)
        else:
            cand_parent.append(index[path[:-1]])
            cand_prob.append(float(pos_prob[len(path) - 1][path[-1]]))
            cand_token.append(int(pos_token[len(path) - 1][path[-1]]))
        cum.append(P)
    return cand_parent, cand_prob, cand_token, cum
