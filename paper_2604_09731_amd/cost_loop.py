#!/usr/bin/env python3
"""Cost-model loop on the device (Sec. 3.1 "Cost Modeling" -> Sec. 3.2 of the paper), for the
attention layer this library implements.

For each batch size: time tree_verify_attention for trees of 1, 4, 8, 16, 32 and 64 nodes per
sequence (the paper profiles a handful of forward passes per device), take the plain decoding
step (a tree that is only its root) as c_T, fit the power-exponential model of Eq. "exp_model"
to the EXTRA time over that step as a function of the drafted tokens batch * (n - 1), and the
line of Eq. "linear_model" to the draft side's time for the same tokens; the library builds the
cost tables from the fits (smart_cost_tables_biased: cost[n] = 1 + (draft + verify model) / c_T,
and the differentiated marginal cost of Eq. "marginal_cost") and smart_select_tree chooses trees
over the same candidate forests, once with the exact difference cost[n+1] - cost[n] and once
with the differentiated marginal cost (--forest product: the forests of a drafter with
independent positions, the Cartesian-product tree of the paper's appendix).  The
likelihood-maximising expand-and-rerank policy (Sec. 3.1, first paragraph) is run over the same
forests for comparison: its modelled speedup under the same cost table, and the measured
attention time of both policies' trees.  Prints one JSON row per batch size.

The draft side is a stand-in (no draft model is part of this library): a drafter of
--draft-layers layers shaped like the target's (an EAGLE-style head is one), whose time for the
drafted tokens is that many times the measured extra time of ONE layer, against a target of
--target-layers such layers; with the default --draft-layers 0 there is no draft leg.

This measures ONE attention layer (times --target-layers), not a whole target model: the point is
the loop (measure, fit, select) on this hardware, not the absolute speedups.  A caller may pass
`extra_us(tokens)`, the time of whatever else a layer does for that many tokens (bench.py
--cost-loop --with-dense adds a layer's dense products that way).

    python -m paper_2604_09731_amd.cost_loop [--batches 1 8 32 128] [--prefix 3584]
"""
from __future__ import annotations

import argparse
import json
import sys

import numpy as np


def main(argv=None, extra_us=None):
    import torch
    from . import binding as B
    from . import workloads as W
    ap = argparse.ArgumentParser()
    ap.add_argument("--batches", type=int, nargs="+", default=[1, 8, 32, 128])
    ap.add_argument("--prefix", type=int, default=3584)
    ap.add_argument("--sizes", type=int, nargs="+", default=[1, 4, 8, 16, 32, 64])
    ap.add_argument("--reps", type=int, default=50)
    ap.add_argument("--baseline-k", type=int, default=8)
    ap.add_argument("--baseline-depth", type=int, default=6)
    ap.add_argument("--baseline-g", type=int, default=59)
    ap.add_argument("--forest", choices=["autoregressive", "product"], default="autoregressive",
                    help="candidate forests: the workloads' autoregressive drafts (children conditioned on the path), "
                         "or the Cartesian product of independent per-position top-k candidates (the tree the paper's "
                         "appendix builds for a block-diffusion drafter), cut at 1024 candidates")
    ap.add_argument("--target-layers", type=int, default=1, help="the verification pass is this many of the measured layer")
    ap.add_argument("--draft-layers", type=int, default=0,
                    help="stand-in draft model: this many layers of the target's shape run over the drafted tokens "
                         "(0: no draft leg, lambda = 0)")
    args = ap.parse_args(argv)
    assert torch.cuda.is_available(), "needs the MI355X"
    lib = B.SmartTree(0)
    base = W.WORKLOADS["cfg3a"]
    rows = []

    def time_attention(w, cu, parent):
        """Microseconds per tree_verify_attention call for these trees (cache and queries synthetic)."""
        inp = W.make_attention_inputs(w, cu, poison_unused=False)
        dev = "cuda"
        t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
        el = lambda a: torch.from_numpy(np.ascontiguousarray(a)).view(torch.int16).view(torch.bfloat16).to(dev)
        kc, vc = B.interleave_kv_cache(el(inp.k_cache), el(inp.v_cache))
        d_cu, d_par, d_len = t(cu), t(parent), t(inp.prefix_len)
        _, _, _, mask, _ = lib.tree_pack(d_cu, d_par, d_len)
        q, kt, vt, bt = el(inp.q), el(inp.k_tree), el(inp.v_tree), t(inp.block_table)
        run = lambda: lib.tree_verify_attention(q, kt, vt, kc, vc, bt, d_len, d_cu, mask, inp.scale,
                                                B.SMART_KV_INTERLEAVED)
        for _ in range(5):
            run()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(args.reps):
            run()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e3 / args.reps

    def layer_us(w, cu, parent):
        """One layer for these trees: the library's attention, plus the caller's extra for the same tokens."""
        return time_attention(w, cu, parent) + (extra_us(int(cu[-1])) if extra_us else 0.0)

    def tiled(sel, batch):
        """The trees of a selection result, repeated until there are `batch` of them."""
        n_seq = sel["cu_nodes"].shape[0] - 1
        sizes = np.diff(sel["cu_nodes"])
        order = [b % n_seq for b in range(batch)]
        cu = np.concatenate([[0], np.cumsum(sizes[order])]).astype(np.int32)
        parent = np.concatenate([sel["parent"][sel["cu_nodes"][b]:sel["cu_nodes"][b + 1]] for b in order])
        return cu, parent.astype(np.int32), float(np.mean(sel["L"][order]))

    for batch in args.batches:
        w = base.scaled(batch=batch, prefix_min=args.prefix, prefix_max=args.prefix)
        rng = np.random.default_rng(7)
        big = W.random_tree(max(args.sizes), rng, "random")           # nested trees: the first n nodes of one tree
        times = []
        for n in args.sizes:
            cu = (np.arange(batch + 1) * n).astype(np.int32)
            times.append(layer_us(w, cu, np.tile(big[:n], batch).astype(np.int32)))
        sizes = np.array(args.sizes, np.float64)
        layer = np.array(times)
        layer_1 = layer[0] if args.sizes[0] == 1 else float(np.interp(1.0, sizes, layer))
        times = args.target_layers * layer                   # a verification pass
        c_T = args.target_layers * layer_1                    # a plain decoding step of the target
        x = batch * (sizes[1:] - 1.0)                         # drafted tokens
        extra = np.maximum(times[1:] - c_T, 1e-3)
        draft = args.draft_layers * np.maximum(layer[1:] - layer_1, 1e-3) if args.draft_layers else None
        fit = B.smart_fit_cost_models(x, draft, extra)
        lam = fit.get("lambda", 0.0)
        n_max = base.budget
        # cost[n] = (c_T + draft + extra verification time of the n - 1 drafted nodes) / c_T, and its derivative
        cost, dcost = B.smart_cost_tables_biased(lam, 0.0, fit["gamma"], fit["delta"], fit["rho"], c_T, c_T, float(batch),
                                                 1, n_max)
        if args.forest == "product":
            import types
            rng_f = np.random.default_rng(base.seed + 7)
            n_f = min(batch, 32)
            logits = rng_f.normal(0.0, 2.0, size=(n_f, base.max_depth, base.top_k))
            pos_prob = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)      # softmax over the k candidates
            pos_token = rng_f.integers(0, 32000, size=pos_prob.shape).astype(np.int32)
            forest = types.SimpleNamespace(**B.smart_product_forest(pos_prob, pos_token, 1024))
        else:
            forest = W.make_forest(base.scaled(batch=min(batch, 32)))
        sel = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost,
                                  alpha=base.alpha, max_depth=base.max_depth, budget=n_max)
        sel_d = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost, dcost,
                                    alpha=base.alpha, max_depth=base.max_depth, budget=n_max)
        n_sel, n_sel_d = np.diff(sel["cu_nodes"]), np.diff(sel_d["cu_nodes"])
        row = dict(batch=batch, forest=args.forest, extra=bool(extra_us), target_layers=args.target_layers,
                   draft_layers=args.draft_layers, sizes=args.sizes, us=[round(float(v), 2) for v in times],
                   c_T_us=round(float(c_T), 2), lam=lam,
                   gamma=fit["gamma"], delta=fit["delta"], rho=fit["rho"],
                   rms_us=round(float(np.sqrt(fit["sse"] / len(x))), 3),
                   tree_nodes_min_median_max=[int(n_sel.min()), int(np.median(n_sel)), int(n_sel.max())],
                   L_mean=round(float(sel["L"].mean()), 3), R_mean=round(float(sel["R"].mean()), 3),
                   derivative_tree_nodes_min_median_max=[int(n_sel_d.min()), int(np.median(n_sel_d)), int(n_sel_d.max())],
                   derivative_R_mean=round(float(sel_d["R"].mean()), 3))
        # The fixed expand-and-rerank policy over the same forests, under the same cost table: its modelled
        # speedup, and what the kernel really takes for both policies' trees (measured R = L c_T / time).
        fixed = B.smart_baseline_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost,
                                      k=args.baseline_k, max_depth=args.baseline_depth, g=min(args.baseline_g, n_max - 1))
        for name, res in (("smart", sel), ("baseline", fixed)):
            cu, parent, L_mean = tiled(res, batch)
            one = layer_us(w, cu, parent)
            # a verification pass of these trees, and the draft side's time for their drafted tokens
            us = args.target_layers * one + args.draft_layers * max(one - layer_1, 0.0)
            row[name + "_us"] = round(float(us), 2)
            row[name + "_measured_R"] = round(L_mean * float(c_T) / float(us), 3)
        row["baseline_nodes"] = int(np.median(np.diff(fixed["cu_nodes"])))
        row["baseline_L_mean"] = round(float(fixed["L"].mean()), 3)
        row["baseline_R_mean"] = round(float(fixed["R"].mean()), 3)
        rows.append(row)
        print(json.dumps(row), flush=True)
    return rows


if __name__ == "__main__":
    sys.exit(0 if main() else 1)
