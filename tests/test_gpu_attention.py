"""GPU parity of tree_verify_attention against the fp64 CPU oracle, through the
C ABI.  Tolerances (max |out - ref| / max |ref| over the output tensor):
1e-5 for fp32 inputs, 2e-2 for bf16 inputs with fp32 accumulation."""
import numpy as np
import pytest

from oracle import pack_accept as PA
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return B.SmartTree(0)


class Case:
    """A workload instance on the host (numpy) and on the GPU (torch)."""

    def __init__(self, w, cu, parent, inp, layout):
        import torch
        self.w, self.cu, self.parent, self.inp, self.layout = w, cu, parent, inp, layout
        dev = "cuda"
        self.q = H.torch_elems(inp.q, w.dtype, dev)
        self.k_tree = H.torch_elems(inp.k_tree, w.dtype, dev)
        self.v_tree = H.torch_elems(inp.v_tree, w.dtype, dev)
        kc = H.torch_elems(inp.k_cache, w.dtype, dev)
        vc = H.torch_elems(inp.v_cache, w.dtype, dev)
        if layout == B.SMART_KV_INTERLEAVED:
            kc, vc = B.interleave_kv_cache(kc, vc)
        self.k_cache, self.v_cache = kc, vc
        self.block_table = torch.from_numpy(inp.block_table).to(dev)
        self.prefix_len = torch.from_numpy(inp.prefix_len).to(dev)
        self.cu_nodes = torch.from_numpy(np.ascontiguousarray(cu)).to(dev)
        self.parent_d = torch.from_numpy(np.ascontiguousarray(parent)).to(dev)

    def run(self, lib, want_lse=True):
        _, _, _, mask, status = lib.tree_pack(self.cu_nodes, self.parent_d, self.prefix_len)
        assert not status.cpu().numpy().any()
        out, lse = lib.tree_verify_attention(self.q, self.k_tree, self.v_tree, self.k_cache,
                                             self.v_cache, self.block_table, self.prefix_len,
                                             self.cu_nodes, mask, self.inp.scale, self.layout,
                                             want_lse=True)
        import torch
        torch.cuda.synchronize()
        return out, lse

    def oracle(self, oracle_attention, sel=None):
        i = self.inp
        return oracle_attention.tree_attention(i.q, i.k_tree, i.v_tree, i.k_cache, i.v_cache,
                                               i.block_table, i.prefix_len, self.cu, self.parent,
                                               i.scale, sel=sel)


def make_case(w, layout, prefix_len=None, trees=None, seed=None):
    if trees is None:
        cu, parent, _, _ = H.trees_from_library(w)
    else:
        cu, parent = trees
    inp = W.make_attention_inputs(w, cu, seed=seed, prefix_len=prefix_len)
    return Case(w, cu, parent, inp, layout)


def check_full(lib, oracle_attention, case, tol=None):
    out, lse = case.run(lib)
    ref, ref_lse = case.oracle(oracle_attention)
    err = H.rel_err(H.out_to_f64(out, case.w.dtype), ref)
    tol = tol or H.TOL[case.w.dtype]
    assert np.isfinite(H.out_to_f64(out, case.w.dtype)).all()
    assert err <= tol, f"{case.w.name}: rel err {err:.3e} > {tol}"
    lse_err = np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max()
    assert lse_err <= (1e-4 if case.w.dtype == "f32" else 2e-2), lse_err
    return err


# ----- the two small fp32 configurations, both cache layouts ---------------------------
@pytest.mark.parametrize("name", ["cfg1", "cfg1_sharp"])
@pytest.mark.parametrize("layout", [B.SMART_KV_PLAIN, B.SMART_KV_INTERLEAVED])
def test_fp32_tiny_configs(lib, oracle_attention, name, layout):
    check_full(lib, oracle_attention, make_case(W.WORKLOADS[name], layout))


# ----- bf16: small shapes spanning several tiles with ragged tails, both kernels --------
def _ragged_case(layout, dtype="bf16", Hq=8, Hkv=2, D=128, seed=21):
    rng = np.random.default_rng(seed)
    sizes = [1, 3, 9, 17, 40, 2]
    shapes = ["random", "chain", "random", "star", "random", "random"]
    trees = [W.random_tree(n, rng, s) for n, s in zip(sizes, shapes)]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = np.array([0, 1, 31, 32, 33, 517], np.int32)         # empty, sub-tile, exact, ragged, multi-tile
    w = W.Workload("ragged", dtype, len(sizes), Hq, Hkv, D, 0, 0, seed=seed)
    return make_case(w, layout, prefix_len=lens, trees=(cu, parent), seed=seed)


@pytest.mark.parametrize("force_general", [0, 1])
def test_bf16_ragged_small(lib, oracle_attention, force_general):
    lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, force_general)
    try:
        check_full(lib, oracle_attention, _ragged_case(B.SMART_KV_INTERLEAVED))
        if force_general:
            check_full(lib, oracle_attention, _ragged_case(B.SMART_KV_PLAIN))
            check_full(lib, oracle_attention, _ragged_case(B.SMART_KV_PLAIN, D=64))
            check_full(lib, oracle_attention, _ragged_case(B.SMART_KV_INTERLEAVED, dtype="f32", D=64))
    finally:
        lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 0)


@pytest.mark.parametrize("G,Hkv", [(4, 8), (7, 4), (8, 2), (1, 4), (32, 1)])
def test_bf16_group_sizes_and_big_trees(lib, oracle_attention, G, Hkv):
    rng = np.random.default_rng(G)
    sizes = [128, 96, 5, 33]
    trees = [W.random_tree(n, rng, "chain" if i == 1 else "random") for i, n in enumerate(sizes)]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    w = W.Workload("groups", "bf16", 4, G * Hkv, Hkv, 128, 0, 0, seed=30 + G)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([300, 77, 1000, 64], np.int32),
                     trees=(cu, np.concatenate(trees).astype(np.int32)))
    check_full(lib, oracle_attention, case)


def test_many_sequences_all_classes_and_window_reload(lib, oracle_attention):
    """More than 64 sequences (the plan lookup leaves its 64-sequence window), all three row
    classes in one batch, empty prefixes and one-node trees in between."""
    rng = np.random.default_rng(77)
    B_ = 150
    sizes = rng.choice([1, 2, 5, 8, 9, 14, 16, 17, 30, 64, 65, 100], size=B_)
    trees = [W.random_tree(int(n), rng) for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    lens = rng.integers(0, 200, size=B_).astype(np.int32)
    lens[::7] = 0
    lens[3] = 1500                      # one long prefix: pieces longer than the block-id window
    w = W.Workload("many", "bf16", B_, 8, 2, 128, 0, 0, seed=55)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=lens,
                     trees=(cu, np.concatenate(trees).astype(np.int32)))
    check_full(lib, oracle_attention, case)
    for workers in (3, 1000):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            check_full(lib, oracle_attention, case)
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)


# ----- the bf16 configurations ------------------------------------------------------------
def test_cfg2_full(lib, oracle_attention):
    check_full(lib, oracle_attention, make_case(W.WORKLOADS["cfg2"], B.SMART_KV_INTERLEAVED))


@pytest.mark.parametrize("name", ["cfg3a", "cfg3b", "cfg4", "cfg5a", "cfg5b"])
def test_reduced_configs_full_compare(lib, oracle_attention, name):
    """Same shapes and tree recipe, fewer sequences and a shorter (still ragged,
    multi-tile) prefix, so the oracle covers every output element."""
    w = W.WORKLOADS[name]
    w = w.scaled(batch=min(w.batch, 6), prefix_min=max(200, w.prefix_min // 16),
                 prefix_max=w.prefix_max // 16 + 13, image_prefix=w.image_prefix // 16)
    check_full(lib, oracle_attention, make_case(w, B.SMART_KV_INTERLEAVED))


def _library_trees_checked_against_oracle(w):
    """The trees the library's smart_select_tree builds for this workload, after checking that
    the oracle's selection builds exactly the same ones (node order, parents, tokens)."""
    forest = W.make_forest(w)
    cu, parent, token, cand = H.trees_from_library(w, forest)
    cu_o, parent_o, token_o, cand_o = H.trees_from_oracle(w, forest)
    assert np.array_equal(cu, cu_o) and np.array_equal(parent, parent_o)
    assert np.array_equal(token, token_o) and np.array_equal(cand, cand_o)
    return cu, parent


def test_cfg3a_full_size_every_row(lib, oracle_attention):
    """The benchmark's workload at full size, in the launch configuration the benchmark times:
    every output element and every lse against the oracle."""
    w = W.WORKLOADS["cfg3a"]
    case = make_case(w, B.SMART_KV_INTERLEAVED, trees=_library_trees_checked_against_oracle(w))
    check_full(lib, oracle_attention, case)


@pytest.mark.parametrize("name", ["cfg3b", "cfg4", "cfg5a", "cfg5b"])
def test_full_size_configs_sampled(lib, oracle_attention, name):
    """Full size, in the launch configuration the benchmark times; the oracle computes a seeded
    sample of (node, head) rows one by one: at least one row of every (sequence, kv head) segment
    (so every piece of every worker's share is merged into some compared row), the first and the
    last node of the smallest and the largest tree of every row class, and 64 rows drawn freely;
    plus finiteness of every output and lse."""
    w = W.WORKLOADS[name]
    cu, parent = _library_trees_checked_against_oracle(w)
    case = make_case(w, B.SMART_KV_INTERLEAVED, trees=(cu, parent))
    out, lse = case.run(lib)
    o = H.out_to_f64(out, w.dtype)
    assert np.isfinite(o).all() and np.isfinite(lse.cpu().numpy()).all()
    rng = np.random.default_rng(9)
    N = int(cu[-1])
    G = w.num_q_heads // w.num_kv_heads
    sizes = np.diff(cu)
    nodes, heads = [], []
    for b in range(w.batch):                                   # one row per (sequence, kv head)
        for g in range(w.num_kv_heads):
            nodes.append(int(cu[b]) + int(rng.integers(0, sizes[b])))
            heads.append(g * G + int(rng.integers(0, G)))
    rows = sizes * G
    for in_class in (rows <= 32, (rows > 32) & (rows <= 64), rows > 64):
        members = np.flatnonzero(in_class)
        if len(members) == 0:
            continue
        for b in (members[np.argmin(sizes[members])], members[np.argmax(sizes[members])]):
            for node in (int(cu[b]), int(cu[b + 1]) - 1):
                for h in (0, w.num_q_heads - 1):
                    nodes.append(node)
                    heads.append(h)
    nodes += rng.integers(0, N, 64).tolist()
    heads += rng.integers(0, w.num_q_heads, 64).tolist()
    nodes, heads = np.array(nodes, np.int32), np.array(heads, np.int32)
    ref, ref_lse = case.oracle(oracle_attention, sel=(nodes, heads))
    got = o[nodes, heads]
    scale = np.abs(ref).max()
    err = np.abs(got - ref).max() / scale
    assert err <= H.TOL[w.dtype], f"{name}: rel err {err:.3e}"
    assert np.abs(lse.cpu().numpy()[nodes, heads] - ref_lse).max() <= 2e-2


# ----- invariances the kernel must have at any size ---------------------------------------
def test_paging_split_and_determinism(lib, oracle_attention):
    import torch
    w = W.WORKLOADS["cfg3b"].scaled(batch=5, prefix_min=300, prefix_max=900)
    case = make_case(w, B.SMART_KV_INTERLEAVED)
    out1, lse1 = case.run(lib)
    out2, _ = case.run(lib)
    assert torch.equal(out1, out2)                              # determinism
    # paging invariance: permute physical blocks and the table -> bit-identical
    nb = case.k_cache.shape[0]
    perm = torch.randperm(nb, device="cuda", generator=torch.Generator("cuda").manual_seed(1))
    k2 = torch.empty_like(case.k_cache)
    v2 = torch.empty_like(case.v_cache)
    k2[perm] = case.k_cache
    v2[perm] = case.v_cache
    bt = case.block_table.clone()
    valid = bt >= 0
    bt[valid] = perm[bt[valid].long()].int()
    keep = (case.k_cache, case.v_cache, case.block_table)
    case.k_cache, case.v_cache, case.block_table = k2, v2, bt
    out3, _ = case.run(lib)
    case.k_cache, case.v_cache, case.block_table = keep
    assert torch.equal(out1, out3)
    # split invariance: any number of workers gives the same result up to fp32 merge order
    ref = out1.float()
    for workers in (1, 7, 64, 4096):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            o, l = case.run(lib)
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)
        assert (o.float() - ref).abs().max().item() <= 2 ** -7 * ref.abs().max().item()
        assert (l - lse1).abs().max().item() <= 1e-4
    # matrix-core path and general kernel agree to bf16 output rounding
    lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 1)
    try:
        og, _ = case.run(lib)
    finally:
        lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 0)
    assert (og.float() - ref).abs().max().item() <= 2e-2 * ref.abs().max().item()


def test_tree_masking_perturbation_and_relabelling(lib, oracle_attention):
    import torch
    rng = np.random.default_rng(5)
    n = 24
    tree = W.random_tree(n, rng)
    w = W.Workload("mask", "bf16", 1, 8, 2, 128, 0, 0, seed=41)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([75], np.int32),
                     trees=(np.array([0, n], np.int32), tree))
    out, _ = case.run(lib)
    anc = []
    for i in range(n):
        s, j = set(), i
        while j >= 0:
            s.add(j)
            j = int(tree[j])
        anc.append(s)
    for j in (3, 11, 23):
        kt, vt = case.k_tree.clone(), case.v_tree.clone()
        case.k_tree[j] = -case.k_tree[j] * 2
        case.v_tree[j] = case.v_tree[j] + 3
        out2, _ = case.run(lib)
        case.k_tree, case.v_tree = kt, vt
        for i in range(n):
            same = torch.equal(out[i], out2[i])
            assert same == (j not in anc[i]), (i, j)
    # topological relabelling permutes the outputs
    placed, order = set(), []
    while len(order) < n:
        ready = [i for i in range(n) if i not in placed and (tree[i] < 0 or tree[i] in placed)]
        pick = int(rng.choice(ready))
        placed.add(pick)
        order.append(pick)
    new_of_old = {o: i for i, o in enumerate(order)}
    tree2 = np.array([-1 if tree[o] < 0 else new_of_old[int(tree[o])] for o in order], np.int32)
    idx = torch.tensor(order, device="cuda")
    case2 = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([75], np.int32),
                      trees=(np.array([0, n], np.int32), tree2))
    case2.q, case2.k_tree, case2.v_tree = case.q[idx], case.k_tree[idx], case.v_tree[idx]
    out3, _ = case2.run(lib)
    assert (out3.float() - out[idx].float()).abs().max().item() <= 2 ** -7 * out.float().abs().max().item()


def test_chain_single_node_and_empty_batch(lib, oracle_attention):
    import torch
    w = W.Workload("chain", "bf16", 3, 32, 8, 128, 0, 0, seed=43)
    trees = [W.random_tree(1, None, "chain"), W.random_tree(20, None, "chain"), W.random_tree(1, None, "chain")]
    cu = np.array([0, 1, 21, 22], np.int32)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([130, 64, 0], np.int32),
                     trees=(cu, np.concatenate(trees).astype(np.int32)))
    check_full(lib, oracle_attention, case)
    # empty batch / no nodes: nothing launched, nothing written
    empty = torch.empty((0, 32, 128), dtype=torch.bfloat16, device="cuda")
    out = lib.tree_verify_attention(empty, empty[:, :8], empty[:, :8], case.k_cache, case.v_cache,
                                    case.block_table[:0], case.prefix_len[:0],
                                    torch.zeros(1, dtype=torch.int32, device="cuda"),
                                    torch.empty((0, 2), dtype=torch.int64, device="cuda"),
                                    0.1, B.SMART_KV_INTERLEAVED)
    assert out.shape[0] == 0


def test_two_steps_of_the_loop_through_commit(lib, oracle_attention):
    """verify -> accept -> commit -> verify again.  The second step's attention runs on the
    device over the cache the device grew; the oracle does the same walk on its own cache.
    Accept decisions are integers (bit-exact), so both sides commit the same nodes; the
    second step's output must match to the bf16 tolerance, and the rows must see the new
    tokens (their output changes when the committed V rows are what they were not)."""
    import torch
    from oracle import pack_accept as PA
    w = W.Workload("loop", "bf16", 5, 8, 2, 128, 0, 0)
    rng = np.random.default_rng(77)
    sizes = [9, 30, 4, 17, 12]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, "random") for n in sizes]).astype(np.int32)
    N = int(cu[-1])
    max_depth = 6
    prefix_len = np.array([200, 1000, 40, 520, 8], np.int32)      # 8 free slots in every last block
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=prefix_len, trees=(cu, parent))
    token = rng.integers(0, 3, size=N).astype(np.int32)           # few distinct tokens: long accepted paths
    target = rng.integers(0, 3, size=N).astype(np.int32)
    # step 1 on the device
    out1, _ = case.run(lib)
    acc_len, acc_path, _ = lib.tree_accept(case.cu_nodes, case.parent_d, torch.from_numpy(token).cuda(),
                                           torch.from_numpy(target).cuda(), max_depth)
    nb = case.inp.meta["num_blocks"]
    new_len, status = lib.tree_commit(case.cu_nodes, acc_len, acc_path, case.k_tree, case.v_tree, case.k_cache,
                                      case.v_cache, case.block_table, case.prefix_len, B.SMART_KV_INTERLEAVED, 16, nb,
                                      w.num_kv_heads * 16 * 128, 16 * 128)
    torch.cuda.synchronize()
    assert not status.cpu().numpy().any()
    # the same walk on the oracle's side
    ref_len, ref_path, _ = PA.accept(cu, parent, token, target, max_depth)
    assert acc_len.cpu().numpy().tolist() == ref_len and acc_path.cpu().numpy().tolist() == ref_path
    assert max(ref_len) >= 2
    i = case.inp
    ok, oc = i.k_cache.copy(), i.v_cache.copy()
    grown, st = PA.commit(cu, ref_len, ref_path, i.k_tree, i.v_tree, ok, oc, i.block_table, prefix_len, max_depth)
    assert st == [0] * w.batch and new_len.cpu().numpy().tolist() == grown
    # step 2: new trees, new queries, over the grown prefixes
    sizes2 = [5, 3, 20, 8, 33]
    cu2 = np.concatenate([[0], np.cumsum(sizes2)]).astype(np.int32)
    parent2 = np.concatenate([W.random_tree(n, rng, "random") for n in sizes2]).astype(np.int32)
    N2 = int(cu2[-1])
    q2 = W._normal(5, 1, (N2, w.num_q_heads, 128), 1.0, "bf16")
    k2 = W._normal(5, 2, (N2, w.num_kv_heads, 128), 1.0, "bf16")
    v2 = W._normal(5, 3, (N2, w.num_kv_heads, 128), 1.0, "bf16")
    d = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    _, _, _, mask2, st2 = lib.tree_pack(d(cu2), d(parent2), new_len)
    assert not st2.cpu().numpy().any()
    out2, _ = lib.tree_verify_attention(H.torch_elems(q2, "bf16", "cuda"), H.torch_elems(k2, "bf16", "cuda"),
                                        H.torch_elems(v2, "bf16", "cuda"), case.k_cache, case.v_cache, case.block_table,
                                        new_len, d(cu2), mask2, i.scale, B.SMART_KV_INTERLEAVED, want_lse=True)
    torch.cuda.synchronize()
    grown = np.array(grown, np.int32)
    ref2, _ = oracle_attention.tree_attention(q2, k2, v2, ok, oc, i.block_table, grown, cu2, parent2, i.scale)
    got2 = H.out_to_f64(out2, "bf16")
    assert np.isfinite(got2).all()
    assert H.rel_err(got2, ref2) <= H.TOL["bf16"]
    # and the committed tokens matter: without them the oracle's answer is measurably different
    stale, _ = oracle_attention.tree_attention(q2, k2, v2, i.k_cache, i.v_cache, i.block_table, prefix_len, cu2, parent2, i.scale)
    assert H.rel_err(stale, ref2) > 10 * H.TOL["bf16"] or np.abs(stale - ref2).max() > 0.05


def test_medium_trees_every_tail_of_the_two_tile_iteration(lib, oracle_attention):
    """Class 1 (33 .. 64 rows per kv head) consumes two tiles per iteration, one per key group,
    with three iterations of fetches in flight: prefixes of 1 .. 12 tiles, ragged or not, with
    9 .. 16 nodes at G = 4, hit every phase of that pipeline (short segments, odd tile counts,
    a ragged last tile in either key group)."""
    rng = np.random.default_rng(5)
    lens = np.array([32, 33, 63, 64, 65, 96, 97, 128, 159, 161, 223, 224, 257, 300, 352, 383], np.int32)
    sizes = [9 + (i % 8) for i in range(len(lens))]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, "random") for n in sizes]).astype(np.int32)
    w = W.Workload("medium", "bf16", len(sizes), 16, 4, 128, 0, 0, seed=9)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=lens, trees=(cu, parent), seed=9)
    check_full(lib, oracle_attention, case)
    # the same with few workers (long shares crossing many segments) and with many (pieces of a tile or two)
    for workers in (3, 64):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            check_full(lib, oracle_attention, case)
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)


def test_offsets_that_are_no_running_sum(lib):
    """d_cu_nodes must be a running sum inside [0, total_nodes].  Overlapping or decreasing offsets
    would make the trees' sizes add up to more than total_nodes, the bound every buffer of the call
    is sized by: the matrix-core path then writes no output row at all, the general kernel zero-fills
    what no well-formed range owns, and neither reads or writes outside the arrays."""
    import torch
    rng = np.random.default_rng(8)
    sizes = [128, 0, 0, 0]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    w = W.Workload("offsets", "bf16", 4, 8, 2, 128, 0, 0, seed=12)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([300, 200, 100, 50], np.int32),
                     trees=(cu, W.random_tree(128, rng, "random").astype(np.int32)))
    _, _, _, mask, _ = lib.tree_pack(case.cu_nodes, case.parent_d, case.prefix_len)
    for bad in ([0, 128, 0, 128, 128], [0, 128, 128, 64, 128], [-1, 128, 128, 128, 128], [0, 64, 128, 200, 128]):
        d_bad = torch.tensor(bad, dtype=torch.int32, device="cuda")
        for force_general in (0, 1):
            lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, force_general)
            try:
                out = torch.full_like(case.q, 7.0)
                lib.tree_verify_attention(case.q, case.k_tree, case.v_tree, case.k_cache, case.v_cache,
                                          case.block_table, case.prefix_len, d_bad, mask, case.inp.scale,
                                          B.SMART_KV_INTERLEAVED, out=out)
                torch.cuda.synchronize()
            finally:
                lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 0)
            assert torch.isfinite(out.float()).all()
            if not force_general:
                assert (out.float() == 7.0).all()


@pytest.mark.parametrize("force_general", [0, 1])
def test_block_table_entries_outside_the_cache_are_reported(lib, force_general):
    """Entries of the block table that the call reads and that lie outside [0, num_blocks) are read as the nearest
    valid block (nothing leaves the cache) and reported per sequence; entries past a sequence's prefix are never
    read and never reported; a later call with a sound table clears the report."""
    import torch
    rng = np.random.default_rng(4)
    sizes = [5, 20, 70, 3, 9]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, "random") for n in sizes]).astype(np.int32)
    w = W.Workload("table", "bf16", len(sizes), 8, 2, 128, 0, 0, seed=19)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([100, 333, 64, 0, 50], np.int32), trees=(cu, parent))
    _, _, _, mask, _ = lib.tree_pack(case.cu_nodes, case.parent_d, case.prefix_len)
    nb = case.k_cache.shape[0]
    bt = case.block_table.clone()
    bt[1, 3] = -5                       # read: sequence 1 uses blocks 0 .. 20
    bt[2, 3] = nb + 3                   # read: the last block sequence 2 uses (64 tokens = blocks 0 .. 3)
    bt[0, 7] = nb + 100                 # not read: sequence 0 uses blocks 0 .. 6
    bt[4, 4:] = -9                      # not read: sequence 4 uses blocks 0 .. 3
    lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, force_general)
    try:
        for table, expect in ((bt, [0, 1, 1, 0, 0]), (case.block_table, [0, 0, 0, 0, 0])):
            status = torch.full((len(sizes),), 77, dtype=torch.int32, device="cuda")
            out = lib.tree_verify_attention(case.q, case.k_tree, case.v_tree, case.k_cache, case.v_cache, table,
                                            case.prefix_len, case.cu_nodes, mask, case.inp.scale, B.SMART_KV_INTERLEAVED,
                                            status=status)
            torch.cuda.synchronize()
            assert status.cpu().tolist() == [e * B.SMART_TVA_BAD_BLOCK for e in expect]
            ok_rows = torch.cat([out[cu[b]:cu[b + 1]] for b in (0, 3, 4)])
            assert torch.isfinite(ok_rows.float()).all()
    finally:
        lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 0)


# ----- seeded random shapes: batch sizes around the 64-sequence plan window, group sizes 1..16, ------
# ----- all three row classes mixed in one call, chains / stars / random trees, ragged and empty prefixes
@pytest.mark.parametrize("seed", [1, 2])
def test_random_shapes(lib, oracle_attention, seed):
    rng = np.random.default_rng(seed)
    worst = 0.0
    for case in range(40):
        batch = int(rng.choice([1, 2, 3, 5, 8, 17, 33, 64, 65, 70]))
        Hkv, G = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 7, 8, 16]))
        kind = str(rng.choice(["small", "mixed", "big"]))
        lo, hi = {"small": (1, 9), "mixed": (1, 129), "big": (40, 129)}[kind]
        sizes = rng.integers(lo, hi, batch)
        if batch * int(sizes.max()) * Hkv * G > 40000:
            sizes = np.minimum(sizes, 24)
        trees = [W.random_tree(int(n), rng, str(rng.choice(["random", "chain", "star"]))) for n in sizes]
        cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        parent = np.concatenate(trees).astype(np.int32)
        lens = rng.integers(0, int(rng.choice([40, 300, 1500])), batch).astype(np.int32)
        lens[rng.integers(0, batch)] = int(rng.choice([0, 1, 31, 32, 33, 64]))
        w = W.Workload("random_shapes", "bf16", batch, Hkv * G, Hkv, 128, 0, 0, seed=1000 * seed + case)
        c = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=lens, trees=(cu, parent), seed=1000 * seed + case)
        worst = max(worst, check_full(lib, oracle_attention, c))
    assert worst <= H.TOL["bf16"]


# ----- the softmax reference follows the maximum in steps: drifting and jumping maxima ------------
@pytest.mark.parametrize("pattern", ["drift", "spikes", "decay"])
def test_maxima_that_drift_and_jump_along_the_prefix(lib, oracle_attention, pattern):
    """The kernels rescale their accumulators only when the running maximum has moved well above the value the
    exponentials are taken against.  Keys whose scores grow slowly along the prefix keep that value stale for many
    tiles, planted spikes force the rescale, decaying scores never trigger it after the first tile; trees of every
    class (8, 40 and 128 rows per kv head at G = 4), prefixes long enough for many tiles per wavefront."""
    rng = np.random.default_rng(77)
    sizes = [2, 10, 32, 7]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    w = W.Workload("maxima_" + pattern, "bf16", 4, 16, 4, 128, 0, 0, seed=91)
    lens = np.array([4000, 3333, 2900, 517], np.int32)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=lens, trees=(cu, np.concatenate(trees).astype(np.int32)))
    inp = case.inp
    k = W.bf16_bits_to_f32(inp.k_cache)
    for b in range(4):
        t = np.arange(int(lens[b]))
        if pattern == "drift":
            f = 0.1 + 5.0 * t / lens[b]                                       # score spread grows 50-fold
        elif pattern == "decay":
            f = 5.0 * (1.0 - t / lens[b]) + 0.05
        else:
            f = np.where(rng.random(len(t)) < 0.004, 9.0, 0.3)               # rare keys with 30-fold scores
        blk, slot = inp.block_table[b][t // 16], t % 16
        k[blk, :, slot, :] *= f[:, None, None].astype(np.float32)
    inp.k_cache[...] = np.where(np.isnan(k), inp.k_cache, W.f32_to_bf16_bits(k))
    case = Case(w, cu, case.parent, inp, B.SMART_KV_INTERLEAVED)
    check_full(lib, oracle_attention, case)


# ----- a wavefront's share of a piece longer than the 64 tiles its block-id registers hold -----------
def test_long_prefix_few_workers_shares_of_several_chunks(lib, oracle_attention):
    """One sequence with 1251 tiles (ragged end) and a tree of one row tile: with one or two workers a piece is a
    whole (sequence, kv head) segment and every wavefront's share of it is about 156 tiles, i.e. three refills of
    its block-id registers.  (The fp8 cache streams through the same loop: tests/test_gpu_fp8_cache.py.)"""
    rng = np.random.default_rng(3)
    sizes = [2, 3]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, "random") for n in sizes]).astype(np.int32)
    w = W.Workload("long", "bf16", 2, 8, 2, 128, 0, 0, seed=17)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([40011, 70], np.int32), trees=(cu, parent), seed=17)
    for workers in (1, 2, 0):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            check_full(lib, oracle_attention, case)
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)


# ----- class 2: shares cut in a space of costs, for every number of workers from 1 to 40 ---------------
def test_large_trees_with_every_number_of_workers(lib, oracle_attention):
    """Trees of 96, 160 and 280 rows per kv head (three, five and eight + one row tiles: the last one has two row
    groups of unequal cost) over ragged prefixes of 22 to 33 tiles, split among 1 .. 40 workers: the share boundaries
    fall everywhere inside the segments, also less than a tile into one (a share that holds no tile of a segment it
    touches leaves an empty partial) and inside a tree's second row group."""
    rng = np.random.default_rng(23)
    sizes = [12, 20, 35]                                             # x 8 heads per kv head
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, s) for n, s in zip(sizes, ["random", "chain", "random"])]).astype(np.int32)
    w = W.Workload("large_workers", "bf16", 3, 16, 2, 128, 0, 0, seed=29)
    case = make_case(w, B.SMART_KV_INTERLEAVED, prefix_len=np.array([700, 1043, 801], np.int32), trees=(cu, parent), seed=29)
    ref, ref_lse = case.oracle(oracle_attention)
    first = None
    for workers in range(1, 41):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            out, lse = case.run(lib)
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)
        got = H.out_to_f64(out, "bf16")
        assert np.isfinite(got).all(), workers
        err = H.rel_err(got, ref)
        assert err <= H.TOL["bf16"], (workers, err)
        assert np.abs(lse.cpu().numpy().astype(np.float64) - ref_lse).max() <= 2e-2, workers
        if first is None:
            first = lse.cpu().numpy().copy()
        # however the prefix is split, the log-sum-exp of a row is the same up to rounding
        assert np.abs(lse.cpu().numpy() - first).max() <= 1e-4, workers
