"""Pins for the fp64 attention oracle (CPU only).

The paper prints no attention values, so the oracle is pinned to library
routines on special cases that cover every part of it: torch's fp64
scaled_dot_product_attention on the path of each node (chain = causal
attention, single node = decode attention, star), scipy's softmax through
one-hot values, and invariances a correct implementation must have.
"""
import numpy as np
import pytest
import torch
from scipy.special import softmax as sp_softmax

from paper_2604_09731_amd import workloads as W

BS = 16


def _small_inputs(seed, B=2, Hq=4, Hkv=2, D=16, lens=(37, 5), trees=None, dtype="f32"):
    rng = np.random.default_rng(seed)
    if trees is None:
        trees = [W.random_tree(int(rng.integers(1, 12)), rng) for _ in range(B)]
    cu = np.concatenate([[0], np.cumsum([len(t) for t in trees])]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    w = W.Workload("t", dtype, B, Hq, Hkv, D, 0, 0, seed=seed)
    inp = W.make_attention_inputs(w, cu, seed=seed, prefix_len=np.array(lens, np.int32))
    return inp, parent


def _as_f64(x, dtype):
    return (W.bf16_bits_to_f32(x) if dtype == "bf16" else x).astype(np.float64)


def _logical_kv(inp, b, g):
    """[len_b, D] prefix K and V of (sequence, kv head), through the block table."""
    L = int(inp.prefix_len[b])
    t = np.arange(L)
    blk = inp.block_table[b, t // BS]
    k = _as_f64(inp.k_cache, inp.dtype)[blk, g, t % BS]
    v = _as_f64(inp.v_cache, inp.dtype)[blk, g, t % BS]
    return k, v


def _sdpa_path(inp, parent, node, h, causal_tail=False):
    """torch fp64 SDPA of `node`'s query over [prefix ; root..node path]."""
    b = int(np.searchsorted(inp.cu_nodes, node, side="right") - 1)
    base = int(inp.cu_nodes[b])
    G = inp.q.shape[1] // inp.k_tree.shape[1]
    g = h // G
    path = []
    j = node - base
    while j >= 0:
        path.append(base + j)
        j = int(parent[base + j])
    path.reverse()
    kp, vp = _logical_kv(inp, b, g)
    kt = _as_f64(inp.k_tree, inp.dtype)[path, g]
    vt = _as_f64(inp.v_tree, inp.dtype)[path, g]
    K = torch.from_numpy(np.concatenate([kp, kt]))[None, None]
    V = torch.from_numpy(np.concatenate([vp, vt]))[None, None]
    q = torch.from_numpy(_as_f64(inp.q, inp.dtype)[node, h])[None, None, None]
    o = torch.nn.functional.scaled_dot_product_attention(q, K, V, scale=inp.scale)
    return o[0, 0, 0].numpy()


def _run(oracle_attention, inp, parent, sel=None):
    return oracle_attention.tree_attention(inp.q, inp.k_tree, inp.v_tree, inp.k_cache, inp.v_cache,
                                           inp.block_table, inp.prefix_len, inp.cu_nodes, parent,
                                           inp.scale, sel=sel)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_every_node_equals_sdpa_over_its_path(oracle_attention, dtype):
    inp, parent = _small_inputs(3, dtype=dtype)
    out, _ = _run(oracle_attention, inp, parent)
    N, Hq, _ = out.shape
    for node in range(N):
        for h in range(Hq):
            np.testing.assert_allclose(out[node, h], _sdpa_path(inp, parent, node, h),
                                       rtol=0, atol=1e-13)


def test_chain_tree_is_causal_attention(oracle_attention):
    n = 9
    inp, parent = _small_inputs(4, B=1, lens=(21,), trees=[W.random_tree(n, None, "chain")])
    out, _ = _run(oracle_attention, inp, parent)
    L = int(inp.prefix_len[0])
    Hq, Hkv = inp.q.shape[1], inp.k_tree.shape[1]
    G = Hq // Hkv
    for h in range(Hq):
        kp, vp = _logical_kv(inp, 0, h // G)
        K = torch.from_numpy(np.concatenate([kp, inp.k_tree[:, h // G].astype(np.float64)]))
        V = torch.from_numpy(np.concatenate([vp, inp.v_tree[:, h // G].astype(np.float64)]))
        # queries are the n appended tokens of a length L+n sequence: pad the
        # query side with zeros for the prefix positions and use is_causal
        Q = torch.zeros(L + n, inp.q.shape[2], dtype=torch.float64)
        Q[L:] = torch.from_numpy(inp.q[:, h].astype(np.float64))
        o = torch.nn.functional.scaled_dot_product_attention(
            Q[None, None], K[None, None], V[None, None], is_causal=True, scale=inp.scale)
        np.testing.assert_allclose(out[:, h], o[0, 0, L:].numpy(), rtol=0, atol=1e-13)


def test_single_node_is_decode_attention(oracle_attention):
    inp, parent = _small_inputs(5, B=3, lens=(16, 1, 33), trees=[np.array([-1], np.int32)] * 3)
    out, _ = _run(oracle_attention, inp, parent)
    for node in range(3):
        for h in range(out.shape[1]):
            np.testing.assert_allclose(out[node, h], _sdpa_path(inp, parent, node, h), atol=1e-13)


def test_star_tree_children_see_prefix_root_self_only(oracle_attention):
    inp, parent = _small_inputs(6, B=1, lens=(10,), trees=[W.random_tree(6, None, "star")])
    out, _ = _run(oracle_attention, inp, parent)
    # perturbing a sibling's K/V must not move a child's output at all
    k2, v2 = inp.k_tree.copy(), inp.v_tree.copy()
    k2[3] += 5.0
    v2[3] -= 7.0
    out2, _ = oracle_attention.tree_attention(inp.q, k2, v2, inp.k_cache, inp.v_cache,
                                              inp.block_table, inp.prefix_len, inp.cu_nodes,
                                              parent, inp.scale)
    for child in (1, 2, 4, 5):
        assert np.array_equal(out[child], out2[child])
    assert np.array_equal(out[0], out2[0])
    assert not np.array_equal(out[3], out2[3])


def test_probabilities_via_one_hot_values_match_scipy_softmax(oracle_attention):
    # D >= number of keys: V row x = e_x, so out = the softmax weights themselves
    D, L = 32, 11
    tree = np.array([-1, 0, 0, 1, 3], np.int32)      # node 4: path 0-1-3-4
    inp, parent = _small_inputs(7, B=1, Hq=2, Hkv=1, D=D, lens=(L,), trees=[tree])
    inp.v_cache[...] = 0
    inp.v_tree[...] = 0
    for t in range(L):
        inp.v_cache[inp.block_table[0, t // BS], 0, t % BS, t] = 1.0
    for j in range(5):
        inp.v_tree[j, 0, L + j] = 1.0
    out, lse = _run(oracle_attention, inp, parent)
    kp, _ = _logical_kv(inp, 0, 0)
    anc = {0: [0], 1: [0, 1], 2: [0, 2], 3: [0, 1, 3], 4: [0, 1, 3, 4]}
    for node, path in anc.items():
        for h in range(2):
            keys = np.concatenate([kp, inp.k_tree[path, 0].astype(np.float64)])
            s = inp.scale * keys @ inp.q[node, h].astype(np.float64)
            p = sp_softmax(s)
            expect = np.zeros(D)
            expect[:L] = p[:L]
            for a, j in enumerate(path):
                expect[L + j] = p[L + a]
            np.testing.assert_allclose(out[node, h], expect, atol=1e-14)
            assert abs(out[node, h].sum() - 1.0) < 1e-13
            from scipy.special import logsumexp
            assert abs(lse[node, h] - logsumexp(s)) < 1e-12


def test_non_ancestor_perturbation_is_invisible_and_ancestor_is_not(oracle_attention):
    rng = np.random.default_rng(8)
    tree = W.random_tree(12, rng)
    inp, parent = _small_inputs(8, B=1, lens=(19,), trees=[tree])
    out, _ = _run(oracle_attention, inp, parent)
    anc = []
    for i in range(12):
        s, j = set(), i
        while j >= 0:
            s.add(j)
            j = int(parent[j])
        anc.append(s)
    for j in range(12):
        k2, v2 = inp.k_tree.copy(), inp.v_tree.copy()
        k2[j] *= -3.0
        v2[j] += 11.0
        out2, _ = oracle_attention.tree_attention(inp.q, k2, v2, inp.k_cache, inp.v_cache,
                                                  inp.block_table, inp.prefix_len, inp.cu_nodes,
                                                  parent, inp.scale)
        for i in range(12):
            same = np.array_equal(out[i], out2[i])
            assert same == (j not in anc[i]), (i, j)


def test_topological_relabelling_permutes_outputs(oracle_attention):
    rng = np.random.default_rng(9)
    n = 10
    tree = W.random_tree(n, rng)
    inp, parent = _small_inputs(9, B=1, lens=(23,), trees=[tree])
    out, lse = _run(oracle_attention, inp, parent)
    # random topological order: repeatedly pick any node whose parent is placed
    placed, order = set(), []
    while len(order) < n:
        ready = [i for i in range(n) if i not in placed and (parent[i] < 0 or parent[i] in placed)]
        pick = int(rng.choice(ready))
        placed.add(pick)
        order.append(pick)
    assert order != list(range(n))
    new_of_old = {o: i for i, o in enumerate(order)}
    parent2 = np.array([-1 if parent[o] < 0 else new_of_old[int(parent[o])] for o in order], np.int32)
    out2, lse2 = oracle_attention.tree_attention(inp.q[order], inp.k_tree[order], inp.v_tree[order],
                                                 inp.k_cache, inp.v_cache, inp.block_table,
                                                 inp.prefix_len, inp.cu_nodes, parent2, inp.scale)
    np.testing.assert_allclose(out2, out[order], rtol=0, atol=1e-12)
    np.testing.assert_allclose(lse2, lse[order], rtol=0, atol=1e-12)


def test_shared_key_shift_changes_nothing_and_gqa_groups(oracle_attention):
    inp, parent = _small_inputs(10, B=1, Hq=4, Hkv=2, lens=(30,))
    inp.q[:, 1] = inp.q[:, 0]      # same group (G = 2): identical outputs
    inp.q[:, 2] = inp.q[:, 0]      # other group: different K/V, different output
    out, lse = _run(oracle_attention, inp, parent)
    assert np.array_equal(out[:, 0], out[:, 1])
    assert not np.allclose(out[:, 0], out[:, 2])
    c = np.random.default_rng(1).standard_normal(inp.q.shape[2]).astype(np.float32)
    k_tree2 = inp.k_tree + c
    k_cache2 = inp.k_cache + c
    out2, lse2 = oracle_attention.tree_attention(inp.q, k_tree2, inp.v_tree, k_cache2, inp.v_cache,
                                                 inp.block_table, inp.prefix_len, inp.cu_nodes,
                                                 parent, inp.scale)
    np.testing.assert_allclose(out2, out, rtol=0, atol=1e-5)   # f32 rounding of k + c only
    shift = inp.scale * (inp.q.astype(np.float64) @ c.astype(np.float64))
    np.testing.assert_allclose(lse2 - lse, shift, atol=1e-4)


def test_paging_invariance_and_poison(oracle_attention):
    inp, parent = _small_inputs(11, B=2, lens=(37, 20))
    out, _ = _run(oracle_attention, inp, parent)
    assert np.isfinite(out).all()                 # NaN-filled unused slots are never read
    assert np.isnan(inp.k_cache).any()
    nb = inp.k_cache.shape[0]
    perm = np.random.default_rng(2).permutation(nb)
    k2 = np.empty_like(inp.k_cache)
    v2 = np.empty_like(inp.v_cache)
    k2[perm] = inp.k_cache
    v2[perm] = inp.v_cache
    bt2 = np.where(inp.block_table >= 0, perm[np.maximum(inp.block_table, 0)], 0).astype(np.int32)
    bt_clean = np.where(inp.block_table >= 0, inp.block_table, 0).astype(np.int32)
    out_a, _ = oracle_attention.tree_attention(inp.q, inp.k_tree, inp.v_tree, inp.k_cache, inp.v_cache,
                                               bt_clean, inp.prefix_len, inp.cu_nodes, parent, inp.scale)
    out_b, _ = oracle_attention.tree_attention(inp.q, inp.k_tree, inp.v_tree, k2, v2, bt2,
                                               inp.prefix_len, inp.cu_nodes, parent, inp.scale)
    assert np.array_equal(out_a, out_b)
    assert np.array_equal(out_a, out)


def test_bf16_inputs_are_upcast_exactly_and_selection_mode(oracle_attention):
    inp, parent = _small_inputs(12, dtype="bf16")
    out, lse = _run(oracle_attention, inp, parent)
    f = lambda a: W.bf16_bits_to_f32(a)
    out32, _ = oracle_attention.tree_attention(f(inp.q), f(inp.k_tree), f(inp.v_tree),
                                               np.nan_to_num(f(inp.k_cache)), np.nan_to_num(f(inp.v_cache)),
                                               inp.block_table, inp.prefix_len, inp.cu_nodes, parent, inp.scale)
    assert np.array_equal(out, out32)
    nodes = np.array([0, out.shape[0] - 1, 1], np.int32)
    heads = np.array([3, 0, 2], np.int32)
    o_sel, l_sel = _run(oracle_attention, inp, parent, sel=(nodes, heads))
    assert np.array_equal(o_sel, out[nodes, heads])
    assert np.array_equal(l_sel, lse[nodes, heads])


def test_empty_prefix_and_rejects_bad_tree(oracle_attention):
    inp, parent = _small_inputs(13, B=2, lens=(0, 3))
    out, _ = _run(oracle_attention, inp, parent)
    for node in range(out.shape[0]):
        np.testing.assert_allclose(out[node, 0], _sdpa_path(inp, parent, node, 0), atol=1e-13)
    bad = parent.copy()
    if len(bad) > 1:
        bad[1] = 1
        with pytest.raises(ValueError):
            _run(oracle_attention, inp, bad)
