"""GPU parity of Algorithm 1 one layer at a time on the device (smart_select_begin_device,
smart_select_layer_device) and of tree_compact_pack, against the CPU oracle, through the C ABI.
Everything here is compared bit for bit: decisions, node order, P, L and R are binary64 values
that both sides must compute with the same operations in the same order."""
import numpy as np
import pytest

from oracle import pack_accept as PA
from oracle import selection as S
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return B.SmartTree(0)


def _dev(a, dtype):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype)).to("cuda")


def _forests(seed, batch, k_range=(2, 5), d_range=(2, 5), cap=600):
    rng = np.random.default_rng(seed)
    forests = []
    for _ in range(batch):
        k, d = int(rng.integers(*k_range)), int(rng.integers(*d_range))
        parent, prob, depth = [-1], [1.0], [0]
        i = 0
        while i < len(parent) and len(parent) < cap:
            if depth[i] < d:
                p = rng.dirichlet(np.ones(k + 1))[:k]
                for j in np.argsort(-p):
                    parent.append(i)
                    prob.append(float(p[j]))
                    depth.append(depth[i] + 1)
            i += 1
        forests.append((parent, prob, [int(t) for t in rng.integers(0, 32000, len(parent))]))
    return forests


def _device_layers(lib, forests, cost, dcost, alpha, max_depth, budget, dilution):
    """Runs the device form over the forests' layers; returns (state, candidate index per node)."""
    import torch
    nb = len(forests)
    st = B.DeviceLayerState(nb, budget, "cuda")
    d_cost = _dev(cost, np.float64)
    d_dcost = None if dcost is None else _dev(dcost, np.float64)
    lib.select_begin(st, _dev([f[2][0] for f in forests], np.int32), d_cost)

    def step(cu, parent_nodes, offered):
        prob = [forests[b][1][u] for b in range(nb) for u in offered[b]]
        tok = [forests[b][2][u] for b in range(nb) for u in offered[b]]
        out, status = lib.select_layer(st, _dev(cu, np.int32), _dev(parent_nodes, np.int32), _dev(prob, np.float64),
                                       _dev(tok, np.int32), d_cost, d_dcost, alpha=alpha, dilution=dilution)
        torch.cuda.synchronize()
        assert status.cpu().numpy().tolist() == [0] * nb
        return out.cpu().numpy().tolist()

    cand = H.drive_layers_batch([f[0] for f in forests], max_depth, step)
    torch.cuda.synchronize()
    return st, cand


def _host_state(st):
    return {k: getattr(st, k).cpu().numpy() for k in
            ("n", "layer_begin", "sum_P", "parent", "token", "pathprob", "path_sum", "L", "R")}


def _check_against_oracle(st, cand, forests, cost, dcost, alpha, max_depth, budget, dilution):
    h = _host_state(st)
    for b, (parent, prob, token) in enumerate(forests):
        t = S.select_tree(parent, prob, token, list(cost), None if dcost is None else list(dcost), alpha=alpha,
                          max_depth=max_depth, budget=budget, schedule=S.LAYERWISE, dilution=dilution)
        n, o = int(h["n"][b]), b * budget
        assert n == len(t) and cand[b] == t.cand_index, (b, n, len(t))
        assert h["parent"][o:o + n].tolist() == t.parent and h["token"][o:o + n].tolist() == t.token
        assert h["pathprob"][o:o + n].tolist() == t.pathprob          # bit for bit
        assert h["L"][b] == t.L and h["R"][b] == t.R, (b, h["L"][b], t.L)


@pytest.mark.parametrize("dilution", [B.SMART_DILUTION_NONE, B.SMART_DILUTION_PATH_MEAN])
@pytest.mark.parametrize("seed", range(3))
def test_device_layers_bit_exact_against_the_oracle(lib, seed, dilution):
    forests = _forests(seed, batch=33)
    cost = np.array([1.0 + 0.01 * n + 0.0005 * n * n for n in range(130)])
    dcost = np.array([0.01 + 0.001 * n for n in range(129)]) if seed % 2 else None
    for budget, max_depth in ((128, 4), (12, 4), (3, 3), (1, 2)):
        st, cand = _device_layers(lib, forests, cost, dcost, 0.85, max_depth, budget, dilution)
        _check_against_oracle(st, cand, forests, cost, dcost, 0.85, max_depth, budget, dilution)


@pytest.mark.parametrize("dilution", [B.SMART_DILUTION_NONE, B.SMART_DILUTION_PATH_MEAN])
def test_wide_layers_over_several_lane_chunks_and_a_budget_that_cuts_them(lib, dilution):
    """Fan-out 12: layers of 12, 144 and up to 1500 candidates (many 64-lane chunks), a cheap cost so
    that far more pass the rule than the budget admits, and equal probabilities among them (ties)."""
    rng = np.random.default_rng(5)
    forests = []
    for _ in range(5):
        parent, prob, depth = [-1], [1.0], [0]
        i = 0
        while i < len(parent):
            if depth[i] < 3 and len(parent) < 1700:
                p = np.round(rng.dirichlet(np.ones(13))[:12] * 16) / 16      # coarse values: many exact ties
                for j in range(12):
                    parent.append(i)
                    prob.append(float(min(max(p[j], 1 / 16), 1.0)))
                    depth.append(depth[i] + 1)
            i += 1
        forests.append((parent, prob, list(range(len(parent)))))
    cost = np.array([1.0 + 1e-4 * n for n in range(130)])
    for budget in (128, 100, 30):
        st, cand = _device_layers(lib, forests, cost, None, 1.0, 3, budget, dilution)
        _check_against_oracle(st, cand, forests, cost, None, 1.0, 3, budget, dilution)
        if dilution == B.SMART_DILUTION_NONE:
            assert _host_state(st)["n"].max() == budget                  # the cut really happened


def test_device_layer_statuses_and_untouched_state(lib):
    import torch
    cost = np.array([1.0 + n / 8.0 for n in range(12)])
    d_cost = _dev(cost, np.float64)
    st = B.DeviceLayerState(4, 8, "cuda")
    lib.select_begin(st, _dev([5, 6, 7, 8], np.int32), d_cost)
    out, status = lib.select_layer(st, _dev([0, 2, 3, 4, 5], np.int32), _dev([0] * 5, np.int32),
                                   _dev([0.5, 0.25, 0.5, 0.5, 0.5], np.float64), _dev([1, 2, 3, 4, 5], np.int32),
                                   d_cost, alpha=1.0)
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [0, 0, 0, 0] and out.cpu().numpy().tolist() == [1, 2, 1, 1, 1]
    before = _host_state(st)
    # seq 0: parent no longer in the newest layer; seq 1: fine; seq 2: not a probability; seq 3: offers nothing
    out, status = lib.select_layer(st, _dev([0, 1, 2, 3, 3], np.int32), _dev([0, 1, 1], np.int32),
                                   _dev([0.5, 0.5, 1.5], np.float64), _dev([9, 9, 9], np.int32), d_cost, alpha=1.0)
    torch.cuda.synchronize()
    after = _host_state(st)
    assert status.cpu().numpy().tolist() == [B.SMART_ETREE, 0, B.SMART_ETREE, 0]
    assert out.cpu().numpy().tolist() == [-1, 2, -1]
    for b in (0, 2):
        for k in ("n", "layer_begin", "sum_P", "L", "R"):
            assert after[k][b] == before[k][b], (k, b)
        assert np.array_equal(after["parent"][b * 8:b * 8 + 8], before["parent"][b * 8:b * 8 + 8])
    assert after["n"].tolist() == [3, 3, 2, 2] and after["layer_begin"].tolist() == [1, 2, 1, 2]
    # offsets that leave the candidate arrays: nothing of that sequence is touched
    out, status = lib.select_layer(st, _dev([0, 0, 9, 9, 9], np.int32), _dev([2, 2], np.int32),
                                   _dev([0.5, 0.5], np.float64), _dev([1, 1], np.int32), d_cost, alpha=1.0)
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [0, B.SMART_ETREE, B.SMART_ETREE, B.SMART_ETREE]
    assert _host_state(st)["n"].tolist() == [3, 3, 2, 2]
    # more candidates than one launch takes
    big = B.SMART_MAX_LAYER_CAND + 1
    st1 = B.DeviceLayerState(1, 8, "cuda")
    lib.select_begin(st1, _dev([1], np.int32), d_cost)
    out, status = lib.select_layer(st1, _dev([0, big], np.int32), _dev([0] * big, np.int32),
                                   _dev([0.5] * big, np.float64), _dev([1] * big, np.int32), d_cost)
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [B.SMART_ECAP] and (out.cpu().numpy() == -1).all()
    assert _host_state(st1)["n"].tolist() == [1]
    # exactly the limit is fine
    big = B.SMART_MAX_LAYER_CAND
    out, status = lib.select_layer(st1, _dev([0, big], np.int32), _dev([0] * big, np.int32),
                                   _dev([0.5] * big, np.float64), _dev(np.arange(big), np.int32), d_cost, alpha=1.0)
    torch.cuda.synchronize()
    assert status.cpu().numpy().tolist() == [0]
    assert out.cpu().numpy()[:8].tolist() == [1, 2, 3, 4, 5, 6, 7, -1] and _host_state(st1)["n"].tolist() == [8]


def test_compact_pack_then_attention_with_a_capacity_instead_of_a_size(lib, oracle_attention):
    """The whole device-side front end: layers -> tree_compact_pack -> tree_verify_attention called with
    total_nodes = capacity, compared with the oracle on the trees the oracle selects."""
    import torch
    budget, max_depth = 24, 4
    forests = _forests(11, batch=7)
    cost = np.array([1.0 + 0.02 * n for n in range(130)])
    st, cand = _device_layers(lib, forests, cost, None, 0.9, max_depth, budget, B.SMART_DILUTION_NONE)
    h = _host_state(st)
    sizes = h["n"].tolist()
    assert len(set(sizes)) > 2 and max(sizes) > 8
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([h["parent"][b * budget:b * budget + sizes[b]] for b in range(7)]).astype(np.int32)
    token = np.concatenate([h["token"][b * budget:b * budget + sizes[b]] for b in range(7)]).astype(np.int32)
    N, cap = int(cu[-1]), 7 * budget
    for dtype, layout, Hq, Hkv in (("bf16", B.SMART_KV_INTERLEAVED, 8, 2), ("f32", B.SMART_KV_PLAIN, 4, 2)):
        w = W.Workload("device_front_end", dtype, 7, Hq, Hkv, 128, 0, 0, seed=3)
        lens = np.array([0, 5, 31, 64, 100, 517, 33], np.int32)
        inp = W.make_attention_inputs(w, cu, seed=3, prefix_len=lens)
        d_len = _dev(lens, np.int32)
        d_cu, d_par, d_tok, depth, pos, seq, mask, status = lib.tree_compact_pack(st, d_len)
        torch.cuda.synchronize()
        assert status.cpu().numpy().tolist() == [0] * 7
        assert d_cu.cpu().numpy().tolist() == cu.tolist() and d_par.shape[0] == cap
        assert d_par.cpu().numpy()[:N].tolist() == parent.tolist() and d_tok.cpu().numpy()[:N].tolist() == token.tolist()
        o_depth, o_pos, o_seq, o_mask = PA.pack(cu, parent, lens)
        assert depth.cpu().numpy()[:N].tolist() == o_depth and pos.cpu().numpy()[:N].tolist() == o_pos
        assert seq.cpu().numpy()[:N].tolist() == o_seq
        words = np.stack([np.array([m[0] for m in o_mask], np.uint64), np.array([m[1] for m in o_mask], np.uint64)], 1)
        assert np.array_equal(mask.cpu().numpy().view(np.uint64)[:N], words)

        def padded(x):                      # per-node inputs in arrays of `cap` rows, the tail poisoned
            t = H.torch_elems(x, dtype, "cuda")
            full = torch.full((cap,) + tuple(t.shape[1:]), float("nan"), dtype=t.dtype, device="cuda")
            full[:N] = t
            return full
        kc, vc = H.torch_elems(inp.k_cache, dtype, "cuda"), H.torch_elems(inp.v_cache, dtype, "cuda")
        if layout == B.SMART_KV_INTERLEAVED:
            kc, vc = B.interleave_kv_cache(kc, vc)
        out = torch.full((cap, Hq, 128), 7.0, dtype=kc.dtype, device="cuda")
        out, lse = lib.tree_verify_attention(padded(inp.q), padded(inp.k_tree), padded(inp.v_tree), kc, vc,
                                             _dev(inp.block_table, np.int32), d_len, d_cu, mask, inp.scale, layout,
                                             out=out, want_lse=True)
        torch.cuda.synchronize()
        ref, _ = oracle_attention.tree_attention(inp.q, inp.k_tree, inp.v_tree, inp.k_cache, inp.v_cache,
                                                 inp.block_table, inp.prefix_len, cu, parent, inp.scale)
        got = H.out_to_f64(out, dtype)
        assert H.rel_err(got[:N], ref) <= H.TOL[dtype]
        tail = got[N:]
        assert np.isfinite(tail).all() and (np.all(tail == 7.0) or np.all(tail == 0.0))   # untouched or zero-filled
