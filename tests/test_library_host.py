"""CPU-only checks of the C-ABI library: it loads, exports every declared
symbol, rejects bad arguments before touching a device, and its host-side
selection is bit-exact against the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import selection as S
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "smart_tree.h")).read()
    declared = set(re.findall(r"^(?:int32_t|const char\*)\s+(\w+)\s*\(", header, flags=re.M))
    assert declared == set(B.EXPORTS)
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in declared:
        assert hasattr(lib, name), name
    assert B._strerror(0) == "ok" and "tree" in B._strerror(B.SMART_ETREE)


def test_timeline_build_exports_the_library_and_its_two_calls():
    """The timeline build (stamps in the attention kernels, for python -m paper_2604_09731_amd.timeline) is the
    same library plus smart_timeline_read / smart_timeline_clear; the ordinary library has neither."""
    from paper_2604_09731_amd import timeline
    assert os.path.exists(timeline.TIMELINE_LIB), "build it with python -m paper_2604_09731_amd.build"
    stamped = ctypes.CDLL(timeline.TIMELINE_LIB)
    for name in list(B.EXPORTS) + ["smart_timeline_read", "smart_timeline_clear"]:
        assert hasattr(stamped, name), name
    plain = ctypes.CDLL(B.LIB_PATH)
    assert not hasattr(plain, "smart_timeline_read") and not hasattr(plain, "smart_timeline_clear")


@pytest.mark.parametrize("name", ["cfg2", "cfg3a", "cfg3b", "cfg4", "cfg5a", "cfg5b"])
def test_selection_bit_exact_on_workloads(name):
    w = W.WORKLOADS[name]
    w = w.scaled(batch=min(w.batch, 12))
    forest = W.make_forest(w)
    a = H.trees_from_oracle(w, forest)
    b = H.trees_from_library(w, forest)
    for x, y in zip(a, b):
        assert np.array_equal(x, y)


@pytest.mark.parametrize("schedule", [B.SMART_BEST_FIRST, B.SMART_LAYERWISE])
@pytest.mark.parametrize("dilution", [B.SMART_DILUTION_NONE, B.SMART_DILUTION_PATH_MEAN])
@pytest.mark.parametrize("alpha", [1.0, 0.8, 0.55])
def test_selection_all_modes_bit_exact_including_L_R_pathprob(schedule, dilution, alpha):
    for wname, budget, depth in [("cfg2", 128, 8), ("cfg4", 96, 6), ("cfg2", 17, 3), ("cfg4", 1, 6)]:
        w = W.WORKLOADS[wname].scaled(batch=5)
        f = W.make_forest(w, seed=77 + budget)
        cost = W.cost_table(w, n_max=budget)
        dcost = None
        r = B.smart_select_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, dcost,
                                alpha=alpha, max_depth=depth, budget=budget, schedule=schedule,
                                dilution=dilution)
        trees = S.select_batch(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, dcost,
                               alpha=alpha, max_depth=depth, budget=budget, schedule=schedule,
                               dilution=dilution)
        for b, t in enumerate(trees):
            lo, hi = r["cu_nodes"][b], r["cu_nodes"][b + 1]
            assert r["parent"][lo:hi].tolist() == t.parent
            assert r["token"][lo:hi].tolist() == t.token
            assert r["cand_index"][lo:hi].tolist() == t.cand_index
            assert r["pathprob"][lo:hi].tolist() == t.pathprob      # bit-exact doubles
            assert r["L"][b] == t.L and r["R"][b] == t.R


def test_selection_with_derivative_table_and_knee_costs():
    w = W.WORKLOADS["cfg3a"].scaled(batch=6)
    f = W.make_forest(w)
    cost = W.cost_table(w)
    dcost = np.gradient(cost)[: w.budget + 1] * 0.9
    r = B.smart_select_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, dcost,
                            alpha=0.9, max_depth=8, budget=w.budget)
    trees = S.select_batch(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, dcost,
                           alpha=0.9, max_depth=8, budget=w.budget)
    assert r["cand_index"].tolist() == sum((t.cand_index for t in trees), [])


def test_selection_error_paths():
    w = W.WORKLOADS["cfg2"].scaled(batch=2)
    f = W.make_forest(w)
    cost = W.cost_table(w)
    ok = dict(alpha=0.8, max_depth=8, budget=64)
    call = lambda **kw: B.smart_select_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost,
                                            **{**ok, **kw})
    for bad in (dict(alpha=0.0), dict(alpha=1.5), dict(alpha=float("nan")), dict(budget=0),
                dict(budget=129), dict(max_depth=-1), dict(schedule=7), dict(dilution=-1)):
        if bad.get("budget") == 129:
            with pytest.raises((B.SmartError, ValueError)):
                call(**bad)
            continue
        with pytest.raises(B.SmartError) as e:
            call(**bad)
        assert e.value.code == B.SMART_EINVAL
    with pytest.raises(B.SmartError) as e:
        call(out_cap=10)
    assert e.value.code == B.SMART_ECAP
    bad_parent = f.cand_parent.copy()
    bad_parent[5] = 9
    with pytest.raises(B.SmartError) as e:
        B.smart_select_tree(f.cand_cu, bad_parent, f.cand_prob, f.cand_token, cost, **ok)
    assert e.value.code == B.SMART_ETREE
    bad_prob = f.cand_prob.copy()
    bad_prob[3] = 1.5
    with pytest.raises(B.SmartError) as e:
        B.smart_select_tree(f.cand_cu, f.cand_parent, bad_prob, f.cand_token, cost, **ok)
    assert e.value.code == B.SMART_ETREE
    two_roots = f.cand_parent.copy()
    two_roots[1] = -1
    with pytest.raises(B.SmartError) as e:
        B.smart_select_tree(f.cand_cu, two_roots, f.cand_prob, f.cand_token, cost, **ok)
    assert e.value.code == B.SMART_ETREE
    # empty batch is fine
    r = B.smart_select_tree(np.zeros(1, np.int32), np.zeros(0, np.int32), np.zeros(0), np.zeros(0, np.int32),
                            cost, **ok)
    assert r["cu_nodes"].tolist() == [0]


def test_device_entry_points_validate_on_the_host_first():
    """Every case below is invalid, so each call must return its error code
    before it looks at the context or the device (there is no GPU here): a
    zeroed buffer stands in for the context."""
    lib = B._lib()
    fake = ctypes.create_string_buffer(512)
    ctx = ctypes.cast(fake, ctypes.c_void_p)
    one = ctypes.create_string_buffer(64)
    ptr = ctypes.cast(one, ctypes.c_void_p)
    assert lib.tree_pack(None, None, 1, 1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.tree_pack(ctx, None, -1, 1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.tree_pack(ctx, None, 1, 1, None, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.tree_pack(ctx, None, 1, 1, ptr, ptr, ptr, ptr, ptr, ptr, None, ptr) == B.SMART_EINVAL
    assert lib.tree_accept(ctx, None, 1, -1, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.tree_accept(ctx, None, 1, 8, ptr, None, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.tree_accept(None, None, 1, 8, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert lib.kv_cache_write(ctx, None, 5, 0, 1, 8, 128, 16, 4, ptr, ptr, ptr, ptr, ptr, 16384, 2048, 128) == B.SMART_EINVAL
    assert lib.kv_cache_write(ctx, None, 1, 1, 1, 8, 128, 12, 4, ptr, ptr, ptr, ptr, ptr, 16384, 2048, 128) == B.SMART_EINVAL
    assert lib.kv_cache_write(ctx, None, 1, 1, 1, 8, 128, 16, 4, ptr, ptr, ptr, ptr, ptr, 16384, 100, 128) == B.SMART_EINVAL
    commit = lambda **kw: lib.tree_commit(*[kw.get(k, v) for k, v in dict(
        ctx=ctx, stream=None, dtype=1, layout=1, batch=2, max_depth=4, Hkv=8, D=128, bs=16, max_blocks=4, nb=8,
        cu=ptr, alen=ptr, apath=ptr, kt=ptr, vt=ptr, bt=ptr, plen=ptr, kc=ptr, vc=ptr, bstride=16384,
        hstride=2048, tstride=128, nlen=ctypes.cast(fake, ctypes.c_void_p), st=ptr).items()])
    assert commit(ctx=None) == B.SMART_EINVAL
    assert commit(dtype=7) == B.SMART_EINVAL
    assert commit(layout=3) == B.SMART_EINVAL
    assert commit(max_depth=-1) == B.SMART_EINVAL
    assert commit(bs=12) == B.SMART_EINVAL            # interleaved layout needs multiples of 8
    assert commit(hstride=100) == B.SMART_EINVAL
    assert commit(kt=None) == B.SMART_EINVAL
    assert commit(nlen=ptr) == B.SMART_EINVAL         # new lengths may not alias the old ones
    assert commit(batch=0) == B.SMART_OK
    up = lambda *a: lib.tree_upload_pack(*a)
    assert up(None, None, 1, 1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert up(ctx, None, 1, 1, None, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL
    assert up(ctx, None, 1, 1, ptr, ptr, None, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL   # token: both or none
    assert up(ctx, None, 1, 1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, None, ptr) == B.SMART_EINVAL
    assert up(ctx, None, 0, 0, ptr, None, None, ptr, None, None, ptr, None, None, None, None, ptr) == B.SMART_OK
    assert up(ctx, None, 1, 1, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr, ptr) == B.SMART_EINVAL   # pageable
    assert lib.smart_set_option(None, 1, 0) == B.SMART_EINVAL
    assert lib.smart_set_option(ctx, B.SMART_OPT_TVA_PROFILE_STRIDE, 0) == B.SMART_EINVAL
    assert lib.tree_upload(None, None, ptr, ptr, 4) == B.SMART_EINVAL
    assert lib.tree_upload(ctx, None, ptr, ptr, -1) == B.SMART_EINVAL
    assert lib.tree_upload(ctx, None, None, ptr, 4) == B.SMART_EINVAL
    assert lib.tree_upload(ctx, None, ptr, None, 4) == B.SMART_EINVAL
    assert lib.tree_upload(ctx, None, None, None, 0) == B.SMART_OK
    # pageable host memory is refused before anything is launched (here: no device at all)
    assert lib.tree_upload(ctx, None, ptr, ptr, 4) == B.SMART_EINVAL
    assert lib.smart_create(None, 0) == B.SMART_EINVAL
    assert lib.smart_destroy(None) == B.SMART_EINVAL

    def tva(**kw):
        p = B.TvaParams()
        base = dict(dtype=1, kv_layout=1, batch=1, total_nodes=1, num_q_heads=32, num_kv_heads=8,
                    head_dim=128, block_size=16, max_blocks_per_seq=4, num_blocks=4,
                    softmax_scale=0.088, cache_block_stride=8 * 2048, cache_head_stride=2048,
                    cache_token_stride=128)
        base.update(kw)
        for k, v in base.items():
            setattr(p, k, v)
        for f in ("d_q", "d_k_tree", "d_v_tree", "d_k_cache", "d_v_cache", "d_block_table",
                  "d_prefix_len", "d_cu_nodes", "d_anc_mask", "d_out"):
            if f not in kw:
                setattr(p, f, ptr.value)
        return lib.tree_verify_attention(ctx, None, ctypes.byref(p))

    assert lib.tree_verify_attention(None, None, None) == B.SMART_EINVAL
    for bad in (dict(dtype=3), dict(kv_layout=2), dict(num_q_heads=30), dict(head_dim=96),
                dict(block_size=12), dict(block_size=128), dict(softmax_scale=0.0),
                dict(softmax_scale=float("nan")), dict(cache_head_stride=100),
                dict(cache_block_stride=1024), dict(batch=-1), dict(d_q=None), dict(d_anc_mask=None),
                dict(d_k_cache=None), dict(kv_layout=0, cache_token_stride=64), dict(num_blocks=0)):
        assert tva(**bad) == B.SMART_EINVAL, bad


def _hand_worked():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "selection_hand_worked.json")) as f:
        return json.load(f)


def test_hand_worked_example_library():
    """The same hand-worked forest through the C ABI."""
    g = _hand_worked()
    fo = g["forest"]
    cost = np.array([1.0 + n / 8.0 for n in range(9)])
    modes = {"BEST_FIRST": B.SMART_BEST_FIRST, "LAYERWISE": B.SMART_LAYERWISE}
    dil = {"NONE": B.SMART_DILUTION_NONE, "PATH_MEAN": B.SMART_DILUTION_PATH_MEAN}
    for case in g["cases"]:
        r = B.smart_select_tree(np.array([0, 6], np.int32), fo["parent"], fo["prob"], fo["token"], cost,
                                alpha=case["alpha"], max_depth=g["max_depth"], budget=g["budget"],
                                schedule=modes[case["schedule"]], dilution=dil[case["dilution"]])
        assert r["cand_index"].tolist() == case["cand_index"], case["name"]
        assert r["parent"].tolist() == case["parent"], case["name"]
        assert r["pathprob"].tolist() == [fo["path_prob"][i] for i in case["cand_index"]]
        assert r["L"][0] == case["L"] and r["R"][0] == case["R"], case["name"]


# ---------------------------------------------------------------------------
# Algorithm 1 one layer at a time (host form)
# ---------------------------------------------------------------------------
def _layered_forests(seed, batch):
    rng = np.random.default_rng(seed)
    forests = []
    for _ in range(batch):
        k, d = int(rng.integers(2, 5)), int(rng.integers(2, 5))
        parent, prob, depth = [-1], [1.0], [0]
        i = 0
        while i < len(parent) and len(parent) < 400:
            if depth[i] < d:
                p = rng.dirichlet(np.ones(k + 1))[:k]
                for j in np.argsort(-p):
                    parent.append(i)
                    prob.append(float(p[j]))
                    depth.append(depth[i] + 1)
            i += 1
        forests.append((parent, prob, list(rng.integers(0, 32000, len(parent)))))
    return forests


def _library_layers(forests, cost, dcost, alpha, max_depth, budget, dilution):
    from tests.helpers import drive_layers_batch
    st = B.HostLayerState(len(forests), budget)
    st.begin([f[2][0] for f in forests], cost)

    def step(cu, parent_nodes, offered):
        prob = [forests[b][1][u] for b in range(len(forests)) for u in offered[b]]
        tok = [forests[b][2][u] for b in range(len(forests)) for u in offered[b]]
        return st.layer(cu, parent_nodes, prob, tok, cost, dcost, alpha=alpha, dilution=dilution)

    cand = drive_layers_batch([f[0] for f in forests], max_depth, step)
    return st, cand


@pytest.mark.parametrize("dilution", [B.SMART_DILUTION_NONE, B.SMART_DILUTION_PATH_MEAN])
@pytest.mark.parametrize("seed", range(4))
def test_layer_at_a_time_bit_exact_against_the_oracle(seed, dilution):
    forests = _layered_forests(seed, batch=9)
    cost = np.array([1.0 + 0.01 * n + 0.0005 * n * n for n in range(130)])
    dcost = np.array([0.01 + 0.001 * n for n in range(129)]) if seed % 2 else None
    for budget, max_depth in ((128, 4), (12, 4), (3, 3), (1, 2)):
        st, cand = _library_layers(forests, cost, dcost, 0.85, max_depth, budget, dilution)
        for b, (parent, prob, token) in enumerate(forests):
            t = S.select_tree(parent, prob, token, cost.tolist(), None if dcost is None else dcost.tolist(),
                              alpha=0.85, max_depth=max_depth, budget=budget, schedule=S.LAYERWISE,
                              dilution=dilution)
            par_b, tok_b, pp_b = st.tree(b)
            assert cand[b] == t.cand_index and par_b == t.parent and tok_b == [int(x) for x in t.token]
            assert pp_b == t.pathprob                               # bit for bit
            assert st.L[b] == t.L and st.R[b] == t.R


def test_layer_at_a_time_hand_worked_example_library():
    from tests.helpers import drive_layers_batch
    g = _hand_worked()
    fo = g["forest"]
    cost = np.array([1.0 + n / 8.0 for n in range(9)])
    for case in g["cases"]:
        if case["schedule"] != "LAYERWISE":
            continue
        st, cand = _library_layers([(fo["parent"], fo["prob"], fo["token"])], cost, None, case["alpha"],
                                   g["max_depth"], g["budget"], getattr(B, "SMART_DILUTION_" + case["dilution"]))
        par, tok, _ = st.tree(0)
        assert cand[0] == case["cand_index"] and par == case["parent"], case["name"]
        assert st.L[0] == case["L"] and st.R[0] == case["R"], case["name"]


def test_layer_at_a_time_error_paths_leave_the_state_alone():
    cost = np.array([1.0 + n / 8.0 for n in range(12)])
    st = B.HostLayerState(2, 8)
    st.begin([5, 6], cost)
    st.layer([0, 2, 3], [0, 0, 0], [0.5, 0.25, 0.5], [1, 2, 3], cost, alpha=1.0)
    snap = {k: getattr(st, k).copy() for k in ("n", "layer_begin", "sum_P", "parent", "token", "pathprob", "L", "R")}

    def refused(code, *a, **kw):
        with pytest.raises(B.SmartError) as e:
            st.layer(*a, **kw)
        assert e.value.code == code
        for k, v in snap.items():
            assert np.array_equal(getattr(st, k), v), k

    refused(B.SMART_ETREE, [0, 1, 1], [0], [0.5], [1], cost)              # node 0 is no longer in the newest layer
    refused(B.SMART_ETREE, [0, 1, 2], [1, 5], [0.5, 0.5], [1, 2], cost)   # node 5 does not exist
    refused(B.SMART_ETREE, [0, 1, 1], [1], [1.5], [1], cost)              # not a probability
    refused(B.SMART_ETREE, [0, 1, 1], [1], [float("nan")], [1], cost)
    refused(B.SMART_ETREE, [1, 1, 1], [1], [0.5], [1], cost)              # offsets must start at 0
    refused(B.SMART_ETREE, [0, 1, 0], [1], [0.5], [1], cost)              # ... and ascend
    refused(B.SMART_EINVAL, [0, 1, 1], [1], [0.5], [1], cost, alpha=0.0)
    refused(B.SMART_EINVAL, [0, 1, 1], [1], [0.5], [1], cost, dilution=7)
    no_sum = B.HostLayerState(1, 8, path_sum=False)
    no_sum.begin([1], cost)
    with pytest.raises(B.SmartError) as e:
        no_sum.layer([0, 1], [0], [0.5], [1], cost, dilution=B.SMART_DILUTION_PATH_MEAN)
    assert e.value.code == B.SMART_EINVAL
    assert no_sum.layer([0, 1], [0], [0.5], [9], cost, alpha=1.0).tolist() == [1]   # fine without dilution
    # a layer that offers nothing ends the tree: no active node is left
    assert st.layer([0, 0, 0], [], [], [], cost).tolist() == []
    assert st.layer_begin.tolist() == st.n.tolist()
    refused2 = pytest.raises(B.SmartError)
    with refused2 as e:
        st.layer([0, 1, 1], [1], [0.5], [1], cost)
    assert e.value.code == B.SMART_ETREE


def test_device_layer_entry_points_validate_on_the_host_first():
    import ctypes
    lib = B._lib()
    st = B.LayerStateStruct(batch=1, budget=8)
    one = ctypes.c_void_p(8)
    assert lib.smart_select_begin_device(None, None, ctypes.byref(st), one, one) == B.SMART_EINVAL
    assert lib.smart_select_layer_device(None, None, ctypes.byref(st), one, one, one, one, 4, one, None, 0.8, 0,
                                         one, one) == B.SMART_EINVAL
    assert lib.tree_compact_pack(None, None, ctypes.byref(st), 8, one, one, one, one, one, one, one, one,
                                 one) == B.SMART_EINVAL
    assert lib.smart_select_begin(None, one, one) == B.SMART_EINVAL
    bad = B.LayerStateStruct(batch=1, budget=129)
    assert lib.smart_select_begin(ctypes.byref(bad), one, one) == B.SMART_EINVAL


# ---------------------------------------------------------------------------
# The likelihood-maximising baseline policy
# ---------------------------------------------------------------------------
def test_baseline_policy_hand_worked_example_library():
    import json
    import os
    with open(os.path.join(os.path.dirname(__file__), "golden", "baseline_hand_worked.json")) as f:
        g = json.load(f)
    fo = g["forest"]
    cost = np.array([1.0 + n / 8.0 for n in range(70)])
    for case in g["cases"]:
        r = B.smart_baseline_tree([0, len(fo["parent"])], fo["parent"], fo["prob"], fo["token"], cost, k=case["k"],
                                  max_depth=case.get("max_depth", g["max_depth"]), g=case["g"])
        assert r["cand_index"].tolist() == case["cand_index"] and r["parent"].tolist() == case["parent"], case["name"]
        assert r["L"][0] == case["L"] and r["R"][0] == case["R"], case["name"]


@pytest.mark.parametrize("name", ["cfg2", "cfg4"])
def test_baseline_policy_bit_exact_on_workload_forests(name):
    w = W.WORKLOADS[name].scaled(batch=6)
    f = W.make_forest(w)
    cost = np.array([1.0 + 0.004 * n for n in range(130)])
    for k, d, g in ((10, 6, 60), (3, 3, 8), (5, 7, 127), (7, 4, 0), (1, 8, 30)):
        r = B.smart_baseline_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, k=k, max_depth=d, g=g)
        for b in range(w.batch):
            lo, hi = int(f.cand_cu[b]), int(f.cand_cu[b + 1])
            t = S.baseline_tree(f.cand_parent[lo:hi].tolist(), f.cand_prob[lo:hi].tolist(),
                                f.cand_token[lo:hi].tolist(), cost.tolist(), k=k, max_depth=d, g=g)
            a, e = int(r["cu_nodes"][b]), int(r["cu_nodes"][b + 1])
            assert r["cand_index"][a:e].tolist() == t.cand_index and r["parent"][a:e].tolist() == t.parent
            assert r["token"][a:e].tolist() == t.token and r["pathprob"][a:e].tolist() == t.pathprob
            assert r["L"][b] == t.L and r["R"][b] == t.R


def test_baseline_policy_error_paths():
    cost = np.ones(130)
    ok = dict(cand_cu=[0, 3], cand_parent=[-1, 0, 0], cand_prob=[1.0, 0.5, 0.25], cand_token=[1, 2, 3], cost=cost)
    assert B.smart_baseline_tree(**ok, k=2, max_depth=2, g=5)["cu_nodes"].tolist() == [0, 3]
    for bad, code in ((dict(k=0), B.SMART_EINVAL), (dict(max_depth=-1), B.SMART_EINVAL), (dict(g=128), None),
                      (dict(cand_parent=[-1, 0, 2]), B.SMART_ETREE), (dict(cand_prob=[1.0, 1.5, 0.2]), B.SMART_ETREE),
                      (dict(cand_cu=[1, 3]), B.SMART_ETREE)):
        kw = dict(ok, k=2, max_depth=2, g=5)
        kw.update(bad)
        if code is None:
            with pytest.raises((B.SmartError, ValueError)):
                B.smart_baseline_tree(**kw)
            continue
        with pytest.raises(B.SmartError) as e:
            B.smart_baseline_tree(**kw)
        assert e.value.code == code, bad


def test_per_sequence_budgets_equal_one_call_per_sequence():
    w = W.WORKLOADS["cfg3b"].scaled(batch=12)
    f = W.make_forest(w)
    cost = W.cost_table(w)
    budgets = W.topn_budgets(w)
    assert len(set(budgets.tolist())) > 3
    for schedule in (B.SMART_BEST_FIRST, B.SMART_LAYERWISE):
        r = B.smart_select_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, alpha=w.alpha,
                                max_depth=w.max_depth, budget=int(budgets.max()), budgets=budgets, schedule=schedule)
        for b in range(w.batch):
            lo, hi = int(f.cand_cu[b]), int(f.cand_cu[b + 1])
            t = S.select_tree(f.cand_parent[lo:hi].tolist(), f.cand_prob[lo:hi].tolist(), f.cand_token[lo:hi].tolist(),
                              cost, alpha=w.alpha, max_depth=w.max_depth, budget=int(budgets[b]), schedule=schedule)
            a, e = int(r["cu_nodes"][b]), int(r["cu_nodes"][b + 1])
            assert r["cand_index"][a:e].tolist() == t.cand_index and r["parent"][a:e].tolist() == t.parent
            assert r["L"][b] == t.L and r["R"][b] == t.R
    for bad in ([0] + [4] * 11, [4] * 11 + [int(budgets.max()) + 1]):
        with pytest.raises(B.SmartError) as e:
            B.smart_select_tree(f.cand_cu, f.cand_parent, f.cand_prob, f.cand_token, cost, budget=int(budgets.max()),
                                budgets=bad)
        assert e.value.code == B.SMART_EINVAL


# ---------------------------------------------------------------------------
# Cartesian-product candidate forest (drafter with independent positions)
# ---------------------------------------------------------------------------
def test_product_forest_hand_worked_example_library():
    import json
    with open(os.path.join(os.path.dirname(__file__), "golden", "product_forest_hand_worked.json")) as f:
        g = json.load(f)
    for cap in range(1, 9):
        r = B.smart_product_forest([g["pos_prob"]], [g["pos_token"]], cap)
        n = min(cap, 7)
        assert r["cand_cu"].tolist() == [0, n]
        assert r["cand_parent"].tolist() == g["parent"][:n] and r["cand_prob"].tolist() == g["prob"][:n]
        assert r["cand_token"].tolist() == g["token"][:n]
    t = g["tie_case"]
    r = B.smart_product_forest([t["pos_prob"]], [[[1, 2], [3, 4]]], 7)
    assert r["cand_parent"].tolist() == t["parent"]


@pytest.mark.parametrize("seed", range(5))
def test_product_forest_bit_exact_against_the_oracle(seed):
    """Softmax-of-normal position distributions (the recipe of the workloads' drafts), full products small enough
    for the oracle to enumerate; also repeated probabilities, which exercise the tie order."""
    rng = np.random.default_rng(100 + seed)
    batch, d, k = 5, int(rng.integers(1, 6)), int(rng.integers(1, 5))
    logits = rng.normal(0.0, 2.0, size=(batch, d, k + 2))
    pp = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    pp = pp[..., :k]
    if seed % 2:
        pp = np.round(pp * 8) / 8                                              # many equal products, some zeros
    tok = rng.integers(0, 32000, size=(batch, d, k)).astype(np.int32)
    total = sum(k ** l for l in range(d + 1))
    for cap in (1, 2, 7, total // 2 + 1, total, total + 3):
        r = B.smart_product_forest(pp, tok, cap)
        for b in range(batch):
            parent, prob, token, _P = S.product_forest(pp[b].tolist(), tok[b].tolist(), cap)
            lo, hi = int(r["cand_cu"][b]), int(r["cand_cu"][b + 1])
            assert hi - lo == min(cap, total)
            assert r["cand_parent"][lo:hi].tolist() == parent and r["cand_prob"][lo:hi].tolist() == prob
            assert r["cand_token"][lo:hi].tolist() == token


def test_product_forest_feeds_both_policies():
    """A forest cut at a cap well above the budget gives the rule the same tree as the whole product, and the
    tree cut to its g most probable nodes is the head of the list."""
    rng = np.random.default_rng(5)
    logits = rng.normal(0.0, 2.0, size=(3, 6, 8))
    pp = np.exp(logits) / np.exp(logits).sum(-1, keepdims=True)
    tok = rng.integers(0, 32000, size=(3, 6, 8)).astype(np.int32)
    cost = np.array([1.0 + 0.01 * n for n in range(66)])
    small, large = B.smart_product_forest(pp, tok, 200), B.smart_product_forest(pp, tok, 2000)
    sel = [B.smart_select_tree(f["cand_cu"], f["cand_parent"], f["cand_prob"], f["cand_token"], cost, alpha=0.8,
                               max_depth=6, budget=64) for f in (small, large)]
    assert sel[0]["cu_nodes"].tolist() == sel[1]["cu_nodes"].tolist() and sel[0]["L"].tolist() == sel[1]["L"].tolist()
    assert sel[0]["token"].tolist() == sel[1]["token"].tolist() and sel[0]["parent"].tolist() == sel[1]["parent"].tolist()
    fixed = B.smart_baseline_tree(small["cand_cu"], small["cand_parent"], small["cand_prob"], small["cand_token"], cost,
                                  k=200, max_depth=6, g=59)
    for b in range(3):
        lo, hi = int(fixed["cu_nodes"][b]), int(fixed["cu_nodes"][b + 1])
        assert sorted(fixed["cand_index"][lo:hi].tolist()) == list(range(60))
    # a forest of a drafter with few confident positions is smaller than the cap
    r = B.smart_product_forest(np.full((2, 3, 2), 0.5), np.zeros((2, 3, 2), np.int32), 100)
    assert r["cand_cu"].tolist() == [0, 15, 30]


def test_product_forest_error_paths():
    pp, tok = np.full((1, 2, 2), 0.5), np.zeros((1, 2, 2), np.int32)
    assert B.smart_product_forest(pp, tok, 3)["cand_cu"].tolist() == [0, 3]
    for bad_pp, cap in ((np.full((1, 2, 2), 1.5), 3), (np.full((1, 2, 2), np.nan), 3), (np.full((1, 2, 2), -0.1), 3),
                        (pp, 0), (np.full((1, 32, 4), 0.5), 3)):
        with pytest.raises(B.SmartError) as e:
            B.smart_product_forest(bad_pp, np.zeros(bad_pp.shape, np.int32), cap)
        assert e.value.code == B.SMART_EINVAL
    with pytest.raises(ValueError):
        B.smart_product_forest(pp, np.zeros((1, 2, 3), np.int32), 3)
    # capacity: the C entry point writes nothing when the outputs are too small
    lib = B._lib()
    cu, par, tk = np.full(2, -7, np.int32), np.full(2, -7, np.int32), np.full(2, -7, np.int32)
    pr = np.full(2, -7.0)
    p = lambda a: ctypes.c_void_p(a.ctypes.data)
    rc = lib.smart_product_forest(1, 2, 2, p(pp), p(tok), 3, p(cu), p(par), p(pr), p(tk), 2)
    assert rc == B.SMART_ECAP and cu.tolist() == [-7, -7] and par.tolist() == [-7, -7]
    # depth 0: the root alone
    r = B.smart_product_forest(np.zeros((2, 0, 3)), np.zeros((2, 0, 3), np.int32), 4)
    assert r["cand_cu"].tolist() == [0, 1, 2] and r["cand_parent"].tolist() == [-1, -1]
