"""tree_verify_attention_static -- the entry point for callers that cannot allocate device
memory (its partial results and launch plan live in a static device array) -- against
tree_verify_attention on the same inputs, through the C ABI: two calls in a row, the second
with a smaller input, so that what the first call left in the array is still there."""
import numpy as np
import pytest

from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _inputs(w, dev):
    import torch
    cu, parent, _, _ = H.trees_from_library(w)
    inp = W.make_attention_inputs(w, cu)
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    kc, vc = B.interleave_kv_cache(H.torch_elems(inp.k_cache, w.dtype, dev), H.torch_elems(inp.v_cache, w.dtype, dev))
    return dict(w=w, cu=cu, parent=parent, inp=inp, q=H.torch_elems(inp.q, w.dtype, dev),
                k_tree=H.torch_elems(inp.k_tree, w.dtype, dev), v_tree=H.torch_elems(inp.v_tree, w.dtype, dev),
                kc=kc, vc=vc, block_table=t(inp.block_table), prefix_len=t(inp.prefix_len), d_cu=t(cu),
                d_parent=t(parent))


def _call(lib, c, static, hint=True):
    import torch
    _, _, _, mask, status = lib.tree_pack(c["d_cu"], c["d_parent"], c["prefix_len"])
    assert not status.cpu().numpy().any()
    out = torch.full_like(c["q"], float("nan"))
    lse = torch.full(c["q"].shape[:2], float("nan"), dtype=torch.float32, device=c["q"].device)
    lib.tree_verify_attention(c["q"], c["k_tree"], c["v_tree"], c["kc"], c["vc"], c["block_table"], c["prefix_len"],
                              c["d_cu"], mask, c["inp"].scale, B.SMART_KV_INTERLEAVED, out=out, lse=lse,
                              h_cu_nodes=c["cu"] if hint else None, static=static)
    torch.cuda.synchronize()
    return out, lse


def test_static_entry_point_matches_the_allocating_one(oracle_attention):
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = B.SmartTree(0)
    dev = "cuda"
    # all three row classes (cfg3b: 4 .. 64 nodes x 4 group heads), several workers per segment; then a smaller call
    big = _inputs(W.WORKLOADS["cfg3b"].scaled(batch=9, prefix_min=700, prefix_max=1500), dev)
    small = _inputs(W.WORKLOADS["cfg3a"].scaled(batch=3, prefix_min=150, prefix_max=420), dev)
    for c in (big, small):
        ref_out, ref_lse = _call(lib, c, static=False)
        out, lse = _call(lib, c, static=True)
        # same kernels, same plan, same merge order: bit-identical
        assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))
        assert torch.equal(lse, ref_lse)
        # and both within the stated tolerance of the oracle
        i = c["inp"]
        want, want_lse = oracle_attention.tree_attention(i.q, i.k_tree, i.v_tree, i.k_cache, i.v_cache, i.block_table,
                                                         i.prefix_len, c["cu"], c["parent"], i.scale)
        assert H.rel_err(H.out_to_f64(out, "bf16"), want) <= H.TOL["bf16"]
        assert np.abs(lse.cpu().numpy().astype(np.float64) - want_lse).max() <= 2e-2
    # without the host copy of the offsets the room is counted from the totals alone
    out, _ = _call(lib, small, static=True, hint=False)
    ref_out, _ = _call(lib, small, static=False)
    assert torch.equal(out.view(torch.int16), ref_out.view(torch.int16))


def test_static_entry_point_rejects_what_does_not_fit():
    import torch
    assert torch.cuda.is_available(), "this test needs the MI355X"
    lib = B.SmartTree(0)
    dev = "cuda"
    c = _inputs(W.WORKLOADS["cfg3a"].scaled(batch=3, prefix_min=150, prefix_max=420), dev)
    _, _, _, mask, _ = lib.tree_pack(c["d_cu"], c["d_parent"], c["prefix_len"])
    out = torch.zeros_like(c["q"])
    args = (c["q"], c["k_tree"], c["v_tree"], c["kc"], c["vc"], c["block_table"], c["prefix_len"], c["d_cu"], mask,
            c["inp"].scale, B.SMART_KV_INTERLEAVED)
    # a host copy of the offsets that is no running sum
    bad = c["cu"].copy()
    bad[1] = bad[2] + 1
    with pytest.raises(B.SmartError) as e:
        lib.tree_verify_attention(*args, out=out, h_cu_nodes=bad, static=True)
    assert e.value.code == B.SMART_EINVAL
    # more partial results than the array holds: a capacity (total_nodes) far beyond the trees, no host offsets
    N_cap = 1 << 16
    q_big = torch.zeros((N_cap,) + tuple(c["q"].shape[1:]), dtype=c["q"].dtype, device=dev)
    kt_big = torch.zeros((N_cap,) + tuple(c["k_tree"].shape[1:]), dtype=c["q"].dtype, device=dev)
    mask_big = torch.zeros((N_cap, 2), dtype=torch.int64, device=dev)
    with pytest.raises(B.SmartError) as e:
        lib.tree_verify_attention(q_big, kt_big, kt_big, c["kc"], c["vc"], c["block_table"], c["prefix_len"], c["d_cu"],
                                  mask_big, c["inp"].scale, B.SMART_KV_INTERLEAVED, out=torch.empty_like(q_big),
                                  static=True)
    assert e.value.code == B.SMART_ECAP
    torch.cuda.synchronize()
