"""The device part of a verify step (upload + pack, attention, accept) captured in a HIP graph: every replay,
with eager launches and synchronisations in between, must reproduce the eager result bit for bit (the library
enqueues no memset, allocates nothing once the workspace is reserved, and never synchronises)."""
import numpy as np
import pytest

from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def test_graph_replays_equal_the_eager_step():
    import torch
    lib = B.SmartTree(0)
    w = W.WORKLOADS["cfg3a"].scaled(batch=6, prefix_min=300, prefix_max=900)
    cu, parent, token, cand = H.trees_from_library(w)
    inp = W.make_attention_inputs(w, cu, poison_unused=False)
    forest = W.make_forest(w)
    N = int(cu[-1])
    q, kt, vt = (H.torch_elems(x, "bf16", "cuda") for x in (inp.q, inp.k_tree, inp.v_tree))
    kc, vc = B.interleave_kv_cache(H.torch_elems(inp.k_cache, "bf16", "cuda"), H.torch_elems(inp.v_cache, "bf16", "cuda"))
    t = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    bt, plen = t(inp.block_table), t(inp.prefix_len)
    target = t(W.make_target_next(forest, cu, cand, seed=3))
    pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
    p_cu, p_par, p_tok = pin(cu), pin(parent), pin(token)
    lib.reserve(w.batch, N, w.num_q_heads, w.num_kv_heads)          # no allocation inside the capture
    out = torch.empty_like(q)

    def device_step():
        d_cu, d_par, d_tok, _, _, _, mask, _ = lib.tree_upload_pack(p_cu, p_par, p_tok, plen)
        lib.tree_verify_attention(q, kt, vt, kc, vc, bt, plen, d_cu, mask, inp.scale, B.SMART_KV_INTERLEAVED, out=out)
        return lib.tree_accept(d_cu, d_par, d_tok, target, w.max_depth)

    ref = device_step()
    torch.cuda.synchronize()
    ref_out, ref_len, ref_path, ref_bonus = out.clone(), ref[0].clone(), ref[1].clone(), ref[2].clone()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        device_step()
    torch.cuda.current_stream().wait_stream(side)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        res = device_step()
    for i in range(5):
        out.zero_()
        res[0].fill_(-7)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out), i
        assert torch.equal(res[0], ref_len) and torch.equal(res[1], ref_path) and torch.equal(res[2], ref_bonus), i
        # the program's own eager work between the replays, other trees included
        p_par[1:3] = 0
        device_step()
        torch.cuda.synchronize()
        p_par.copy_(torch.from_numpy(parent))
    # A replay reads the pinned arrays when it runs, not what they held at capture: other tokens (same trees)
    # change what is accepted, and the replay must follow them.
    p_tok.copy_(torch.from_numpy(np.ascontiguousarray(token[::-1] + 1)))
    ref2 = device_step()
    torch.cuda.synchronize()
    ref2 = [x.clone() for x in ref2]
    assert not all(torch.equal(a, b) for a, b in zip(ref2, (ref_len, ref_path, ref_bonus))), "tokens changed nothing"
    res[0].fill_(-7)
    graph.replay()
    torch.cuda.synchronize()
    assert all(torch.equal(a, b) for a, b in zip(res, ref2))
