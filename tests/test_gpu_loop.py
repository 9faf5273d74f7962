"""Three steps of the whole loop on the device, every call of the library in its place, against the same
loop built from the oracles: layer-at-a-time selection (draft candidates arrive per layer) -> tree_compact_pack
-> tree_rope -> tree_verify_attention (total_nodes as a capacity) -> tree_accept -> tree_commit, the prefix
growing by the accepted tokens."""
import numpy as np
import pytest

from oracle import pack_accept as PA
from oracle import rope as R
from oracle import selection as S
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


def _dev(a, dtype=None):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a, dtype)).to("cuda")


def _forest(rng, k, d):
    parent, prob, depth = [-1], [1.0], [0]
    i = 0
    while i < len(parent):
        if depth[i] < d:
            p = rng.dirichlet(np.ones(k + 1))[:k]
            for j in np.argsort(-p):
                parent.append(i)
                prob.append(float(p[j]))
                depth.append(depth[i] + 1)
        i += 1
    return parent, prob, [int(t) for t in rng.integers(0, 5, len(parent))]


def test_three_steps_of_the_whole_loop(oracle_attention):
    import torch
    lib = B.SmartTree(0)
    rng = np.random.default_rng(2024)
    nb_seq, Hq, Hkv, D, bs, budget, max_depth = 5, 8, 2, 128, 16, 12, 3
    max_blocks = 40
    nblk = nb_seq * max_blocks
    lens = np.array([0, 17, 100, 333, 64], np.int32)
    block_table = rng.permutation(nblk).reshape(nb_seq, max_blocks).astype(np.int32)
    bf = lambda x: W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, np.float32))).astype(np.float64)
    # the cache before the first step: keys rotated by their positions (what earlier steps would have left)
    k_plain = bf(rng.standard_normal((nblk, Hkv, bs, D)))
    v_plain = bf(rng.standard_normal((nblk, Hkv, bs, D)))
    for b in range(nb_seq):
        for t in range(int(lens[b])):
            blk, slot = int(block_table[b, t // bs]), t % bs
            k_plain[blk, :, slot] = bf(R.rope(k_plain[blk, :, slot][None], [t])[0])
    to_dev = lambda x: torch.from_numpy(W.f32_to_bf16_bits(x.astype(np.float32))).view(torch.int16).view(torch.bfloat16).cuda()
    kc, vc = B.interleave_kv_cache(to_dev(k_plain), to_dev(v_plain))
    d_bt = _dev(block_table)
    d_len = _dev(lens)
    cost = np.array([1.0 + 0.03 * n for n in range(budget + 2)])
    d_cost = _dev(cost, np.float64)
    cap = nb_seq * budget
    scale = 1.0 / np.sqrt(D)
    for step in range(3):
        forests = [_forest(rng, 3, max_depth) for _ in range(nb_seq)]
        # ---- device: the tree grows layer by layer
        st = B.DeviceLayerState(nb_seq, budget, "cuda")
        lib.select_begin(st, _dev([f[2][0] for f in forests], np.int32), d_cost)

        def layer(cu, parent_nodes, offered):
            prob = [forests[b][1][u] for b in range(nb_seq) for u in offered[b]]
            tok = [forests[b][2][u] for b in range(nb_seq) for u in offered[b]]
            out, status = lib.select_layer(st, _dev(cu, np.int32), _dev(parent_nodes, np.int32),
                                           _dev(prob, np.float64), _dev(tok, np.int32), d_cost, alpha=0.9)
            assert not status.cpu().numpy().any()
            return out.cpu().numpy().tolist()

        cand = H.drive_layers_batch([f[0] for f in forests], max_depth, layer)
        d_cu, d_par, d_tok, depth, position, _, mask, status = lib.tree_compact_pack(st, d_len)
        assert not status.cpu().numpy().any()
        cu = d_cu.cpu().numpy()
        N = int(cu[-1])
        # ---- oracle: the same trees
        trees = [S.select_tree(f[0], f[1], f[2], cost.tolist(), alpha=0.9, max_depth=max_depth, budget=budget,
                               schedule=S.LAYERWISE) for f in forests]
        assert [t.cand_index for t in trees] == cand
        parent = np.concatenate([t.parent for t in trees]).astype(np.int32)
        token = np.concatenate([t.token for t in trees]).astype(np.int32)
        assert cu.tolist() == np.concatenate([[0], np.cumsum([len(t) for t in trees])]).tolist()
        assert d_par.cpu().numpy()[:N].tolist() == parent.tolist() and d_tok.cpu().numpy()[:N].tolist() == token.tolist()
        o_depth, o_pos, _, _ = PA.pack(cu, parent, lens)
        assert position.cpu().numpy()[:N].tolist() == o_pos
        # ---- the target model's q / k / v for the tree nodes (synthetic), in arrays of `cap` rows
        q = bf(rng.standard_normal((N, Hq, D)))
        k_tree = bf(rng.standard_normal((N, Hkv, D)))
        v_tree = bf(rng.standard_normal((N, Hkv, D)))
        pad = lambda x: torch.cat([to_dev(x), torch.zeros((cap - N,) + x.shape[1:], dtype=torch.bfloat16, device="cuda")])
        d_q, d_kt, d_vt = pad(q), pad(k_tree), pad(v_tree)
        lib.tree_rope(position, d_q, d_kt)
        out = lib.tree_verify_attention(d_q, d_kt, d_vt, kc, vc, d_bt, d_len, d_cu, mask, scale, B.SMART_KV_INTERLEAVED)
        target_next = rng.integers(0, 5, N).astype(np.int32)
        d_target = _dev(np.concatenate([target_next, np.zeros(cap - N, np.int32)]))
        acc_len, acc_path, bonus = lib.tree_accept(d_cu, d_par, d_tok, d_target, max_depth)
        new_len, c_status = lib.tree_commit(d_cu, acc_len, acc_path, d_kt, d_vt, kc, vc, d_bt, d_len,
                                            B.SMART_KV_INTERLEAVED, bs, nblk, kc.stride(0), kc.stride(1))
        torch.cuda.synchronize()
        # ---- oracle chain
        q_r, k_r = R.rope(q, o_pos), bf(R.rope(k_tree, o_pos))
        ref, _ = oracle_attention.tree_attention(q_r, k_r, v_tree, k_plain, v_plain, block_table, lens, cu, parent, scale)
        got = H.out_to_f64(out, "bf16")[:N]
        assert H.rel_err(got, ref) <= H.TOL["bf16"], (step, H.rel_err(got, ref))
        o_len, o_path, o_bonus = PA.accept(cu, parent, token, target_next, max_depth)
        assert acc_len.cpu().numpy().tolist() == o_len and acc_path.cpu().numpy().tolist() == o_path
        assert bonus.cpu().numpy().tolist() == o_bonus
        o_new, o_status = PA.commit(cu, o_len, o_path, k_r, v_tree, k_plain, v_plain, block_table, lens, max_depth)
        assert c_status.cpu().numpy().tolist() == o_status == [0] * nb_seq
        assert new_len.cpu().numpy().tolist() == o_new
        assert sum(o_len) >= 1 or step > 0
        lens = np.array(o_new, np.int32)
        d_len = new_len
    # after three steps the two caches hold the same values (rotated keys: the device rotates in binary32 and
    # rounds once, the oracle in binary64: at most one bf16 unit apart)
    nbk, hk, _, _, _ = kc.shape
    k_back = kc.float().cpu().numpy().transpose(0, 1, 3, 2, 4).reshape(nbk, hk, bs, D)   # [blk][h][slot][d]
    v_back = vc.float().cpu().numpy().transpose(0, 1, 2, 4, 3).reshape(nbk, hk, bs, D)
    assert np.array_equal(v_back, v_plain)
    assert np.abs(k_back - k_plain).max() <= 2.0 ** -7 * np.abs(k_plain).max()
    assert lens.sum() > np.array([0, 17, 100, 333, 64]).sum() + 3
