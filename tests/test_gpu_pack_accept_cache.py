"""GPU parity (bit-exact) of tree_pack, tree_accept and kv_cache_write against
the CPU oracle, called through the C ABI."""
import numpy as np
import pytest

from oracle import kv_layout as KL
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


def _dev(a, dtype=None):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a)).to("cuda")


def _random_batch(seed, sizes, shapes=None):
    rng = np.random.default_rng(seed)
    ts = [W.random_tree(n, rng, (shapes or ["random"] * len(sizes))[i]) for i, n in enumerate(sizes)]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    return cu, np.concatenate(ts).astype(np.int32), rng


def _mask_words(mask):
    lo = np.array([m[0] for m in mask], dtype=np.uint64)
    hi = np.array([m[1] for m in mask], dtype=np.uint64)
    return np.stack([lo, hi], 1)


@pytest.mark.parametrize("seed", range(3))
def test_tree_pack_bit_exact(lib, seed):
    sizes = [1, 2, 15, 63, 64, 65, 127, 128, 40, 7] + list(np.random.default_rng(seed).integers(1, 129, 40))
    shapes = ["random"] * len(sizes)
    shapes[5], shapes[7], shapes[8] = "chain", "chain", "star"
    cu, parent, rng = _random_batch(seed, sizes, shapes)
    plen = rng.integers(0, 20000, len(sizes)).astype(np.int32)
    depth, pos, seq, mask = PA.pack(cu, parent, plen)
    d, p, s, m, st = lib.tree_pack(_dev(cu), _dev(parent), _dev(plen))
    assert st.cpu().numpy().tolist() == [0] * len(sizes)
    assert d.cpu().numpy().tolist() == depth
    assert p.cpu().numpy().tolist() == pos
    assert s.cpu().numpy().tolist() == seq
    assert np.array_equal(m.cpu().numpy().view(np.uint64), _mask_words(mask))


def test_tree_pack_workload_trees_and_malformed(lib):
    w = W.WORKLOADS["cfg4"]
    cu, parent, token, _ = H.trees_from_library(w)
    plen = W.make_prefix_len(w)
    depth, pos, seq, mask = PA.pack(cu, parent, plen)
    d, p, s, m, st = lib.tree_pack(_dev(cu), _dev(parent), _dev(plen))
    assert d.cpu().numpy().tolist() == depth and p.cpu().numpy().tolist() == pos
    assert np.array_equal(m.cpu().numpy().view(np.uint64), _mask_words(mask))
    # malformed sequences are flagged and zero-filled; the others are untouched
    cu2 = np.array([0, 3, 6, 6, 10, 140], np.int32)         # seq 2 empty, seq 4 has 130 nodes
    par2 = np.concatenate([[-1, 0, 1], [-1, 2, 0], [0, 0, 1, 2], [-1] + list(range(129))]).astype(np.int32)
    plen2 = np.array([5, 6, 7, 8, 9], np.int32)
    d, p, s, m, st = lib.tree_pack(_dev(cu2), _dev(par2), _dev(plen2))
    assert st.cpu().numpy().tolist() == [0, B.SMART_ETREE, B.SMART_ETREE, B.SMART_ETREE, B.SMART_ETREE]
    assert d.cpu().numpy()[:3].tolist() == [0, 1, 2]
    assert not m.cpu().numpy()[3:].any() and not d.cpu().numpy()[3:].any()


@pytest.mark.parametrize("seed", range(3))
def test_tree_accept_bit_exact(lib, seed):
    sizes = [1, 5, 12, 30, 64, 65, 128, 100]
    cu, parent, rng = _random_batch(seed, sizes, ["random"] * 6 + ["chain", "random"])
    N = cu[-1]
    token = rng.integers(0, 6, N).astype(np.int32)
    target = rng.integers(0, 6, N).astype(np.int32)
    for b in range(len(sizes)):
        for i in range(1, sizes[b]):
            if rng.random() < 0.7:
                target[cu[b] + parent[cu[b] + i]] = token[cu[b] + i]
    for max_depth in (128, 8, 0):
        alen, paths, bonus = PA.accept(cu, parent, token, target, max_depth)
        a, p, bo = lib.tree_accept(_dev(cu), _dev(parent), _dev(token), _dev(target), max_depth)
        assert a.cpu().numpy().tolist() == alen
        assert p.cpu().numpy().tolist() == paths
        assert bo.cpu().numpy().tolist() == bonus


def test_tree_accept_on_workload_and_expected_length(lib):
    """Monte-Carlo form of the acceptance-length identity: with acceptance
    probability = draft probability, mean(accept_len + 1) over many target
    draws approaches sum_u P(u) (the L that selection reports)."""
    w = W.WORKLOADS["cfg2"].scaled(batch=64)
    forest = W.make_forest(w)
    r = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token,
                            W.cost_table(w), alpha=w.alpha, max_depth=w.max_depth, budget=w.budget)
    cu, parent, token, cand = r["cu_nodes"], r["parent"], r["token"], r["cand_index"]
    dcu, dpar, dtok = _dev(cu), _dev(parent), _dev(token)
    emitted = np.zeros(w.batch)
    trials = 300
    for trial in range(trials):
        target = W.make_target_next(forest, cu, cand, seed=5000 + trial)
        a, p, bo = lib.tree_accept(dcu, dpar, dtok, _dev(target), w.max_depth)
        if trial < 3:
            alen, paths, bonus = PA.accept(cu, parent, token, target, w.max_depth)
            assert a.cpu().numpy().tolist() == alen and bo.cpu().numpy().tolist() == bonus
            assert p.cpu().numpy().tolist() == paths
        emitted += a.cpu().numpy() + 1
    mean = emitted.sum() / (trials * w.batch)
    expect = r["L"].mean()
    # per-draw std of emitted tokens is < 3; 19200 draws -> 3 sigma < 0.07
    assert abs(mean - expect) < 0.07, (mean, expect)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("D", [64, 128])
def test_kv_cache_write_layouts(lib, dtype, D):
    import torch
    rng = np.random.default_rng(3)
    nb, Hkv, bs, n = 9, 3, 16, 70
    w = W.Workload("t", dtype, 1, Hkv, Hkv, D, 0, 0)
    k_src = W._normal(1, 1, (n, Hkv, D), 1.0, dtype)
    v_src = W._normal(1, 2, (n, Hkv, D), 1.0, dtype)
    slots = rng.permutation(nb * bs)[:n].astype(np.int64)
    slots[5] = -1                                            # skipped
    zero = np.zeros((nb, Hkv, bs, D), k_src.dtype)
    plain_k, plain_v = zero.copy(), zero.copy()
    for t in range(n):
        if slots[t] >= 0:
            plain_k[slots[t] // bs, :, slots[t] % bs] = k_src[t]
            plain_v[slots[t] // bs, :, slots[t] % bs] = v_src[t]
    tk = H.torch_elems(k_src, dtype, "cuda")
    tv = H.torch_elems(v_src, dtype, "cuda")
    raw = lambda t: t.cpu().view(torch.int16 if dtype == "bf16" else torch.float32).numpy().view(k_src.dtype)
    for layout in (B.SMART_KV_PLAIN, B.SMART_KV_INTERLEAVED):
        kc = torch.zeros((nb, Hkv, bs * D), dtype=tk.dtype, device="cuda")
        vc = torch.zeros_like(kc)
        lib.kv_cache_write(tk, tv, _dev(slots), kc, vc, layout, bs, nb, Hkv * bs * D, bs * D, D)
        if layout == B.SMART_KV_PLAIN:
            assert np.array_equal(raw(kc).reshape(plain_k.shape), plain_k)
            assert np.array_equal(raw(vc).reshape(plain_v.shape), plain_v)
        else:
            assert np.array_equal(raw(kc), KL.interleave_plain_cache(plain_k, "k"))
            assert np.array_equal(raw(vc), KL.interleave_plain_cache(plain_v, "v"))
            # the binding's layout converter moves data the same way
            ik, iv = B.interleave_kv_cache(H.torch_elems(plain_k, dtype, "cuda"),
                                           H.torch_elems(plain_v, dtype, "cuda"))
            assert np.array_equal(raw(ik).reshape(nb, Hkv, -1), raw(kc))
            assert np.array_equal(raw(iv).reshape(nb, Hkv, -1), raw(vc))


@pytest.mark.parametrize("n_words,src_off,dst_off", [(1, 0, 0), (4, 0, 0), (4099, 0, 0), (1000, 1, 0), (1000, 0, 3),
                                                     (70000, 4, 8)])
def test_tree_upload_copies_pinned_host_words(lib, n_words, src_off, dst_off):
    """The copy is bit-exact for aligned and unaligned ends and leaves the words around the
    destination alone."""
    import torch
    rng = np.random.default_rng(n_words)
    host = torch.empty(n_words + src_off + 5, dtype=torch.int32).pin_memory()
    host.numpy()[:] = rng.integers(-2**31, 2**31 - 1, size=host.numel(), dtype=np.int64).astype(np.int32)
    dev = torch.full((n_words + dst_off + 7,), -77, dtype=torch.int32, device="cuda")
    lib.tree_upload(host[src_off:src_off + n_words], dev[dst_off:dst_off + n_words])
    torch.cuda.synchronize()
    got = dev.cpu().numpy()
    assert (got[dst_off:dst_off + n_words] == host.numpy()[src_off:src_off + n_words]).all()
    assert (got[:dst_off] == -77).all() and (got[dst_off + n_words:] == -77).all()


def test_tree_upload_refuses_pageable_memory(lib):
    import torch
    host = torch.zeros(64, dtype=torch.int32)          # not pinned: the device cannot address it
    dev = torch.full((64,), 5, dtype=torch.int32, device="cuda")
    with pytest.raises(B.SmartError) as e:
        lib.tree_upload(host, dev)
    assert e.value.code == B.SMART_EINVAL
    torch.cuda.synchronize()
    assert (dev.cpu().numpy() == 5).all()


@pytest.mark.parametrize("dtype,D", [("bf16", 128), ("f32", 64)])
@pytest.mark.parametrize("seed", range(2))
def test_tree_commit_matches_oracle(lib, dtype, D, seed):
    """Accepted paths from the library's own accept walk are committed on the device in both
    cache layouts; caches, new lengths and status equal the oracle's, bit for bit.  One
    sequence has no room left in its block table, one has a corrupted path."""
    import torch
    rng = np.random.default_rng(100 + seed)
    Bsz, Hkv, bs, max_depth, max_blocks = 7, 2, 16, 6, 5
    sizes = [int(x) for x in rng.integers(1, 40, size=Bsz)]
    cu, parent, _ = _random_batch(seed + 50, sizes)
    N = int(cu[-1])
    token = rng.integers(0, 6, size=N).astype(np.int32)
    target = rng.integers(0, 6, size=N).astype(np.int32)
    prefix_len = rng.integers(0, (max_blocks - 1) * bs, size=Bsz).astype(np.int32)
    nb = Bsz * max_blocks + 3
    block_table = rng.permutation(nb)[:Bsz * max_blocks].reshape(Bsz, max_blocks).astype(np.int32)
    k_tree = W._normal(seed, 1, (N, Hkv, D), 1.0, dtype)
    v_tree = W._normal(seed, 2, (N, Hkv, D), 1.0, dtype)
    plain_k = W._normal(seed, 3, (nb, Hkv, bs, D), 1.0, dtype)
    plain_v = W._normal(seed, 4, (nb, Hkv, bs, D), 1.0, dtype)
    acc_len, acc_path, _ = lib.tree_accept(_dev(cu), _dev(parent), _dev(token), _dev(target), max_depth)
    h_len, h_path = acc_len.cpu().numpy().copy(), acc_path.cpu().numpy().copy()
    assert h_len.max() >= 1                                   # some draft token is accepted
    prefix_len[2] = max_blocks * bs - int(h_len[2])           # one token too many for sequence 2
    h_path[4, 0] = sizes[4]                                   # not a node of sequence 4's tree
    ref_k, ref_v = plain_k.copy(), plain_v.copy()
    ref_len, ref_status = PA.commit(cu, h_len, h_path, k_tree, v_tree, ref_k, ref_v, block_table, prefix_len, max_depth)
    assert ref_status[2] == B.SMART_ECAP and ref_status[4] == B.SMART_ETREE and sum(s == 0 for s in ref_status) == Bsz - 2
    raw = lambda t: t.cpu().view(torch.int16 if dtype == "bf16" else torch.float32).numpy().view(k_tree.dtype)
    tk, tv = H.torch_elems(k_tree, dtype, "cuda"), H.torch_elems(v_tree, dtype, "cuda")
    for layout in (B.SMART_KV_PLAIN, B.SMART_KV_INTERLEAVED):
        kc, vc = H.torch_elems(plain_k, dtype, "cuda"), H.torch_elems(plain_v, dtype, "cuda")
        if layout == B.SMART_KV_INTERLEAVED:
            kc, vc = B.interleave_kv_cache(kc, vc)
        new_len, status = lib.tree_commit(_dev(cu), _dev(h_len), _dev(h_path), tk, tv, kc, vc, _dev(block_table),
                                          _dev(prefix_len), layout, bs, nb, Hkv * bs * D, bs * D, D)
        torch.cuda.synchronize()
        assert status.cpu().numpy().tolist() == ref_status
        assert new_len.cpu().numpy().tolist() == ref_len
        if layout == B.SMART_KV_PLAIN:
            assert np.array_equal(raw(kc).reshape(ref_k.shape), ref_k)
            assert np.array_equal(raw(vc).reshape(ref_v.shape), ref_v)
        else:
            assert np.array_equal(raw(kc).reshape(nb, Hkv, -1), KL.interleave_plain_cache(ref_k, "k"))
            assert np.array_equal(raw(vc).reshape(nb, Hkv, -1), KL.interleave_plain_cache(ref_v, "v"))


@pytest.mark.parametrize("seed", range(2))
def test_tree_upload_pack_equals_upload_then_pack(lib, seed):
    """The fused launch leaves the same device copies and the same packing as the oracle's
    pack of the host arrays; a malformed sequence is reported, not packed."""
    import torch
    sizes = [1, 7, 128, 64, 65, 3, 30]
    shapes = ["random", "chain", "random", "star", "random", "chain", "random"]
    cu, parent, rng = _random_batch(300 + seed, sizes, shapes)
    N = int(cu[-1])
    token = rng.integers(0, 1000, size=N).astype(np.int32)
    prefix_len = rng.integers(0, 5000, size=len(sizes)).astype(np.int32)
    bad = 3
    parent_bad = parent.copy()
    parent_bad[cu[bad] + 5] = 7                      # a parent that does not precede its child
    pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
    d_cu, d_par, d_tok, depth, position, node_seq, mask, status = lib.tree_upload_pack(
        pin(cu), pin(parent_bad), pin(token), _dev(prefix_len))
    torch.cuda.synchronize()
    assert np.array_equal(d_cu.cpu().numpy(), cu)
    assert np.array_equal(d_par.cpu().numpy(), parent_bad)
    assert np.array_equal(d_tok.cpu().numpy(), token)
    st = status.cpu().numpy()
    assert st[bad] == B.SMART_ETREE and not np.delete(st, bad).any()
    r_depth, r_pos, r_seq, r_mask = PA.pack(cu, parent, prefix_len)
    keep = np.ones(N, bool)
    keep[cu[bad]:cu[bad + 1]] = False
    assert np.array_equal(depth.cpu().numpy()[keep], np.array(r_depth)[keep])
    assert np.array_equal(position.cpu().numpy()[keep], np.array(r_pos)[keep])
    assert np.array_equal(node_seq.cpu().numpy()[keep], np.array(r_seq)[keep])
    assert np.array_equal(mask.cpu().numpy().view(np.uint64)[keep], _mask_words(r_mask)[keep])
    assert not depth.cpu().numpy()[~keep].any() and not mask.cpu().numpy()[~keep].any()
    # pageable memory is refused
    with pytest.raises(B.SmartError):
        lib.tree_upload_pack(torch.from_numpy(cu), pin(parent), pin(token), _dev(prefix_len))


@pytest.mark.parametrize("batch", [64, 65, 150])
def test_tree_upload_pack_offsets_in_the_arguments_or_fetched(lib, batch):
    """Up to 64 sequences the offsets travel with the launch, above that the kernel fetches them from the pinned
    array: both leave the same copies and packing; offsets that leave the node arrays are reported per sequence."""
    import torch
    rng0 = np.random.default_rng(batch)
    sizes = [int(n) for n in rng0.integers(1, 12, size=batch)]
    cu, parent, rng = _random_batch(500 + batch, sizes, ["random"] * batch)
    N = int(cu[-1])
    token = rng.integers(0, 1000, size=N).astype(np.int32)
    prefix_len = rng.integers(0, 5000, size=batch).astype(np.int32)
    pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
    d_cu, d_par, d_tok, depth, position, node_seq, mask, status = lib.tree_upload_pack(
        pin(cu), pin(parent), pin(token), _dev(prefix_len))
    torch.cuda.synchronize()
    assert np.array_equal(d_cu.cpu().numpy(), cu) and np.array_equal(d_par.cpu().numpy(), parent)
    assert np.array_equal(d_tok.cpu().numpy(), token) and not status.cpu().numpy().any()
    r_depth, r_pos, r_seq, r_mask = PA.pack(cu, parent, prefix_len)
    assert np.array_equal(depth.cpu().numpy(), np.array(r_depth)) and np.array_equal(position.cpu().numpy(), np.array(r_pos))
    assert np.array_equal(node_seq.cpu().numpy(), np.array(r_seq))
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), _mask_words(r_mask))
    # a sequence whose offsets run backwards is reported and left alone (its neighbours' ranges are their own)
    cu_bad = cu.copy()
    cu_bad[5] = cu[4] - 1 if cu[4] > 0 else cu[6] + 1
    out = lib.tree_upload_pack(pin(cu_bad), pin(parent), pin(token), _dev(prefix_len))
    torch.cuda.synchronize()
    st = out[-1].cpu().numpy()
    assert st[4] == B.SMART_ETREE or st[5] == B.SMART_ETREE


@pytest.mark.parametrize("total", [383, 447, 448, 449, 700])
@pytest.mark.parametrize("with_tokens", [True, False])
def test_tree_upload_pack_trees_in_the_arguments_or_fetched(lib, total, with_tokens):
    """With at most 448 nodes in all (and at most 64 sequences) parents and tokens travel with the launch as well,
    above that the kernel fetches them from the pinned arrays: both sides of the limit leave the same copies and the
    oracle's packing, with and without tokens; a malformed tree is reported either way."""
    import torch
    sizes = [128, 100, 90, 1, 33]
    rest = total - sum(sizes)
    while rest > 128:
        sizes.append(64)
        rest -= 64
    sizes.append(rest)
    assert sum(sizes) == total and all(1 <= n <= 128 for n in sizes)
    cu, parent, rng = _random_batch(900 + total, sizes, [["random", "chain", "star"][i % 3] for i in range(len(sizes))])
    token = rng.integers(0, 1 << 30, size=total).astype(np.int32)
    prefix_len = rng.integers(0, 5000, size=len(sizes)).astype(np.int32)
    pin = lambda a: torch.from_numpy(np.ascontiguousarray(a)).pin_memory()
    out = lib.tree_upload_pack(pin(cu), pin(parent), pin(token) if with_tokens else None, _dev(prefix_len))
    torch.cuda.synchronize()
    d_cu, d_par, d_tok, depth, position, node_seq, mask, status = out
    assert np.array_equal(d_cu.cpu().numpy(), cu) and np.array_equal(d_par.cpu().numpy(), parent)
    assert (d_tok is None) if not with_tokens else np.array_equal(d_tok.cpu().numpy(), token)
    assert not status.cpu().numpy().any()
    r_depth, r_pos, r_seq, r_mask = PA.pack(cu, parent, prefix_len)
    assert np.array_equal(depth.cpu().numpy(), np.array(r_depth)) and np.array_equal(position.cpu().numpy(), np.array(r_pos))
    assert np.array_equal(node_seq.cpu().numpy(), np.array(r_seq))
    assert np.array_equal(mask.cpu().numpy().view(np.uint64), _mask_words(r_mask))
    parent_bad = parent.copy()
    parent_bad[cu[1] + 3] = 50                       # a parent that does not precede its child
    st = lib.tree_upload_pack(pin(cu), pin(parent_bad), pin(token) if with_tokens else None, _dev(prefix_len))[-1]
    torch.cuda.synchronize()
    st = st.cpu().numpy()
    assert st[1] == B.SMART_ETREE and not np.delete(st, 1).any()
