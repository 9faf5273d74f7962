"""GPU parity of the fp8 (E4M3) KV-cache variant against the CPU oracle, through the C ABI: the cache writer
is bit-exact, attention over an fp8 cache meets the same tolerance as over a bf16 cache (the oracle is fed
the decoded cache, so the comparison measures kernel arithmetic, not the quantisation)."""
import numpy as np
import pytest

from oracle import fp8 as F
from oracle import kv_layout as KL
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
    return torch.from_numpy(np.ascontiguousarray(a, dtype)).to("cuda")


def _f32(raw, dtype):
    return W.bf16_bits_to_f32(raw) if dtype == "bf16" else raw.astype(np.float32)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
@pytest.mark.parametrize("k_scale,v_scale", [(1.0, 1.0), (0.37, 2.0 ** -3), (3.0, 0.011)])
def test_kv_cache_write_fp8_bit_exact(lib, dtype, k_scale, v_scale):
    import torch
    rng = np.random.default_rng(4)
    nb, Hkv, bs, D, n = 7, 3, 16, 128, 60
    k_src = W._normal(2, 1, (n, Hkv, D), 1.0, dtype)
    v_src = W._normal(2, 2, (n, Hkv, D), 1.0, dtype)
    # special values: zeros of both signs, ties, values beyond the range, tiny values
    special = np.array([0.0, -0.0, 1.0625, 1.1875, 500.0, -1e6, 2.0 ** -10, 3 * 2.0 ** -10, 447.9, 17.0], np.float32)
    if dtype == "bf16":
        k_src[0, 0, :10] = W.f32_to_bf16_bits(special * np.float32(k_scale))
    else:
        k_src[0, 0, :10] = special * np.float32(k_scale)
    slots = rng.permutation(nb * bs)[:n].astype(np.int64)
    slots[7] = -1
    want_k = np.zeros((nb, Hkv, bs, D), np.uint8)
    want_v = np.zeros((nb, Hkv, bs, D), np.uint8)
    ek = F.encode(_f32(k_src, dtype) / np.float32(k_scale))             # binary32 division, as the kernel does
    ev = F.encode(_f32(v_src, dtype) / np.float32(v_scale))
    for t in range(n):
        if slots[t] >= 0:
            want_k[slots[t] // bs, :, slots[t] % bs] = ek[t]
            want_v[slots[t] // bs, :, slots[t] % bs] = ev[t]
    tk, tv = H.torch_elems(k_src, dtype, "cuda"), H.torch_elems(v_src, dtype, "cuda")
    for layout in (B.SMART_KV_PLAIN, B.SMART_KV_INTERLEAVED):
        kc = torch.zeros((nb, Hkv, bs * D), dtype=torch.uint8, device="cuda")
        vc = torch.zeros_like(kc)
        lib.kv_cache_write_fp8(tk, tv, _dev(slots), kc, vc, layout, bs, nb, Hkv * bs * D, bs * D, k_scale, v_scale,
                               token_stride=D)
        torch.cuda.synchronize()
        if layout == B.SMART_KV_PLAIN:
            assert np.array_equal(kc.cpu().numpy().reshape(want_k.shape), want_k)
            assert np.array_equal(vc.cpu().numpy().reshape(want_v.shape), want_v)
        else:
            assert np.array_equal(kc.cpu().numpy(), KL.interleave_plain_cache(want_k, "k"))
            assert np.array_equal(vc.cpu().numpy(), KL.interleave_plain_cache(want_v, "v"))


def _fp8_case(lib, w, cu, parent, lens, k_scale, v_scale, layout, seed):
    """Builds an fp8 cache with the library's writer from the workload's bf16 / f32 cache contents; returns the
    device tensors and the decoded cache (float64, scales applied) for the oracle."""
    import torch
    inp = W.make_attention_inputs(w, cu, seed=seed, prefix_len=lens, poison_unused=False)
    nb, Hkv, bs, D = inp.k_cache.shape
    # every slot of the cache as one "token": the writer quantises the whole cache
    slots = np.arange(nb * bs, dtype=np.int64)
    k_rows = np.ascontiguousarray(inp.k_cache.transpose(0, 2, 1, 3)).reshape(nb * bs, Hkv, D)
    v_rows = np.ascontiguousarray(inp.v_cache.transpose(0, 2, 1, 3)).reshape(nb * bs, Hkv, D)
    kc = torch.zeros((nb, Hkv, bs * D), dtype=torch.uint8, device="cuda")
    vc = torch.zeros_like(kc)
    lib.kv_cache_write_fp8(H.torch_elems(k_rows, w.dtype, "cuda"), H.torch_elems(v_rows, w.dtype, "cuda"), _dev(slots),
                           kc, vc, layout, bs, nb, Hkv * bs * D, bs * D, k_scale, v_scale, token_stride=D)
    torch.cuda.synchronize()
    kq = F.decode(F.encode(_f32(inp.k_cache, w.dtype) / np.float32(k_scale))) * float(np.float32(k_scale))
    vq = F.decode(F.encode(_f32(inp.v_cache, w.dtype) / np.float32(v_scale))) * float(np.float32(v_scale))
    return inp, kc, vc, kq, vq


@pytest.mark.parametrize("dtype,layout,D", [("bf16", B.SMART_KV_INTERLEAVED, 128), ("bf16", B.SMART_KV_PLAIN, 64),
                                            ("f32", B.SMART_KV_INTERLEAVED, 64)])
def test_attention_over_an_fp8_cache(lib, oracle_attention, dtype, layout, D):
    import torch
    rng = np.random.default_rng(8)
    sizes = [1, 3, 9, 17, 40, 2]
    trees = [W.random_tree(n, rng, s) for n, s in zip(sizes, ["random", "chain", "random", "star", "random", "random"])]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = np.array([0, 1, 31, 32, 33, 517], np.int32)
    w = W.Workload("fp8", dtype, len(sizes), 8, 2, D, 0, 0, seed=31)
    k_scale, v_scale = 0.05, 0.02                                    # unit-variance inputs use most of the range
    inp, kc, vc, kq, vq = _fp8_case(lib, w, cu, parent, lens, k_scale, v_scale, layout, 31)
    f64 = (lambda x: W.bf16_bits_to_f32(x).astype(np.float64)) if dtype == "bf16" else (lambda x: x.astype(np.float64))
    d_cu, d_par, d_len = _dev(cu), _dev(parent), _dev(lens)
    _, _, _, mask, _ = lib.tree_pack(d_cu, d_par, d_len)
    nb, Hkv, bs, _ = inp.k_cache.shape
    kc4 = kc.view(nb, Hkv, bs, D) if layout == B.SMART_KV_PLAIN else kc.view(nb, Hkv, D // 8, bs, 8)
    vc4 = vc.view(nb, Hkv, bs, D) if layout == B.SMART_KV_PLAIN else vc.view(nb, Hkv, bs // 8, D, 8)
    out, lse = lib.tree_verify_attention(H.torch_elems(inp.q, dtype, "cuda"), H.torch_elems(inp.k_tree, dtype, "cuda"),
                                         H.torch_elems(inp.v_tree, dtype, "cuda"), kc4, vc4,
                                         _dev(inp.block_table), d_len, d_cu, mask, inp.scale, layout, block_size=bs,
                                         want_lse=True, k_scale=k_scale, v_scale=v_scale)
    torch.cuda.synchronize()
    ref, ref_lse = oracle_attention.tree_attention(f64(inp.q), f64(inp.k_tree), f64(inp.v_tree), kq, vq,
                                                   inp.block_table, lens, cu, parent, inp.scale)
    got = H.out_to_f64(out, dtype)
    assert np.isfinite(got).all()
    assert H.rel_err(got, ref) <= H.TOL[dtype], H.rel_err(got, ref)
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= (1e-4 if dtype == "f32" else 2e-2)
    # the quantisation itself is visible: against the unquantised cache the error is well above the tolerance
    ref0, _ = oracle_attention.tree_attention(f64(inp.q), f64(inp.k_tree), f64(inp.v_tree), f64(inp.k_cache),
                                              f64(inp.v_cache), inp.block_table, lens, cu, parent, inp.scale)
    assert H.rel_err(ref, ref0) > 1e-3


def test_fp8_long_prefix_few_workers_shares_of_several_chunks(lib, oracle_attention):
    """A wavefront's share of a piece longer than the 64 tiles its block-id registers hold (one or two workers, one
    sequence of 1251 tiles with a ragged end), for trees of one row tile, of two (the halves of the workgroup stream
    the same tiles) and of several row groups."""
    import torch
    rng = np.random.default_rng(3)
    sizes = [2, 12, 40]                                              # 8, 48 and 160 rows per kv head at G = 4
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate([W.random_tree(n, rng, "random") for n in sizes]).astype(np.int32)
    lens = np.array([40011, 20500, 70], np.int32)
    w = W.Workload("fp8long", "bf16", 3, 8, 2, 128, 0, 0, seed=19)
    ks, vs = 0.05, 0.02
    inp, kc, vc, kq, vq = _fp8_case(lib, w, cu, parent, lens, ks, vs, B.SMART_KV_INTERLEAVED, 19)
    f64 = lambda x: W.bf16_bits_to_f32(x).astype(np.float64)
    d_cu, d_par, d_len = _dev(cu), _dev(parent), _dev(lens)
    _, _, _, mask, _ = lib.tree_pack(d_cu, d_par, d_len)
    nb, Hkv, bs, D = inp.k_cache.shape
    kc4, vc4 = kc.view(nb, Hkv, D // 8, bs, 8), vc.view(nb, Hkv, bs // 8, D, 8)
    ref, _ = oracle_attention.tree_attention(f64(inp.q), f64(inp.k_tree), f64(inp.v_tree), kq, vq, inp.block_table,
                                             lens, cu, parent, inp.scale)
    q, kt, vt = (H.torch_elems(x, "bf16", "cuda") for x in (inp.q, inp.k_tree, inp.v_tree))
    for workers in (1, 2, 0):
        lib.set_option(B.SMART_OPT_TVA_WORKERS, workers)
        try:
            out, _ = lib.tree_verify_attention(q, kt, vt, kc4, vc4, _dev(inp.block_table), d_len, d_cu, mask, inp.scale,
                                               B.SMART_KV_INTERLEAVED, block_size=bs, want_lse=True, k_scale=ks, v_scale=vs)
            torch.cuda.synchronize()
        finally:
            lib.set_option(B.SMART_OPT_TVA_WORKERS, 0)
        got = H.out_to_f64(out, "bf16")
        assert np.isfinite(got).all()
        assert H.rel_err(got, ref) <= H.TOL["bf16"], (workers, H.rel_err(got, ref))


def test_fp8_argument_checks(lib):
    import ctypes
    import torch
    x = torch.zeros(16 * 128, dtype=torch.bfloat16, device="cuda")
    c = torch.zeros(16 * 128, dtype=torch.uint8, device="cuda")
    sm = torch.zeros(1, dtype=torch.int64, device="cuda")
    L = B._lib()
    vp = lambda t: ctypes.c_void_p(t.data_ptr())
    call = lambda ks, vs, dt=B.SMART_BF16: L.kv_cache_write_fp8(lib._h, None, dt, B.SMART_KV_INTERLEAVED, 1, 1, 128, 16, 1,
                                                                vp(x), vp(x), vp(sm), vp(c), vp(c), 2048, 2048, 128,
                                                                ctypes.c_float(ks), ctypes.c_float(vs))
    assert call(1.0, 1.0) == B.SMART_OK
    for ks, vs in ((0.0, 1.0), (1.0, -1.0), (float("nan"), 1.0), (1.0, float("inf"))):
        assert call(ks, vs) == B.SMART_EINVAL
    assert call(1.0, 1.0, dt=B.SMART_FP8_E4M3) == B.SMART_EINVAL
    torch.cuda.synchronize()


def _run_fp8(lib, oracle_attention, w, cu, parent, lens, seed, k_scale=0.05, v_scale=0.02):
    import torch
    inp, kc, vc, kq, vq = _fp8_case(lib, w, cu, parent, lens, k_scale, v_scale, B.SMART_KV_INTERLEAVED, seed)
    f64 = lambda x: W.bf16_bits_to_f32(x).astype(np.float64)
    d_cu, d_par, d_len = _dev(cu), _dev(parent), _dev(lens)
    _, _, _, mask, _ = lib.tree_pack(d_cu, d_par, d_len)
    nb, Hkv, bs, D = inp.k_cache.shape
    out, lse = lib.tree_verify_attention(H.torch_elems(inp.q, "bf16", "cuda"), H.torch_elems(inp.k_tree, "bf16", "cuda"),
                                         H.torch_elems(inp.v_tree, "bf16", "cuda"), kc.view(nb, Hkv, D // 8, bs, 8),
                                         vc.view(nb, Hkv, bs // 8, D, 8), _dev(inp.block_table), d_len, d_cu, mask,
                                         inp.scale, B.SMART_KV_INTERLEAVED, block_size=bs, want_lse=True,
                                         k_scale=k_scale, v_scale=v_scale)
    torch.cuda.synchronize()
    ref, ref_lse = oracle_attention.tree_attention(f64(inp.q), f64(inp.k_tree), f64(inp.v_tree), kq, vq,
                                                   inp.block_table, lens, cu, parent, inp.scale)
    got = H.out_to_f64(out, "bf16")
    assert np.isfinite(got).all()
    err = H.rel_err(got, ref)
    assert err <= H.TOL["bf16"], err
    assert np.abs(lse.cpu().numpy() - ref_lse).max() <= 2e-2
    return got


@pytest.mark.parametrize("batch,G,Hkv,maxlen", [(32, 4, 8, 1200), (5, 8, 2, 3000), (70, 4, 2, 400), (1, 1, 4, 2500)])
def test_fp8_small_trees_on_the_matrix_cores(lib, oracle_attention, batch, G, Hkv, maxlen):
    """Every sequence has at most 32 rows per kv head: all of them go through the fp8 streaming kernel
    (ragged prefixes, empty prefixes, several workers per segment, more than 64 sequences)."""
    rng = np.random.default_rng(batch + G)
    sizes = rng.integers(1, 32 // G + 1, batch)
    trees = [W.random_tree(int(n), rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = rng.integers(0, maxlen, batch).astype(np.int32)
    lens[0] = maxlen
    if batch > 3:
        lens[1], lens[2], lens[3] = 0, 33, 31
    w = W.Workload("fp8_small", "bf16", batch, Hkv * G, Hkv, 128, 0, 0, seed=77)
    a = _run_fp8(lib, oracle_attention, w, cu, parent, lens, 77)
    # the general kernel over the same fp8 cache agrees (two implementations of one definition)
    lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 1)
    try:
        g = _run_fp8(lib, oracle_attention, w, cu, parent, lens, 77)
    finally:
        lib.set_option(B.SMART_OPT_TVA_FORCE_GENERAL, 0)
    assert H.rel_err(a, g) <= H.TOL["bf16"]


def test_fp8_scales_are_applied(lib, oracle_attention):
    """Large and small scales, keys and values scaled apart: the result follows the decoded cache."""
    rng = np.random.default_rng(2)
    sizes = [4, 6, 2]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = np.array([700, 64, 129], np.int32)
    w = W.Workload("fp8_scales", "bf16", 3, 8, 2, 128, 0, 0, seed=5)
    for ks, vs in ((0.01, 0.3), (0.2, 0.01), (1.0, 1.0)):
        _run_fp8(lib, oracle_attention, w, cu, parent, lens, 5, k_scale=ks, v_scale=vs)


def test_fp8_scales_and_row_groups_of_large_trees(lib, oracle_attention):
    """Trees of more than 64 rows per kv head go through the LDS-staged loop (fp8 bytes converted to bf16 in LDS):
    one, two and three row groups of 256 rows at 8 heads per kv head, the last group with 1, 3 and 8 row tiles,
    ragged and exact prefix ends, an empty prefix, keys and values scaled apart."""
    rng = np.random.default_rng(12)
    sizes = [9, 33, 35, 64, 12, 60]                 # 72, 264, 280, 512, 96 and 480 rows per kv head
    trees = [W.random_tree(n, rng, s) for n, s in zip(sizes, ["random", "chain", "random", "random", "star", "random"])]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = np.array([1500, 257, 96, 1029, 0, 33], np.int32)
    w = W.Workload("fp8_large", "bf16", len(sizes), 16, 2, 128, 0, 0, seed=44)
    for ks, vs in ((0.05, 0.02), (0.011, 0.4)):
        _run_fp8(lib, oracle_attention, w, cu, parent, lens, 44, k_scale=ks, v_scale=vs)


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tree_commit_into_an_fp8_cache(lib, dtype):
    """The accepted path's rows go into the fp8 cache as the writer would quantise them; the oracle commits the
    oracle-encoded rows into a byte cache.  Lengths, status and every cache byte agree."""
    import torch
    from oracle import pack_accept as PA
    rng = np.random.default_rng(12)
    Bsz, Hkv, bs, D, max_depth, max_blocks = 6, 2, 16, 128, 5, 4
    sizes = [int(x) for x in rng.integers(2, 30, size=Bsz)]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    N = int(cu[-1])
    token = rng.integers(0, 4, size=N).astype(np.int32)
    target = rng.integers(0, 4, size=N).astype(np.int32)
    prefix_len = rng.integers(0, (max_blocks - 1) * bs, size=Bsz).astype(np.int32)
    nb = Bsz * max_blocks + 2
    block_table = rng.permutation(nb)[:Bsz * max_blocks].reshape(Bsz, max_blocks).astype(np.int32)
    k_tree = W._normal(12, 1, (N, Hkv, D), 1.0, dtype)
    v_tree = W._normal(12, 2, (N, Hkv, D), 1.0, dtype)
    k_scale, v_scale = 0.04, 0.25
    acc_len, acc_path, _ = lib.tree_accept(_dev(cu), _dev(parent), _dev(token), _dev(target), max_depth)
    h_len, h_path = acc_len.cpu().numpy().copy(), acc_path.cpu().numpy().copy()
    assert h_len.max() >= 1
    prefix_len[1] = max_blocks * bs - int(h_len[1])           # one token too many for sequence 1
    ref_k = rng.integers(0, 255, (nb, Hkv, bs, D)).astype(np.uint8)
    ref_v = rng.integers(0, 255, (nb, Hkv, bs, D)).astype(np.uint8)
    start_k, start_v = ref_k.copy(), ref_v.copy()
    ek = F.encode(_f32(k_tree, dtype) / np.float32(k_scale))
    ev = F.encode(_f32(v_tree, dtype) / np.float32(v_scale))
    ref_len, ref_status = PA.commit(cu, h_len, h_path, ek, ev, ref_k, ref_v, block_table, prefix_len, max_depth)
    assert ref_status[1] == B.SMART_ECAP
    tk, tv = H.torch_elems(k_tree, dtype, "cuda"), H.torch_elems(v_tree, dtype, "cuda")
    for layout in (B.SMART_KV_PLAIN, B.SMART_KV_INTERLEAVED):
        if layout == B.SMART_KV_PLAIN:
            kc, vc = _dev(start_k.reshape(nb, Hkv, bs * D)), _dev(start_v.reshape(nb, Hkv, bs * D))
        else:
            kc, vc = _dev(KL.interleave_plain_cache(start_k, "k")), _dev(KL.interleave_plain_cache(start_v, "v"))
        new_len, status = lib.tree_commit(_dev(cu), _dev(h_len), _dev(h_path), tk, tv, kc, vc, _dev(block_table),
                                          _dev(prefix_len), layout, bs, nb, Hkv * bs * D, bs * D, D,
                                          k_scale=k_scale, v_scale=v_scale)
        torch.cuda.synchronize()
        assert status.cpu().numpy().tolist() == ref_status and new_len.cpu().numpy().tolist() == ref_len
        if layout == B.SMART_KV_PLAIN:
            assert np.array_equal(kc.cpu().numpy().reshape(ref_k.shape), ref_k)
            assert np.array_equal(vc.cpu().numpy().reshape(ref_v.shape), ref_v)
        else:
            assert np.array_equal(kc.cpu().numpy(), KL.interleave_plain_cache(ref_k, "k"))
            assert np.array_equal(vc.cpu().numpy(), KL.interleave_plain_cache(ref_v, "v"))


def test_fp8_random_shapes(lib, oracle_attention):
    """Seeded random shapes over an fp8 cache: batches around the 64-sequence plan window, group sizes 1..16,
    one- and two-tile row groups and trees that need several groups, ragged and empty prefixes."""
    rng = np.random.default_rng(31)
    for case in range(30):
        batch = int(rng.choice([1, 2, 5, 8, 17, 33, 64, 65, 70]))
        Hkv, G = int(rng.choice([1, 2, 4, 8])), int(rng.choice([1, 2, 4, 7, 8, 16]))
        lo, hi = {"small": (1, 9), "mixed": (1, 129), "big": (40, 129)}[str(rng.choice(["small", "mixed", "big"]))]
        sizes = rng.integers(lo, hi, batch)
        if batch * int(sizes.max()) * Hkv * G > 30000:
            sizes = np.minimum(sizes, 20)
        trees = [W.random_tree(int(n), rng, str(rng.choice(["random", "chain", "star"]))) for n in sizes]
        cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
        parent = np.concatenate(trees).astype(np.int32)
        lens = rng.integers(0, int(rng.choice([40, 300, 1200])), batch).astype(np.int32)
        lens[rng.integers(0, batch)] = int(rng.choice([0, 1, 31, 32, 33, 64]))
        w = W.Workload("fp8_random", "bf16", batch, Hkv * G, Hkv, 128, 0, 0, seed=4000 + case)
        _run_fp8(lib, oracle_attention, w, cu, parent, lens, 4000 + case,
                 k_scale=float(rng.choice([0.02, 0.05, 0.3])), v_scale=float(rng.choice([0.02, 0.05, 0.3])))
