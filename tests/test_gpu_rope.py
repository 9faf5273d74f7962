"""GPU parity of tree_rope against the CPU oracle, through the C ABI, and the rotated tree through
tree_verify_attention."""
import numpy as np
import pytest

from oracle import pack_accept as PA
from oracle import rope as R
from paper_2604_09731_amd import binding as B
from paper_2604_09731_amd import workloads as W
from tests import helpers as H

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lib():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    return B.SmartTree(0)


def _elems(rng, shape, dtype):
    x = rng.standard_normal(shape).astype(np.float32)
    if dtype == "bf16":
        bits = W.f32_to_bf16_bits(x)
        return bits, W.bf16_bits_to_f32(bits).astype(np.float64)
    return x, x.astype(np.float64)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("pairing", [B.SMART_ROPE_HALF_SPLIT, B.SMART_ROPE_INTERLEAVED])
@pytest.mark.parametrize("D,rot,base", [(128, 128, 10000.0), (128, 64, 500000.0), (64, 64, 10000.0), (64, 2, 7.5)])
def test_tree_rope_against_the_oracle(lib, dtype, pairing, D, rot, base):
    import torch
    rng = np.random.default_rng(D + rot + pairing)
    N, Hq, Hkv = 77, 8, 2
    pos = np.concatenate([[0, 1, 2, 131071, 99999], rng.integers(0, 131072, N - 5)]).astype(np.int32)
    q_raw, q64 = _elems(rng, (N, Hq, D), dtype)
    k_raw, k64 = _elems(rng, (N, Hkv, D), dtype)
    q, k = H.torch_elems(q_raw, dtype, "cuda"), H.torch_elems(k_raw, dtype, "cuda")
    lib.tree_rope(torch.from_numpy(pos).cuda(), q, k, base=base, rotary_dim=rot, pairing=pairing)
    torch.cuda.synchronize()
    for got, ref in ((q, R.rope(q64, pos, base, rot, pairing)), (k, R.rope(k64, pos, base, rot, pairing))):
        got = H.out_to_f64(got, dtype)
        assert H.rel_err(got, ref) <= (2e-6 if dtype == "f32" else 2 ** -8), H.rel_err(got, ref)
        # what lies past rotary_dim is bit-identical to the input
        assert np.array_equal(got[..., rot:], (q64 if got.shape[1] == Hq else k64)[..., rot:])
        # binary32 rotation of unit-scale inputs: every element within rounding of the exact value
        tol = 4e-6 if dtype == "f32" else 2 ** -8 * np.maximum(np.abs(ref), 1e-3) + 1e-6
        assert (np.abs(got - ref) <= tol * (4.0 if dtype == "f32" else 1.0)).all()


def test_tree_rope_argument_checks(lib):
    import ctypes
    import torch
    L = B._lib()
    x = torch.zeros(4 * 2 * 128, dtype=torch.float32, device="cuda")
    pos = torch.zeros(4, dtype=torch.int32, device="cuda")
    ok = dict(dtype=B.SMART_F32, n=4, hq=1, hkv=1, d=128, rot=128, pairing=0, base=10000.0,
              pos=pos.data_ptr(), q=x.data_ptr(), k=x.data_ptr())

    def call(**kw):
        a = dict(ok, **kw)
        return L.tree_rope(lib._h, None, a["dtype"], a["n"], a["hq"], a["hkv"], a["d"], a["rot"], a["pairing"],
                           ctypes.c_double(a["base"]), ctypes.c_void_p(a["pos"]) if a["pos"] else None,
                           ctypes.c_void_p(a["q"]) if a["q"] else None, ctypes.c_void_p(a["k"]) if a["k"] else None)

    assert call() == B.SMART_OK and call(n=0, pos=0) == B.SMART_OK
    for bad in (dict(dtype=5), dict(n=-1), dict(d=130, rot=130), dict(rot=127), dict(rot=0), dict(rot=130),
                dict(pairing=2), dict(base=0.0), dict(base=float("nan")), dict(pos=0), dict(q=0), dict(hq=0, hkv=0)):
        assert call(**bad) == B.SMART_EINVAL, bad
    assert call(hq=0, q=0) == B.SMART_OK                      # keys only
    torch.cuda.synchronize()


def test_rotated_tree_through_attention(lib, oracle_attention):
    """pack -> tree_rope -> attention over a cache of rotated keys, against the oracle fed the oracle's
    own rotation; and the same step with every position shifted by a constant (scores depend on relative
    positions only, so the output must not move)."""
    import torch
    rng = np.random.default_rng(3)
    sizes = [5, 17, 40, 1]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    lens = np.array([64, 100, 517, 33], np.int32)
    w = W.Workload("rope", "bf16", 4, 8, 2, 128, 0, 0, seed=9)
    inp = W.make_attention_inputs(w, cu, seed=9, prefix_len=lens)
    f64 = lambda bits: W.bf16_bits_to_f32(bits).astype(np.float64)
    bs = inp.k_cache.shape[2]
    outs = []
    for shift in (0, 1000):
        # rotate the cached keys by their token positions (host side, rounded to bf16: what the cache holds)
        k_cache = f64(inp.k_cache)
        for b in range(4):
            for t in range(int(lens[b])):
                blk, slot = int(inp.block_table[b, t // bs]), t % bs
                k_cache[blk, :, slot, :] = R.rope(k_cache[blk, :, slot, :][None], [t + shift])[0]
        k_cache_bits = W.f32_to_bf16_bits(k_cache.astype(np.float32))
        depth, pos, _, _ = PA.pack(cu, parent, lens + shift)
        d_cu, d_par = torch.from_numpy(cu).cuda(), torch.from_numpy(parent).cuda()
        d_len = torch.from_numpy(lens).cuda()
        _, position, _, mask, status = lib.tree_pack(d_cu, d_par, torch.from_numpy(lens + shift).cuda())
        assert position.cpu().numpy().tolist() == pos
        q, kt = H.torch_elems(inp.q, "bf16", "cuda"), H.torch_elems(inp.k_tree, "bf16", "cuda")
        lib.tree_rope(position, q, kt)
        kc, vc = B.interleave_kv_cache(H.torch_elems(k_cache_bits, "bf16", "cuda"),
                                       H.torch_elems(inp.v_cache, "bf16", "cuda"))
        out = lib.tree_verify_attention(q, kt, H.torch_elems(inp.v_tree, "bf16", "cuda"), kc, vc,
                                        torch.from_numpy(inp.block_table).cuda(), d_len, d_cu, mask, inp.scale,
                                        B.SMART_KV_INTERLEAVED)
        torch.cuda.synchronize()
        ref, _ = oracle_attention.tree_attention(R.rope(f64(inp.q), pos), R.rope(f64(inp.k_tree), pos),
                                                 f64(inp.v_tree), f64(k_cache_bits), f64(inp.v_cache),
                                                 inp.block_table, lens, cu, parent, inp.scale)
        got = H.out_to_f64(out, "bf16")
        assert H.rel_err(got, ref) <= H.TOL["bf16"], H.rel_err(got, ref)
        outs.append(got)
    assert H.rel_err(outs[1], outs[0]) <= H.TOL["bf16"]
