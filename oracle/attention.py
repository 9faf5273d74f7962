"""CPU oracle: tree-verification attention (fp64).  TEST INFRASTRUCTURE ONLY.

Thin ctypes wrapper around ``tree_attention_ref.c`` (which holds the definition
and its citation) plus a helper that compiles it with gcc.  Only ``tests/``,
``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline`` leg may use
this module; the product package never imports it.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tree_attention_ref.c")
_LIB = os.path.join(_HERE, "libtree_attention_ref.so")
_lib = None

DTYPE_F32, DTYPE_BF16, DTYPE_F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the C oracle (gcc, -O2, no FMA contraction, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        c_i32p = ctypes.POINTER(ctypes.c_int32)
        lib.tree_attention_ref.restype = ctypes.c_int
        lib.tree_attention_ref.argtypes = [
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int64, ctypes.c_int64, ctypes.c_int64,
            c_i32p, ctypes.c_int, c_i32p, c_i32p, c_i32p,
            ctypes.c_int64, c_i32p, c_i32p,
            ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
        lib.tree_attention_ref_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def num_threads() -> int:
    return int(_load().tree_attention_ref_threads())


def _dtype_code(a: np.ndarray) -> int:
    if a.dtype == np.float32:
        return DTYPE_F32
    if a.dtype == np.float64:
        return DTYPE_F64
    if a.dtype == np.uint16:
        return DTYPE_BF16          # raw bfloat16 bit patterns
    raise TypeError(f"unsupported element type {a.dtype}")


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def tree_attention(q, k_tree, v_tree, k_cache, v_cache, block_table, prefix_len,
                   cu_nodes, parent, scale, sel=None):
    """out, lse = attention of every tree node over its prefix + ancestors-or-self.

    q        [N, Hq, D]; k_tree, v_tree [N, Hkv, D];
    k_cache, v_cache [num_blocks, Hkv, block_size, D] (plain layout);
    all float32 / float64 / uint16 (= bf16 bits), one shared type.
    block_table [B, max_blocks]; prefix_len [B]; cu_nodes [B+1]; parent [N].
    sel: optional (nodes, heads) int arrays -> only those rows, out [n_sel, D].
    """
    lib = _load()
    q = np.ascontiguousarray(q)
    code = _dtype_code(q)
    arrs = [np.ascontiguousarray(x) for x in (k_tree, v_tree, k_cache, v_cache)]
    for a in arrs:
        if _dtype_code(a) != code:
            raise TypeError("q, k, v must share one element type")
    k_tree, v_tree, k_cache, v_cache = arrs
    N, Hq, D = q.shape
    Hkv = k_tree.shape[1]
    nb, Hkv2, bs, D2 = k_cache.shape
    assert Hkv2 == Hkv and D2 == D and v_cache.shape == k_cache.shape
    assert k_tree.shape == (N, Hkv, D) and v_tree.shape == (N, Hkv, D)
    block_table = np.ascontiguousarray(block_table, dtype=np.int32)
    B, max_blocks = block_table.shape
    bt, bt_p = _i32(block_table)
    pl, pl_p = _i32(prefix_len)
    cu, cu_p = _i32(cu_nodes)
    pa, pa_p = _i32(parent)
    assert cu.shape == (B + 1,) and pl.shape == (B,) and int(cu[-1]) == N and pa.shape == (N,)
    if pl.size:
        used = (pl.max() + bs - 1) // bs
        assert used <= max_blocks
        for b in range(B):      # only the entries a sequence's prefix reaches are read
            ub = bt[b, :(int(pl[b]) + bs - 1) // bs]
            assert ub.size == 0 or (ub.min() >= 0 and ub.max() < nb)
    if sel is None:
        n_sel = -1
        sn_p = sh_p = None
        out = np.empty((N, Hq, D), dtype=np.float64)
        lse = np.empty((N, Hq), dtype=np.float64)
    else:
        sn, sn_p = _i32(sel[0])
        sh, sh_p = _i32(sel[1])
        n_sel = int(sn.shape[0])
        assert sh.shape == sn.shape
        assert n_sel == 0 or (sn.min() >= 0 and sn.max() < N and sh.min() >= 0 and sh.max() < Hq)
        out = np.empty((n_sel, D), dtype=np.float64)
        lse = np.empty((n_sel,), dtype=np.float64)
    ptr = lambda a: ctypes.c_void_p(a.ctypes.data)
    rc = lib.tree_attention_ref(
        code, B, Hq, Hkv, D, bs, float(scale),
        ptr(q), ptr(k_tree), ptr(v_tree), ptr(k_cache), ptr(v_cache),
        k_cache.strides[0] // k_cache.itemsize, k_cache.strides[1] // k_cache.itemsize,
        k_cache.strides[2] // k_cache.itemsize,
        bt_p, max_blocks, pl_p, cu_p, pa_p,
        n_sel, sn_p, sh_p,
        out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)),
        lse.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"tree_attention_ref rejected its input (code {rc})")
    return out, lse
