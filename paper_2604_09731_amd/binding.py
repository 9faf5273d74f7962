"""Thin ctypes binding of libsmart_tree.so (argument marshalling only).

Every step runs in the library's kernels (or, for selection, its host C++).
PyTorch supplies device memory and streams.  There is no fallback: if the
library has not been built, or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("SMART_TREE_LIB") or os.path.join(_HERE, "libsmart_tree.so")

SMART_OK, SMART_EINVAL, SMART_ETREE, SMART_ECAP, SMART_EHIP, SMART_ENOMEM = 0, -1, -2, -3, -4, -5
SMART_F32, SMART_BF16 = 0, 1
SMART_FP8_E4M3 = 2
SMART_TVA_BAD_BLOCK = 1
SMART_KV_PLAIN, SMART_KV_INTERLEAVED = 0, 1
SMART_BEST_FIRST, SMART_LAYERWISE = 0, 1
SMART_DILUTION_NONE, SMART_DILUTION_PATH_MEAN = 0, 1
SMART_OPT_TVA_WORKERS, SMART_OPT_TVA_FORCE_GENERAL, SMART_OPT_TVA_PROFILE = 1, 2, 3
SMART_OPT_TVA_PROFILE_STRIDE = 4
SMART_ROPE_HALF_SPLIT, SMART_ROPE_INTERLEAVED = 0, 1
SMART_MAX_NODES = 128
SMART_MAX_LAYER_CAND = 2048

EXPORTS = ["smart_strerror", "smart_last_hip_error", "smart_create", "smart_destroy",
           "smart_reserve", "smart_set_option", "smart_tva_profile_read", "smart_select_tree", "smart_select_tree_budgets", "smart_baseline_tree", "smart_product_forest", "smart_select_begin", "smart_select_layer",
           "smart_select_begin_device", "smart_select_layer_device", "tree_compact_pack", "tree_rope", "smart_cost_tables", "smart_cost_tables_biased", "smart_fit_cost_models", "tree_upload",
           "tree_upload_pack", "tree_pack",
           "kv_cache_write", "kv_cache_write_fp8", "tree_verify_attention", "tree_verify_attention_static", "tree_accept", "tree_accept_sample", "tree_commit", "tree_commit_fp8"]


class SmartError(RuntimeError):
    def __init__(self, code: int, what: str):
        self.code = code
        super().__init__(f"{what}: {_strerror(code)} (code {code}, hip error {_lib().smart_last_hip_error()})")


class TvaParams(ctypes.Structure):
    _fields_ = [
        ("dtype", ctypes.c_int32), ("kv_layout", ctypes.c_int32),
        ("batch", ctypes.c_int32), ("total_nodes", ctypes.c_int32),
        ("num_q_heads", ctypes.c_int32), ("num_kv_heads", ctypes.c_int32),
        ("head_dim", ctypes.c_int32),
        ("block_size", ctypes.c_int32), ("max_blocks_per_seq", ctypes.c_int32),
        ("num_blocks", ctypes.c_int32),
        ("softmax_scale", ctypes.c_float), ("kv_cache_dtype", ctypes.c_int32),
        ("d_q", ctypes.c_void_p), ("d_k_tree", ctypes.c_void_p), ("d_v_tree", ctypes.c_void_p),
        ("d_k_cache", ctypes.c_void_p), ("d_v_cache", ctypes.c_void_p),
        ("cache_block_stride", ctypes.c_int64), ("cache_head_stride", ctypes.c_int64),
        ("cache_token_stride", ctypes.c_int64),
        ("d_block_table", ctypes.c_void_p), ("d_prefix_len", ctypes.c_void_p),
        ("d_cu_nodes", ctypes.c_void_p), ("d_anc_mask", ctypes.c_void_p),
        ("d_out", ctypes.c_void_p), ("d_lse", ctypes.c_void_p),
        ("h_cu_nodes", ctypes.c_void_p),
        ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float),
        ("d_status", ctypes.c_void_p),
    ]


class LayerStateStruct(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("budget", ctypes.c_int32),
                ("n", ctypes.c_void_p), ("layer_begin", ctypes.c_void_p), ("sum_P", ctypes.c_void_p),
                ("parent", ctypes.c_void_p), ("token", ctypes.c_void_p), ("pathprob", ctypes.c_void_p),
                ("path_sum", ctypes.c_void_p), ("L", ctypes.c_void_p), ("R", ctypes.c_void_p)]


_STATE_FIELDS = (("n", "i4", False), ("layer_begin", "i4", False), ("sum_P", "f8", False),
                 ("parent", "i4", True), ("token", "i4", True), ("pathprob", "f8", True),
                 ("path_sum", "f8", True), ("L", "f8", False), ("R", "f8", False))

_libh = None


def _lib():
    global _libh
    if _libh is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with "
                               "`python -m paper_2604_09731_amd.build` (there is no fallback)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32, i64, f64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_double
        lib.smart_strerror.restype = ctypes.c_char_p
        lib.smart_strerror.argtypes = [i32]
        lib.smart_last_hip_error.restype = i32
        lib.smart_create.restype = i32
        lib.smart_create.argtypes = [ctypes.POINTER(vp), i32]
        lib.smart_destroy.restype = i32
        lib.smart_destroy.argtypes = [vp]
        lib.smart_reserve.restype = i32
        lib.smart_reserve.argtypes = [vp, i32, i32, i32, i32]
        lib.smart_set_option.restype = i32
        lib.smart_set_option.argtypes = [vp, i32, i64]
        lib.smart_tva_profile_read.restype = i32
        lib.smart_tva_profile_read.argtypes = [vp, vp, i32, vp]
        lib.smart_select_tree.restype = i32
        lib.smart_select_tree.argtypes = [i32, vp, vp, vp, vp, vp, vp, f64, i32, i32, i32, i32,
                                          vp, vp, vp, vp, vp, i64, vp, vp]
        lib.smart_select_tree_budgets.restype = i32
        lib.smart_select_tree_budgets.argtypes = [i32, vp, vp, vp, vp, vp, vp, f64, i32, i32, vp, i32, i32,
                                                  vp, vp, vp, vp, vp, i64, vp, vp]
        lib.smart_baseline_tree.restype = i32
        lib.smart_baseline_tree.argtypes = [i32, vp, vp, vp, vp, vp, i32, i32, i32, vp, vp, vp, vp, vp, i64, vp, vp]
        lib.smart_product_forest.restype = i32
        lib.smart_product_forest.argtypes = [i32, i32, i32, vp, vp, i32, vp, vp, vp, vp, i64]
        sp = ctypes.POINTER(LayerStateStruct)
        lib.smart_select_begin.restype = i32
        lib.smart_select_begin.argtypes = [sp, vp, vp]
        lib.smart_select_layer.restype = i32
        lib.smart_select_layer.argtypes = [sp, vp, vp, vp, vp, vp, vp, f64, i32, vp]
        lib.smart_select_begin_device.restype = i32
        lib.smart_select_begin_device.argtypes = [vp, vp, sp, vp, vp]
        lib.smart_select_layer_device.restype = i32
        lib.smart_select_layer_device.argtypes = [vp, vp, sp, vp, vp, vp, vp, i64, vp, vp, f64, i32, vp, vp]
        lib.tree_compact_pack.restype = i32
        lib.tree_compact_pack.argtypes = [vp, vp, sp, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.tree_rope.restype = i32
        lib.tree_rope.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, f64, vp, vp, vp]
        lib.smart_cost_tables.restype = i32
        lib.smart_cost_tables.argtypes = [f64, f64, f64, f64, f64, f64, i32, vp, vp]
        lib.smart_cost_tables_biased.restype = i32
        lib.smart_cost_tables_biased.argtypes = [f64, f64, f64, f64, f64, f64, f64, f64, i32, i32, vp, vp]
        lib.smart_fit_cost_models.restype = i32
        lib.smart_fit_cost_models.argtypes = [i32, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.tree_upload.restype = i32
        lib.tree_upload.argtypes = [vp, vp, vp, vp, i64]
        lib.tree_upload_pack.restype = i32
        lib.tree_upload_pack.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.tree_pack.restype = i32
        lib.tree_pack.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp, vp]
        lib.kv_cache_write.restype = i32
        lib.kv_cache_write.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                       i64, i64, i64]
        lib.kv_cache_write_fp8.restype = i32
        lib.kv_cache_write_fp8.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                           i64, i64, i64, ctypes.c_float, ctypes.c_float]
        lib.tree_verify_attention.restype = i32
        lib.tree_verify_attention.argtypes = [vp, vp, ctypes.POINTER(TvaParams)]
        lib.tree_verify_attention_static.restype = i32
        lib.tree_verify_attention_static.argtypes = [vp, vp, ctypes.POINTER(TvaParams)]
        lib.tree_commit.restype = i32
        lib.tree_commit.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp, vp,
                                    vp, vp, i64, i64, i64, vp, vp]
        lib.tree_accept_sample.restype = i32
        lib.tree_accept_sample.argtypes = [vp, vp, i32, i32, i32, i32, vp, vp, vp, vp, i64, ctypes.c_uint64,
                                           ctypes.c_uint64, vp, vp, vp]
        lib.tree_commit_fp8.restype = i32
        lib.tree_commit_fp8.argtypes = [vp, vp, i32, i32, i32, i32, i32, i32, i32, i32, i32, vp, vp, vp, vp, vp, vp,
                                        vp, vp, vp, i64, i64, i64, vp, vp, ctypes.c_float, ctypes.c_float]
        lib.tree_accept.restype = i32
        lib.tree_accept.argtypes = [vp, vp, i32, i32, vp, vp, vp, vp, vp, vp, vp]
        _libh = lib
    return _libh


def _strerror(code: int) -> str:
    return _lib().smart_strerror(code).decode()


def _check(code: int, what: str):
    if code != SMART_OK:
        raise SmartError(code, what)


# ---------------------------------------------------------------------------
# host: selection
# ---------------------------------------------------------------------------
def smart_select_tree(cand_cu, cand_parent, cand_prob, cand_token, cost, dcost=None, alpha=0.8,
                      max_depth=8, budget=64, schedule=SMART_BEST_FIRST,
                      dilution=SMART_DILUTION_NONE, out_cap: Optional[int] = None, budgets=None):
    """Returns dict(cu_nodes, parent, token, cand_index, pathprob, L, R) of numpy arrays.
    ``budgets``: optional per-sequence budgets (each at most ``budget``, which sizes the tables)."""
    cand_cu = np.ascontiguousarray(cand_cu, np.int32)
    cand_parent = np.ascontiguousarray(cand_parent, np.int32)
    cand_prob = np.ascontiguousarray(cand_prob, np.float64)
    cand_token = np.ascontiguousarray(cand_token, np.int32)
    cost = np.ascontiguousarray(cost, np.float64)
    if dcost is not None:
        dcost = np.ascontiguousarray(dcost, np.float64)
        if dcost.shape[0] < budget + 1:
            raise ValueError("dcost needs budget + 1 entries")
    if cost.shape[0] < budget + 2:
        raise ValueError("cost needs budget + 2 entries")
    batch = cand_cu.shape[0] - 1
    cap = int(out_cap if out_cap is not None else batch * max(budget, 1))
    o_cu = np.zeros(batch + 1, np.int32)
    o_parent = np.zeros(max(cap, 1), np.int32)
    o_token = np.zeros(max(cap, 1), np.int32)
    o_cand = np.zeros(max(cap, 1), np.int32)
    o_pp = np.zeros(max(cap, 1), np.float64)
    o_L = np.zeros(max(batch, 1), np.float64)
    o_R = np.zeros(max(batch, 1), np.float64)
    p = lambda a: ctypes.c_void_p(a.ctypes.data) if a is not None else None
    if budgets is None:
        rc = _lib().smart_select_tree(batch, p(cand_cu), p(cand_parent), p(cand_prob), p(cand_token),
                                      p(cost), p(dcost), float(alpha), int(max_depth), int(budget),
                                      int(schedule), int(dilution), p(o_cu), p(o_parent), p(o_token),
                                      p(o_cand), p(o_pp), cap, p(o_L), p(o_R))
    else:
        budgets = np.ascontiguousarray(budgets, np.int32)
        if budgets.shape[0] != batch:
            raise ValueError("one budget per sequence")
        rc = _lib().smart_select_tree_budgets(batch, p(cand_cu), p(cand_parent), p(cand_prob), p(cand_token),
                                              p(cost), p(dcost), float(alpha), int(max_depth), int(budget),
                                              p(budgets), int(schedule), int(dilution), p(o_cu), p(o_parent),
                                              p(o_token), p(o_cand), p(o_pp), cap, p(o_L), p(o_R))
    _check(rc, "smart_select_tree")
    n = int(o_cu[-1])
    return dict(cu_nodes=o_cu, parent=o_parent[:n], token=o_token[:n], cand_index=o_cand[:n],
                pathprob=o_pp[:n], L=o_L[:batch], R=o_R[:batch])


def smart_baseline_tree(cand_cu, cand_parent, cand_prob, cand_token, cost, k=10, max_depth=6, g=60):
    """The expand-top-k / keep-top-g policy; same result dict as smart_select_tree."""
    cand_cu = np.ascontiguousarray(cand_cu, np.int32)
    cand_parent = np.ascontiguousarray(cand_parent, np.int32)
    cand_prob = np.ascontiguousarray(cand_prob, np.float64)
    cand_token = np.ascontiguousarray(cand_token, np.int32)
    cost = np.ascontiguousarray(cost, np.float64)
    if cost.shape[0] < g + 2:
        raise ValueError("cost needs g + 2 entries")
    batch = cand_cu.shape[0] - 1
    cap = max(1, batch * (g + 1))
    o_cu = np.zeros(batch + 1, np.int32)
    o_parent, o_token, o_cand = (np.zeros(cap, np.int32) for _ in range(3))
    o_pp = np.zeros(cap, np.float64)
    o_L, o_R = np.zeros(max(batch, 1), np.float64), np.zeros(max(batch, 1), np.float64)
    p = lambda a: ctypes.c_void_p(a.ctypes.data)
    rc = _lib().smart_baseline_tree(batch, p(cand_cu), p(cand_parent), p(cand_prob), p(cand_token), p(cost), int(k),
                                    int(max_depth), int(g), p(o_cu), p(o_parent), p(o_token), p(o_cand), p(o_pp),
                                    cap, p(o_L), p(o_R))
    _check(rc, "smart_baseline_tree")
    n = int(o_cu[-1])
    return dict(cu_nodes=o_cu, parent=o_parent[:n], token=o_token[:n], cand_index=o_cand[:n], pathprob=o_pp[:n],
                L=o_L[:batch], R=o_R[:batch])


def smart_product_forest(pos_prob, pos_token, cap):
    """Candidate forests of a drafter with independent positions: pos_prob, pos_token [batch][depth][k]; the `cap`
    most probable nodes of the Cartesian product per sequence.  Returns cand_cu / cand_parent / cand_prob /
    cand_token as smart_select_tree and smart_baseline_tree read them."""
    pos_prob = np.ascontiguousarray(pos_prob, np.float64)
    pos_token = np.ascontiguousarray(pos_token, np.int32)
    if pos_prob.ndim != 3 or pos_prob.shape != pos_token.shape:
        raise ValueError("pos_prob and pos_token must both be [batch][depth][k]")
    batch, depth, k = (int(v) for v in pos_prob.shape)
    total = max(1, batch * int(cap))
    cu = np.zeros(batch + 1, np.int32)
    parent, token = np.zeros(total, np.int32), np.zeros(total, np.int32)
    prob = np.zeros(total, np.float64)
    p = lambda a: ctypes.c_void_p(a.ctypes.data)
    rc = _lib().smart_product_forest(batch, depth, k, p(pos_prob), p(pos_token), int(cap), p(cu), p(parent), p(prob),
                                     p(token), total)
    _check(rc, "smart_product_forest")
    n = int(cu[-1])
    return dict(cand_cu=cu, cand_parent=parent[:n], cand_prob=prob[:n], cand_token=token[:n])


class HostLayerState:
    """Trees under construction by Algorithm 1 one layer at a time, in host (numpy) arrays."""

    def __init__(self, batch: int, budget: int, path_sum: bool = True):
        self.batch, self.budget = int(batch), int(budget)
        self.struct = LayerStateStruct(batch=self.batch, budget=self.budget)
        for name, kind, per_node in _STATE_FIELDS:
            if name == "path_sum" and not path_sum:
                arr = None
            else:
                arr = np.zeros(max(1, self.batch * (self.budget if per_node else 1)), np.dtype(kind))
            setattr(self, name, arr)
            setattr(self.struct, name, arr.ctypes.data if arr is not None else None)

    def begin(self, root_token, cost):
        root_token = np.ascontiguousarray(root_token, np.int32)
        cost = np.ascontiguousarray(cost, np.float64)
        assert root_token.shape[0] == self.batch and cost.shape[0] >= self.budget + 2
        rc = _lib().smart_select_begin(ctypes.byref(self.struct), root_token.ctypes.data, cost.ctypes.data)
        _check(rc, "smart_select_begin")

    def layer(self, cand_cu, cand_parent_node, cand_prob, cand_token, cost, dcost=None, alpha=0.8,
              dilution=SMART_DILUTION_NONE):
        """Offers one layer of candidates; returns the node id (or -1) of each."""
        cand_cu = np.ascontiguousarray(cand_cu, np.int32)
        cand_parent_node = np.ascontiguousarray(cand_parent_node, np.int32)
        cand_prob = np.ascontiguousarray(cand_prob, np.float64)
        cand_token = np.ascontiguousarray(cand_token, np.int32)
        cost = np.ascontiguousarray(cost, np.float64)
        assert cand_cu.shape[0] == self.batch + 1 and cost.shape[0] >= self.budget + 2
        if dcost is not None:
            dcost = np.ascontiguousarray(dcost, np.float64)
            assert dcost.shape[0] >= self.budget + 1
        out = np.full(max(1, cand_parent_node.shape[0]), -1, np.int32)
        p = lambda a: ctypes.c_void_p(a.ctypes.data) if a is not None else None
        rc = _lib().smart_select_layer(ctypes.byref(self.struct), p(cand_cu), p(cand_parent_node), p(cand_prob),
                                       p(cand_token), p(cost), p(dcost), float(alpha), int(dilution), p(out))
        _check(rc, "smart_select_layer")
        return out[:cand_parent_node.shape[0]]

    def tree(self, b: int):
        """(parent, token, pathprob) lists of sequence b."""
        n, o = int(self.n[b]), b * self.budget
        return self.parent[o:o + n].tolist(), self.token[o:o + n].tolist(), self.pathprob[o:o + n].tolist()


class DeviceLayerState:
    """The same state in device (torch) tensors."""

    def __init__(self, batch: int, budget: int, device, path_sum: bool = True):
        torch = _torch()
        self.batch, self.budget = int(batch), int(budget)
        self.struct = LayerStateStruct(batch=self.batch, budget=self.budget)
        for name, kind, per_node in _STATE_FIELDS:
            if name == "path_sum" and not path_sum:
                t = None
            else:
                t = torch.zeros(max(1, self.batch * (self.budget if per_node else 1)),
                                dtype=torch.int32 if kind == "i4" else torch.float64, device=device)
            setattr(self, name, t)
            setattr(self.struct, name, t.data_ptr() if t is not None else None)


def smart_cost_tables(lam, gamma, delta, rho, c_T, tokens_per_node, n_max, want_dcost=True):
    """(cost[n_max + 2], dcost[n_max + 1] or None) of the fitted device cost models."""
    cost = np.zeros(n_max + 2, np.float64)
    dcost = np.zeros(n_max + 1, np.float64) if want_dcost else None
    p = lambda a: ctypes.c_void_p(a.ctypes.data) if a is not None else None
    rc = _lib().smart_cost_tables(float(lam), float(gamma), float(delta), float(rho), float(c_T),
                                  float(tokens_per_node), int(n_max), p(cost), p(dcost))
    _check(rc, "smart_cost_tables")
    return cost, dcost


def smart_cost_tables_biased(lam, beta, gamma, delta, rho, eta, c_T, tokens_per_node, undrafted_nodes, n_max,
                             want_dcost=True):
    """The tables with the models' bias terms kept and the first undrafted_nodes nodes (the root) left out of
    the drafted tokens; (cost[n_max + 2], dcost[n_max + 1] or None)."""
    cost = np.zeros(n_max + 2, np.float64)
    dcost = np.zeros(n_max + 1, np.float64) if want_dcost else None
    p = lambda a: ctypes.c_void_p(a.ctypes.data) if a is not None else None
    rc = _lib().smart_cost_tables_biased(float(lam), float(beta), float(gamma), float(delta), float(rho), float(eta),
                                         float(c_T), float(tokens_per_node), int(undrafted_nodes), int(n_max),
                                         p(cost), p(dcost))
    _check(rc, "smart_cost_tables_biased")
    return cost, dcost


def smart_fit_cost_models(x, t_draft=None, t_verify=None):
    """Least-squares fits; returns dict with lambda (if t_draft) and gamma, delta, rho, sse (if t_verify)."""
    x = np.ascontiguousarray(x, np.float64)
    td = None if t_draft is None else np.ascontiguousarray(t_draft, np.float64)
    tv = None if t_verify is None else np.ascontiguousarray(t_verify, np.float64)
    out = [ctypes.c_double(0.0) for _ in range(5)]
    p = lambda a: ctypes.c_void_p(a.ctypes.data) if a is not None else None
    rc = _lib().smart_fit_cost_models(x.shape[0], p(x), p(td), p(tv), *[ctypes.byref(o) for o in out])
    _check(rc, "smart_fit_cost_models")
    res = {}
    if td is not None:
        res["lambda"] = out[0].value
    if tv is not None:
        res.update(gamma=out[1].value, delta=out[2].value, rho=out[3].value, sse=out[4].value)
    return res


# ---------------------------------------------------------------------------
# device
# ---------------------------------------------------------------------------
def _torch():
    import torch
    return torch


def _stream_ptr():
    torch = _torch()
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else None


def _dtype_code(t):
    torch = _torch()
    if t.dtype == torch.float32:
        return SMART_F32
    if t.dtype == torch.bfloat16:
        return SMART_BF16
    raise TypeError(f"unsupported element type {t.dtype}")


def interleave_kv_cache(k_plain, v_plain):
    """[num_blocks, Hkv, block_size, D] plain caches -> the interleaved layout
    (pure data movement; shapes [nb, Hkv, D/8, bs, 8] and [nb, Hkv, bs/8, D, 8])."""
    nb, Hkv, bs, D = k_plain.shape
    k = k_plain.reshape(nb, Hkv, bs, D // 8, 8).permute(0, 1, 3, 2, 4).contiguous()
    v = v_plain.reshape(nb, Hkv, bs // 8, 8, D).permute(0, 1, 2, 4, 3).contiguous()
    return k, v


class SmartTree:
    """Owns one smart_ctx on one device."""

    def __init__(self, device: int = 0):
        torch = _torch()
        if not torch.cuda.is_available():
            raise RuntimeError("no GPU visible: the tree-verification library needs an MI355X")
        self.device = int(device)
        torch.cuda.set_device(self.device)
        torch.cuda.init()
        h = ctypes.c_void_p()
        _check(_lib().smart_create(ctypes.byref(h), self.device), "smart_create")
        self._h = h

    def close(self):
        if getattr(self, "_h", None):
            _check(_lib().smart_destroy(self._h), "smart_destroy")
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def set_option(self, key: int, value: int):
        _check(_lib().smart_set_option(self._h, key, int(value)), "smart_set_option")

    def reserve(self, max_batch, max_total_nodes, max_q_heads, max_kv_heads):
        _check(_lib().smart_reserve(self._h, max_batch, max_total_nodes, max_q_heads, max_kv_heads),
               "smart_reserve")

    def profile_read(self, cap: int = 65536):
        """Durations (ms) of the dominant attention kernel of the calls recorded
        since the last read; the caller synchronises first."""
        buf = (ctypes.c_float * cap)()
        cnt = ctypes.c_int32(0)
        _check(_lib().smart_tva_profile_read(self._h, buf, cap, ctypes.byref(cnt)),
               "smart_tva_profile_read")
        return [buf[i] for i in range(cnt.value)]

    # -- tree_upload -------------------------------------------------------
    def tree_upload(self, pinned_src, dst):
        """Copies a pinned host int32 tensor into a device int32 tensor of the same length."""
        if pinned_src.numel() != dst.numel():
            raise ValueError("tree_upload: sizes differ")
        rc = _lib().tree_upload(self._h, _stream_ptr(), _ptr(pinned_src), _ptr(dst), pinned_src.numel())
        _check(rc, "tree_upload")
        return dst

    # -- tree_upload_pack --------------------------------------------------
    def tree_upload_pack(self, pinned_cu_nodes, pinned_parent, pinned_token, prefix_len):
        """Pinned host tree CSR -> device copies + tree_pack outputs, one launch.  Returns
        (cu_nodes, parent, token, depth, position, node_seq, anc_mask, status) on the device."""
        torch = _torch()
        B = pinned_cu_nodes.shape[0] - 1
        N = int(pinned_cu_nodes[B])
        dev = prefix_len.device
        i32 = lambda n: torch.empty(n, dtype=torch.int32, device=dev)
        cu, par, tok = i32(B + 1), i32(N), (i32(N) if pinned_token is not None else None)
        depth, position, node_seq, status = i32(N), i32(N), i32(N), i32(B)
        anc_mask = torch.empty((N, 2), dtype=torch.int64, device=dev)
        rc = _lib().tree_upload_pack(self._h, _stream_ptr(), B, N, _ptr(pinned_cu_nodes), _ptr(pinned_parent),
                                     _ptr(pinned_token), _ptr(cu), _ptr(par), _ptr(tok), _ptr(prefix_len),
                                     _ptr(depth), _ptr(position), _ptr(node_seq), _ptr(anc_mask), _ptr(status))
        _check(rc, "tree_upload_pack")
        return cu, par, tok, depth, position, node_seq, anc_mask, status

    # -- Algorithm 1 one layer at a time, on the device ---------------------
    def select_begin(self, state: DeviceLayerState, root_token, cost):
        rc = _lib().smart_select_begin_device(self._h, _stream_ptr(), ctypes.byref(state.struct), _ptr(root_token),
                                              _ptr(cost))
        _check(rc, "smart_select_begin_device")

    def select_layer(self, state: DeviceLayerState, cand_cu, cand_parent_node, cand_prob, cand_token, cost,
                     dcost=None, alpha=0.8, dilution=SMART_DILUTION_NONE, out_node=None, status=None):
        """Device tensors in, (out_node, status) device tensors out; nothing synchronises."""
        torch = _torch()
        cap = cand_parent_node.shape[0]
        if out_node is None:
            out_node = torch.empty(max(1, cap), dtype=torch.int32, device=cand_cu.device)
        if status is None:
            status = torch.empty(max(1, state.batch), dtype=torch.int32, device=cand_cu.device)
        rc = _lib().smart_select_layer_device(self._h, _stream_ptr(), ctypes.byref(state.struct), _ptr(cand_cu),
                                              _ptr(cand_parent_node), _ptr(cand_prob), _ptr(cand_token), cap,
                                              _ptr(cost), _ptr(dcost), float(alpha), int(dilution), _ptr(out_node),
                                              _ptr(status))
        _check(rc, "smart_select_layer_device")
        return out_node[:cap], status[:state.batch]

    def tree_compact_pack(self, state: DeviceLayerState, prefix_len, total_cap=None):
        """Returns (cu_nodes, parent, token, depth, position, node_seq, anc_mask, status); the per-node
        tensors have total_cap rows of which cu_nodes[-1] are in use."""
        torch = _torch()
        B = state.batch
        N = int(total_cap if total_cap is not None else B * state.budget)
        dev = prefix_len.device
        i32 = lambda n: torch.zeros(max(1, n), dtype=torch.int32, device=dev)
        cu, par, tok = i32(B + 1), i32(N), i32(N)
        depth, position, node_seq, status = i32(N), i32(N), i32(N), i32(B)
        anc_mask = torch.zeros((max(1, N), 2), dtype=torch.int64, device=dev)
        rc = _lib().tree_compact_pack(self._h, _stream_ptr(), ctypes.byref(state.struct), N, _ptr(prefix_len),
                                      _ptr(cu), _ptr(par), _ptr(tok), _ptr(depth), _ptr(position), _ptr(node_seq),
                                      _ptr(anc_mask), _ptr(status))
        _check(rc, "tree_compact_pack")
        return cu, par[:N], tok[:N], depth[:N], position[:N], node_seq[:N], anc_mask[:N], status[:B]

    # -- tree_rope ---------------------------------------------------------
    def tree_rope(self, position, q, k_tree, base=10000.0, rotary_dim=None, pairing=SMART_ROPE_HALF_SPLIT):
        """Rotates q [N, Hq, D] and k_tree [N, Hkv, D] in place by the nodes' position ids."""
        N, Hq, D = q.shape
        Hkv = k_tree.shape[1]
        rc = _lib().tree_rope(self._h, _stream_ptr(), _dtype_code(q), N, Hq, Hkv, D,
                              int(D if rotary_dim is None else rotary_dim), int(pairing), float(base),
                              _ptr(position), _ptr(q), _ptr(k_tree))
        _check(rc, "tree_rope")

    # -- tree_pack ---------------------------------------------------------
    def tree_pack(self, cu_nodes, parent, prefix_len):
        torch = _torch()
        B = cu_nodes.shape[0] - 1
        N = parent.shape[0]
        dev = cu_nodes.device
        depth = torch.empty(N, dtype=torch.int32, device=dev)
        position = torch.empty(N, dtype=torch.int32, device=dev)
        node_seq = torch.empty(N, dtype=torch.int32, device=dev)
        anc_mask = torch.empty((N, 2), dtype=torch.int64, device=dev)
        status = torch.empty(B, dtype=torch.int32, device=dev)
        rc = _lib().tree_pack(self._h, _stream_ptr(), B, N, _ptr(cu_nodes), _ptr(parent),
                              _ptr(prefix_len), _ptr(depth), _ptr(position), _ptr(node_seq),
                              _ptr(anc_mask), _ptr(status))
        _check(rc, "tree_pack")
        return depth, position, node_seq, anc_mask, status

    # -- kv_cache_write ----------------------------------------------------
    def kv_cache_write(self, k_src, v_src, slot_mapping, k_cache, v_cache, layout, block_size,
                       num_blocks, block_stride, head_stride, token_stride=0):
        n, Hkv, D = k_src.shape
        rc = _lib().kv_cache_write(self._h, _stream_ptr(), _dtype_code(k_src), layout, n, Hkv, D,
                                   block_size, num_blocks, _ptr(k_src), _ptr(v_src),
                                   _ptr(slot_mapping), _ptr(k_cache), _ptr(v_cache),
                                   block_stride, head_stride, token_stride)
        _check(rc, "kv_cache_write")

    def kv_cache_write_fp8(self, k_src, v_src, slot_mapping, k_cache, v_cache, layout, block_size,
                           num_blocks, block_stride, head_stride, k_scale, v_scale, token_stride=0):
        """k_cache / v_cache: uint8 tensors (E4M3); strides in elements."""
        n, Hkv, D = k_src.shape
        rc = _lib().kv_cache_write_fp8(self._h, _stream_ptr(), _dtype_code(k_src), layout, n, Hkv, D,
                                       block_size, num_blocks, _ptr(k_src), _ptr(v_src), _ptr(slot_mapping),
                                       _ptr(k_cache), _ptr(v_cache), block_stride, head_stride, token_stride,
                                       float(k_scale), float(v_scale))
        _check(rc, "kv_cache_write_fp8")

    # -- tree_verify_attention ---------------------------------------------
    def tree_verify_attention(self, q, k_tree, v_tree, k_cache, v_cache, block_table, prefix_len,
                              cu_nodes, anc_mask, softmax_scale, kv_layout, block_size=16,
                              out=None, lse=None, want_lse=False, h_cu_nodes=None, k_scale=None, v_scale=None,
                              static=False, status=None):
        """k_cache / v_cache: [num_blocks, Hkv, ...] with one contiguous page of
        block_size * D elements per (block, head) (any of the two layouts).
        ``status``: optional int32 [B] tensor that receives the per-sequence block-table check.
        ``static``: call tree_verify_attention_static (no device allocation inside the library;
        pass ``out`` / ``lse`` so that nothing is allocated here either)."""
        torch = _torch()
        N, Hq, D = q.shape
        Hkv = k_tree.shape[1]
        B = cu_nodes.shape[0] - 1
        if out is None:
            out = torch.empty_like(q)
        if lse is None and want_lse:
            lse = torch.empty((N, Hq), dtype=torch.float32, device=q.device)
        p = TvaParams()
        p.dtype = _dtype_code(q)
        p.kv_layout = kv_layout
        p.batch, p.total_nodes, p.num_q_heads, p.num_kv_heads, p.head_dim = B, N, Hq, Hkv, D
        p.block_size = block_size
        p.max_blocks_per_seq = block_table.shape[1] if block_table is not None else 0
        p.num_blocks = k_cache.shape[0] if k_cache is not None else 0
        p.softmax_scale = float(softmax_scale)
        p.d_q, p.d_k_tree, p.d_v_tree = q.data_ptr(), k_tree.data_ptr(), v_tree.data_ptr()
        if k_cache is not None:
            assert k_cache.stride(0) == v_cache.stride(0) and k_cache.stride(1) == v_cache.stride(1)
            p.d_k_cache, p.d_v_cache = k_cache.data_ptr(), v_cache.data_ptr()
            p.cache_block_stride, p.cache_head_stride = k_cache.stride(0), k_cache.stride(1)
            p.cache_token_stride = k_cache.stride(2) if kv_layout == SMART_KV_PLAIN else D
            p.d_block_table = block_table.data_ptr()
        else:
            p.cache_block_stride = p.cache_head_stride = block_size * D
            p.cache_token_stride = D
        if k_cache is not None and k_cache.dtype == torch.uint8:      # an fp8 (E4M3) cache
            p.kv_cache_dtype = SMART_FP8_E4M3
            p.k_scale, p.v_scale = float(k_scale), float(v_scale)
        p.d_prefix_len, p.d_cu_nodes = prefix_len.data_ptr(), cu_nodes.data_ptr()
        p.d_anc_mask = anc_mask.data_ptr()
        p.d_out = out.data_ptr()
        p.d_lse = lse.data_ptr() if lse is not None else None
        p.d_status = status.data_ptr() if status is not None else None
        if h_cu_nodes is not None:      # numpy int32 [B+1], host copy of cu_nodes
            h_cu_nodes = np.ascontiguousarray(h_cu_nodes, np.int32)
            assert h_cu_nodes.shape[0] == B + 1
            p.h_cu_nodes = h_cu_nodes.ctypes.data
        entry = _lib().tree_verify_attention_static if static else _lib().tree_verify_attention
        _check(entry(self._h, _stream_ptr(), ctypes.byref(p)),
               "tree_verify_attention_static" if static else "tree_verify_attention")
        return (out, lse) if (want_lse or lse is not None) else out

    # -- tree_accept -------------------------------------------------------
    def tree_accept(self, cu_nodes, parent, token, target_next, max_depth):
        torch = _torch()
        B = cu_nodes.shape[0] - 1
        dev = cu_nodes.device
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        accept_path = torch.empty((B, max_depth + 1), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        rc = _lib().tree_accept(self._h, _stream_ptr(), B, max_depth, _ptr(cu_nodes), _ptr(parent),
                                _ptr(token), _ptr(target_next), _ptr(accept_len), _ptr(accept_path),
                                _ptr(bonus))
        _check(rc, "tree_accept")
        return accept_len, accept_path, bonus

    # -- tree_accept_sample ------------------------------------------------
    def tree_accept_sample(self, cu_nodes, parent, token, target_prob, max_depth, seed, step):
        """Temperature-1 verification; target_prob [N, V] float32 (rows may be strided)."""
        torch = _torch()
        B = cu_nodes.shape[0] - 1
        dev = cu_nodes.device
        N, V = target_prob.shape
        assert target_prob.dtype == torch.float32 and target_prob.stride(1) == 1
        accept_len = torch.empty(B, dtype=torch.int32, device=dev)
        accept_path = torch.empty((B, max_depth + 1), dtype=torch.int32, device=dev)
        bonus = torch.empty(B, dtype=torch.int32, device=dev)
        rc = _lib().tree_accept_sample(self._h, _stream_ptr(), B, N, max_depth, V, _ptr(cu_nodes), _ptr(parent),
                                       _ptr(token), _ptr(target_prob), target_prob.stride(0), int(seed), int(step),
                                       _ptr(accept_len), _ptr(accept_path), _ptr(bonus))
        _check(rc, "tree_accept_sample")
        return accept_len, accept_path, bonus

    # -- tree_commit -------------------------------------------------------
    def tree_commit(self, cu_nodes, accept_len, accept_path, k_tree, v_tree, k_cache, v_cache, block_table,
                    prefix_len, layout, block_size, num_blocks, block_stride, head_stride, token_stride=0,
                    k_scale=None, v_scale=None):
        """Appends the accepted path's K/V rows to the paged cache (in place); returns
        (new_prefix_len, status)."""
        torch = _torch()
        B = cu_nodes.shape[0] - 1
        _, Hkv, D = k_tree.shape
        new_len = torch.empty(B, dtype=torch.int32, device=cu_nodes.device)
        status = torch.empty(B, dtype=torch.int32, device=cu_nodes.device)
        args = (self._h, _stream_ptr(), _dtype_code(k_tree), layout, B, accept_path.shape[1] - 1,
                Hkv, D, block_size, block_table.shape[1], num_blocks, _ptr(cu_nodes),
                _ptr(accept_len), _ptr(accept_path), _ptr(k_tree), _ptr(v_tree), _ptr(block_table),
                _ptr(prefix_len), _ptr(k_cache), _ptr(v_cache), block_stride, head_stride,
                token_stride, _ptr(new_len), _ptr(status))
        if k_cache.dtype == torch.uint8:                          # an fp8 (E4M3) cache
            rc = _lib().tree_commit_fp8(*args, float(k_scale), float(v_scale))
        else:
            rc = _lib().tree_commit(*args)
        _check(rc, "tree_commit")
        return new_len, status
