"""Seeded synthetic workloads (inputs only).

This module is the one piece shared by the CPU oracle's tests and the HIP
library's tests and benchmark.  It holds none of the method's arithmetic: it
draws random draft distributions, queries, keys, values, block tables and
target tokens with the shapes of the evaluated workloads, and tabulates the
cost functions the workloads name.  Tree selection, packing, attention and
acceptance are computed elsewhere (by the library, or by the oracle).

Everything is numpy on the host; bf16 tensors are carried as uint16 bit
patterns (round-to-nearest-even from float32).
"""
from __future__ import annotations

from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field, replace
from typing import Callable, Optional

import numpy as np

BLOCK_SIZE = 16
BF16_NAN = 0x7FC0
VOCAB = 32000


# --------------------------------------------------------------------------
# workload table
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    dtype: str                 # "f32" | "bf16"
    batch: int
    num_q_heads: int
    num_kv_heads: int
    head_dim: int
    prefix_min: int            # prefix length is uniform in [prefix_min, prefix_max]
    prefix_max: int
    image_prefix: int = 0      # first tokens whose K/V come from N(0, 1.5^2)
    qkv_scale: float = 1.0     # elements = N(0,1) * qkv_scale
    tree: str = "rule"         # "binary3" | "rule" | "topn"
    top_k: int = 8             # children drawn per expanded node
    max_depth: int = 8
    budget: int = 128          # per-sequence node budget B (root included)
    alpha: float = 0.8
    topn_min: int = 0          # "topn": n_b uniform in [topn_min, topn_max]
    topn_max: int = 0
    cost_name: str = ""
    seed: int = 0

    @property
    def group(self) -> int:
        return self.num_q_heads // self.num_kv_heads

    def scaled(self, name=None, **kw) -> "Workload":
        return replace(self, name=name or (self.name + "_small"), **kw)


def _cost_cfg2(n):   # c(n) = 1 + 0.004 n
    return 1.0 + 0.004 * n


def _knee(N, a, b, knee):  # c(N) = 1 + a N + b max(0, N - knee) / 64
    return 1.0 + a * N + b * max(0.0, N - knee) / 64.0


_COSTS: dict[str, Callable[[int, int], float]] = {
    # cost of a verify step when every one of `batch` sequences carries n nodes
    "cfg2": lambda n, batch: _cost_cfg2(n),
    "cfg3": lambda n, batch: _knee(batch * n, 0.002, 0.02, 512.0),
    "cfg4": lambda n, batch: 1.0 + 0.003 * n,
    "cfg5": lambda n, batch: _knee(batch * n, 0.001, 0.05, 1024.0),
    "flat": lambda n, batch: 1.0 + 1e-9 * n,
}


def cost_table(w: Workload, n_max: Optional[int] = None, name: Optional[str] = None) -> np.ndarray:
    """cost[n] for n = 0 .. n_max + 1 (n counts the root).  For the workloads
    whose cost function takes the batch-wide token count, every sequence
    assumes the batch is split evenly: cost[n] = c(batch * n)."""
    n_max = w.budget if n_max is None else n_max
    f = _COSTS[name or w.cost_name]
    return np.array([f(n, w.batch) for n in range(n_max + 2)], dtype=np.float64)


WORKLOADS: dict[str, Workload] = {}


def _reg(w: Workload):
    WORKLOADS[w.name] = w


_reg(Workload("cfg1", "f32", 1, 8, 2, 64, 128, 128, qkv_scale=0.125, tree="binary3", seed=1001))
_reg(Workload("cfg1_sharp", "f32", 1, 8, 2, 64, 128, 128, qkv_scale=1.0, tree="binary3", seed=1011))
_reg(Workload("cfg2", "bf16", 4, 32, 8, 128, 2048, 2048, tree="rule", top_k=8, max_depth=8,
              budget=128, cost_name="cfg2", seed=1002))
_reg(Workload("cfg3a", "bf16", 32, 32, 8, 128, 3072, 4096, tree="rule", top_k=8, max_depth=8,
              budget=64, cost_name="cfg3", seed=1003))
_reg(Workload("cfg3b", "bf16", 32, 32, 8, 128, 3072, 4096, tree="topn", top_k=8, max_depth=8,
              budget=64, topn_min=4, topn_max=64, cost_name="flat", seed=1003))
_reg(Workload("cfg4", "bf16", 12, 28, 4, 128, 8192, 8192, image_prefix=1024, tree="rule",
              top_k=4, max_depth=6, budget=96, cost_name="cfg4", seed=1004))
_reg(Workload("cfg5a", "bf16", 64, 64, 8, 128, 16384, 16384, tree="rule", top_k=8, max_depth=8,
              budget=48, cost_name="cfg5", seed=1005))
_reg(Workload("cfg5b", "bf16", 64, 64, 8, 128, 16384, 16384, tree="topn", top_k=8, max_depth=8,
              budget=48, topn_min=1, topn_max=48, cost_name="flat", seed=1005))


# --------------------------------------------------------------------------
# random streams
# --------------------------------------------------------------------------
def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[seed, stream]))


def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round-to-nearest-even float32 -> bfloat16 bit patterns (finite inputs)."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def _normal(seed: int, stream: int, shape, scale: float, dtype: str) -> np.ndarray:
    """N(0, scale^2) tensor in the workload's element type, filled in parallel
    from independent Philox streams (fixed chunking, so it is reproducible)."""
    n = int(np.prod(shape))
    out = np.empty(n, dtype=np.float32 if dtype == "f32" else np.uint16)
    chunk = 1 << 22
    n_chunks = (n + chunk - 1) // chunk

    def fill(c):
        g = np.random.Generator(np.random.Philox(key=[seed, stream], counter=[0, 0, c, 0]))
        lo, hi = c * chunk, min(n, (c + 1) * chunk)
        x = g.standard_normal(hi - lo, dtype=np.float32)
        if scale != 1.0:
            x *= np.float32(scale)
        out[lo:hi] = x if dtype == "f32" else f32_to_bf16_bits(x)

    if n_chunks <= 1:
        for c in range(n_chunks):
            fill(c)
    else:
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(fill, range(n_chunks)))
    return out.reshape(shape)


# --------------------------------------------------------------------------
# candidate forests (draft distributions)
# --------------------------------------------------------------------------
@dataclass
class Forest:
    cand_cu: np.ndarray       # [B+1] int32
    cand_parent: np.ndarray   # [C] int32, local, -1 = root
    cand_prob: np.ndarray     # [C] float64 conditional draft probability (root 1.0)
    cand_token: np.ndarray    # [C] int32


def make_forest(w: Workload, seed: Optional[int] = None, floor: float = 1e-3,
                sigma: float = 2.0) -> Forest:
    """Per sequence: a root, then for every node above the materialisation
    floor and shallower than max_depth, top_k children whose conditional
    probabilities are softmax(N(0, sigma^2) logits), sorted descending, with
    distinct tokens.  Children whose running product of probabilities falls
    under `floor` are not materialised (the floor only bounds the input size;
    it lies below every threshold the selection rule can produce here).
    Candidates are in breadth-first order, so parents precede children."""
    seed = w.seed if seed is None else seed
    cu = [0]
    parent, prob, token = [], [], []
    for b in range(w.batch):
        g = _rng(seed, 100 + b)
        lp = [-1]
        pp = [1.0]
        tk = [int(g.integers(VOCAB))]
        cum = [1.0]
        dep = [0]
        i = 0
        while i < len(lp):
            if dep[i] < w.max_depth:
                logits = g.normal(0.0, sigma, w.top_k)
                e = np.exp(logits - logits.max())
                p = np.sort(e / e.sum())[::-1]
                toks = g.choice(VOCAB, size=w.top_k, replace=False)
                for j in range(w.top_k):
                    c = cum[i] * float(p[j])
                    if c >= floor:
                        lp.append(i)
                        pp.append(float(p[j]))
                        tk.append(int(toks[j]))
                        cum.append(c)
                        dep.append(dep[i] + 1)
            i += 1
        parent += lp
        prob += pp
        token += tk
        cu.append(len(parent))
    return Forest(np.array(cu, np.int32), np.array(parent, np.int32),
                  np.array(prob, np.float64), np.array(token, np.int32))


def topn_budgets(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    """Per-sequence node counts of the range-filling stand-in workloads."""
    seed = w.seed if seed is None else seed
    return _rng(seed, 7).integers(w.topn_min, w.topn_max + 1, size=w.batch).astype(np.int32)


BINARY3_PARENT = np.array([-1, 0, 0, 1, 1, 2, 2, 3, 3, 4, 4, 5, 5, 6, 6], np.int32)


def fixed_tree(w: Workload):
    """cu_nodes, parent, token for the workloads with a prescribed tree."""
    assert w.tree == "binary3"
    n = len(BINARY3_PARENT)
    cu = np.arange(w.batch + 1, dtype=np.int32) * n
    parent = np.tile(BINARY3_PARENT, w.batch)
    token = _rng(w.seed, 8).integers(VOCAB, size=w.batch * n).astype(np.int32)
    return cu, parent, token


def random_tree(n: int, rng: np.random.Generator, shape: str = "random") -> np.ndarray:
    """A parent array in topological order: 'random' (uniform random parent
    among earlier nodes), 'chain', or 'star'."""
    parent = np.full(n, -1, np.int32)
    for i in range(1, n):
        if shape == "chain":
            parent[i] = i - 1
        elif shape == "star":
            parent[i] = 0
        else:
            parent[i] = int(rng.integers(0, i))
    return parent


# --------------------------------------------------------------------------
# attention inputs
# --------------------------------------------------------------------------
@dataclass
class AttentionInputs:
    dtype: str
    q: np.ndarray             # [N, Hq, D]
    k_tree: np.ndarray        # [N, Hkv, D]
    v_tree: np.ndarray        # [N, Hkv, D]
    k_cache: np.ndarray       # [num_blocks, Hkv, 16, D]  plain layout
    v_cache: np.ndarray       # [num_blocks, Hkv, 16, D]  plain layout
    block_table: np.ndarray   # [B, max_blocks] int32, unused entries = -1
    prefix_len: np.ndarray    # [B] int32
    cu_nodes: np.ndarray      # [B+1] int32
    scale: float
    meta: dict = field(default_factory=dict)


def make_prefix_len(w: Workload, seed: Optional[int] = None) -> np.ndarray:
    seed = w.seed if seed is None else seed
    return _rng(seed, 1).integers(w.prefix_min, w.prefix_max + 1, size=w.batch).astype(np.int32)


def make_attention_inputs(w: Workload, cu_nodes: np.ndarray, seed: Optional[int] = None,
                          prefix_len: Optional[np.ndarray] = None, spare_blocks: int = 3,
                          poison_unused: bool = True) -> AttentionInputs:
    """Q, tree K/V, a block-permuted paged cache and its block table.

    Slots of a sequence's last block past its prefix, and the spare blocks no
    sequence owns, are filled with NaN: nothing may ever read them."""
    seed = w.seed if seed is None else seed
    N = int(cu_nodes[-1])
    Hq, Hkv, D = w.num_q_heads, w.num_kv_heads, w.head_dim
    if prefix_len is None:
        prefix_len = make_prefix_len(w, seed)
    prefix_len = np.asarray(prefix_len, np.int32)
    blocks_per_seq = (prefix_len + BLOCK_SIZE - 1) // BLOCK_SIZE
    max_blocks = max(1, int(blocks_per_seq.max()) if len(blocks_per_seq) else 1)
    used = int(blocks_per_seq.sum())
    nb = used + spare_blocks

    q = _normal(seed, 2, (N, Hq, D), w.qkv_scale, w.dtype)
    k_tree = _normal(seed, 3, (N, Hkv, D), w.qkv_scale, w.dtype)
    v_tree = _normal(seed, 4, (N, Hkv, D), w.qkv_scale, w.dtype)
    k_cache = _normal(seed, 5, (nb, Hkv, BLOCK_SIZE, D), w.qkv_scale, w.dtype)
    v_cache = _normal(seed, 6, (nb, Hkv, BLOCK_SIZE, D), w.qkv_scale, w.dtype)

    perm = _rng(seed, 9).permutation(nb).astype(np.int32)
    block_table = np.full((w.batch, max_blocks), -1, np.int32)
    nan = np.float32(np.nan) if w.dtype == "f32" else np.uint16(BF16_NAN)
    pos = 0
    for b in range(w.batch):
        nblk = int(blocks_per_seq[b])
        phys = perm[pos:pos + nblk]
        block_table[b, :nblk] = phys
        pos += nblk
        if w.image_prefix > 0:
            # image-patch keys/values: a wider distribution on the leading tokens
            n_img_blocks = min(nblk, w.image_prefix // BLOCK_SIZE)
            for cache, stream in ((k_cache, 15), (v_cache, 16)):
                img = _normal(seed, stream * 1000 + b, (n_img_blocks, Hkv, BLOCK_SIZE, D),
                              1.5 * w.qkv_scale, w.dtype)
                cache[phys[:n_img_blocks]] = img
        tail = int(prefix_len[b]) % BLOCK_SIZE
        if poison_unused and nblk > 0 and tail != 0:
            k_cache[phys[-1], :, tail:, :] = nan
            v_cache[phys[-1], :, tail:, :] = nan
    if poison_unused:
        k_cache[perm[pos:]] = nan
        v_cache[perm[pos:]] = nan
    return AttentionInputs(w.dtype, q, k_tree, v_tree, k_cache, v_cache, block_table,
                           prefix_len, np.asarray(cu_nodes, np.int32),
                           1.0 / float(np.sqrt(D)),
                           {"num_blocks": nb, "max_blocks": max_blocks})


# --------------------------------------------------------------------------
# target tokens for the accept walk
# --------------------------------------------------------------------------
def make_target_next(forest: Forest, cu_nodes, cand_index, seed: int) -> np.ndarray:
    """For every selected node, the token the target model would emit next:
    one of that node's candidate children, drawn with the child's conditional
    draft probability (the workloads equate acceptance and draft probability),
    otherwise a token no child carries."""
    N = int(cu_nodes[-1])
    out = np.empty(N, np.int32)
    g = _rng(seed, 11)
    for b in range(len(cu_nodes) - 1):
        lo, hi = int(forest.cand_cu[b]), int(forest.cand_cu[b + 1])
        par = forest.cand_parent[lo:hi]
        kids: dict[int, list[int]] = {}
        for u in range(1, hi - lo):
            kids.setdefault(int(par[u]), []).append(u)
        for i in range(int(cu_nodes[b]), int(cu_nodes[b + 1])):
            c = int(cand_index[i])
            r = float(g.random())
            tok = VOCAB + 1  # never drafted
            acc = 0.0
            for u in kids.get(c, []):
                acc += float(forest.cand_prob[lo + u])
                if r < acc:
                    tok = int(forest.cand_token[lo + u])
                    break
            out[i] = tok
    return out


def algorithmic_work(w: Workload, prefix_len, cu_nodes, depth_plus_one_sum: int) -> dict:
    """Bytes that must cross HBM and flops that must be done in one verify step:
    every prefix K/V byte once per (sequence, kv head); Q, tree K/V and the
    output once; 4*D flops per (query row, attended key)."""
    e = 4 if w.dtype == "f32" else 2
    Hq, Hkv, D = w.num_q_heads, w.num_kv_heads, w.head_dim
    N = int(cu_nodes[-1])
    n = np.diff(np.asarray(cu_nodes)).astype(np.int64)
    L = np.asarray(prefix_len).astype(np.int64)
    kv_bytes = int(L.sum()) * Hkv * D * 2 * e
    io_bytes = N * (2 * Hkv + 2 * Hq) * D * e
    attended = int((n * L).sum()) + int(depth_plus_one_sum)
    return {"kv_bytes": kv_bytes, "io_bytes": io_bytes, "bytes": kv_bytes + io_bytes,
            "attended_tokens": attended, "flops": 4 * D * Hq * attended}
