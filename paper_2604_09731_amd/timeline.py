"""Timeline of one tree_verify_attention call, from wall-clock stamps inside its two kernels.

    python -m paper_2604_09731_amd.timeline cfg3a [cfg3b ...] [--reps 20] [--kv fp8]

Loads the timeline build of the library (libsmart_tree_timeline.so: the same sources with
-DSMART_TVA_TIMELINE, built beside the ordinary one by `python -m paper_2604_09731_amd.build`), runs the
attention call of a named workload on synthetic inputs of its shape (trees selected by the library, as in
bench.py) and prints, averaged over `--reps` launches after warm-up:

  * per class of the prefix kernel: workgroups, and the time each took (start of the workgroup to the end of its
    last wavefront), in us;
  * per XCD (workgroup index mod 8): mean time and shader clock (cycles / wall time);
  * when the kernel's first workgroup starts, its last one ends, and how far apart the ends are;
  * for the combine kernel: when its wavefronts start and end relative to the prefix kernel's last end, and how
    long a wavefront lives.

The stamps cost a few hundred nanoseconds per workgroup; the figures are for reading the structure of a launch,
the durations quoted elsewhere come from rocprofv3 on the ordinary library.
"""
from __future__ import annotations

import argparse
import ctypes
import os
import sys

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
TIMELINE_LIB = os.path.join(_HERE, "libsmart_tree_timeline.so")
TICKS_PER_US = 100.0          # the wall-clock counter runs at 100 MHz
WG_SLOTS, WAVE_SLOTS = 1024, 16384


def _select_trees(B, W, w):
    """The workload's trees, selected by the library (rule, per-sequence budgets or the fixed tree)."""
    if w.tree == "binary3":
        cu, parent, _ = W.fixed_tree(w)
        return np.asarray(cu, np.int32), np.asarray(parent, np.int32)
    forest = W.make_forest(w)
    cost = W.cost_table(w)
    kw = dict(alpha=w.alpha, max_depth=w.max_depth)
    if w.tree == "rule":
        r = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost,
                                budget=w.budget, **kw)
    else:
        budgets = W.topn_budgets(w)
        r = B.smart_select_tree(forest.cand_cu, forest.cand_parent, forest.cand_prob, forest.cand_token, cost,
                                budget=int(budgets.max()), budgets=budgets, **kw)
    return r["cu_nodes"], r["parent"]


def run(workload: str, reps: int, kv: str) -> None:
    import torch
    from . import binding as B
    from . import workloads as W

    L = B._lib()
    L.smart_timeline_read.argtypes = [ctypes.c_void_p, ctypes.c_void_p]
    L.smart_timeline_read.restype = ctypes.c_int32
    L.smart_timeline_clear.restype = ctypes.c_int32
    w = W.WORKLOADS[workload]
    lib = B.SmartTree(0)
    dev = "cuda:0"
    cu, parent = _select_trees(B, W, w)
    inp = W.make_attention_inputs(w, cu)

    def elems(x):
        t = torch.from_numpy(np.ascontiguousarray(x))
        if w.dtype == "bf16":
            t = t.view(torch.int16).view(torch.bfloat16)
        return t.to(dev)

    q, k_tree, v_tree = elems(inp.q), elems(inp.k_tree), elems(inp.v_tree)
    kc, vc = B.interleave_kv_cache(elems(inp.k_cache), elems(inp.v_cache))
    scales = {}
    if kv == "fp8":
        nb, Hkv, bs, D = inp.k_cache.shape
        rows = lambda x: elems(np.ascontiguousarray(x.transpose(0, 2, 1, 3)).reshape(nb * bs, Hkv, D))
        kc8 = torch.zeros((nb, Hkv, D // 8, bs, 8), dtype=torch.uint8, device=dev)
        vc8 = torch.zeros((nb, Hkv, bs // 8, D, 8), dtype=torch.uint8, device=dev)
        lib.kv_cache_write_fp8(rows(inp.k_cache), rows(inp.v_cache), torch.arange(nb * bs, device=dev), kc8, vc8,
                               B.SMART_KV_INTERLEAVED, bs, nb, Hkv * bs * D, bs * D, 2.0 ** -5, 2.0 ** -5)
        kc, vc = kc8, vc8
        scales = dict(k_scale=2.0 ** -5, v_scale=2.0 ** -5)
    # two copies of the cache used in turn, so that a small cache is not served by the last-level cache
    caches = [(kc, vc), (kc.clone(), vc.clone())]
    d_cu, d_par, d_len = (torch.from_numpy(np.ascontiguousarray(x)).to(dev) for x in (cu, parent, inp.prefix_len))
    bt = torch.from_numpy(inp.block_table).to(dev)
    _, _, _, mask, _ = lib.tree_pack(d_cu, d_par, d_len)

    def call(i):
        k, v = caches[i & 1]
        lib.tree_verify_attention(q, k_tree, v_tree, k, v, bt, d_len, d_cu, mask, inp.scale, B.SMART_KV_INTERLEAVED,
                                  **scales)

    for i in range(6):
        call(i)
    torch.cuda.synchronize()
    wg_buf = np.zeros(WG_SLOTS * 4, np.uint64)
    wave_buf = np.zeros(WAVE_SLOTS * 2, np.uint64)
    wg_runs, wave_runs = [], []
    for i in range(reps):
        if L.smart_timeline_clear():
            raise RuntimeError("smart_timeline_clear failed")
        call(i)
        if L.smart_timeline_read(wg_buf.ctypes.data, wave_buf.ctypes.data):
            raise RuntimeError("smart_timeline_read failed")
        wg_runs.append(wg_buf.reshape(-1, 4).copy())
        wave_runs.append(wave_buf.reshape(-1, 2).copy())

    sizes = np.diff(cu)
    print(f"== {workload} ({kv} cache): batch {w.batch}, {int(cu[-1])} tree nodes ({sizes.min()}-{sizes.max()} per sequence), "
          f"prefix {inp.prefix_len.min()}..{inp.prefix_len.max()}, {reps} launches")
    # ---- prefix kernel ----
    used = (wg_runs[0][:, 3] >> np.uint64(63)) == 1
    idx = np.nonzero(used)[0]
    cls = (wg_runs[0][used, 3] & np.uint64(0xFF)).astype(int)
    start = np.stack([r[used, 0].astype(np.float64) for r in wg_runs])
    end = np.stack([r[used, 1].astype(np.float64) for r in wg_runs])
    cyc = np.stack([r[used, 2].astype(np.float64) for r in wg_runs])
    t0 = start.min(axis=1, keepdims=True)
    dur = ((end - start) / TICKS_PER_US).mean(axis=0)
    ghz = (cyc / (end - start) * TICKS_PER_US * 1e-3).mean(axis=0)
    print(f"prefix kernel: {used.sum()} workgroups; first start 0, last start "
          f"{((start - t0).max(axis=1) / TICKS_PER_US).mean():.2f} us, ends {((end - t0).min(axis=1) / TICKS_PER_US).mean():.1f} .. "
          f"{((end - t0).max(axis=1) / TICKS_PER_US).mean():.1f} us")
    for c in range(3):
        v = np.sort(dur[cls == c])
        if len(v):
            print(f"  class {c}: {len(v):3d} workgroups, time per workgroup min {v[0]:.1f}  median {v[len(v) // 2]:.1f}  "
                  f"mean {v.mean():.1f}  max {v[-1]:.1f} us")
    print("  per XCD (workgroup index mod 8), mean time us / shader clock GHz: " +
          "  ".join(f"{x}: {dur[idx % 8 == x].mean():.1f} / {ghz[idx % 8 == x].mean():.2f}" for x in range(8)
                    if (idx % 8 == x).any()))
    # ---- combine kernel ----
    ran = wave_runs[0][:, 1] > 0
    if ran.any():
        last_end = end.max(axis=1, keepdims=True)
        ws = np.stack([r[ran, 0].astype(np.float64) for r in wave_runs]) - last_end
        we = np.stack([r[ran, 1].astype(np.float64) for r in wave_runs]) - last_end
        s_us, e_us = ws / TICKS_PER_US, we / TICKS_PER_US
        life = (e_us - s_us)
        note = "" if ran.sum() < WAVE_SLOTS else f" (the first {WAVE_SLOTS} only)"
        print(f"combine kernel: {ran.sum()} wavefronts{note}; after the prefix kernel's last end: starts "
              f"{s_us.min(axis=1).mean():.2f} .. {s_us.max(axis=1).mean():.2f} us (median {np.median(s_us, axis=1).mean():.2f}), "
              f"ends {e_us.min(axis=1).mean():.2f} .. {e_us.max(axis=1).mean():.2f} us; a wavefront lives "
              f"{life.mean():.2f} us on average, {life.max(axis=1).mean():.2f} at most")


def main(argv=None) -> int:
    ap = argparse.ArgumentParser(description=__doc__.split("\n\n")[0])
    ap.add_argument("workloads", nargs="+")
    ap.add_argument("--reps", type=int, default=20)
    ap.add_argument("--kv", choices=["bf16", "fp8"], default="bf16")
    args = ap.parse_args(argv)
    if not os.path.exists(TIMELINE_LIB):
        sys.exit(f"{TIMELINE_LIB} is missing: build it with `python -m paper_2604_09731_amd.build`")
    # the binding loads whatever SMART_TREE_LIB names, once per process: set it before the binding is imported
    os.environ["SMART_TREE_LIB"] = TIMELINE_LIB
    if "paper_2604_09731_amd.binding" in sys.modules:
        sys.exit("the library binding is already loaded in this process: run this module on its own")
    for wl in args.workloads:
        run(wl, args.reps, args.kv)
    return 0


if __name__ == "__main__":
    sys.exit(main())
