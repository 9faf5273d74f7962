"""Plain CPU oracle for the tree-verification hot path.

TEST INFRASTRUCTURE ONLY.  Written from the paper and from plain definitions,
independent of the HIP library: no shared code, headers, tables or helpers.
Only ``tests/``, ``__graft_entry__.smoke()`` and ``bench.py``'s ``cpu_baseline``
leg may import it.

  attention.py + tree_attention_ref.c   fp64 per-node softmax attention
  selection.py                          SMART marginal rule, both schedules,
                                        brute-force optimum on tiny forests
  pack_accept.py                        depth / position / ancestor masks,
                                        greedy accept walk
  kv_layout.py                          where an element of the paged cache
                                        lives in the interleaved layout
"""
