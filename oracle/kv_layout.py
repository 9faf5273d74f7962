"""CPU oracle: element addresses of the interleaved paged KV-cache layout.
TEST INFRASTRUCTURE ONLY.

The paper is silent on cache layout (it never describes verification beyond a
target forward pass).  The library stores a paged cache so that one aligned
group of 8 elements is exactly one matrix-core operand register group:

  K:  [block][kv head][D / 8][block_size][8]
      element (slot, d) of a (block, head) page sits at
      ((d // 8) * block_size + slot) * 8 + d % 8
  V:  [block][kv head][block_size / 8][D][8]
      element (slot, d) sits at
      ((slot // 8) * D + d) * 8 + slot % 8

This file writes those two formulas out element by element (slow loops over
index arrays via numpy fancy indexing) so that the library's cache writer and
layout converter can be checked against something that is not themselves.
"""
from __future__ import annotations

import numpy as np

VEC = 8


def k_offset(slot, d, block_size, head_dim):
    return ((d // VEC) * block_size + slot) * VEC + d % VEC


def v_offset(slot, d, block_size, head_dim):
    return ((slot // VEC) * head_dim + d) * VEC + slot % VEC


def interleave_plain_cache(plain: np.ndarray, which: str) -> np.ndarray:
    """plain [num_blocks, Hkv, block_size, D] -> flat pages [num_blocks, Hkv, block_size*D]
    holding the same elements at the interleaved offsets."""
    nb, Hkv, bs, D = plain.shape
    assert bs % VEC == 0 and D % VEC == 0
    slot, d = np.meshgrid(np.arange(bs), np.arange(D), indexing="ij")
    off = k_offset(slot, d, bs, D) if which == "k" else v_offset(slot, d, bs, D)
    assert sorted(off.ravel().tolist()) == list(range(bs * D))  # a permutation of the page
    out = np.empty((nb, Hkv, bs * D), dtype=plain.dtype)
    out[:, :, off.ravel()] = plain.reshape(nb, Hkv, bs * D)
    return out
