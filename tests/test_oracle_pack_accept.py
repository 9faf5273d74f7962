"""Pins for the pack and accept oracles (CPU only): cross-checks against
independent statements of the same results (ancestor walk, path enumeration)."""
import numpy as np
import pytest

from oracle import pack_accept as PA
from paper_2604_09731_amd import workloads as W


def _trees(seed, sizes, shapes=None):
    rng = np.random.default_rng(seed)
    ts = [W.random_tree(n, rng, (shapes or ["random"] * len(sizes))[i]) for i, n in enumerate(sizes)]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    return cu, np.concatenate(ts).astype(np.int32), rng


def test_pack_masks_depths_positions():
    cu, parent, rng = _trees(1, [1, 15, 64, 65, 128, 7], ["random", "random", "chain", "random", "random", "star"])
    plen = rng.integers(0, 5000, size=len(cu) - 1).astype(np.int32)
    depth, pos, seq, mask = PA.pack(cu, parent, plen)
    for b in range(len(cu) - 1):
        base = cu[b]
        for i in range(cu[b + 1] - base):
            anc, j = set(), i
            while j >= 0:
                anc.add(j)
                j = int(parent[base + j])
            full = mask[base + i][0] | (mask[base + i][1] << 64)
            assert {x for x in range(128) if (full >> x) & 1} == anc
            assert bin(full).count("1") == depth[base + i] + 1 == len(anc)
            assert full >> (i + 1) == 0                     # only bits <= i
            assert pos[base + i] == plen[b] + depth[base + i]
            assert seq[base + i] == b
    # chain: depth = index; star: depth 1
    assert depth[cu[2]:cu[3]] == list(range(64))
    assert depth[cu[5] + 1:cu[6]] == [1] * 6


def test_pack_rejects_malformed_trees():
    with pytest.raises(ValueError):
        PA.pack([0, 3], [-1, 0, 2], [5])
    with pytest.raises(ValueError):
        PA.pack([0, 2], [0, 0], [5])
    with pytest.raises(ValueError):
        PA.pack([0, 129], [-1] + list(range(128)), [5])


@pytest.mark.parametrize("seed", range(8))
def test_accept_walk_equals_longest_matched_path(seed):
    sizes = [1, 5, 12, 30, 64]
    cu, parent, rng = _trees(seed, sizes)
    N = cu[-1]
    token = rng.integers(0, 6, size=N).astype(np.int32)       # few tokens: duplicates among siblings
    target = rng.integers(0, 6, size=N).astype(np.int32)
    # make long matches likely: copy some child's token into the parent's target
    for b in range(len(sizes)):
        for i in range(1, sizes[b]):
            if rng.random() < 0.6:
                target[cu[b] + parent[cu[b] + i]] = token[cu[b] + i]
    D = 64
    alen, paths, bonus = PA.accept(cu, parent, token, target, D)
    lens2, ends2 = PA.accept_by_path_enumeration(cu, parent, token, target, D)
    assert alen == lens2
    for b in range(len(sizes)):
        p = [v for v in paths[b] if v >= 0]
        assert p[0] == 0 and len(p) == alen[b] + 1
        assert p[-1] == ends2[b]
        for a, c in zip(p[:-1], p[1:]):
            assert parent[cu[b] + c] == a
            assert token[cu[b] + c] == target[cu[b] + a]      # only target-chosen tokens are emitted
        assert bonus[b] == target[cu[b] + p[-1]]
        # nothing further could have been accepted
        last = p[-1]
        assert not any(parent[cu[b] + j] == last and token[cu[b] + j] == target[cu[b] + last]
                       for j in range(sizes[b]))


def test_accept_degenerate_cases():
    cu, parent, _ = _trees(3, [6, 4], ["chain", "star"])
    token = np.array([9, 1, 2, 3, 4, 5, 9, 7, 7, 8], np.int32)
    # all mismatch
    alen, paths, bonus = PA.accept(cu, parent, token, np.full(10, 99, np.int32), 8)
    assert alen == [0, 0] and bonus == [99, 99] and paths[0][:2] == [0, -1]
    # full chain accepted, depth cap truncates
    target = np.array([1, 2, 3, 4, 5, 42, 7, 0, 0, 0], np.int32)
    alen, paths, bonus = PA.accept(cu, parent, token, target, 8)
    assert alen == [5, 1] and bonus[0] == 42 and paths[1][:2] == [0, 1]   # smallest sibling wins the tie
    alen, _, bonus = PA.accept(cu, parent, token, target, 3)
    assert alen[0] == 3 and bonus[0] == 4
