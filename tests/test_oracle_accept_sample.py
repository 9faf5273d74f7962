"""Pins for the temperature-1 verification oracle (CPU only)."""
from fractions import Fraction as F

import numpy as np
import pytest

from oracle import accept_sample as A
from oracle import pack_accept as PA


def test_philox_known_answers():
    """Known-answer vectors published with the generator (Random123's kat_vectors)."""
    assert A.philox4x32_10((0, 0, 0, 0), (0, 0)) == (0x6627e8d5, 0xe169c58d, 0xbc57ac4c, 0x9b00dbd8)
    f = 0xffffffff
    assert A.philox4x32_10((f, f, f, f), (f, f)) == (0x408f276d, 0x41c83b0e, 0xa20bc7c6, 0x6d5451fd)
    assert A.philox4x32_10((0x243f6a88, 0x85a308d3, 0x13198a2e, 0x03707344), (0xa4093822, 0x299f31d0)) == \
        (0xd16cfe09, 0x94fdcceb, 0x5001e420, 0x24126ea1)


def test_weights_are_exact_fixed_point():
    w = A.weights(np.array([0.5, 0.25, 2.0 ** -32, 2.0 ** -33, 0.0, -1.0, float("nan"), 1.0, 3.0], np.float32))
    assert w == [1 << 31, 1 << 30, 1, 0, 0, 0, 0, 1 << 32, 1 << 32]


def _grid_draws(values):
    """Every combination of the given 64-bit draws for the first len(values) draws of sequence 0."""
    import itertools
    return itertools.product(*values)


def test_emitted_token_is_distributed_exactly_as_the_target():
    """Integrate over the random numbers.  Draw i decides the i-th test of the step, so a grid of
    mid-points per draw whose spacing divides every threshold that draw can meet integrates exactly:
    the fraction of grid points that emit token x as the FIRST token of the step -- an accepted child
    of the root, or the bonus when all are rejected -- must be exactly p(x)."""
    V = 6
    p_root = np.array([4, 2, 1, 6, 0, 3], np.float64) / 16.0          # exact in binary32
    prob = np.tile(p_root, (4, 1)).astype(np.float32)
    cu, parent, token = [0, 4], [-1, 0, 0, 0], [9, 3, 0, 5]           # children propose tokens 3, 0, 5
    # thresholds: draw 0 at 6/16 (token 3 of mass 16/16); draw 1 at 4/10 (token 0 of what is left, 10/16);
    # draw 2 at 3/6 (token 5 of 6/16); draw 3, the bonus among tokens 1, 2 (3/16 left), at 2/3
    grids = [[((2 * k + 1) << 64) // (2 * G) for k in range(G)] for G in (16, 10, 2, 3)]
    counts = [F(0)] * V
    for r0 in grids[0]:
        for r1 in grids[1]:
            for r2 in grids[2]:
                for r3 in grids[3]:
                    seq = [r0, r1, r2, r3]
                    # a step that accepts early draws its bonus with the next index: any value will do there
                    al, path, bonus = A.accept_sample(cu, parent, token, prob, 0, 0, 1, draws=lambda b, i: seq[i])
                    first = token[path[0][1]] if al[0] >= 1 else bonus[0]
                    counts[first] += 1
    total = sum(counts)
    assert [c / total for c in counts] == [F(int(x), 16) for x in p_root * 16]


def test_statistics_with_the_generator_itself():
    """The same property through Philox: 20000 steps, chi-square against the target."""
    rng = np.random.default_rng(0)
    V = 12
    p = rng.dirichlet(np.ones(V)).astype(np.float32)
    prob = np.tile(p, (3, 1))
    cu, parent, token = [0, 3], [-1, 0, 0], [0, int(np.argmax(p)), int(np.argmin(p))]
    hist = np.zeros(V)
    n = 20000
    for step in range(n):
        al, path, bonus = A.accept_sample(cu, parent, token, prob, 1234, step, 1)
        hist[token[path[0][1]] if al[0] else bonus[0]] += 1
    w = np.array(A.weights(p), np.float64)
    expect = w / w.sum() * n
    chi2 = float(((hist - expect) ** 2 / expect).sum())
    assert chi2 < 40.0, chi2                        # 11 degrees of freedom: P(chi2 > 40) < 4e-5


def test_point_mass_target_reduces_to_the_greedy_walk():
    """If the target puts all its mass on one token after every node, sampling and the greedy walk agree
    (accept_len, path and bonus), whatever the random numbers."""
    rng = np.random.default_rng(3)
    from paper_2604_09731_amd import workloads as W
    sizes = [1, 7, 30, 64]
    trees = [W.random_tree(n, rng, "random") for n in sizes]
    cu = np.concatenate([[0], np.cumsum(sizes)]).astype(np.int32)
    parent = np.concatenate(trees).astype(np.int32)
    N, V = int(cu[-1]), 5
    token = rng.integers(0, V, N).astype(np.int32)
    target_next = rng.integers(0, V, N).astype(np.int32)
    prob = np.zeros((N, V), np.float32)
    prob[np.arange(N), target_next] = 1.0
    for seed in range(3):
        al, path, bonus = A.accept_sample(cu, parent, token, prob, seed, 7, 6)
        gl, gpath, gbonus = PA.accept(cu, parent, token, target_next, 6)
        assert al == gl and path == gpath and bonus == gbonus


def test_depth_cap_duplicates_and_empty_mass():
    prob = np.zeros((4, 4), np.float32)
    prob[:, 1] = 1.0
    # chain 0 -> 1 -> 2 -> 3, all proposing token 1: accepted until the cap
    al, path, bonus = A.accept_sample([0, 4], [-1, 0, 1, 2], [0, 1, 1, 1], prob, 0, 0, 2)
    assert al == [2] and path == [[0, 1, 2]] and bonus == [1]
    # two siblings with the same token: the second one's mass is already gone, it is never drawn for
    prob2 = np.array([[0.5, 0.5, 0, 0]] * 3, np.float32)
    seen = set()
    for step in range(64):
        al, path, bonus = A.accept_sample([0, 3], [-1, 0, 0], [0, 1, 1], prob2, 5, step, 4)
        seen.add((al[0], tuple(path[0][:2]), bonus[0]))
        assert path[0][1] in (-1, 1)                                  # node 2 can never be accepted
        if al[0] == 0:
            assert bonus[0] == 0                                      # token 1 was rejected: only token 0 is left
    assert len(seen) >= 2
    # no mass at all: nothing is accepted, no bonus
    al, path, bonus = A.accept_sample([0, 2], [-1, 0], [0, 1], np.zeros((2, 4), np.float32), 0, 0, 4)
    assert al == [0] and bonus == [-1]
