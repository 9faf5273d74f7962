"""CPU oracle: temperature-1 (sampling) verification of a draft tree.  TEST INFRASTRUCTURE ONLY.

The paper evaluates at temperatures 0 and 1, as the work it builds on does, and relies on verification
being lossless (Sec. 4, evaluation paragraph); the tree-based drafters it builds on propose a
node's children deterministically (the draft model's top-k tokens), and for deterministic
proposals the lossless rule is:

    at node `cur` with target distribution p over the vocabulary, visit its children in node
    order; child c with token x is accepted with probability p(x) / (mass not yet rejected at
    this node); on rejection x's mass is removed; if every child is rejected (or there is
    none) the step ends and the bonus token is drawn from what is left of p.

    (P(first child accepted) = p(x1); P(second) = (1 - p(x1)) p(x2) / (1 - p(x1)) = p(x2); ...;
    so the emitted token is distributed exactly as p.)

To make every decision independent of floating-point summation order, probabilities are turned
into integer weights once, w(x) = floor(p(x) * 2^32) (exact in binary64 for binary32 inputs;
NaN and negatives count as 0, values above 1 as 1), and all further arithmetic is on integers:
with a uniform 64-bit draw r and remaining weight R, mulhi(r, R) = floor(r R / 2^64) is uniform
on [0, R); child x is accepted iff mulhi(r, R) < w(x), and the bonus token is the first index
whose running weight sum exceeds mulhi(r, R).  The emitted distribution is w / sum(w).

Random draws come from Philox-4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers:
as easy as 1, 2, 3", SC 2011), counter = (draw index, step low, step high, sequence), key =
(seed low, seed high); a draw is the first two output words, low word first.
"""
from __future__ import annotations

import numpy as np

M32 = 0xFFFFFFFF
PHILOX_M0, PHILOX_M1 = 0xD2511F53, 0xCD9E8D57
PHILOX_W0, PHILOX_W1 = 0x9E3779B9, 0xBB67AE85


def philox4x32_10(counter, key):
    """counter: 4 words, key: 2 words (32-bit each).  Returns 4 words."""
    c0, c1, c2, c3 = (int(x) & M32 for x in counter)
    k0, k1 = (int(x) & M32 for x in key)
    for _ in range(10):
        p0 = PHILOX_M0 * c0
        p1 = PHILOX_M1 * c2
        c0, c1, c2, c3 = ((p1 >> 32) ^ c1 ^ k0) & M32, p1 & M32, ((p0 >> 32) ^ c3 ^ k1) & M32, p0 & M32
        k0 = (k0 + PHILOX_W0) & M32
        k1 = (k1 + PHILOX_W1) & M32
    return c0, c1, c2, c3


def rand64(seed, step, seq, draw):
    x = philox4x32_10((draw, step & M32, (step >> 32) & M32, seq), (seed & M32, (seed >> 32) & M32))
    return x[0] | (x[1] << 32)


def weights(p_row):
    """Integer weights of one distribution (a list of Python ints)."""
    out = []
    for p in np.asarray(p_row, np.float64):
        if not (p > 0.0):          # NaN, zero, negative
            out.append(0)
        elif p >= 1.0:
            out.append(1 << 32)
        else:
            out.append(int(np.floor(p * 4294967296.0)))
    return out


def mulhi(r, R):
    return (r * R) >> 64


def accept_sample(cu_nodes, parent, token, target_prob, seed, step, max_depth, draws=None):
    """Returns (accept_len, accept_path, bonus_token) like the greedy walk.

    target_prob: [N, V] distribution the target model assigns after each node.
    draws: optional callable (b, i) -> 64-bit int replacing the generator (used by the pins
    that integrate over the random numbers).
    A sequence whose remaining weight is 0 when the bonus is due gets bonus -1.
    """
    B = len(cu_nodes) - 1
    V = target_prob.shape[1]
    accept_len, paths, bonus = [0] * B, [[-1] * (max_depth + 1) for _ in range(B)], [0] * B
    for b in range(B):
        base = int(cu_nodes[b])
        n_b = int(cu_nodes[b + 1]) - base
        n_draw = 0

        def draw():
            nonlocal n_draw
            r = draws(b, n_draw) if draws is not None else rand64(seed, step, b, n_draw)
            n_draw += 1
            return r

        cur, path = 0, [0]
        while True:
            w = weights(target_prob[base + cur])
            R = sum(w)
            rejected = set()
            nxt = -1
            if len(path) <= max_depth:
                for c in range(cur + 1, n_b):
                    if int(parent[base + c]) != cur:
                        continue
                    x = int(token[base + c])
                    if not (0 <= x < V) or x in rejected:
                        continue                      # nothing of its mass is left
                    if R > 0 and mulhi(draw(), R) < w[x]:
                        nxt = c
                        break
                    R -= w[x]
                    rejected.add(x)
            if nxt < 0:
                break
            cur = nxt
            path.append(cur)
        if R > 0:
            T = mulhi(draw(), R)
            acc = 0
            tok = -1
            for v in range(V):
                if v in rejected:
                    continue
                acc += w[v]
                if acc > T:
                    tok = v
                    break
            bonus[b] = tok
        else:
            bonus[b] = -1
        accept_len[b] = len(path) - 1
        for d, v in enumerate(path):
            paths[b][d] = v
    return accept_len, paths, bonus
