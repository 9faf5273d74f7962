"""Pins for the rotary-embedding oracle (CPU only): the properties that define the rotation."""
import numpy as np
import pytest

from oracle import rope as R


@pytest.mark.parametrize("pairing", [R.HALF_SPLIT, R.INTERLEAVED])
def test_position_zero_is_identity_and_lengths_are_kept(pairing):
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, 16))
    assert np.array_equal(R.rope(x, [0] * 5, pairing=pairing), x)
    y = R.rope(x, [7, 1, 300, 4095, 12], pairing=pairing)
    assert np.allclose((y ** 2).sum(-1), (x ** 2).sum(-1), rtol=1e-12)
    assert not np.allclose(y, x)


@pytest.mark.parametrize("pairing", [R.HALF_SPLIT, R.INTERLEAVED])
def test_scores_depend_on_relative_position_only(pairing):
    """<R_m q, R_n k> = <R_{m-n} q, k>: the property rotary embeddings are built for."""
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((1, 2, 32)), rng.standard_normal((1, 2, 32))
    for m, n in ((5, 3), (100, 100), (4000, 3990), (17, 40)):
        lhs = (R.rope(q, [m], pairing=pairing) * R.rope(k, [n], pairing=pairing)).sum(-1)
        if m >= n:
            rhs = (R.rope(q, [m - n], pairing=pairing) * k).sum(-1)
        else:
            rhs = (q * R.rope(k, [n - m], pairing=pairing)).sum(-1)
        assert np.allclose(lhs, rhs, rtol=0, atol=1e-9)


def test_known_angles_and_the_two_pairings():
    # head of 4, base 100: pair 0 turns by pos, pair 1 by pos / 10
    x = np.array([[[1.0, 2.0, 3.0, 4.0]]])
    y = R.rope(x, [1], base=100.0, pairing=R.HALF_SPLIT)       # pairs (x0, x2), (x1, x3)
    c0, s0, c1, s1 = np.cos(1.0), np.sin(1.0), np.cos(0.1), np.sin(0.1)
    assert np.allclose(y[0, 0], [1 * c0 - 3 * s0, 2 * c1 - 4 * s1, 1 * s0 + 3 * c0, 2 * s1 + 4 * c1], atol=1e-15)
    y = R.rope(x, [1], base=100.0, pairing=R.INTERLEAVED)      # pairs (x0, x1), (x2, x3)
    assert np.allclose(y[0, 0], [1 * c0 - 2 * s0, 1 * s0 + 2 * c0, 3 * c1 - 4 * s1, 3 * s1 + 4 * c1], atol=1e-15)
    # a quarter turn of the fastest pair: (x, y) -> (-y, x)
    y = R.rope(np.array([[[1.0, 0.0, 0.0, 0.0]]]), [1], base=1.0, pairing=R.INTERLEAVED)
    assert np.allclose(R.rope(np.array([[[1.0, 0.0]]]), [1], base=1.0)[0, 0], [np.cos(1.0), np.sin(1.0)])
    assert np.allclose(y[0, 0], [np.cos(1.0), np.sin(1.0), 0.0, 0.0])


def test_rotations_compose_and_partial_rotary_dim_leaves_the_rest():
    rng = np.random.default_rng(2)
    x = rng.standard_normal((2, 2, 12))
    a = R.rope(R.rope(x, [3, 10]), [4, 20])
    assert np.allclose(a, R.rope(x, [7, 30]), atol=1e-12)
    y = R.rope(x, [9, 9], rotary_dim=8)
    assert np.array_equal(y[..., 8:], x[..., 8:]) and not np.allclose(y[..., :8], x[..., :8])
    with pytest.raises(ValueError):
        R.rope(x, [0, 0], rotary_dim=7)
