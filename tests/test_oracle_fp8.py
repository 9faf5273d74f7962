"""Pins for the E4M3 codec of the fp8 KV-cache variant (CPU only)."""
import numpy as np

from oracle import fp8 as F


def test_values_the_format_specification_names():
    assert F.decode_one(0x7E) == 448.0 and F.decode_one(0xFE) == -448.0          # largest finite
    assert F.decode_one(0x01) == 2.0 ** -9 and F.decode_one(0x07) == 7 * 2.0 ** -9  # subnormals
    assert F.decode_one(0x08) == 2.0 ** -6                                        # smallest normal
    assert F.decode_one(0x38) == 1.0 and F.decode_one(0x3C) == 1.5 and F.decode_one(0x40) == 2.0
    assert F.decode_one(0x00) == 0.0 and np.signbit(F.decode_one(0x80)) and F.decode_one(0x80) == 0.0
    assert np.isnan(F.decode_one(0x7F)) and np.isnan(F.decode_one(0xFF))          # the only NaNs
    assert np.isfinite(F.TABLE).sum() == 254                                      # no infinities


def test_round_trip_monotone_and_ties_to_even():
    finite = [c for c in range(256) if c & 0x7F != 0x7F]
    for c in finite:
        assert F.encode_one(F.decode_one(c)) == c
    pos = F.TABLE[:0x7F]
    assert (np.diff(pos) > 0).all()
    # half-way points go to the even mantissa
    assert F.encode_one(1.0625) == 0x38 and F.encode_one(1.1875) == 0x3A          # 1.0 | 1.25
    assert F.encode_one(2.0 ** -10) == 0x00 and F.encode_one(3 * 2.0 ** -10) == 0x02   # 0 | 2 * 2^-9
    assert F.encode_one(464.0) == 0x7E and F.encode_one(1e9) == 0x7E and F.encode_one(-1e9) == 0xFE  # saturation
    assert F.encode_one(float("nan")) == 0x7F and F.encode_one(float("inf")) == 0x7E


def test_encode_is_the_nearest_grid_point_by_brute_force():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(3000), rng.standard_normal(1000) * 100, rng.standard_normal(1000) * 1e-3,
                        rng.uniform(-460, 460, 1000)])
    grid = F.TABLE[np.isfinite(F.TABLE)]
    got = F.decode(F.encode(x))
    for xi, gi in zip(x, got):
        best = np.abs(grid - np.clip(xi, -448, 448)).min()
        assert abs(gi - np.clip(xi, -448, 448)) == best


def test_array_form_equals_the_scalar_definition():
    rng = np.random.default_rng(1)
    x = np.concatenate([rng.standard_normal(4000) * 3, rng.uniform(-500, 500, 2000), rng.standard_normal(2000) * 0.01,
                        F.TABLE[np.isfinite(F.TABLE)], [0.0, -0.0, np.inf, -np.inf, np.nan, 1.0625, 1.1875, 2.0 ** -10,
                                                         3 * 2.0 ** -10, 464.0, 447.99, 448.0, -448.0]])
    mid = (F.TABLE[:0x7E] + F.TABLE[1:0x7F]) / 2             # every half-way point of the grid, both signs
    x = np.concatenate([x, mid, -mid])
    assert F.encode(x).tolist() == [F.encode_one(v) for v in x]
