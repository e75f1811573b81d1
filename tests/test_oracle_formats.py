"""Pins for the oracle's number-format helpers (decode to fp64, round-to-nearest-even).

Every other oracle function leans on these two, so they are checked against things that are
not the oracle: numpy's own float16 conversion (a library routine), the IEEE-754 definition
evaluated by exhaustive search in exact rational arithmetic, and hand-picked boundary values.
"""
import bisect
from fractions import Fraction

import numpy as np
import pytest

from oracle import pdelta_oracle as orc


def _finite_table(decode_all):
    """Sorted (value, bits) of all finite non-negative patterns of a 16-bit format."""
    vals = []
    for bits in range(0x8000):
        x = decode_all[bits]
        if np.isfinite(x):
            vals.append((Fraction(float(x)), bits))
    vals.sort()
    return vals


def _rne_by_search(x: Fraction, table, overflow_bits, max_next: Fraction):
    """IEEE round-to-nearest-even by brute force over every finite value of the format."""
    sign = 0x8000 if x < 0 else 0
    a = abs(x)
    keys = [t[0] for t in table]
    largest = keys[-1]
    # Overflow rule: values at or beyond largest + half an ulp (of the top binade) go to inf.
    if a >= largest + (max_next - largest) / 2:
        return sign | overflow_bits
    j = bisect.bisect_left(keys, a)
    if j < len(keys) and keys[j] == a:
        return sign | table[j][1]
    lo, hi = table[j - 1], table[min(j, len(keys) - 1)]
    dlo, dhi = a - lo[0], hi[0] - a
    if dlo < dhi:
        return sign | lo[1]
    if dhi < dlo:
        return sign | hi[1]
    return sign | (lo[1] if lo[1] % 2 == 0 else hi[1])


def test_decode_f16_matches_numpy_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = bits.view(np.float16).astype(np.float64)
    got = orc.decode(bits, orc.F16)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])
    assert np.array_equal(np.signbit(got[~nan]), np.signbit(want[~nan]))   # -0 keeps its sign


def test_decode_bf16_is_the_top_half_of_fp32_for_every_pattern():
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    want = (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)
    got = orc.decode(bits, orc.BF16)
    nan = np.isnan(want)
    assert np.array_equal(np.isnan(got), nan)
    assert np.array_equal(got[~nan], want[~nan])


def test_decode_hand_values():
    # value, fp16 pattern, bf16 pattern: written out from the format definitions
    cases = [(1.0, 0x3C00, 0x3F80), (-2.0, 0xC000, 0xC000), (0.5, 0x3800, 0x3F00),
             (65504.0, 0x7BFF, None), (2.0 ** -24, 0x0001, None), (2.0 ** -14, 0x0400, None),
             (2.0 ** -133, None, 0x0001), (2.0 ** -126, None, 0x0080), (1.5, 0x3E00, 0x3FC0)]
    for val, h, b in cases:
        if h is not None:
            assert orc.decode(np.array([h], np.uint16), orc.F16)[0] == val
        if b is not None:
            assert orc.decode(np.array([b], np.uint16), orc.BF16)[0] == val


@pytest.mark.parametrize("dtype", [orc.F16, orc.BF16])
def test_rne_round_trips_every_finite_pattern(dtype):
    bits = np.arange(65536, dtype=np.uint32).astype(np.uint16)
    vals = orc.decode(bits, dtype)
    keep = np.isfinite(vals)
    assert np.array_equal(orc.rne(vals[keep], dtype), bits[keep])   # includes -0 -> 0x8000


def test_rne_f16_matches_numpy_on_random_and_boundary_doubles():
    rng = np.random.default_rng(7)
    x = np.concatenate([
        rng.standard_normal(20000) * 10.0 ** rng.uniform(-9, 5, 20000),
        rng.uniform(-2.0 ** -13, 2.0 ** -13, 5000),                  # subnormal range
        np.array([65504.0, 65519.999, 65520.0, 65536.0, 1e9, -65520.0, 2.0 ** -25,
                  2.0 ** -25 * (1 + 2.0 ** -40), 2.0 ** -26, 0.0, -0.0]),
    ])
    with np.errstate(over="ignore"):
        want = x.astype(np.float16).view(np.uint16)                   # numpy rounds once, RNE
    assert np.array_equal(orc.rne(x, orc.F16), want)


@pytest.mark.parametrize("dtype,overflow_bits,max_next", [
    (orc.F16, 0x7C00, Fraction(2) ** 16),
    (orc.BF16, 0x7F80, Fraction(2) ** 128),
])
def test_rne_agrees_with_exhaustive_search_including_ties(dtype, overflow_bits, max_next):
    bits = np.arange(0x8000, dtype=np.uint32).astype(np.uint16)
    table = _finite_table(orc.decode(bits, dtype))
    rng = np.random.default_rng(11)
    idx = rng.integers(0, len(table) - 1, 300)
    xs = []
    for j in idx:
        lo, hi = table[j][0], table[j + 1][0]
        mid = (lo + hi) / 2
        xs += [mid, mid + (hi - lo) / 1024, mid - (hi - lo) / 1024]    # exact ties and near ties
    xs += [Fraction(float(v)) for v in rng.standard_normal(300) * 3.0]
    xs += [-x for x in xs[:50]]
    # only doubles can be passed to the oracle: keep those Fractions that are exact doubles
    xs = [x for x in xs if Fraction(float(x)) == x]
    assert len(xs) > 600
    got = orc.rne(np.array([float(x) for x in xs]), dtype)
    want = [_rne_by_search(x, table, overflow_bits, max_next) for x in xs]
    assert [int(g) for g in got] == want
