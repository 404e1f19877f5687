"""Pins for the oracle's bfloat16 conversions and for the CheckFree+ copy
(paper, section "CheckFree+: First and Last Stage Recovery": an end stage is
restored from its neighbour and the (de)embedding without any loss)."""
from fractions import Fraction

import numpy as np
import pytest

import exactmath as em
import oracle


def test_bf16_widening_all_patterns():
    bits = np.arange(65536, dtype=np.uint32)
    with np.errstate(invalid="ignore"):
        f = (bits << 16).view(np.float32).astype(np.float64)
    for h in range(0, 65536, 7):
        v = oracle.bf16_to_f64(h)
        assert (np.isnan(v) and np.isnan(f[h])) or v == f[h]


def test_bf16_narrowing_is_one_correct_rounding():
    rng = np.random.default_rng(0)
    xs = list(rng.normal(size=3000) * 10.0 ** rng.uniform(-42, 39, 3000))
    # exact ties, values just beside ties, subnormals, overflow threshold
    for h in range(0, 0x7F7F, 97):
        lo = em.bf16_bits_to_fraction(h)
        hi = em.bf16_bits_to_fraction(h + 1)
        mid = float((lo + hi) / 2)
        xs += [mid, np.nextafter(mid, np.inf), np.nextafter(mid, -np.inf), -mid]
    xs += [0.0, -0.0, 2.0 ** -133, 2.0 ** -134, 1.5 * 2.0 ** -134, 2.0 ** -134 * 0.99, 3.3895313892515355e38,
           3.3961775292304e38, 3.4e38, 1e39, -1e39, 1e-300, 5e-324]
    for x in xs:
        want = em.fraction_to_bf16_bits(Fraction(float(x)))
        if x == 0.0 and np.signbit(x):
            want = 0x8000
        assert oracle.f64_to_bf16(float(x)) == want, x
    assert oracle.f64_to_bf16(float("inf")) == 0x7F80
    assert oracle.f64_to_bf16(float("-inf")) == 0xFF80
    n = oracle.f64_to_bf16(float("nan"))
    assert (n & 0x7F80) == 0x7F80 and (n & 0x7F) != 0


def test_bf16_roundtrip_identity():
    for h in list(range(0, 0x7F80, 13)) + list(range(0x8000, 0xFF80, 13)):
        assert oracle.f64_to_bf16(oracle.bf16_to_f64(h)) == h


def test_copy_is_bytewise_including_nan_payloads():
    rng = np.random.default_rng(1)
    raw = rng.integers(0, 2 ** 32, size=10007, dtype=np.uint64).astype(np.uint32)
    raw[:6] = [0x7FC00001, 0xFFC12345, 0x7F800001, 0x80000000, 0x00000001, 0x807FFFFF]
    f = raw.view(np.float32)
    h = rng.integers(0, 2 ** 16, size=33, dtype=np.uint64).astype(np.uint16)
    for th in (1, 3):
        out = oracle.copy_stage([f, h, np.zeros(0, np.float32)], threads=th)
        assert np.array_equal(out[0].view(np.uint32), raw)
        assert np.array_equal(out[1], h)
        assert out[2].size == 0
        assert out[0].ctypes.data != f.ctypes.data


def test_copy_equals_weighted_average_with_zero_weight():
    # "copy previous" is the omega_{i+1} = 0 case of the recovery formula.
    rng = np.random.default_rng(2)
    a = rng.normal(0, 0.02, 1000).astype(np.float32)
    b = rng.normal(0, 0.02, 1000).astype(np.float32)
    assert np.array_equal(oracle.copy_stage([a])[0], oracle.recover_stage_weighted_avg([a], [b], 2.0, 0.0)[0])


def test_range_copy_moves_the_named_elements_and_nothing_else():
    """Slices of a replica refresh: numpy's own slice assignment is the reference."""
    rng = np.random.default_rng(3)
    src = [rng.integers(0, 2 ** 32, size=5000, dtype=np.uint64).astype(np.uint32).view(np.float32),
           rng.integers(0, 2 ** 16, size=777, dtype=np.uint64).astype(np.uint16),
           np.zeros(0, np.float32)]
    ranges = [(0, 0, 1), (0, 17, 1000), (0, 4999, 1), (1, 3, 0), (1, 700, 77)]
    dst = [np.full(5000, np.nan, np.float32), np.full(777, 0xABCD, np.uint16), np.zeros(0, np.float32)]
    want = [d.copy() for d in dst]
    for t, first, count in ranges:
        want[t][first:first + count] = src[t][first:first + count]
    got = oracle.copy_stage_ranges(src, dst, ranges)
    for g, w in zip(got, want):
        assert g.tobytes() == w.tobytes()
    assert np.isnan(got[0][1:17]).all() and np.isnan(got[0][1017:4999]).all()       # guard bands untouched
    assert (got[1][:700] == 0xABCD).all()
    # ranges that tile every tensor add up to the whole-stage copy
    dst2 = [np.zeros_like(s) for s in src]
    tiles = [(0, lo, min(1024, 5000 - lo)) for lo in range(0, 5000, 1024)] + [(1, 0, 400), (1, 400, 377)]
    got2 = oracle.copy_stage_ranges(src, dst2, tiles)
    for g, w in zip(got2, oracle.copy_stage(src)):
        assert g.tobytes() == w.tobytes()
    with pytest.raises(ValueError):
        oracle.copy_stage_ranges(src, dst2, [(1, 700, 78)])
