"""Pins for the oracle's weighted-average recovery (paper, section "CheckFree:
Memoryless Recovery", display equation; Algorithm 1, third step).

The pins are the special cases the section itself names (omega_{i+1} = 0 is a
copy of the previous stage; equal omegas are the uniform average), hand-worked
values, algebraic invariants and exact rational arithmetic with a correct
rounding written independently (tests/exactmath.py).  A swapped weight, the
algorithm box's misprint (omega_{i-1} on both terms), a missing denominator or
a double rounding each break at least one of them."""
import os
from fractions import Fraction

import numpy as np
import pytest

import exactmath as em
import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "blend_hand_cases.txt")


def _bf16(x):
    """float32 array -> bf16 bits (RNE) via exact rounding of each value."""
    return np.array([em.fraction_to_bf16_bits(Fraction(float(v))) for v in np.ravel(x)],
                    dtype=np.uint16).reshape(np.shape(x))


def _rand_weights(rng, n, dtype):
    a = rng.normal(0, 0.02, n).astype(np.float32)
    b = rng.normal(0, 0.02, n).astype(np.float32)
    if dtype == "bf16":
        return _bf16(a), _bf16(b)
    return a, b


def test_hand_worked_cases():
    rows = [l.split() for l in open(GOLDEN) if l.strip() and not l.startswith("#")]
    assert len(rows) >= 10
    for wp, wn, a, b, want in rows:
        a32 = np.array([float(a)], np.float32)
        b32 = np.array([float(b)], np.float32)
        assert float(a32[0]) == float(a) and float(b32[0]) == float(b)
        out = oracle.recover_stage_weighted_avg([a32], [b32], float(wp), float(wn))[0]
        assert out[0] == np.float32(float(want)), (wp, wn, a, b, want, out)
        outb = oracle.recover_stage_weighted_avg([_bf16(a32)], [_bf16(b32)], float(wp), float(wn))[0]
        assert outb[0] == _bf16(np.array([float(want)], np.float32))[0]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_zero_weight_on_one_neighbour_is_exact_copy_of_the_other(dtype):
    rng = np.random.default_rng(1)
    a, b = _rand_weights(rng, 3000, dtype)
    for w in (1.0, 3.7e-3, 1.9e-9, 12345.678):
        out = oracle.recover_stage_weighted_avg([a], [b], w, 0.0)[0]
        assert np.array_equal(out, a)                     # "copy previous": omega_{i+1} = 0
        out = oracle.recover_stage_weighted_avg([a], [b], 0.0, w)[0]
        assert np.array_equal(out, b)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_identical_neighbours_give_back_that_stage(dtype):
    rng = np.random.default_rng(2)
    a, _ = _rand_weights(rng, 3000, dtype)
    for wp, wn in [(1.0, 1.0), (3.7e-3, 1.9e-2), (1e-9, 5.0), (7.0, 1e-12)]:
        out = oracle.recover_stage_weighted_avg([a], [a.copy()], wp, wn)[0]
        assert np.array_equal(out, a)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_equal_omegas_are_the_correctly_rounded_uniform_average(dtype):
    """omega_{i-1} = omega_{i+1}: the uniform average.  (a+b)/2 of two floats sits
    on a rounding tie quite often, so the result is pinned bit for bit where the
    products omega*w are exact (omega a power of two) and, for any other equal
    pair, everywhere except on exact ties, where binary64's own rounding of
    omega*w may break the tie either way (one ulp)."""
    rng = np.random.default_rng(3)
    a, b = _rand_weights(rng, 400, dtype)
    for w in (0.5, 2.0 ** -20, 0.37):
        out = oracle.recover_stage_weighted_avg([a], [b], w, w)[0]
        for k in range(a.size):
            if dtype == "f32":
                exact = (Fraction(float(a[k])) + Fraction(float(b[k]))) / 2
                want = em.fraction_to_f32_bits(exact)
                got = int(out.view(np.uint32)[k])
                sign, m, q = em.round_fraction(exact, "f32")
            else:
                exact = (em.bf16_bits_to_fraction(a[k]) + em.bf16_bits_to_fraction(b[k])) / 2
                want = em.fraction_to_bf16_bits(exact)
                got = int(out[k])
                sign, m, q = em.round_fraction(exact, "bf16")
            tie = abs(abs(exact) / Fraction(2) ** q - m) == Fraction(1, 2)
            if w != 0.37 or not tie:
                assert got == want
            else:
                assert abs(got - want) <= 1


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_rational_brute_force(dtype):
    """Exact value of the formula, correctly rounded: the oracle may differ only
    where binary64's own rounding moved the value across a rounding boundary
    (at most one ulp, and rarely)."""
    rng = np.random.default_rng(4)
    worst, off = 0, 0
    for trial in range(12):
        a, b = _rand_weights(rng, 120, dtype)
        wp, wn = (10.0 ** rng.uniform(-10, 1, 2)).tolist()
        out = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
        for k in range(a.size):
            if dtype == "f32":
                fa, fb = Fraction(float(a[k])), Fraction(float(b[k]))
            else:
                fa, fb = em.bf16_bits_to_fraction(a[k]), em.bf16_bits_to_fraction(b[k])
            exact = (Fraction(wp) * fa + Fraction(wn) * fb) / (Fraction(wp) + Fraction(wn))
            if dtype == "f32":
                want = np.array([em.fraction_to_f32_bits(exact)], np.uint32).view(np.float32)
                d = int(em.ulp_distance(out[k:k + 1], want)[0])
            else:
                want = np.array([em.fraction_to_bf16_bits(exact)], np.uint16)
                d = int(em.ulp_distance(out[k:k + 1], want)[0])
            worst = max(worst, d)
            off += d != 0
    assert worst <= 1
    assert off <= 2          # double rounding through binary64 is a ~1e-8 event per element


def test_bf16_result_is_rounded_once_not_through_fp32():
    """A value a hair above a bf16 tie: one rounding goes up; rounding to fp32
    first lands on the tie and then goes to even (down).  a = 1, b = 1 + 2^-7,
    weights 1 and 1 + 2^-20 give 1 + 2^-8 + about 2^-29."""
    a = np.array([0x3F80], np.uint16)
    b = np.array([0x3F81], np.uint16)
    wp, wn = 1.0, 1.0 + 2.0 ** -20
    exact = (Fraction(wp) * 1 + Fraction(wn) * (1 + Fraction(1, 128))) / (Fraction(wp) + Fraction(wn))
    assert exact > 1 + Fraction(1, 256) and exact - (1 + Fraction(1, 256)) < Fraction(1, 2 ** 28)
    assert em.fraction_to_bf16_bits(exact) == 0x3F81
    assert oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0][0] == 0x3F81
    # mirrored: a hair below the tie goes down
    assert oracle.recover_stage_weighted_avg([a], [b], wn, wp)[0][0] == 0x3F80


def test_unrounded_value_matches_exact_rational():
    rng = np.random.default_rng(14)
    a = rng.normal(0, 0.02, 200).astype(np.float32).astype(np.float64)
    b = rng.normal(0, 0.02, 200).astype(np.float32).astype(np.float64)
    wp, wn = 3.7e-3, 1.9e-2
    out = oracle.blend_unrounded(a, b, wp, wn)
    for k in range(a.size):
        exact = (Fraction(wp) * Fraction(a[k]) + Fraction(wn) * Fraction(b[k])) / (Fraction(wp) + Fraction(wn))
        scale = (Fraction(wp) * abs(Fraction(a[k])) + Fraction(wn) * abs(Fraction(b[k]))) / (Fraction(wp) + Fraction(wn))
        assert abs(Fraction(out[k]) - exact) <= scale * Fraction(4, 2 ** 53)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_convexity(dtype):
    rng = np.random.default_rng(5)
    a, b = _rand_weights(rng, 20000, dtype)
    for wp, wn in [(3.7e-3, 1.9e-2), (1.0, 1e-9), (2.5, 2.5)]:
        out = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
        if dtype == "f32":
            oa, ob, oo = em.ordered_f32(a), em.ordered_f32(b), em.ordered_f32(out)
        else:
            oa, ob, oo = em.ordered_bf16(a), em.ordered_bf16(b), em.ordered_bf16(out)
        assert np.all(oo >= np.minimum(oa, ob)) and np.all(oo <= np.maximum(oa, ob))


def test_weight_moves_result_toward_the_heavier_neighbour():
    # More gradient norm on a neighbour => result closer to that neighbour.
    a = np.array([0.0], np.float32)
    b = np.array([1.0], np.float32)
    lo = oracle.recover_stage_weighted_avg([a], [b], 3.0, 1.0)[0][0]     # heavier prev
    hi = oracle.recover_stage_weighted_avg([a], [b], 1.0, 3.0)[0][0]     # heavier next
    assert lo == np.float32(0.25) and hi == np.float32(0.75)


def test_linearity_of_the_unrounded_value():
    rng = np.random.default_rng(6)
    a1, a2, b1, b2 = (rng.normal(0, 0.02, 5000) for _ in range(4))
    wp, wn = 3.7e-3, 1.9e-2
    lhs = oracle.blend_unrounded(a1 + a2, b1 + b2, wp, wn)
    rhs = oracle.blend_unrounded(a1, b1, wp, wn) + oracle.blend_unrounded(a2, b2, wp, wn)
    scale = np.abs(a1) + np.abs(a2) + np.abs(b1) + np.abs(b2)
    assert np.all(np.abs(lhs - rhs) <= 1e-15 * scale)
    # homogeneity in the weights tensor
    assert np.array_equal(oracle.blend_unrounded(4 * a1, 4 * b1, wp, wn), 4 * oracle.blend_unrounded(a1, b1, wp, wn))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scale_invariance_in_omega(dtype):
    rng = np.random.default_rng(7)
    a, b = _rand_weights(rng, 5000, dtype)
    wp, wn = 3.7e-3, 1.9e-2
    ref = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
    for k in (-40, -3, 1, 17, 60):
        out = oracle.recover_stage_weighted_avg([a], [b], wp * 2.0 ** k, wn * 2.0 ** k)[0]
        assert np.array_equal(out, ref)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_swap_symmetry(dtype):
    rng = np.random.default_rng(8)
    a, b = _rand_weights(rng, 5000, dtype)
    x = oracle.recover_stage_weighted_avg([a], [b], 3.7e-3, 1.9e-2)[0]
    y = oracle.recover_stage_weighted_avg([b], [a], 1.9e-2, 3.7e-3)[0]
    assert np.array_equal(x, y)


def test_one_scalar_pair_blends_every_tensor_of_the_stage():
    rng = np.random.default_rng(9)
    prev = [rng.normal(0, 0.02, s).astype(np.float32) for s in [(4, 5), (7,), (1,), (3, 3, 2)]]
    nxt = [rng.normal(0, 0.02, s).astype(np.float32) for s in [(4, 5), (7,), (1,), (3, 3, 2)]]
    out = oracle.recover_stage_weighted_avg(prev, nxt, 1.0, 3.0)
    assert [o.shape for o in out] == [p.shape for p in prev]
    cat = oracle.recover_stage_weighted_avg([np.concatenate([p.ravel() for p in prev])],
                                            [np.concatenate([n.ravel() for n in nxt])], 1.0, 3.0)[0]
    assert np.array_equal(np.concatenate([o.ravel() for o in out]), cat)


def test_threads_do_not_change_bits():
    rng = np.random.default_rng(10)
    a, b = _rand_weights(rng, 100_003, "f32")
    x = oracle.recover_stage_weighted_avg([a], [b], 3.7e-3, 1.9e-2, threads=1)[0]
    y = oracle.recover_stage_weighted_avg([a], [b], 3.7e-3, 1.9e-2, threads=8)[0]
    assert np.array_equal(x, y)


def test_subnormal_and_extreme_values():
    a = np.array([2.0 ** -149, -2.0 ** -140, np.finfo(np.float32).max, 0.0, -0.0], np.float32)
    b = np.array([2.0 ** -149, 2.0 ** -140, np.finfo(np.float32).max, -0.0, -0.0], np.float32)
    out = oracle.recover_stage_weighted_avg([a], [b], 1.0, 1.0)[0]
    assert out[0] == np.float32(2.0 ** -149)              # subnormals are kept, not flushed
    assert out[1] == 0.0
    assert out[2] == np.finfo(np.float32).max
    assert out[3] == 0.0 and out[4] == 0.0 and np.signbit(out[4])


def test_nan_and_inf_weights_propagate():
    a = np.array([np.nan, np.inf, 1.0], np.float32)
    b = np.array([1.0, 1.0, -np.inf], np.float32)
    out = oracle.recover_stage_weighted_avg([a], [b], 1.0, 3.0)[0]
    assert np.isnan(out[0]) and out[1] == np.inf and out[2] == -np.inf


@pytest.mark.parametrize("wp,wn", [(0.0, 0.0), (np.nan, 1.0), (1.0, np.inf), (-1.0, 2.0), (np.inf, np.inf),
                                   (1e-320, 1e-320), (1e308, 1e308)])
def test_degenerate_omega_rule_is_the_uniform_average(wp, wn):
    """Our reading where the paper is silent (parity unpinned): an unusable
    omega pair falls back to the unweighted (uniform) average the section itself mentions."""
    rng = np.random.default_rng(12)
    a, b = _rand_weights(rng, 500, "f32")
    assert oracle.effective_omega(wp, wn) == (1.0, 1.0, True)
    out = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
    ref = oracle.recover_stage_weighted_avg([a], [b], 1.0, 1.0)[0]
    assert np.array_equal(out, ref)


def test_regular_omegas_pass_through():
    assert oracle.effective_omega(3.0, 0.0) == (3.0, 0.0, False)
    assert oracle.effective_omega(1e-300, 2e-300) == (1e-300, 2e-300, False)


def test_mismatched_stages_are_rejected():
    a = [np.zeros(4, np.float32)]
    with pytest.raises(ValueError):
        oracle.recover_stage_weighted_avg(a, [np.zeros(5, np.float32)], 1, 1)
    with pytest.raises(ValueError):
        oracle.recover_stage_weighted_avg(a, a + a, 1, 1)
    with pytest.raises(ValueError):
        oracle.recover_stage_weighted_avg(a, [np.zeros(4, np.uint16)], 1, 1)


# ----------------------------------------------------------------------------
# the common power-of-two factor taken out of the weights before the blend
# ----------------------------------------------------------------------------

def test_common_scale_is_an_exact_power_of_two_that_normalises_the_sum():
    rng = np.random.default_rng(31)
    for _ in range(300):
        wp, wn = (10.0 ** rng.uniform(-300, 300, 2)).tolist()
        if rng.random() < 0.2:
            wn = 0.0
        sp, sn = oracle.common_scale(wp, wn)
        assert 1.0 <= sp + sn < 2.0
        (big, sbig), (small, ssmall) = sorted([(wp, sp), (wn, sn)], reverse=True)
        f = Fraction(sbig) / Fraction(big)
        assert f.numerator == 1 or f.denominator == 1                      # a power of two ...
        assert (f.numerator & (f.numerator - 1)) == 0 and (f.denominator & (f.denominator - 1)) == 0
        # ... and the same one on both weights, unless the smaller one was pushed below the binary64
        # range, where it is more than 2^1000 times smaller than the other and cannot matter
        assert Fraction(ssmall) == Fraction(small) * f or ssmall < 2.0 ** -1000
    assert oracle.common_scale(1.0, 0.5) == (1.0, 0.5)                      # already in [1, 2): untouched
    assert oracle.common_scale(3.0, 1.0) == (0.75, 0.25)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_scale_invariance_in_omega_over_the_whole_binary64_range(dtype):
    """The equation does not change under a common factor; with the factor taken
    out first the result is the same bits from one end of the range to the other."""
    rng = np.random.default_rng(32)
    a, b = _rand_weights(rng, 3000, dtype)
    wp, wn = 3.7e-3, 1.9e-2
    ref = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
    for k in (-1000, -960, -500, 500, 1000, 1020):
        out = oracle.recover_stage_weighted_avg([a], [b], wp * 2.0 ** k, wn * 2.0 ** k)[0]
        assert np.array_equal(out, ref), k


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_exact_rational_brute_force_at_extreme_omegas(dtype):
    """Omegas near the ends of the binary64 range against weights of ordinary and
    of extreme size: the exact value of the equation, correctly rounded."""
    rng = np.random.default_rng(33)
    worst = 0
    pairs = [(1e300, 3e299), (2e-300, 7e-301), (1.5e-310, 4e-307), (8e307, 1e305), (1e300, 1e-300)]
    a, b = _rand_weights(rng, 60, dtype)
    if dtype == "f32":
        a[:4] = [3e38, -1e-38, 1e-45, 2.5]
        b[:4] = [-2e38, 1e-38, -3e-45, 1e30]
    for wp, wn in pairs:
        out = oracle.recover_stage_weighted_avg([a], [b], wp, wn)[0]
        for k in range(a.size):
            if dtype == "f32":
                fa, fb = Fraction(float(a[k])), Fraction(float(b[k]))
            else:
                fa, fb = em.bf16_bits_to_fraction(a[k]), em.bf16_bits_to_fraction(b[k])
            exact = (Fraction(wp) * fa + Fraction(wn) * fb) / (Fraction(wp) + Fraction(wn))
            if dtype == "f32":
                want = np.array([em.fraction_to_f32_bits(exact)], np.uint32).view(np.float32)
            else:
                want = np.array([em.fraction_to_bf16_bits(exact)], np.uint16)
            worst = max(worst, int(em.ulp_distance(out[k:k + 1], want)[0]))
    assert worst <= 1
