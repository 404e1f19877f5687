"""Pins for the oracle's omega = ||grad W^S_i||^2 (paper, section "CheckFree:
Memoryless Recovery": omega is the squared norm of the stage's last gradient).

None of these re-type the oracle's loop: they are closed forms, exact rational
arithmetic and algebraic invariants that a dropped term, a missing square, a
square root, or a per-tensor mean instead of a sum would break."""
from fractions import Fraction

import numpy as np
import pytest

import oracle

THREADS = [1, 3, 8]


@pytest.mark.parametrize("threads", THREADS)
@pytest.mark.parametrize("n", [1, 7, 4096, 100003])
def test_constant_tensor_closed_form(n, threads):
    c = 2.0 ** -7
    g = np.full(n, c, dtype=np.float32)
    assert oracle.stage_grad_sqnorm([g], threads) == n * c * c          # exact


@pytest.mark.parametrize("threads", THREADS)
def test_ramp_closed_form(threads):
    n = 10_000
    g = np.arange(1, n + 1, dtype=np.float32)
    assert oracle.stage_grad_sqnorm([g], threads) == n * (n + 1) * (2 * n + 1) // 6


def test_ramp_split_over_tensors_is_one_stage():
    # omega is over ALL tensors of the stage: matrices and vectors alike.
    n = 3000
    g = np.arange(1, n + 1, dtype=np.float32)
    parts = [g[:1], g[1:50].reshape(7, 7), g[50:2048], g[2048:]]
    assert oracle.stage_grad_sqnorm(parts) == n * (n + 1) * (2 * n + 1) // 6


@pytest.mark.parametrize("threads", THREADS)
def test_exact_rational_brute_force(threads):
    rng = np.random.default_rng(11)
    for trial in range(20):
        sizes = rng.integers(1, 60, size=rng.integers(1, 6))
        sig = 10.0 ** rng.uniform(-5, -2)
        tensors = [rng.normal(0, sig, size=s).astype(np.float32) for s in sizes]
        exact = sum(Fraction(float(v)) ** 2 for t in tensors for v in t)
        got = Fraction(oracle.stage_grad_sqnorm(tensors, threads))
        assert abs(got - exact) <= exact * Fraction(1, 10 ** 15)


def test_additive_over_tensors_exactly():
    rng = np.random.default_rng(5)
    a = rng.normal(0, 1e-3, 1000).astype(np.float32)
    b = rng.normal(0, 1e-4, 77).astype(np.float32)
    assert oracle.stage_grad_sqnorm([a, b]) == oracle.stage_grad_sqnorm([a]) + oracle.stage_grad_sqnorm([b])


def test_scaling_by_two_is_exact_factor_four():
    rng = np.random.default_rng(6)
    g = rng.normal(0, 1e-3, 5000).astype(np.float32)
    assert oracle.stage_grad_sqnorm([2 * g]) == 4 * oracle.stage_grad_sqnorm([g])
    assert oracle.stage_grad_sqnorm([-g]) == oracle.stage_grad_sqnorm([g])


def test_permutation_invariance_within_fp64_noise():
    rng = np.random.default_rng(7)
    g = rng.normal(0, 1e-3, 50_000).astype(np.float32)
    w = oracle.stage_grad_sqnorm([g])
    w2 = oracle.stage_grad_sqnorm([rng.permutation(g)])
    assert abs(w - w2) <= 1e-13 * w


def test_threaded_split_matches_serial():
    rng = np.random.default_rng(8)
    tensors = [rng.normal(0, s, n).astype(np.float32) for s, n in [(1e-2, 100_001), (1e-5, 17), (3e-4, 4096)]]
    w = oracle.stage_grad_sqnorm(tensors, 1)
    for th in (2, 5, 8, 64):
        assert abs(oracle.stage_grad_sqnorm(tensors, th) - w) <= 1e-12 * w   # n * 2^-53 bound of plain summation


def test_empty_and_single():
    assert oracle.stage_grad_sqnorm([]) == 0.0
    assert oracle.stage_grad_sqnorm([np.zeros(0, np.float32)]) == 0.0
    assert oracle.stage_grad_sqnorm([np.array([-3.0], np.float32)]) == 9.0
    assert oracle.stage_grad_sqnorm([np.zeros(0, np.float32), np.array([0.5], np.float32)], 4) == 0.25


def test_tiny_and_huge_values_do_not_leave_fp64_range():
    # fp32 extremes square inside binary64's range: no underflow to 0, no inf.
    tiny = np.array([2.0 ** -149] * 4, np.float32)
    huge = np.array([np.finfo(np.float32).max] * 4, np.float32)
    assert oracle.stage_grad_sqnorm([tiny]) == 4 * 2.0 ** -298
    assert oracle.stage_grad_sqnorm([huge]) == 4 * float(np.finfo(np.float32).max) ** 2


def test_nonfinite_gradient_propagates():
    g = np.array([1.0, np.inf, 2.0], np.float32)
    assert oracle.stage_grad_sqnorm([g]) == np.inf
    g = np.array([1.0, np.nan, 2.0], np.float32)
    assert np.isnan(oracle.stage_grad_sqnorm([g]))


def test_statistical_expectation_at_model_shape():
    # E[omega] = sum_t n_t sigma_t^2 with relative s.d. sqrt(2/n_t) per tensor: a gross-error check
    import workloads
    wl = workloads.make_workload(1, shape=workloads.StageShape(96, 256, 2))
    shapes = wl.spec.shape.tensor_shapes()
    for s in range(3):
        grads = workloads.stage_to_numpy(wl.grads[s])
        n = np.array([np.prod(sh) for sh in shapes], dtype=np.float64)
        mean = float(np.sum(n * wl.sigmas[s] ** 2))
        sd = float(np.sqrt(np.sum(2 * n * wl.sigmas[s] ** 4)))
        assert abs(oracle.stage_grad_sqnorm(grads) - mean) < 6 * sd


def test_bf16_gradients_closed_form_and_exact_rational():
    # bf16 bit patterns: 0x3C00 = 2^-7; the ramp 1..256 is exact in bf16
    c = np.full(1000, 0x3C00, dtype=np.uint16)
    assert oracle.stage_grad_sqnorm([c]) == 1000 * 2.0 ** -14
    ramp32 = np.arange(1, 257, dtype=np.float32)
    ramp = (ramp32.view(np.uint32) >> 16).astype(np.uint16)
    assert np.all((ramp.astype(np.uint32) << 16).view(np.float32) == ramp32)
    assert oracle.stage_grad_sqnorm([ramp]) == 256 * 257 * 513 // 6
    rng = np.random.default_rng(3)
    bits = rng.integers(0, 0x7F80, 300).astype(np.uint16) | (rng.integers(0, 2, 300).astype(np.uint16) << 15)
    vals = (bits.astype(np.uint32) << 16).view(np.float32)
    keep = np.abs(vals) < 1e10
    bits = bits[keep]
    exact = sum(Fraction(float(v)) ** 2 for v in (bits.astype(np.uint32) << 16).view(np.float32))
    got = Fraction(oracle.stage_grad_sqnorm([bits]))
    assert abs(got - exact) <= exact * Fraction(1, 10 ** 15)
    # mixed stage: fp32 and bf16 tensors add up
    f = np.array([3.0, 4.0], np.float32)
    assert oracle.stage_grad_sqnorm([f, c]) == 25.0 + 1000 * 2.0 ** -14


def test_per_tensor_norms_add_up_to_omega():
    rng = np.random.default_rng(21)
    tensors = [rng.normal(0, s, n).astype(np.float32) for s, n in [(1e-2, 1001), (1e-5, 17), (3e-4, 4096), (1.0, 0)]]
    per = oracle.tensor_grad_sqnorms(tensors)
    assert per[3] == 0.0
    for t, g in zip(per, tensors):
        exact = sum(Fraction(float(v)) ** 2 for v in g)
        assert abs(Fraction(t) - exact) <= exact * Fraction(1, 10 ** 12)      # n * 2^-53 bound of plain summation
    total = 0.0
    for t in per:
        total += t
    assert total == oracle.stage_grad_sqnorm(tensors)          # same association: exact
