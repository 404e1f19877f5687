"""Pins for the oracle's Adam step with omega as a by-product (paper, appendix
"Optimizers": Adam, no weight decay, betas (0.9, 0.999); section "CheckFree:
Memoryless Recovery": every stage keeps the squared norm of its last gradient).

What fixes the function from outside: PyTorch's own Adam (an independent
implementation of the same published algorithm) on the CPU in float64, closed
forms (zero gradient; the first step is a sign step; a constant gradient moves
the weight by the same amount every step), exact invariances (sign flip, a
common power of two on gradient, moments and eps), and the already pinned
squared-norm function for the omega it returns."""
import numpy as np
import pytest
import torch

import exactmath as em
import oracle

LR, B1, B2, EPS = 3e-4, 0.9, 0.999, 1e-8


def _state(rng, n, zero_moments=False):
    w = rng.normal(0, 0.02, n).astype(np.float32)
    g = (rng.normal(0, 1, n) * 10.0 ** rng.uniform(-5, -2)).astype(np.float32)
    if zero_moments:
        return w, np.zeros(n, np.float32), np.zeros(n, np.float32), g
    m = (rng.normal(0, 1, n) * 1e-3).astype(np.float32)
    v = (rng.normal(0, 1, n) ** 2 * 1e-6).astype(np.float32)
    return w, m, v, g


def _ulp32(x):
    return np.spacing(np.abs(x).astype(np.float32)).astype(np.float64)


@pytest.mark.parametrize("step", [1, 2, 7, 1000, 100000])
def test_one_step_against_torch_adam_in_float64(step):
    """torch.optim.Adam keeps everything in float64 here; the oracle stores the moments in binary32, so
    its moments are torch's rounded once, and its weight differs by that rounding's effect on the update
    (relative 2^-24 on mhat, half of that on the square root, so below 2e-7 of the distance moved) plus its
    own rounding to binary32."""
    rng = np.random.default_rng(step)
    w, m, v, g = _state(rng, 4000, zero_moments=(step == 1))
    p = torch.nn.Parameter(torch.tensor(w, dtype=torch.float64))
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS, weight_decay=0.0)
    opt.state[p]["step"] = torch.tensor(float(step - 1))
    opt.state[p]["exp_avg"] = torch.tensor(m, dtype=torch.float64)
    opt.state[p]["exp_avg_sq"] = torch.tensor(v, dtype=torch.float64)
    p.grad = torch.tensor(g, dtype=torch.float64)
    opt.step()
    tm, tv, tw = (opt.state[p]["exp_avg"].numpy(), opt.state[p]["exp_avg_sq"].numpy(), p.detach().numpy())
    ow, om, ov = w.copy(), m.copy(), v.copy()
    oracle.adam_step_with_sqnorm([ow], [om], [ov], [g], LR, B1, B2, EPS, step)
    assert np.all(np.abs(om.astype(np.float64) - tm) <= 0.5000001 * _ulp32(tm))
    assert np.all(np.abs(ov.astype(np.float64) - tv) <= 0.5000001 * _ulp32(tv))
    moved = np.abs(tw - w.astype(np.float64))
    assert np.all(np.abs(ow.astype(np.float64) - tw) <= 0.5000001 * _ulp32(tw) + 2e-7 * moved)
    assert np.median(moved) > 0.1 * LR                      # and the step did move the weights


def test_several_steps_against_torch_adam_in_float32():
    """The trajectory people actually run (everything binary32): the oracle's binary64 arithmetic with
    binary32 storage stays within a few roundings of it over 20 steps."""
    rng = np.random.default_rng(11)
    w, m, v, _ = _state(rng, 3000, zero_moments=True)
    p = torch.nn.Parameter(torch.tensor(w))
    opt = torch.optim.Adam([p], lr=LR, betas=(B1, B2), eps=EPS, weight_decay=0.0)
    ow, om, ov = w.copy(), m.copy(), v.copy()
    for t in range(1, 21):
        g = (rng.normal(0, 1, w.size) * 1e-3).astype(np.float32)
        p.grad = torch.tensor(g)
        opt.step()
        oracle.adam_step_with_sqnorm([ow], [om], [ov], [g], LR, B1, B2, EPS, t)
    tw = p.detach().numpy().astype(np.float64)
    assert np.all(np.abs(ow.astype(np.float64) - tw) <= 20 * 2.0 * _ulp32(tw) + 20 * 1e-6 * LR)
    assert np.max(np.abs(ow - w)) > 5 * LR                  # far more movement than the tolerance


def test_zero_gradient_only_decays_the_moments():
    rng = np.random.default_rng(2)
    w, m, v, g = _state(rng, 1000)
    g[:] = 0.0
    w0, m0, v0 = w.copy(), m.copy(), v.copy()
    omega = oracle.adam_step_with_sqnorm([w], [m], [v], [g], LR, B1, B2, EPS, 5)
    assert omega == 0.0
    assert np.array_equal(m, (B1 * m0.astype(np.float64)).astype(np.float32))
    assert np.array_equal(v, (B2 * v0.astype(np.float64)).astype(np.float32))
    # from zero moments nothing moves at all
    z = np.zeros(1000, np.float32)
    w1 = w0.copy()
    oracle.adam_step_with_sqnorm([w1], [z.copy()], [z.copy()], [g], LR, B1, B2, EPS, 1)
    assert np.array_equal(w1, w0)


def test_first_step_is_a_sign_step():
    """t = 1 from zero moments: mhat = g, vhat = g^2, so w moves by lr * g / (|g| + eps)."""
    rng = np.random.default_rng(3)
    w, m, v, g = _state(rng, 2000, zero_moments=True)
    g[np.abs(g) < 1e-6] = 1e-3
    w0 = w.copy().astype(np.float64)
    oracle.adam_step_with_sqnorm([w], [m], [v], [g], LR, B1, B2, EPS, 1)
    gd = g.astype(np.float64)
    want = w0 - LR * gd / (np.abs(gd) + EPS)
    assert np.all(np.abs(w.astype(np.float64) - want) <= 0.51 * _ulp32(want) + 3e-7 * LR)
    assert np.all(np.abs(m.astype(np.float64) - 0.1 * gd) <= 0.51 * _ulp32(0.1 * gd) + 1e-17)
    assert np.all(np.abs(v.astype(np.float64) - 0.001 * gd * gd) <= 0.51 * _ulp32(0.001 * gd * gd) + 1e-30)


def test_constant_gradient_moves_the_weight_by_the_same_amount_every_step():
    """With g = c at every step the bias corrections cancel exactly: mhat = c, vhat = c^2 for every t, so
    after T steps w has moved by T * lr * c / (|c| + eps).  A missing or off-by-one bias correction, swapped
    betas or a wrong sign all break this."""
    c = np.array([1e-3, -2.5e-4, 7e-2, -1e-5], np.float32)
    w = np.array([0.01, -0.02, 0.03, 0.005], np.float32)
    w0 = w.astype(np.float64)
    m, v = np.zeros(4, np.float32), np.zeros(4, np.float32)
    T = 50
    for t in range(1, T + 1):
        oracle.adam_step_with_sqnorm([w], [m], [v], [c], LR, B1, B2, EPS, t)
        cd = c.astype(np.float64)
        want = w0 - t * LR * cd / (np.abs(cd) + EPS)
        assert np.all(np.abs(w.astype(np.float64) - want) <= t * (0.51 * _ulp32(want) + 3e-7 * LR)), t


def test_sign_flip_is_exact():
    rng = np.random.default_rng(4)
    w, m, v, g = _state(rng, 3000)
    a = [w.copy(), m.copy(), v.copy()]
    b = [-w, -m, v.copy()]
    oa = oracle.adam_step_with_sqnorm([a[0]], [a[1]], [a[2]], [g], LR, B1, B2, EPS, 9)
    ob = oracle.adam_step_with_sqnorm([b[0]], [b[1]], [b[2]], [-g], LR, B1, B2, EPS, 9)
    assert oa == ob
    assert np.array_equal(a[0], -b[0]) and np.array_equal(a[1], -b[1]) and np.array_equal(a[2], b[2])


def test_common_power_of_two_on_gradient_moments_and_eps_is_exact():
    """g -> 2^k g, m -> 2^k m, v -> 4^k v, eps -> 2^k eps leaves the weight update unchanged bit for bit
    (eps sits beside the square root, outside it: inside, it would have to scale by 4^k)."""
    rng = np.random.default_rng(5)
    w, m, v, g = _state(rng, 3000)
    ref = [w.copy(), m.copy(), v.copy()]
    oref = oracle.adam_step_with_sqnorm([ref[0]], [ref[1]], [ref[2]], [g], LR, B1, B2, EPS, 3)
    for k in (-6, 3, 10):
        s = np.float32(2.0 ** k)
        x = [w.copy(), m * s, v * s * s]
        ox = oracle.adam_step_with_sqnorm([x[0]], [x[1]], [x[2]], [g * s], LR, B1, B2, EPS * 2.0 ** k, 3)
        assert np.array_equal(x[0], ref[0])
        assert np.array_equal(x[1], ref[1] * s) and np.array_equal(x[2], ref[2] * s * s)
        assert ox == oref * 4.0 ** k


def test_omega_is_the_pinned_squared_norm_of_the_same_gradients():
    rng = np.random.default_rng(6)
    shapes = [(7, 5), (1,), (300,), (0,), (64, 3)]
    ws = [rng.normal(0, 0.02, s).astype(np.float32) for s in shapes]
    ms = [np.zeros(s, np.float32) for s in shapes]
    vs = [np.zeros(s, np.float32) for s in shapes]
    gs = [(rng.normal(0, 1, s) * 1e-3).astype(np.float32) for s in shapes]
    omega = oracle.adam_step_with_sqnorm(ws, ms, vs, gs, LR, B1, B2, EPS, 1)
    assert omega == oracle.stage_grad_sqnorm(gs)
    assert omega > 0


def test_larger_gradient_moment_means_smaller_step():
    # the second moment divides: the same mhat with a 100 times larger vhat moves the weight 10 times less
    w = np.zeros(2, np.float32)
    m = np.array([1e-3, 1e-3], np.float32)
    v = np.array([1e-6, 1e-4], np.float32)
    g = np.zeros(2, np.float32)
    oracle.adam_step_with_sqnorm([w], [m], [v], [g], LR, 0.0 + B1, B2, 0.0, 10 ** 6)     # corrections ~ 1
    assert w[0] < 0 and w[1] < 0
    assert abs(w[0] / w[1] - 10.0) < 1e-5


def test_argument_errors():
    a = np.zeros(4, np.float32)
    with pytest.raises(ValueError):
        oracle.adam_step_with_sqnorm([a], [a], [a], [np.zeros(5, np.float32)], LR)
    with pytest.raises(ValueError):
        oracle.adam_step_with_sqnorm([a], [a], [a], [a, a], LR)
    with pytest.raises(ValueError):
        oracle.adam_step_with_sqnorm([a], [a], [a], [a], LR, step=0)
    with pytest.raises(ValueError):
        oracle.adam_step_with_sqnorm([a.astype(np.float64)], [a], [a], [a], LR)
