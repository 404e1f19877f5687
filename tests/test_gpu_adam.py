"""GPU parity of the Adam step that yields omega as a by-product
(cf_adam_step_with_sqnorm) against the CPU oracle, through the C ABI.

Bars.  Moments m, v: the kernel performs the oracle's binary64 operations in the
oracle's order and rounds once, so they must be bit-identical.  Weights: the
kernel multiplies by the reciprocals of the bias corrections where the oracle
divides (relative difference below 2^-51 of the update), so at most 1 binary32
ulp and almost always 0.  omega: 1e-5 relative is the stated bar; binary64
accumulation is checked to 1e-12, and against cf_stage_grad_sqnorm (same terms,
another fixed order) to 1e-13."""
import numpy as np
import pytest
import torch

import exactmath as em
import oracle
import paper_2506_15461_amd as cf
import workloads

pytestmark = pytest.mark.gpu

LR, B1, B2, EPS = 3e-4, 0.9, 0.999, 1e-8


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda", 0)


def np_stage(stage):
    return workloads.stage_to_numpy(stage)


def draw_state(dev, shapes, seed, zero_moments=False):
    gen = torch.Generator(device=dev).manual_seed(seed)
    w = workloads.draw_weights(shapes, "f32", gen, dev)
    sig = workloads.draw_sigmas(len(shapes), np.random.default_rng(seed))
    g = workloads.draw_grads(shapes, sig, gen, dev)
    if zero_moments:
        m = [torch.zeros_like(t) for t in w]
        v = [torch.zeros_like(t) for t in w]
    else:
        m = [torch.empty_like(t).normal_(0, 1e-3, generator=gen) for t in w]
        v = [torch.empty_like(t).normal_(0, 1e-3, generator=gen).square_() for t in w]
    return w, m, v, g


def check_step(c, w, m, v, g, step, lr=LR, b1=B1, b2=B2, eps=EPS):
    """One step on the GPU and in the oracle from the same state; returns the GPU's omega."""
    ow, om, ov, og = (np_stage(x) for x in (w, m, v, g))
    want_omega = oracle.adam_step_with_sqnorm(ow, om, ov, og, lr, b1, b2, eps, step)
    sw, sm, sv, sg = (cf.Stage(c, x) for x in (w, m, v, g))
    omega = cf.cf_adam_step_with_sqnorm(c, sw, sm, sv, sg, lr, b1, b2, eps, step)
    plain = cf.cf_stage_grad_sqnorm(c, [sg])
    torch.cuda.synchronize()
    worst = 0
    for t, (gm, gv, gw) in enumerate(zip(np_stage(m), np_stage(v), np_stage(w))):
        assert np.array_equal(gm.view(np.uint32), om[t].view(np.uint32)), f"first moment, tensor {t}"
        assert np.array_equal(gv.view(np.uint32), ov[t].view(np.uint32)), f"second moment, tensor {t}"
        if gw.size:
            d = em.ulp_distance(gw.reshape(-1), ow[t].reshape(-1))
            assert int(d.max()) <= 1, f"weights, tensor {t}: {int(d.max())} ulp"
            worst = max(worst, int(d.max()))
    got = omega.item()
    assert abs(got - want_omega) <= 1e-12 * want_omega
    assert abs(got - plain.item()) <= 1e-13 * want_omega
    return got


def test_adam_ragged_stage_several_steps(dev):
    c = cf.Context(0)
    shapes = workloads.ragged_shapes(41) + [(0,), (3 * 32768 + 5,)]
    w, m, v, g = draw_state(dev, shapes, 101, zero_moments=True)
    gen = torch.Generator(device=dev).manual_seed(102)
    for step in (1, 2, 3):
        check_step(c, w, m, v, g, step)
        for t in g:                                            # a new gradient every step
            t.normal_(0, 1e-3, generator=gen)
    assert c.read_flags() == 0


@pytest.mark.parametrize("chunk_bytes", [4096, 65536, 1 << 20])
def test_adam_other_chunk_sizes_and_late_steps(dev, chunk_bytes):
    c = cf.Context(0, chunk_bytes=chunk_bytes)
    shapes = workloads.ragged_shapes(42, 8) + [(2 * chunk_bytes // 4 + 3,), (1024,), (1025,)]
    w, m, v, g = draw_state(dev, shapes, 103)
    check_step(c, w, m, v, g, 1000)
    check_step(c, w, m, v, g, 123456)
    assert c.read_flags() == 0


def test_adam_misaligned_tensors(dev):
    """Views that start 1-3 elements into their allocations: all four alike (vector path with a head and a
    tail) and all four different (element path); guard elements around the outputs stay untouched."""
    c = cf.Context(0)
    gen = torch.Generator(device=dev).manual_seed(104)
    n = 70_001
    for offs in [(1, 1, 1, 1), (3, 3, 3, 3), (0, 1, 2, 3), (2, 2, 0, 2)]:
        bases = [torch.empty(n + 8, device=dev).normal_(0, 0.02, generator=gen) for _ in range(4)]
        bases[1].mul_(0.05)
        bases[2].square_()
        bases[3].mul_(0.05)
        before = [b.clone() for b in bases]
        w, m, v, g = ([b[o:o + n]] for b, o in zip(bases, offs))
        check_step(c, w, m, v, g, 4)
        for b, b0, o in zip(bases, before, offs):
            assert torch.equal(b[:o], b0[:o]) and torch.equal(b[o + n:], b0[o + n:])
        assert torch.equal(bases[3], before[3])                 # the gradient is only read


def test_adam_special_values(dev):
    """Zero gradient from zero moments moves nothing; subnormal moments are kept; a NaN gradient poisons its
    own element only and raises the omega flag."""
    c = cf.Context(0)
    w = [torch.tensor([0.5, -0.25, 1e-3, 2.0, 1.0], device=dev)]
    m = [torch.tensor([0.0, 2.0 ** -140, 0.0, 1e-3, 0.0], device=dev)]
    v = [torch.tensor([0.0, 2.0 ** -149, 0.0, 1e-6, 0.0], device=dev)]
    g = [torch.tensor([0.0, 0.0, 2.0 ** -80, -1e19, 1e-3], device=dev)]
    ow, om, ov, og = (np_stage(x) for x in (w, m, v, g))
    want = oracle.adam_step_with_sqnorm(ow, om, ov, og, LR, B1, B2, EPS, 2)
    sw, sm, sv, sg = (cf.Stage(c, x) for x in (w, m, v, g))
    omega = cf.cf_adam_step_with_sqnorm(c, sw, sm, sv, sg, LR, B1, B2, EPS, 2)
    torch.cuda.synchronize()
    assert np.array_equal(np_stage(m)[0].view(np.uint32), om[0].view(np.uint32))
    assert np.array_equal(np_stage(v)[0].view(np.uint32), ov[0].view(np.uint32))
    assert int(em.ulp_distance(np_stage(w)[0], ow[0]).max()) <= 1
    assert w[0][0].item() == 0.5 and m[0][1].item() != 0.0
    assert abs(omega.item() - want) <= 1e-12 * want and c.read_flags() == 0
    g[0][1] = float("nan")
    w0 = w[0].clone()
    omega = cf.cf_adam_step_with_sqnorm(c, sw, sm, sv, sg, LR, B1, B2, EPS, 3)
    torch.cuda.synchronize()
    assert np.isnan(omega.item()) and torch.isnan(w[0][1]) and not torch.isnan(w[0][[0, 2, 3, 4]]).any()
    assert w[0][0] == w0[0]
    assert c.read_flags(clear=True) == cf.CF_FLAG_NONFINITE_OMEGA


def test_adam_omega_is_bit_reproducible_and_feeds_a_recovery(dev):
    """The same step from the same state twice gives the same omega bits; the omegas of two stages' optimizer
    steps drive a recovery that matches the oracle's at the oracle's omegas of the same gradients."""
    c = cf.Context(0)
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(192, 512, 2), seed=515)
    omegas, refs = [], []
    for s in (0, 2):
        refs.append(oracle.stage_grad_sqnorm(np_stage(wl.grads[s])))
        runs = []
        for rep in range(2):
            w = [t.clone() for t in wl.weights[s]]
            m = [torch.zeros_like(t) for t in w]
            v = [torch.zeros_like(t) for t in w]
            om = cf.cf_adam_step_with_sqnorm(c, cf.Stage(c, w), cf.Stage(c, m), cf.Stage(c, v), cf.Stage(c, wl.grads[s]),
                                             LR, step=1)
            runs.append(om)
        torch.cuda.synchronize()
        assert runs[0].cpu().numpy().tobytes() == runs[1].cpu().numpy().tobytes()
        omegas.append(runs[0])
    for om, ref in zip(omegas, refs):
        assert abs(om.item() - ref) <= 1e-12 * ref
    prev, nxt, lost = (cf.Stage(c, wl.weights[i]) for i in (0, 2, 1))
    cf.cf_recover_stage_weighted_avg(c, prev, nxt, omegas[0], omegas[1], lost)
    torch.cuda.synchronize()
    want = oracle.recover_stage_weighted_avg(np_stage(wl.weights[0]), np_stage(wl.weights[2]), refs[0], refs[1])
    for got, x in zip(np_stage(wl.weights[1]), want):
        assert int(em.ulp_distance(got.reshape(-1), x.reshape(-1)).max()) <= 2


def test_adam_argument_errors(dev):
    c = cf.Context(0)
    mk = lambda n, dt=torch.float32: cf.Stage(c, [torch.zeros(n, device=dev, dtype=dt)])
    w, m, v, g = mk(5000), mk(5000), mk(5000), mk(5000)

    def status(*a, **k):
        with pytest.raises(cf.CheckFreeError) as e:
            cf.cf_adam_step_with_sqnorm(c, *a, **k)
        return e.value.status
    assert status(w, m, v, mk(5001), LR) == cf.CF_ERR_SHAPE_MISMATCH
    assert status(w, m, v, mk(5000, torch.bfloat16), LR) == cf.CF_ERR_DTYPE
    assert status(w, m, v, g, LR, step=0) == cf.CF_ERR_VALUE
    assert status(w, m, v, g, LR, beta1=1.0) == cf.CF_ERR_VALUE
    assert status(w, m, v, g, float("nan")) == cf.CF_ERR_VALUE
    assert status(w, m, v, g, LR, eps=-1.0) == cf.CF_ERR_VALUE
    assert status(w, m, v, g, LR, scratch=torch.empty(8, dtype=torch.uint8, device=dev)) == cf.CF_ERR_LIMIT
    big = torch.zeros(12000, device=dev)
    assert status(cf.Stage(c, [big[:5000]]), cf.Stage(c, [big[2500:7500]]), v, g, LR) == cf.CF_ERR_ALIAS
    other = cf.Context(0)
    assert status(w, m, v, cf.Stage(other, [torch.zeros(5000, device=dev)]), LR) == cf.CF_ERR_CONTEXT
    assert cf.adam_scratch_bytes(g) >= 8 * 20 and cf.load_library().cf_adam_scratch_bytes(None) == 0
    # an empty stage: nothing to do, omega 0
    e = [cf.Stage(c, []) for _ in range(4)]
    assert cf.cf_adam_step_with_sqnorm(c, *e, LR).item() == 0.0
    torch.cuda.synchronize()
    assert c.read_flags() == 0


def test_adam_full_size_stage(dev):
    """The 1.5B-shape stage (205 537 280 elements) at full size against the oracle."""
    c = cf.Context(0)
    shapes = workloads.SPECS[3].shape.tensor_shapes()
    w, m, v, g = draw_state(dev, shapes, 105)
    got = check_step(c, w, m, v, g, 17)
    assert got > 0 and c.read_flags() == 0
