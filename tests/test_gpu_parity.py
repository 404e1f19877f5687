"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on
the same seeded inputs.

Bars: stage squared norms within 1e-5 relative; fp32 blended weights within
2 ulp; bf16 blended weights within 1 bf16 ulp; copies bit-exact.  The two
floating-point bars cannot both hold end to end (a 1e-5 relative change of omega
moves most blended elements by far more than 2 ulp), so the blend is compared at
one common omega pair -- the oracle's, uploaded to the device -- and the path as
it runs in production (omegas stay on the device) is checked against the same
oracle result within its first-order sensitivity to the omegas.  Expected values
never come from the GPU; the one place where the oracle is *given* a GPU result
is test_two_recoveries_on_two_streams_at_once, which hands the GPU's own omegas
(already checked against the oracle's to 1e-5) to the oracle's blend so that the
blend of that run can be compared to the ulp bar.
"""
import ctypes

import numpy as np
import pytest
import torch

import exactmath as em
import oracle
import paper_2506_15461_amd as cf
import workloads

pytestmark = pytest.mark.gpu

NORM_RTOL = 1e-5
F32_ULP = 2
BF16_ULP = 1
ORACLE_THREADS = 16


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda", 0)


@pytest.fixture(scope="module")
def ctx():
    c = cf.Context(0)
    yield c
    torch.cuda.synchronize()
    assert c.read_flags(clear=True) in (0, 1, 2, 3)


def np_stage(stage):
    return workloads.stage_to_numpy(stage)


def assert_blend_close(got_stage, want_stage, piece=1 << 25):
    worst = 0
    for t, (g, w) in enumerate(zip(got_stage, want_stage)):
        g, w = g.reshape(-1), w.reshape(-1)
        bar = F32_ULP if g.dtype == np.float32 else BF16_ULP
        for lo in range(0, g.size, piece):                     # in pieces: the distance needs int64 temporaries
            d = em.ulp_distance(g[lo:lo + piece], w[lo:lo + piece])
            m = int(d.max())
            assert m <= bar, f"tensor {t}: {m} ulp (bar {bar}), {int((d > bar).sum())} elements off from {lo}"
            worst = max(worst, m)
    return worst


def as_f64(a):
    """Values of an fp32 array or of bf16 bit patterns, as float64."""
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def assert_end_to_end_within_sensitivity_bound(got_stage, want_stage, prev, nxt, omega_gpu, omega_ref, piece=1 << 25):
    """End to end (GPU omegas -> GPU blend against oracle omegas -> oracle blend) the result moves
    with the omegas: out = b + alpha (a - b), alpha = w_p / (w_p + w_n), so to first order
    |d out| <= alpha beta |a - b| (|d_p| + |d_n|), d_* the relative errors of the omegas; on top of
    that each side rounds once to the storage type."""
    wp, wn = omega_ref
    alpha, beta = wp / (wp + wn), wn / (wp + wn)
    dp, dn = abs(omega_gpu[0] - wp) / wp, abs(omega_gpu[1] - wn) / wn
    for g, w, a, b in zip(got_stage, want_stage, prev, nxt):
        g, w, a, b = (x.reshape(-1) for x in (g, w, a, b))
        for lo in range(0, g.size, piece):
            gv, wv, av, bv = (as_f64(x[lo:lo + piece]) for x in (g, w, a, b))
            ulp = np.spacing(np.abs(wv).astype(np.float32)).astype(np.float64) * (65536.0 if g.dtype == np.uint16 else 1.0)
            bound = 1.01 * alpha * beta * np.abs(av - bv) * (dp + dn) + 2.0 * ulp
            assert np.all(np.abs(gv - wv) <= bound)


def check_recovery(ctx, wl, prev_i, lost_i, next_i):
    """The whole hot path against the oracle, three ways.  Nothing the oracle is given comes from
    the GPU: (1) the GPU's omegas against the oracle's; (2) the GPU's blend at the ORACLE's omegas
    (uploaded) against the oracle's blend at the same omegas, to the ulp bar; (3) the path as it
    runs in production -- omegas stay on the device and feed the blend -- against the same oracle
    result, within the first-order sensitivity to the omegas' error."""
    dev = wl.weights[prev_i][0].device
    prev_np, next_np = np_stage(wl.weights[prev_i]), np_stage(wl.weights[next_i])
    refs = [oracle.stage_grad_sqnorm(np_stage(wl.grads[s]), ORACLE_THREADS) for s in (prev_i, next_i)]
    want = oracle.recover_stage_weighted_avg(prev_np, next_np, refs[0], refs[1], ORACLE_THREADS)

    prev, nxt, lost = (cf.Stage(ctx, wl.weights[i]) for i in (prev_i, next_i, lost_i))
    gp, gn = cf.Stage(ctx, wl.grads[prev_i]), cf.Stage(ctx, wl.grads[next_i])
    # (1)
    omega_dev = cf.cf_stage_grad_sqnorm(ctx, [gp, gn])
    omega = omega_dev.cpu().numpy()
    for k in range(2):
        assert abs(omega[k] - refs[k]) <= NORM_RTOL * refs[k], (k, omega[k], refs[k])
    # (2)
    for t in wl.weights[lost_i]:
        t.fill_(float("nan"))                      # the lost stage's content is gone
    omega_ref_dev = torch.tensor(refs, dtype=torch.float64, device=dev)
    cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, omega_ref_dev[0:1], omega_ref_dev[1:2], lost)
    torch.cuda.synchronize()
    worst = assert_blend_close(np_stage(wl.weights[lost_i]), want)
    # (3)
    for t in wl.weights[lost_i]:
        t.fill_(float("nan"))
    cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, omega_dev[0:1], omega_dev[1:2], lost)
    torch.cuda.synchronize()
    assert_end_to_end_within_sensitivity_bound(np_stage(wl.weights[lost_i]), want, prev_np, next_np, omega, refs)
    return omega, worst


# ----------------------------------------------------------------------------
# squared norms
# ----------------------------------------------------------------------------

def test_sqnorm_ragged_stage_and_empty_stages(ctx, dev):
    gen = torch.Generator(device=dev).manual_seed(7)
    shapes = workloads.ragged_shapes(1)
    stages = []
    for s in range(3):
        sig = workloads.draw_sigmas(len(shapes), np.random.default_rng(s))
        stages.append(workloads.draw_grads(shapes, sig, gen, dev))
    stages.insert(1, [])                                            # a stage with no tensors
    stages.append([torch.empty(0, device=dev), torch.ones(3, device=dev)])
    handles = [cf.Stage(ctx, g) for g in stages]
    omega = cf.cf_stage_grad_sqnorm(ctx, handles).cpu().numpy()
    for k, g in enumerate(stages):
        ref = oracle.stage_grad_sqnorm(np_stage(g))
        assert abs(omega[k] - ref) <= NORM_RTOL * ref, (k, omega[k], ref)
    assert omega[1] == 0.0 and omega[4] == 3.0


def test_sqnorm_closed_forms(ctx, dev):
    n = 100_003
    c = torch.full((n,), 2.0 ** -7, device=dev)
    ramp = torch.arange(1, 2049, device=dev, dtype=torch.float32)
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, [c]), cf.Stage(ctx, [ramp])]).cpu().numpy()
    assert omega[0] == n * 2.0 ** -14                     # every partial sum is exact in fp32
    m = 2048
    assert abs(omega[1] - m * (m + 1) * (2 * m + 1) / 6) <= NORM_RTOL * omega[1]


def test_sqnorm_is_bitwise_reproducible_and_launch_shape_independent(dev):
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(192, 512, 2))
    results = []
    for tuning in ({}, {"sqnorm_blocks_per_cu": 1}, {"sqnorm_blocks_per_cu": 3}, {"sqnorm_blocks_per_cu": 8},
                   {"sqnorm_blocks_per_cu": 65}):
        c = cf.Context(0, **tuning)
        handles = [cf.Stage(c, g) for g in wl.grads]
        for rep in range(3):
            results.append(cf.cf_stage_grad_sqnorm(c, handles).cpu().numpy().tobytes())
    assert len(set(results)) == 1


def test_sqnorm_misaligned_views(ctx, dev):
    gen = torch.Generator(device=dev).manual_seed(9)
    base = torch.empty(200_000, device=dev).normal_(0, 1e-3, generator=gen)
    views = [base[1:70_001], base[70_002:70_003], base[70_003:140_010], base[140_011:199_999]]
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, views)]).cpu().numpy()
    ref = oracle.stage_grad_sqnorm(np_stage(views))
    assert abs(omega[0] - ref) <= NORM_RTOL * ref


@pytest.mark.parametrize("chunk_bytes", [131072, 4 << 20])
def test_sqnorm_data_built_against_binary32_accumulation(dev, chunk_bytes):
    """Every accumulator chain starts with 1.0 and is then fed squares of just under half a binary32
    ulp of 1.0: a binary32 accumulator would round every one of them away (a relative loss of about
    1e-6 at the default chunk size and more than the 1e-5 bar at the largest).  Accumulation in
    binary64 keeps them at every chunk size the tuning accepts."""
    c = cf.Context(0, chunk_bytes=chunk_bytes)
    chunk = chunk_bytes // 4                             # elements per chunk
    iters = chunk // 1024                                # vectors per lane
    n_chunks = 3 if chunk_bytes > 131072 else 40
    g = torch.full((n_chunks * chunk,), 2.0 ** -12.6, device=dev)
    v = g.view(n_chunks, iters, 256, 4)                  # [chunk, iteration, lane, vector slot]
    v[:, 0, :, :] = 1.0
    omega = cf.cf_stage_grad_sqnorm(c, [cf.Stage(c, [g])]).item()
    ref = oracle.stage_grad_sqnorm([workloads.to_numpy(g)])
    # The oracle adds the same tiny term to a large running sum over a million times, always rounding the
    # same way: its own error here is a good part of its worst case n * 2^-53.  The closed form is exact.
    from fractions import Fraction
    small = Fraction(float(np.float32(2.0 ** -12.6))) ** 2
    exact = n_chunks * 1024 + n_chunks * (chunk - 1024) * small
    assert abs(Fraction(omega) - exact) <= exact * Fraction(1, 10 ** 13)
    assert abs(Fraction(ref) - exact) <= exact * g.numel() * Fraction(1, 2 ** 53)
    assert abs(omega - ref) <= NORM_RTOL * ref
    assert c.read_flags() == 0


def test_sqnorm_gradients_far_outside_the_binary32_range_of_squares(ctx, dev):
    """|g| near 2^-80 (squares far below the smallest binary32 number) and near 1e19 (squares above
    the largest): in binary64 neither vanishes nor overflows, and the result matches the oracle."""
    gen = torch.Generator(device=dev).manual_seed(61)
    tiny = torch.empty(300_001, device=dev).normal_(0, 1.0, generator=gen) * 2.0 ** -80
    huge = torch.empty(70_003, device=dev).normal_(0, 1.0, generator=gen) * 1e19
    edge = torch.tensor([2.0 ** -149, -2.0 ** -126, 3.4028234663852886e38, 1.0], device=dev)
    tiny16 = (torch.empty(40_001, device=dev).normal_(0, 1.0, generator=gen) * 2.0 ** -100).to(torch.bfloat16)
    stages = [[tiny], [huge], [edge], [tiny16], [tiny, huge]]
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, s) for s in stages]).cpu().numpy()
    for k, st in enumerate(stages):
        ref = oracle.stage_grad_sqnorm(np_stage(st))
        assert ref > 0 and np.isfinite(ref)
        assert abs(omega[k] - ref) <= 1e-12 * ref, (k, omega[k], ref)
    assert omega[0] < 1e-40 and omega[1] > 1e40
    torch.cuda.synchronize()
    assert ctx.read_flags() == 0


def test_sqnorm_nonfinite_raises_flag(dev):
    c = cf.Context(0)
    g = torch.ones(5000, device=dev)
    g[1234] = float("inf")
    omega = cf.cf_stage_grad_sqnorm(c, [cf.Stage(c, [g]), cf.Stage(c, [torch.ones(10, device=dev)])]).cpu().numpy()
    assert np.isinf(omega[0]) and omega[1] == 10.0
    assert c.read_flags(clear=True) & cf.CF_FLAG_NONFINITE_OMEGA
    assert c.read_flags() == 0


def test_sqnorm_more_stages_than_one_launch_holds(ctx, dev):
    stages = [[torch.full((k + 1,), 2.0, device=dev)] for k in range(70)]
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, s) for s in stages]).cpu().numpy()
    assert np.array_equal(omega, 4.0 * np.arange(1, 71))


def test_sqnorm_per_tensor(ctx, dev):
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(192, 512, 2))
    grads = wl.grads[0] + [torch.empty(0, device=dev), torch.full((5,), 2.0, device=dev)]
    st = cf.Stage(ctx, grads)
    omega, per = cf.cf_stage_grad_sqnorm_per_tensor(ctx, st)
    omega2 = cf.cf_stage_grad_sqnorm(ctx, [st])
    torch.cuda.synchronize()
    assert omega.cpu().numpy().tobytes() == omega2.cpu().numpy().tobytes()       # same bits as the plain call
    per = per.cpu().numpy()
    ref = oracle.tensor_grad_sqnorms(np_stage(grads))
    assert len(per) == len(ref) == 20
    for t in range(len(ref)):
        assert abs(per[t] - ref[t]) <= NORM_RTOL * ref[t], (t, per[t], ref[t])
    assert per[18] == 0.0 and per[19] == 20.0
    assert abs(per.sum() - omega.item()) <= 1e-12 * omega.item()
    # a stage of empty tensors only, and a stage with no tensors
    o, p = cf.cf_stage_grad_sqnorm_per_tensor(ctx, cf.Stage(ctx, [torch.empty(0, device=dev)] * 3))
    assert o.item() == 0.0 and p.cpu().tolist() == [0.0, 0.0, 0.0]
    o, p = cf.cf_stage_grad_sqnorm_per_tensor(ctx, cf.Stage(ctx, []))
    assert o.item() == 0.0 and p.numel() == 0


def test_sqnorm_bf16_gradients(ctx, dev):
    gen = torch.Generator(device=dev).manual_seed(17)
    shapes = workloads.ragged_shapes(8) + [(300_001,)]
    g16 = [torch.empty(s, device=dev).normal_(0, 1e-3, generator=gen).to(torch.bfloat16) for s in shapes]
    mixed = [g16[0], torch.empty(70_001, device=dev).normal_(0, 1e-3, generator=gen), g16[-1][5:]]
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, g16), cf.Stage(ctx, mixed)]).cpu().numpy()
    for k, st in enumerate((g16, mixed)):
        ref = oracle.stage_grad_sqnorm(np_stage(st))
        assert abs(omega[k] - ref) <= NORM_RTOL * ref, (k, omega[k], ref)


# ----------------------------------------------------------------------------
# weighted-average recovery
# ----------------------------------------------------------------------------

def _omega(dev, wp, wn):
    return torch.tensor([wp, wn], dtype=torch.float64, device=dev)


def _draw_pair(dev, shapes, dtype, seed):
    gen = torch.Generator(device=dev).manual_seed(seed)
    return (workloads.draw_weights(shapes, dtype, gen, dev), workloads.draw_weights(shapes, dtype, gen, dev))


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blend_ragged_stage(ctx, dev, dtype):
    shapes = workloads.ragged_shapes(2)
    a, b = _draw_pair(dev, shapes, dtype, 21)
    out = [torch.full_like(t, float("nan")) for t in a]
    for wp, wn in [(3.7e-3, 1.9e-2), (1.0, 1e-9), (5e-11, 7e-4), (123.0, 123.0)]:
        w = _omega(dev, wp, wn)
        cf.cf_recover_stage_weighted_avg(ctx, cf.Stage(ctx, a), cf.Stage(ctx, b), w[0:1], w[1:2], cf.Stage(ctx, out))
        torch.cuda.synchronize()
        want = oracle.recover_stage_weighted_avg(np_stage(a), np_stage(b), wp, wn)
        assert_blend_close(np_stage(out), want)


@pytest.mark.parametrize("chunk_bytes", [4096, 8192, 65536, 1 << 20, 4 << 20])
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blend_copy_and_sqnorm_for_other_chunk_sizes(dev, dtype, chunk_bytes):
    """Chunk and tile boundaries move with the chunk size; results must not."""
    c = cf.Context(0, chunk_bytes=chunk_bytes)
    shapes = workloads.ragged_shapes(5) + [(3 * 65536 + 17,), (1024,), (2048,), (1025,), (262144,),
                                           ((1 << 20) + 9,)]          # the last one crosses even a 4 MiB chunk
    a, b = _draw_pair(dev, shapes, dtype, 27)
    out = [torch.full_like(t, float("nan")) for t in a]
    w = _omega(dev, 3.7e-3, 1.9e-2)
    cf.cf_recover_stage_weighted_avg(c, cf.Stage(c, a), cf.Stage(c, b), w[0:1], w[1:2], cf.Stage(c, out))
    torch.cuda.synchronize()
    assert_blend_close(np_stage(out), oracle.recover_stage_weighted_avg(np_stage(a), np_stage(b), 3.7e-3, 1.9e-2))
    dst = [torch.zeros_like(t) for t in a]
    cf.cf_copy_stage(c, cf.Stage(c, a), cf.Stage(c, dst))
    torch.cuda.synchronize()
    for g, wnt in zip(np_stage(dst), oracle.copy_stage(np_stage(a))):
        assert g.tobytes() == wnt.tobytes()
    if dtype == "f32":
        omega = cf.cf_stage_grad_sqnorm(c, [cf.Stage(c, a)]).cpu().numpy()
        ref = oracle.stage_grad_sqnorm(np_stage(a))
        assert abs(omega[0] - ref) <= NORM_RTOL * ref
    assert c.read_flags() == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blend_special_cases_are_exact(ctx, dev, dtype):
    shapes = workloads.ragged_shapes(3)
    a, b = _draw_pair(dev, shapes, dtype, 22)
    out = [torch.full_like(t, float("nan")) for t in a]
    sa, sb, so = cf.Stage(ctx, a), cf.Stage(ctx, b), cf.Stage(ctx, out)
    bits = torch.int32 if dtype == "f32" else torch.int16

    def same(x, y):
        return all(torch.equal(p.view(bits), q.view(bits)) for p, q in zip(x, y))

    w = _omega(dev, 3.7e-3, 0.0)                     # omega_{i+1} = 0: copy of the previous stage
    cf.cf_recover_stage_weighted_avg(ctx, sa, sb, w[0:1], w[1:2], so)
    assert same(out, a)
    w = _omega(dev, 0.0, 2.5)
    cf.cf_recover_stage_weighted_avg(ctx, sa, sb, w[0:1], w[1:2], so)
    assert same(out, b)
    w = _omega(dev, 3.7e-3, 1.9e-2)                  # identical neighbours give back that stage
    cf.cf_recover_stage_weighted_avg(ctx, sa, sa, w[0:1], w[1:2], so)
    assert same(out, a)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_recovery_with_host_weights_matches_device_weights_and_oracle(ctx, dev, dtype):
    """The strategies the paper compares: uniform average, copy of one neighbour,
    and explicit weights; the host-weight entry point must give the same bits as
    the device-weight one."""
    shapes = workloads.ragged_shapes(6)
    a, b = _draw_pair(dev, shapes, dtype, 41)
    out_h = [torch.full_like(t, float("nan")) for t in a]
    out_d = [torch.full_like(t, float("nan")) for t in a]
    sa, sb, sh, sd = cf.Stage(ctx, a), cf.Stage(ctx, b), cf.Stage(ctx, out_h), cf.Stage(ctx, out_d)
    bits = torch.int32 if dtype == "f32" else torch.int16
    for wp, wn in [(1.0, 1.0), (0.37, 0.37), (1.0, 0.0), (0.0, 1.0), (3.7e-3, 1.9e-2)]:
        cf.cf_recover_stage_with_weights(ctx, sa, sb, wp, wn, sh)
        w = _omega(dev, wp, wn)
        cf.cf_recover_stage_weighted_avg(ctx, sa, sb, w[0:1], w[1:2], sd)
        torch.cuda.synchronize()
        assert all(torch.equal(x.view(bits), y.view(bits)) for x, y in zip(out_h, out_d))
        assert_blend_close(np_stage(out_h), oracle.recover_stage_weighted_avg(np_stage(a), np_stage(b), wp, wn))
        if wn == 0.0:
            assert all(torch.equal(x.view(bits), y.view(bits)) for x, y in zip(out_h, a))      # copy previous
        if wp == 0.0:
            assert all(torch.equal(x.view(bits), y.view(bits)) for x, y in zip(out_h, b))


def test_blend_misaligned_and_in_place(ctx, dev):
    gen = torch.Generator(device=dev).manual_seed(23)
    n = 150_001
    A = torch.empty(n + 8, device=dev).normal_(0, 0.02, generator=gen)
    B = torch.empty(n + 8, device=dev).normal_(0, 0.02, generator=gen)
    O = torch.full((n + 8,), float("nan"), device=dev)
    w = _omega(dev, 3.7e-3, 1.9e-2)
    for oa, ob, oo in [(1, 1, 1), (3, 3, 3), (1, 2, 3), (0, 0, 2)]:
        a, b, o = A[oa:oa + n], B[ob:ob + n], O[oo:oo + n]
        O.fill_(float("nan"))
        cf.cf_recover_stage_weighted_avg(ctx, cf.Stage(ctx, [a]), cf.Stage(ctx, [b]), w[0:1], w[1:2], cf.Stage(ctx, [o]))
        torch.cuda.synchronize()
        want = oracle.recover_stage_weighted_avg(np_stage([a]), np_stage([b]), 3.7e-3, 1.9e-2)
        assert_blend_close(np_stage([o]), want)
        assert torch.isnan(O[:oo]).all() and torch.isnan(O[oo + n:]).all()      # nothing outside the tensor
    # in place: the lost stage's memory is the previous stage's
    a, b = A[:n].clone(), B[:n].clone()
    want = oracle.recover_stage_weighted_avg(np_stage([a]), np_stage([b]), 3.7e-3, 1.9e-2)
    sa = cf.Stage(ctx, [a])
    cf.cf_recover_stage_weighted_avg(ctx, sa, cf.Stage(ctx, [b]), w[0:1], w[1:2], sa)
    torch.cuda.synchronize()
    assert_blend_close(np_stage([a]), want)


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blend_subnormals_extremes_and_nonfinite_weights(ctx, dev, dtype):
    if dtype == "f32":
        vals_a = [2.0 ** -149, -2.0 ** -140, 3.4028234663852886e38, 0.0, -0.0, float("nan"), float("inf"), 1.0,
                  2.0 ** -126, 1e-41, -3e-39]
        vals_b = [2.0 ** -149, 2.0 ** -140, 3.4028234663852886e38, -0.0, -0.0, 1.0, 1.0, float("-inf"),
                  2.0 ** -127, -2e-41, 1e-39]
        a = torch.tensor(vals_a, dtype=torch.float32, device=dev)
        b = torch.tensor(vals_b, dtype=torch.float32, device=dev)
    else:
        # every bf16 bit pattern against a shuffled copy of the same set
        allbits = torch.arange(65536, dtype=torch.int32, device=dev).to(torch.int16)
        perm = torch.randperm(65536, generator=torch.Generator(device=dev).manual_seed(5), device=dev)
        a = allbits.view(torch.bfloat16)
        b = allbits[perm].contiguous().view(torch.bfloat16)
    out = torch.zeros_like(a)
    for wp, wn in [(1.0, 1.0), (3.7e-3, 1.9e-2), (1.0, 3.0)]:
        w = _omega(dev, wp, wn)
        cf.cf_recover_stage_weighted_avg(ctx, cf.Stage(ctx, [a]), cf.Stage(ctx, [b]), w[0:1], w[1:2], cf.Stage(ctx, [out]))
        torch.cuda.synchronize()
        want = oracle.recover_stage_weighted_avg(np_stage([a]), np_stage([b]), wp, wn)
        assert_blend_close(np_stage([out]), want)
    if dtype == "f32":
        w = _omega(dev, 1.0, 1.0)
        cf.cf_recover_stage_weighted_avg(ctx, cf.Stage(ctx, [a]), cf.Stage(ctx, [b]), w[0:1], w[1:2], cf.Stage(ctx, [out]))
        o = out.cpu().numpy()
        assert o[0] == np.float32(2.0 ** -149) and o[8] != 0        # subnormal results are kept


@pytest.mark.parametrize("wp,wn", [(0.0, 0.0), (float("nan"), 1.0), (1.0, float("inf")), (-1.0, 2.0),
                                   (1e-320, 1e-320), (1e308, 1e308)])
def test_blend_degenerate_omega_falls_back_to_uniform_average(dev, wp, wn):
    c = cf.Context(0)
    a, b = _draw_pair(dev, workloads.ragged_shapes(4, 6), "f32", 24)
    out = [torch.full_like(t, float("nan")) for t in a]
    w = _omega(dev, wp, wn)
    cf.cf_recover_stage_weighted_avg(c, cf.Stage(c, a), cf.Stage(c, b), w[0:1], w[1:2], cf.Stage(c, out))
    torch.cuda.synchronize()
    want = oracle.recover_stage_weighted_avg(np_stage(a), np_stage(b), wp, wn)
    assert_blend_close(np_stage(out), want)
    assert c.read_flags(clear=True) == cf.CF_FLAG_DEGENERATE_OMEGA
    w = _omega(dev, 1.0, 2.0)
    cf.cf_recover_stage_weighted_avg(c, cf.Stage(c, a), cf.Stage(c, b), w[0:1], w[1:2], cf.Stage(c, out))
    assert c.read_flags() == 0


def test_blend_argument_errors(ctx, dev):
    a = [torch.zeros(100, device=dev), torch.zeros(7, device=dev)]
    b = [torch.zeros(100, device=dev), torch.zeros(7, device=dev)]
    w = _omega(dev, 1.0, 1.0)
    sa, sb = cf.Stage(ctx, a), cf.Stage(ctx, b)
    cases = [
        ([torch.zeros(100, device=dev), torch.zeros(8, device=dev)], cf.CF_ERR_SHAPE_MISMATCH),
        ([torch.zeros(100, device=dev)], cf.CF_ERR_SHAPE_MISMATCH),
        ([torch.zeros(100, device=dev), torch.zeros(7, device=dev, dtype=torch.bfloat16)], cf.CF_ERR_SHAPE_MISMATCH),
    ]
    for out, code in cases:
        with pytest.raises(cf.CheckFreeError) as e:
            cf.cf_recover_stage_weighted_avg(ctx, sa, sb, w[0:1], w[1:2], cf.Stage(ctx, out))
        assert e.value.status == code
    big = torch.zeros(300, device=dev)
    with pytest.raises(cf.CheckFreeError) as e:          # output overlaps an input, shifted
        cf.cf_recover_stage_weighted_avg(ctx, cf.Stage(ctx, [big[0:100]]), cf.Stage(ctx, [big[200:300]]),
                                         w[0:1], w[1:2], cf.Stage(ctx, [big[50:150]]))
    assert e.value.status == cf.CF_ERR_ALIAS
    with pytest.raises(cf.CheckFreeError) as e:          # output tensors overlap one another
        cf.cf_recover_stage_weighted_avg(ctx, sa, sb, w[0:1], w[1:2], cf.Stage(ctx, [big[0:100], big[98:105]]))
    assert e.value.status == cf.CF_ERR_ALIAS
    other = cf.Context(0)
    with pytest.raises(cf.CheckFreeError) as e:
        cf.cf_recover_stage_weighted_avg(other, sa, sb, w[0:1], w[1:2], sa)
    assert e.value.status == cf.CF_ERR_CONTEXT
    with pytest.raises(cf.CheckFreeError) as e:
        cf.Stage(ctx, [torch.zeros(4, device=dev, dtype=torch.float16)])
    assert e.value.status == cf.CF_ERR_DTYPE


# ----------------------------------------------------------------------------
# CheckFree+ copy
# ----------------------------------------------------------------------------

def test_copy_bit_exact_with_guard_bands(ctx, dev):
    gen = torch.Generator(device=dev).manual_seed(31)
    n = 200_003
    raw = torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int32, device=dev, generator=gen)
    raw[:6] = torch.tensor([0x7FC00001, -0x3EDCBB, 0x7F800001, -2 ** 31, 1, -0x7F800001], dtype=torch.int32)
    src = raw.view(torch.float32)
    half = torch.randint(-2 ** 15, 2 ** 15 - 1, (4099,), dtype=torch.int16, device=dev, generator=gen).view(torch.bfloat16)
    for so, do in [(0, 0), (1, 1), (1, 3), (2, 0)]:
        D = torch.full((n + 16,), float("nan"), device=dev)
        DH = torch.zeros(4099 + 16, dtype=torch.bfloat16, device=dev)
        s = [src[so:], half[so:], torch.empty(0, device=dev)]
        d = [D[do:do + n - so], DH[do:do + 4099 - so], torch.empty(0, device=dev)]
        before = D.clone()
        cf.cf_copy_stage(ctx, cf.Stage(ctx, s), cf.Stage(ctx, d))
        torch.cuda.synchronize()
        want = oracle.copy_stage(np_stage(s))
        for g, wnt in zip(np_stage(d), want):
            assert g.tobytes() == wnt.tobytes()
        assert torch.equal(D[:do].view(torch.int32), before[:do].view(torch.int32))
        assert torch.equal(D[do + n - so:].view(torch.int32), before[do + n - so:].view(torch.int32))
        assert (DH[:do] == 0).all() and (DH[do + 4099 - so:] == 0).all()


def test_hot_calls_can_be_captured_in_a_hip_graph(dev):
    """Callers under graph capture: the three hot calls enqueue kernels only (no
    allocation, no copy, no synchronisation), so a captured recovery replays
    correctly on changed inputs.  Replays alternate with eager work and are each
    compared with the eager result bit for bit."""
    c = cf.Context(0)
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(192, 512, 2))
    gp, gn = cf.Stage(c, wl.grads[0]), cf.Stage(c, wl.grads[2])
    prev, nxt = cf.Stage(c, wl.weights[0]), cf.Stage(c, wl.weights[2])
    out_g = [torch.zeros_like(t) for t in wl.weights[1]]
    out_e = [torch.zeros_like(t) for t in wl.weights[1]]
    cp_g = [torch.zeros_like(t) for t in wl.weights[1]]
    lost_g, lost_e, copy_g = cf.Stage(c, out_g), cf.Stage(c, out_e), cf.Stage(c, cp_g)
    om_g = torch.zeros(2, dtype=torch.float64, device=dev)
    om_e = torch.zeros(2, dtype=torch.float64, device=dev)

    def recovery(omega, lost, stream):
        cf.cf_stage_grad_sqnorm(c, [gp, gn], omega, stream)
        cf.cf_recover_stage_weighted_avg(c, prev, nxt, omega[0:1], omega[1:2], lost, stream)

    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    torch.cuda.synchronize()                               # the stage tables were written on the current stream
    with torch.cuda.stream(side):
        recovery(om_g, lost_g, side)                       # warm-up outside the capture
        side.synchronize()
        graph.capture_begin()
        recovery(om_g, lost_g, side)
        cf.cf_copy_stage(c, lost_g, copy_g, side)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(4):
        for g in wl.grads[0]:                              # new gradients => new omegas => new blend
            g.mul_(1.5 + rep)
        wl.weights[0][0].add_(0.001 * (rep + 1))
        torch.cuda.synchronize()
        recovery(om_e, lost_e, torch.cuda.current_stream())
        torch.cuda.synchronize()
        for t in out_g + cp_g:
            t.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert om_g.cpu().numpy().tobytes() == om_e.cpu().numpy().tobytes(), rep
        for x, y, z in zip(out_g, out_e, cp_g):
            assert torch.equal(x.view(torch.int32), y.view(torch.int32)), rep
            assert torch.equal(z.view(torch.int32), y.view(torch.int32)), rep
    assert c.read_flags() == 0


@pytest.mark.parametrize("seed", range(12))
def test_random_stages_all_operations(dev, seed):
    """Seeded random stages: mixed fp32 / bf16 tensors, sizes from 0 to a few
    chunks, random element offsets into their allocations (so the three streams
    of a blend are sometimes mutually misaligned), random chunk size."""
    rng = np.random.default_rng(1000 + seed)
    gen = torch.Generator(device=dev).manual_seed(2000 + seed)
    chunk_bytes = int(rng.choice([4096, 16384, 131072]))
    c = cf.Context(0, chunk_bytes=chunk_bytes)
    n_tensors = int(rng.integers(1, 9))
    prev, nxt, out, grads, guards = [], [], [], [], []
    for _ in range(n_tensors):
        kind = rng.random()
        n = 0 if kind < 0.1 else int(rng.integers(1, 40)) if kind < 0.3 else int(rng.integers(1, 5 * chunk_bytes // 4))
        dtype = torch.bfloat16 if rng.random() < 0.4 else torch.float32
        same_offsets = rng.random() < 0.6
        offs = [int(rng.integers(0, 9))] * 3 if same_offsets else [int(x) for x in rng.integers(0, 9, 3)]
        bufs = []
        for k in range(3):
            base = torch.empty(n + 16, device=dev).normal_(0, 0.02, generator=gen).to(dtype)
            bufs.append(base)
        out_base = torch.full((n + 16,), float("nan"), device=dev).to(dtype)
        prev.append(bufs[0][offs[0]:offs[0] + n])
        nxt.append(bufs[1][offs[1]:offs[1] + n])
        out.append(out_base[offs[2]:offs[2] + n])
        guards.append((out_base, offs[2], n))
        g = torch.empty(n + 8, device=dev).normal_(0, float(10.0 ** rng.uniform(-5, -2)), generator=gen)
        grads.append(g[offs[0] % 8:offs[0] % 8 + n] if rng.random() < 0.8 else g[:n].to(torch.bfloat16))
    wp, wn = (10.0 ** rng.uniform(-8, 2, 2)).tolist()
    sp, sn, so, sg = cf.Stage(c, prev), cf.Stage(c, nxt), cf.Stage(c, out), cf.Stage(c, grads)
    omega, per = cf.cf_stage_grad_sqnorm_per_tensor(c, sg)
    cf.cf_recover_stage_with_weights(c, sp, sn, wp, wn, so)
    torch.cuda.synchronize()
    ref = oracle.stage_grad_sqnorm(np_stage(grads))
    assert abs(omega.item() - ref) <= NORM_RTOL * ref
    for got, want in zip(per.cpu().numpy(), oracle.tensor_grad_sqnorms(np_stage(grads))):
        assert abs(got - want) <= NORM_RTOL * want
    assert_blend_close(np_stage(out), oracle.recover_stage_weighted_avg(np_stage(prev), np_stage(nxt), wp, wn))
    for base, off, n in guards:                               # nothing written outside the tensors
        assert torch.isnan(base[:off].float()).all() and torch.isnan(base[off + n:].float()).all()
    cf.cf_copy_stage(c, sp, so)
    torch.cuda.synchronize()
    for g, w in zip(np_stage(out), oracle.copy_stage(np_stage(prev))):
        assert g.tobytes() == w.tobytes()
    for base, off, n in guards:
        assert torch.isnan(base[:off].float()).all() and torch.isnan(base[off + n:].float()).all()
    assert c.read_flags() == 0


def test_plain_c_client_on_the_device():
    """The C99 client drives the whole path through the C ABI with hipMalloc'd
    buffers: no PyTorch, no C++ on the caller's side."""
    import os
    import subprocess
    from paper_2506_15461_amd import build as hip_build
    assert os.path.exists(hip_build.C_SMOKE_BIN), "run __graft_entry__.build() first"
    r = subprocess.run([hip_build.C_SMOKE_BIN], capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert "c_abi_smoke: ok" in r.stdout


def test_two_recoveries_on_two_streams_at_once(dev):
    """Independent recoveries issued on two streams (default priority), one
    context each, interleaved call by call."""
    wls = [workloads.make_workload(1, device=dev, shape=workloads.StageShape(256, 704, 2), seed=900 + i) for i in (0, 1)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    ctxs = [cf.Context(0), cf.Context(0)]
    torch.cuda.synchronize()
    handles, omegas = [], []
    for wl, c in zip(wls, ctxs):
        for t in wl.weights[1]:
            t.fill_(float("nan"))
        handles.append(dict(gp=cf.Stage(c, wl.grads[0]), gn=cf.Stage(c, wl.grads[2]), prev=cf.Stage(c, wl.weights[0]),
                            nxt=cf.Stage(c, wl.weights[2]), lost=cf.Stage(c, wl.weights[1])))
        omegas.append(torch.zeros(2, dtype=torch.float64, device=dev))
    torch.cuda.synchronize()
    for rep in range(5):
        for h, c, om, st in zip(handles, ctxs, omegas, streams):
            cf.cf_stage_grad_sqnorm(c, [h["gp"], h["gn"]], om, st)
        for h, c, om, st in zip(handles, ctxs, omegas, streams):
            cf.cf_recover_stage_weighted_avg(c, h["prev"], h["nxt"], om[0:1], om[1:2], h["lost"], st)
    torch.cuda.synchronize()
    for wl, om in zip(wls, omegas):
        w = om.cpu().numpy()
        for k, s in enumerate((0, 2)):
            ref = oracle.stage_grad_sqnorm(np_stage(wl.grads[s]))
            assert abs(w[k] - ref) <= NORM_RTOL * ref
        want = oracle.recover_stage_weighted_avg(np_stage(wl.weights[0]), np_stage(wl.weights[2]), float(w[0]), float(w[1]))
        assert_blend_close(np_stage(wl.weights[1]), want)


def test_empty_stages_and_empty_calls(ctx, dev):
    empty = cf.Stage(ctx, [])
    hollow = cf.Stage(ctx, [torch.empty(0, device=dev), torch.empty(0, device=dev, dtype=torch.bfloat16)])
    hollow2 = cf.Stage(ctx, [torch.empty(0, device=dev), torch.empty(0, device=dev, dtype=torch.bfloat16)])
    w = _omega(dev, 1.0, 2.0)
    cf.cf_recover_stage_weighted_avg(ctx, empty, empty, w[0:1], w[1:2], cf.Stage(ctx, []))      # nothing to do
    cf.cf_recover_stage_with_weights(ctx, hollow, hollow2, 1.0, 1.0, cf.Stage(ctx, [torch.empty(0, device=dev), torch.empty(0, device=dev, dtype=torch.bfloat16)]))
    cf.cf_copy_stage(ctx, hollow, hollow2)
    cf.cf_copy_stage(ctx, empty, cf.Stage(ctx, []))
    out = cf.cf_stage_grad_sqnorm(ctx, [])                           # no stages: no launch, empty result
    assert out.numel() == 0
    om = cf.cf_stage_grad_sqnorm(ctx, [empty, hollow]).cpu().numpy()
    assert om.tolist() == [0.0, 0.0]
    g = cf.Stage(ctx, [torch.full((70_000,), 0.5, device=dev)])
    om = cf.cf_stage_grad_sqnorm(ctx, [g, empty, g]).cpu().numpy()   # a handle twice in one call
    assert om.tolist() == [17500.0, 0.0, 17500.0]
    torch.cuda.synchronize()
    assert ctx.read_flags() == 0


def test_handle_lifetimes(dev):
    lib = cf.load_library()
    c = cf.Context(0)
    st = cf.Stage(c, [torch.ones(10, device=dev)])
    assert lib.cf_ctx_destroy(c._h) == cf.CF_ERR_CONTEXT          # a stage is still alive: nothing freed
    omega = cf.cf_stage_grad_sqnorm(c, [st])                      # ... and everything still works
    assert omega.item() == 10.0
    c.close()                                                     # closes its stages first
    assert not st._h and not c._h
    st.close()                                                    # idempotent
    c.close()


def test_copy_argument_errors(ctx, dev):
    a = torch.zeros(300, device=dev)
    with pytest.raises(cf.CheckFreeError) as e:
        cf.cf_copy_stage(ctx, cf.Stage(ctx, [a[:100]]), cf.Stage(ctx, [a[50:150]]))
    assert e.value.status == cf.CF_ERR_ALIAS
    with pytest.raises(cf.CheckFreeError) as e:
        cf.cf_copy_stage(ctx, cf.Stage(ctx, [a[:100]]), cf.Stage(ctx, [a[100:201]]))
    assert e.value.status == cf.CF_ERR_SHAPE_MISMATCH
    s = cf.Stage(ctx, [a[:100]])
    cf.cf_copy_stage(ctx, s, s)                      # identical memory: allowed, a no-op in effect


# ----------------------------------------------------------------------------
# the five workloads: reduced shapes here, full shapes in test_gpu_fullsize.py
# ----------------------------------------------------------------------------

@pytest.mark.parametrize("config,shape", [
    (1, workloads.StageShape(192, 512, 2)),
    (2, workloads.StageShape(256, 704, 4)),
    (3, workloads.StageShape(256, 704, 4)),
])
def test_recovery_reduced_shapes(ctx, dev, config, shape):
    wl = workloads.make_workload(config, device=dev, shape=shape)
    check_recovery(ctx, wl, 0, 1, 2)
