"""GPU parity of a whole pipeline's recovery: several stages of an 8-stage
pipeline are lost at once, the library's plan (Algorithm 1 for intermediate
stages, CheckFree+ copies for the two ends) is carried out with the library's
kernels, and every stage of the pipeline is compared with the oracle carrying
out the oracle's plan on the same seeded inputs."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_15461_amd as cf
import workloads
from test_gpu_parity import NORM_RTOL, ORACLE_THREADS, assert_blend_close, np_stage

pytestmark = pytest.mark.gpu

N_STAGES = 8


def draw_pipeline(dev, dtype_name, seed):
    shape = workloads.StageShape(128, 352, 1)
    shapes = shape.tensor_shapes() + [(1031,), (3,)]          # a ragged tail on every stage
    gen = torch.Generator(device=dev).manual_seed(seed)
    sig = workloads.draw_sigmas(N_STAGES * len(shapes), np.random.default_rng(seed)).reshape(N_STAGES, len(shapes))
    weights = [workloads.draw_weights(shapes, dtype_name, gen, dev) for _ in range(N_STAGES)]
    grads = [workloads.draw_grads(shapes, sig[s], gen, dev) for s in range(N_STAGES)]
    return weights, grads


@pytest.mark.parametrize("dtype_name", ["f32", "bf16"])
@pytest.mark.parametrize("lost,plus", [([3], False), ([2, 5], False), ([0, 3, 7], True), ([6, 1, 4], True), ([7], True)])
def test_lost_stages_are_rebuilt_as_the_plan_says(dtype_name, lost, plus):
    dev = torch.device("cuda", 0)
    ctx = cf.Context(0)
    weights, grads = draw_pipeline(dev, dtype_name, 4200 + 10 * len(lost) + lost[0])
    before = [np_stage(w) for w in weights]
    grads_np = [np_stage(g) for g in grads]

    # the oracle's side: omegas of all stages, its own plan, its own arithmetic
    omega_ref = [oracle.stage_grad_sqnorm(g, ORACLE_THREADS) for g in grads_np]
    want = [list(st) for st in before]
    for i, step in zip(lost, oracle.recovery_plan(N_STAGES, lost, plus)):
        if step[0] == "average":
            p, n = step[1], step[2]
            want[i] = oracle.recover_stage_weighted_avg(before[p], before[n], omega_ref[p], omega_ref[n], ORACLE_THREADS)
        else:
            want[i] = oracle.copy_stage(before[step[1]])

    # the library's side
    w_stage = [cf.Stage(ctx, w) for w in weights]
    g_stage = [cf.Stage(ctx, g) for g in grads]
    omega = cf.cf_stage_grad_sqnorm(ctx, g_stage)              # all eight stages, one call
    got_omega = omega.cpu().numpy()
    for s in range(N_STAGES):
        assert abs(got_omega[s] - omega_ref[s]) <= NORM_RTOL * omega_ref[s]
    for i in lost:                                              # the lost stages' memory holds nothing of use
        for t in weights[i]:
            t.fill_(float("nan"))
    # the blend is compared at one common omega pair: the oracle's, uploaded
    omega_dev = torch.tensor(omega_ref, dtype=torch.float64, device=dev)
    for lost_i, kind, p, n in cf.cf_plan_recovery(N_STAGES, lost, plus):
        if kind == cf.CF_RECOVER_WEIGHTED_AVG:
            cf.cf_recover_stage_weighted_avg(ctx, w_stage[p], w_stage[n], omega_dev[p:p + 1], omega_dev[n:n + 1],
                                             w_stage[lost_i])
        else:
            assert kind == cf.CF_RECOVER_COPY and p == n
            cf.cf_copy_stage(ctx, w_stage[p], w_stage[lost_i])
    torch.cuda.synchronize()
    assert ctx.read_flags(clear=True) == 0
    for s in range(N_STAGES):
        got = np_stage(weights[s])
        if s in lost and 0 < s < N_STAGES - 1:
            assert_blend_close(got, want[s])
        else:                                                   # survivors untouched, copies exact
            for g, w in zip(got, want[s]):
                assert g.tobytes() == w.tobytes()


def test_a_plan_that_cannot_be_carried_out_touches_nothing():
    dev = torch.device("cuda", 0)
    weights, _ = draw_pipeline(dev, "f32", 77)
    before = [np_stage(w) for w in weights]
    for lost, plus in (([3, 4], True), ([0], False), ([6, 7], True)):
        with pytest.raises(cf.CheckFreeError) as e:
            cf.cf_plan_recovery(N_STAGES, lost, plus)
        assert e.value.status == cf.CF_ERR_VALUE
        with pytest.raises(ValueError):
            oracle.recovery_plan(N_STAGES, lost, plus)
    for s in range(N_STAGES):
        for g, w in zip(np_stage(weights[s]), before[s]):
            assert g.tobytes() == w.tobytes()
