"""GPU parity at the full sizes of the five workloads, in the launch
configuration the benchmark times (default tuning), every element compared."""
import numpy as np
import pytest
import torch

import oracle
import paper_2506_15461_amd as cf
import workloads
from test_gpu_parity import (NORM_RTOL, ORACLE_THREADS, assert_blend_close,
                             assert_end_to_end_within_sensitivity_bound, check_recovery, np_stage)

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda", 0)


@pytest.fixture()
def ctx():
    c = cf.Context(0)
    yield c
    torch.cuda.synchronize()
    assert c.read_flags() == 0


@pytest.mark.parametrize("config", [1, 2, 3])
def test_full_recovery(ctx, dev, config):
    print(f"workload {config}: {workloads.SPECS[config].name}", flush=True)
    wl = workloads.make_workload(config, device=dev)
    omega, worst = check_recovery(ctx, wl, 0, 1, 2)
    # gross-error band from the drawing recipe: E[omega] = sum n_t sigma_t^2
    n = np.array([np.prod(s) for s in wl.spec.shape.tensor_shapes()], dtype=np.float64)
    for k, s in enumerate((0, 2)):
        mean = float(np.sum(n * wl.sigmas[s] ** 2))
        sd = float(np.sqrt(np.sum(2 * n * wl.sigmas[s] ** 4)))
        assert abs(omega[k] - mean) < 6 * sd + 1e-5 * mean
    print(f"  omega={omega.tolist()} blend max ulp={worst}", flush=True)


def test_checkfree_plus_copy_full(ctx, dev):
    wl = workloads.make_workload(4, device=dev, with_grads=False)
    src = wl.weights[0] + wl.extra                     # the stage, E, E^-1, final norm
    assert len(src) == 39 and sum(t.numel() for t in src) == 336_611_328
    dst = [torch.full_like(t, float("nan")) for t in src]
    cf.cf_copy_stage(ctx, cf.Stage(ctx, src), cf.Stage(ctx, dst))
    torch.cuda.synchronize()
    for s, d in zip(src, dst):
        assert torch.equal(s.view(torch.int32), d.view(torch.int32))
    # and against the oracle on the largest and the smallest tensor
    for k in (36, 38, 8):
        want = oracle.copy_stage([workloads.to_numpy(src[k])], ORACLE_THREADS)[0]
        assert workloads.to_numpy(dst[k]).tobytes() == want.tobytes()


def test_pipeline_norm_tracking_then_recovery(ctx, dev):
    wl = workloads.make_workload(5, device=dev)
    lost = wl.lost
    assert 1 <= lost <= 6
    print(f"pipeline workload: lost stage {lost}", flush=True)
    refs = [oracle.stage_grad_sqnorm(np_stage(wl.grads[s]), ORACLE_THREADS) for s in range(8)]
    prev_np, next_np = np_stage(wl.weights[lost - 1]), np_stage(wl.weights[lost + 1])
    want = oracle.recover_stage_weighted_avg(prev_np, next_np, refs[lost - 1], refs[lost + 1], ORACLE_THREADS)
    grads = [cf.Stage(ctx, g) for g in wl.grads]
    omega = cf.cf_stage_grad_sqnorm(ctx, grads)                    # all 8 stages, one call
    w = omega.cpu().numpy()
    for s in range(8):
        assert abs(w[s] - refs[s]) <= NORM_RTOL * refs[s], (s, w[s], refs[s])
    prev, nxt, out = (cf.Stage(ctx, wl.weights[i]) for i in (lost - 1, lost + 1, lost))
    # the blend at the oracle's omegas: ulp bar
    for t in wl.weights[lost]:
        t.fill_(float("nan"))
    ref_dev = torch.tensor(refs, dtype=torch.float64, device=dev)
    cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, ref_dev[lost - 1:lost], ref_dev[lost + 1:lost + 2], out)
    torch.cuda.synchronize()
    assert_blend_close(np_stage(wl.weights[lost]), want)
    # the path as it runs: omegas taken from the just-computed device array
    for t in wl.weights[lost]:
        t.fill_(float("nan"))
    cf.cf_recover_stage_weighted_avg(ctx, prev, nxt, omega[lost - 1:lost], omega[lost + 1:lost + 2], out)
    torch.cuda.synchronize()
    assert_end_to_end_within_sensitivity_bound(np_stage(wl.weights[lost]), want, prev_np, next_np,
                                               (w[lost - 1], w[lost + 1]), (refs[lost - 1], refs[lost + 1]))


def test_one_tensor_beyond_four_gib(ctx, dev):
    """Maximum-size case: a single tensor of 2^30 + 12345 fp32 elements (4.3 GB), so that element
    offsets pass 2^30 and byte offsets pass 2^32 inside one tensor; 4.2 million blend tiles."""
    n = (1 << 30) + 12345
    print(f"huge tensor: {n} elements", flush=True)
    const = torch.full((n,), 2.0 ** -7, device=dev)
    omega = cf.cf_stage_grad_sqnorm(ctx, [cf.Stage(ctx, [const])])
    assert omega.item() == n * 2.0 ** -14                      # every partial sum is exact
    del const
    gen = torch.Generator(device=dev).manual_seed(77)
    a = torch.empty(n, device=dev).normal_(0, 0.02, generator=gen)
    b = torch.empty(n, device=dev).normal_(0, 0.02, generator=gen)
    a_host, b_host = workloads.to_numpy(a), workloads.to_numpy(b)
    w = torch.tensor([3.7e-3, 1.9e-2], dtype=torch.float64, device=dev)
    sa = cf.Stage(ctx, [a])
    cf.cf_recover_stage_weighted_avg(ctx, sa, cf.Stage(ctx, [b]), w[0:1], w[1:2], sa)      # in place
    torch.cuda.synchronize()
    want = oracle.recover_stage_weighted_avg([a_host], [b_host], 3.7e-3, 1.9e-2, ORACLE_THREADS)
    assert_blend_close([workloads.to_numpy(a)], want)
    del want, a_host
    cf.cf_copy_stage(ctx, cf.Stage(ctx, [b]), sa)
    torch.cuda.synchronize()
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_norm_bits_do_not_depend_on_the_launch_shape_at_full_size(dev):
    """The two neighbours' gradients of workload 3 (1.6 GB): the automatic choice walks the chunk list with 512
    resident workgroups at this size; one workgroup per chunk, other caps, repeated calls and the entry point
    that works in the library's static array must all give the same bits, per stage and per tensor."""
    wl = workloads.make_workload(3, device=dev)
    refs = [oracle.stage_grad_sqnorm(np_stage(wl.grads[s]), ORACLE_THREADS) for s in (0, 2)]
    seen, seen_tensors = set(), set()
    for tuning in ({}, {"sqnorm_blocks_per_cu": 65}, {"sqnorm_blocks_per_cu": 1}, {"sqnorm_blocks_per_cu": 5}):
        c = cf.Context(0, **tuning)
        handles = [cf.Stage(c, wl.grads[0]), cf.Stage(c, wl.grads[2])]
        for rep in range(3):
            seen.add(cf.cf_stage_grad_sqnorm(c, handles).cpu().numpy().tobytes())
        om, per = cf.cf_stage_grad_sqnorm_per_tensor(c, handles[0])
        seen_tensors.add(per.cpu().numpy().tobytes())
        one = torch.zeros(1, dtype=torch.float64, device=dev)
        cf.cf_stage_grad_sqnorm_static(c, wl.grads[2], one)
        torch.cuda.synchronize()
        got = np.frombuffer(next(iter(seen)), dtype=np.float64)
        assert om.item() == got[0] and one.item() == got[1]
        assert c.read_flags() == 0
    assert len(seen) == 1 and len(seen_tensors) == 1
    got = np.frombuffer(next(iter(seen)), dtype=np.float64)
    for k in range(2):
        assert abs(got[k] - refs[k]) <= 1e-12 * refs[k]
    per = np.frombuffer(next(iter(seen_tensors)), dtype=np.float64)
    want = oracle.tensor_grad_sqnorms(np_stage(wl.grads[0]))
    assert len(per) == 36
    for t in range(36):
        assert abs(per[t] - want[t]) <= 1e-12 * want[t], t


def test_replica_refresh_in_slices_at_full_size(ctx, dev):
    """Embedding and de-embedding of workload 4 (2 x 262 MB) refreshed in 7 uneven slices issued on two
    streams: bit for bit the whole copy, and a slice touches nothing outside its chunks."""
    wl = workloads.make_workload(4, device=dev, with_grads=False)
    src = list(wl.extra[:2])
    dst = [torch.full_like(t, float("nan")) for t in src]
    s, d = cf.Stage(ctx, src), cf.Stage(ctx, dst)
    n = s.num_chunks
    assert n == 4000
    cf.cf_copy_stage_range(ctx, s, d, 1000, 500)
    torch.cuda.synchronize()
    flat = dst[0].view(-1)
    per = 32768                                              # elements per chunk; E has 2000 chunks
    assert torch.equal(flat[1000 * per:1500 * per].view(torch.int32), src[0].view(-1)[1000 * per:1500 * per].view(torch.int32))
    assert torch.isnan(flat[:1000 * per]).all() and torch.isnan(flat[1500 * per:]).all() and torch.isnan(dst[1]).all()
    cuts = [0, 1, 777, 1000, 1500, 2000, 2001, n]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for k in range(len(cuts) - 1):
        cf.cf_copy_stage_range(ctx, s, d, cuts[k], cuts[k + 1] - cuts[k], streams[k % 2])
    torch.cuda.synchronize()
    for a, b in zip(src, dst):
        assert torch.equal(a.view(torch.int32), b.view(torch.int32))
    want = oracle.copy_stage([workloads.to_numpy(src[1])], ORACLE_THREADS)[0]
    assert workloads.to_numpy(dst[1]).tobytes() == want.tobytes()
