"""GPU tests of the boundary itself: handles built in caller-provided device
memory (no allocation, no copy, no wait inside the library), the slice copy
that keeps a CheckFree+ replica current, the atomic flag read, and weights at
the ends of the binary64 range.  Results are compared with the CPU oracle or,
where two routes through the library must agree, bit for bit with each other."""
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


@pytest.fixture(scope="module")
def dev():
    return torch.device("cuda", 0)


def np_stage(stage):
    return workloads.stage_to_numpy(stage)


def bits_equal(xs, ys):
    return all(np.array_equal(a, b) for a, b in zip(np_stage(xs), np_stage(ys)))


def test_handles_in_caller_memory_give_the_same_bits_as_library_owned_ones(dev):
    wl = workloads.make_workload(2, device=dev, shape=workloads.StageShape(192, 512, 2))      # bf16 weights
    results = []
    for owned in (False, True):
        c = cf.Context(0, owned=owned)
        assert (c.workspace is None) == owned
        out = [torch.full_like(t, float("nan")) for t in wl.weights[1]]
        cp = [torch.zeros_like(t) for t in wl.weights[1]]
        prev, nxt, lost, dst = (cf.Stage(c, x, owned=owned) for x in (wl.weights[0], wl.weights[2], out, cp))
        gp, gn = cf.Stage(c, wl.grads[0], owned=owned), cf.Stage(c, wl.grads[2], owned=owned)
        assert (prev.table is None) == owned
        omega = cf.cf_stage_grad_sqnorm(c, [gp, gn])
        o1, per = cf.cf_stage_grad_sqnorm_per_tensor(c, gp)
        cf.cf_recover_stage_weighted_avg(c, prev, nxt, omega[0:1], omega[1:2], lost)
        cf.cf_copy_stage(c, lost, dst)
        torch.cuda.synchronize()
        assert c.read_flags() == 0
        results.append((omega.cpu().numpy().tobytes(), per.cpu().numpy().tobytes(), np_stage(out), np_stage(cp)))
        for k, s in enumerate((0, 2)):
            ref = oracle.stage_grad_sqnorm(np_stage(wl.grads[s]))
            assert abs(omega[k].item() - ref) <= NORM_RTOL * ref
    a, b = results
    assert a[0] == b[0] and a[1] == b[1]
    assert all(np.array_equal(x, y) for x, y in zip(a[2], b[2])) and all(np.array_equal(x, y) for x, y in zip(a[3], b[3]))
    assert all(np.array_equal(x, y) for x, y in zip(a[2], a[3]))


def test_set_up_and_recovery_on_a_side_stream_with_no_wait_in_between(dev):
    """Context, five stage handles and the recovery itself, all enqueued on one non-default stream
    without a single synchronisation until the result is read."""
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(256, 704, 2), seed=4242)
    refs = [oracle.stage_grad_sqnorm(np_stage(wl.grads[s])) for s in (0, 2)]
    for t in wl.weights[1]:
        t.fill_(float("nan"))
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        c = cf.Context(0, stream=side)
        prev, nxt, lost = (cf.Stage(c, wl.weights[i], stream=side) for i in (0, 2, 1))
        gp, gn = cf.Stage(c, wl.grads[0], stream=side), cf.Stage(c, wl.grads[2], stream=side)
        omega = cf.cf_stage_grad_sqnorm(c, [gp, gn], stream=side)
        cf.cf_recover_stage_weighted_avg(c, prev, nxt, omega[0:1], omega[1:2], lost, stream=side)
    side.synchronize()
    w = omega.cpu().numpy()
    for k in range(2):
        assert abs(w[k] - refs[k]) <= NORM_RTOL * refs[k]
    # binary64 accumulation: the device's omegas are the oracle's to within a few units in the last place,
    # which moves a blended element by far less than one rounding step of the storage type
    want = oracle.recover_stage_weighted_avg(np_stage(wl.weights[0]), np_stage(wl.weights[2]), refs[0], refs[1])
    for g, x in zip(np_stage(wl.weights[1]), want):
        assert int(em.ulp_distance(g.reshape(-1), x.reshape(-1)).max()) <= 2
    assert c.read_flags(stream=side) == 0


def test_set_up_can_be_captured_in_a_hip_graph_with_the_recovery(dev):
    """Handle creation enqueues kernels only, so it can sit inside a captured graph: the
    graph below rebuilds the stage tables in preallocated memory and runs the recovery; it is replayed
    on changed inputs, with eager work in between, and compared with the eager path each time."""
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(192, 512, 2), seed=77)
    c = cf.Context(0)
    out_g = [torch.zeros_like(t) for t in wl.weights[1]]
    out_e = [torch.zeros_like(t) for t in wl.weights[1]]
    lists = dict(prev=wl.weights[0], nxt=wl.weights[2], lost=out_g, gp=wl.grads[0], gn=wl.grads[2])
    tables = {k: torch.empty(cf.stage_table_bytes(c, v), dtype=torch.uint8, device=dev) for k, v in lists.items()}
    om_g = torch.zeros(2, dtype=torch.float64, device=dev)
    om_e = torch.zeros(2, dtype=torch.float64, device=dev)
    eager = {k: cf.Stage(c, v) for k, v in dict(lists, lost=out_e).items()}
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.stream(side):
        graph.capture_begin()
        h = {k: cf.Stage(c, v, stream=side, table=tables[k]) for k, v in lists.items()}
        cf.cf_stage_grad_sqnorm(c, [h["gp"], h["gn"]], om_g, side)
        cf.cf_recover_stage_weighted_avg(c, h["prev"], h["nxt"], om_g[0:1], om_g[1:2], h["lost"], side)
        graph.capture_end()
    torch.cuda.synchronize()
    for rep in range(3):
        for g in wl.grads[2]:
            g.mul_(1.25 + rep)
        for tb in tables.values():
            tb.zero_()                                     # the replay has to rebuild every table
        for t in out_g:
            t.zero_()
        torch.cuda.synchronize()
        cf.cf_stage_grad_sqnorm(c, [eager["gp"], eager["gn"]], om_e)
        cf.cf_recover_stage_weighted_avg(c, eager["prev"], eager["nxt"], om_e[0:1], om_e[1:2], eager["lost"])
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert om_g.cpu().numpy().tobytes() == om_e.cpu().numpy().tobytes(), rep
        assert bits_equal(out_g, out_e), rep
    assert c.read_flags() == 0


def test_stage_with_more_tensors_than_one_table_launch_carries(dev):
    """The tensor list reaches the device 128 tensors per launch; 300 tensors of awkward sizes,
    some empty, some bf16."""
    rng = np.random.default_rng(5)
    gen = torch.Generator(device=dev).manual_seed(6)
    c = cf.Context(0, chunk_bytes=4096)
    tensors = []
    for k in range(300):
        n = 0 if k % 37 == 5 else int(rng.integers(1, 5000))
        t = torch.empty(n, device=dev).normal_(0, 1e-2, generator=gen)
        tensors.append(t.to(torch.bfloat16) if k % 11 == 3 else t)
    st = cf.Stage(c, tensors)
    assert st.numel == sum(t.numel() for t in tensors)
    assert st.num_chunks == sum(-(-t.numel() * t.element_size() // 4096) for t in tensors)
    omega, per = cf.cf_stage_grad_sqnorm_per_tensor(c, st)
    dst_t = [torch.zeros_like(t) for t in tensors]
    cf.cf_copy_stage(c, st, cf.Stage(c, dst_t))
    torch.cuda.synchronize()
    ref = oracle.tensor_grad_sqnorms(np_stage(tensors))
    got = per.cpu().numpy()
    assert len(got) == 300
    for t in range(300):
        assert abs(got[t] - ref[t]) <= NORM_RTOL * ref[t], t
    total = oracle.stage_grad_sqnorm(np_stage(tensors))
    assert abs(omega.item() - total) <= NORM_RTOL * total
    for g, w in zip(np_stage(dst_t), oracle.copy_stage(np_stage(tensors))):
        assert g.tobytes() == w.tobytes()


def test_caller_memory_argument_errors(dev):
    lib = cf.load_library()
    assert lib.cf_workspace_bytes() >= 8
    ws = torch.zeros(int(lib.cf_workspace_bytes()) + 64, dtype=torch.uint8, device=dev)
    h = ctypes.c_void_p()
    p = ctypes.c_void_p(ws.data_ptr())
    assert lib.cf_ctx_create_in(0, None, None, 256, None, ctypes.byref(h)) == cf.CF_ERR_NULL
    assert lib.cf_ctx_create_in(0, None, p, 8, None, ctypes.byref(h)) == cf.CF_ERR_LIMIT
    assert lib.cf_ctx_create_in(0, None, ctypes.c_void_p(ws.data_ptr() + 4), 256, None, ctypes.byref(h)) == cf.CF_ERR_ALIGN
    assert lib.cf_ctx_create_in(0, None, p, 256, None, None) == cf.CF_ERR_NULL
    assert not h.value
    c = cf.Context(0)
    t = torch.ones(100_000, device=dev)
    desc = cf.tensor_descriptors([t])
    need = int(lib.cf_stage_table_bytes(c._h, desc, 1))
    assert need == cf.stage_table_bytes(c, [t]) and 0 < need < 4096
    assert lib.cf_stage_table_bytes(c._h, None, 0) == 0
    assert lib.cf_stage_table_bytes(None, desc, 1) == 2 ** 64 - 1
    assert lib.cf_stage_table_bytes(c._h, None, 1) == 2 ** 64 - 1
    bad = cf.tensor_descriptors([t])
    bad[0].dtype = 9
    assert lib.cf_stage_table_bytes(c._h, bad, 1) == 2 ** 64 - 1
    table = torch.zeros(need + 64, dtype=torch.uint8, device=dev)
    tp = ctypes.c_void_p(table.data_ptr())
    assert lib.cf_stage_create_in(c._h, desc, 1, tp, need - 1, None, ctypes.byref(h)) == cf.CF_ERR_LIMIT
    assert lib.cf_stage_create_in(c._h, desc, 1, None, need, None, ctypes.byref(h)) == cf.CF_ERR_NULL
    assert lib.cf_stage_create_in(c._h, desc, 1, ctypes.c_void_p(table.data_ptr() + 8), need, None,
                                  ctypes.byref(h)) == cf.CF_ERR_ALIGN
    assert lib.cf_stage_create_in(c._h, bad, 1, tp, need, None, ctypes.byref(h)) == cf.CF_ERR_DTYPE
    assert not h.value
    assert lib.cf_stage_create_in(c._h, None, 0, None, 0, None, ctypes.byref(h)) == cf.CF_OK          # empty stage: no memory
    assert lib.cf_stage_num_chunks(h) == 0 and lib.cf_stage_destroy(h) == cf.CF_OK
    torch.cuda.synchronize()
    assert (table == 0).all()                                  # refused calls wrote nothing


@pytest.mark.parametrize("chunk_bytes", [4096, 131072])
def test_slice_copy_against_the_oracle(dev, chunk_bytes):
    """A replica refresh in pieces: each call moves the chunks it names and nothing else."""
    gen = torch.Generator(device=dev).manual_seed(71)
    c = cf.Context(0, chunk_bytes=chunk_bytes)
    sizes = [3 * chunk_bytes // 4 + 17, 5, 0, chunk_bytes // 4, 2 * chunk_bytes // 4 + 1, 40_001]
    src = [torch.randint(-2 ** 31, 2 ** 31 - 1, (n,), dtype=torch.int32, device=dev, generator=gen).view(torch.float32)
           for n in sizes]
    src[3] = src[3][: sizes[3] // 2].contiguous().view(torch.bfloat16)                       # one bf16 tensor, same bytes
    src[5] = src[5][1:]                                                                      # one misaligned tensor
    plan = []                                     # (tensor, first element, count) of every chunk: a tensor starts a new chunk
    for t, x in enumerate(src):
        per = chunk_bytes // x.element_size()
        plan += [(t, lo, min(per, x.numel() - lo)) for lo in range(0, x.numel(), per)]
    s = cf.Stage(c, src)
    assert s.num_chunks == len(plan)
    n = len(plan)
    for first, count in [(0, 1), (1, 2), (n - 1, 1), (2, n - 3), (0, n), (3, 0)]:
        dst = [torch.full_like(t, float("nan")) for t in src]
        d = cf.Stage(c, dst)
        cf.cf_copy_stage_range(c, s, d, first, count)
        torch.cuda.synchronize()
        host = [np.full_like(a, np.nan) if a.dtype == np.float32 else np.full_like(a, 0x7FC0) for a in np_stage(src)]
        want = oracle.copy_stage_ranges(np_stage(src), host, plan[first:first + count])
        for g, w in zip(np_stage(dst), want):
            assert g.tobytes() == w.tobytes(), (first, count)
    # pieces issued on two streams add up to the whole copy
    dst = [torch.zeros_like(t) for t in src]
    d = cf.Stage(c, dst)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    half = n // 2
    cf.cf_copy_stage_range(c, s, d, 0, half, s1)
    cf.cf_copy_stage_range(c, s, d, half, n - half, s2)
    torch.cuda.synchronize()
    for g, w in zip(np_stage(dst), oracle.copy_stage(np_stage(src))):
        assert g.tobytes() == w.tobytes()
    with pytest.raises(cf.CheckFreeError) as e:
        cf.cf_copy_stage_range(c, s, d, n - 1, 2)
    assert e.value.status == cf.CF_ERR_LIMIT
    with pytest.raises(cf.CheckFreeError) as e:
        cf.cf_copy_stage_range(c, s, d, n + 1, 0)
    assert e.value.status == cf.CF_ERR_LIMIT


def test_flags_are_read_and_cleared_in_one_step(dev):
    c = cf.Context(0)
    a = cf.Stage(c, [torch.ones(1000, device=dev)])
    out = cf.Stage(c, [torch.zeros(1000, device=dev)])
    bad = cf.Stage(c, [torch.full((10,), float("inf"), device=dev)])
    assert c.read_flags() == 0
    cf.cf_recover_stage_with_weights(c, a, a, 0.0, 0.0, out)
    assert c.read_flags() == cf.CF_FLAG_DEGENERATE_OMEGA            # reading without clear keeps it
    cf.cf_stage_grad_sqnorm(c, [bad])
    assert c.read_flags(clear=True) == cf.CF_FLAG_DEGENERATE_OMEGA | cf.CF_FLAG_NONFINITE_OMEGA
    assert c.read_flags() == 0
    # a flag raised on another stream after the clearing read is kept for the next read
    side = torch.cuda.Stream()
    cf.cf_stage_grad_sqnorm(c, [bad], stream=side)
    side.synchronize()
    assert c.read_flags(clear=True) == cf.CF_FLAG_NONFINITE_OMEGA
    assert c.read_flags(clear=True) == 0


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_blend_with_omegas_at_the_ends_of_the_binary64_range(dev, dtype):
    """A common factor on both omegas does not change the equation; the kernel takes the power of two
    out first, so omegas near 1e300 or 1e-300 blend as well as ordinary ones (checked against the
    oracle, whose own handling of such weights is pinned by exact rational arithmetic)."""
    c = cf.Context(0)
    gen = torch.Generator(device=dev).manual_seed(81)
    shapes = workloads.ragged_shapes(9, 8)
    a = workloads.draw_weights(shapes, dtype, gen, dev)
    b = workloads.draw_weights(shapes, dtype, gen, dev)
    if dtype == "f32":
        a[4][:4] = torch.tensor([3e38, -1e-38, 1e-45, 2.5], device=dev)
        b[4][:4] = torch.tensor([-2e38, 1e-38, -3e-45, 1e30], device=dev)
    out = [torch.full_like(t, float("nan")) for t in a]
    sa, sb, so = cf.Stage(c, a), cf.Stage(c, b), cf.Stage(c, out)
    ref = None
    for wp, wn in [(1e300, 3e299), (2e-300, 7e-301), (1.5e-310, 4e-307), (8e307, 1e305), (1e300, 1e-300),
                   (3.7e-3 * 2.0 ** 900, 1.9e-2 * 2.0 ** 900), (3.7e-3 * 2.0 ** -900, 1.9e-2 * 2.0 ** -900), (3.7e-3, 1.9e-2)]:
        w = torch.tensor([wp, wn], dtype=torch.float64, device=dev)
        cf.cf_recover_stage_weighted_avg(c, sa, sb, w[0:1], w[1:2], so)
        torch.cuda.synchronize()
        got = np_stage(out)
        want = oracle.recover_stage_weighted_avg(np_stage(a), np_stage(b), wp, wn)
        for g, x in zip(got, want):
            assert int(em.ulp_distance(g.reshape(-1), x.reshape(-1)).max()) <= (2 if dtype == "f32" else 1), (wp, wn)
        if wp in (3.7e-3 * 2.0 ** 900, 3.7e-3 * 2.0 ** -900):
            ref = got if ref is None else ref
            assert all(np.array_equal(x, y) for x, y in zip(got, ref))        # the same bits at both ends
        if (wp, wn) == (3.7e-3, 1.9e-2):
            assert all(np.array_equal(x, y) for x, y in zip(got, ref))        # ... and in the middle
        cf.cf_recover_stage_with_weights(c, sa, sb, wp, wn, so)
        torch.cuda.synchronize()
        assert all(np.array_equal(x, y) for x, y in zip(np_stage(out), got))
    assert c.read_flags() == 0


def test_the_same_gradients_through_two_handles_on_two_streams_at_once(dev):
    """A handle's block holds the norm's scratch, so ONE handle must not be in two norm calls that may overlap;
    the supported way to take the norm of the same tensors concurrently is one handle per stream."""
    c = cf.Context(0)
    wl = workloads.make_workload(1, device=dev, shape=workloads.StageShape(256, 704, 2), seed=616)
    grads = wl.grads[0]
    ref = oracle.stage_grad_sqnorm(np_stage(grads))
    handles = [cf.Stage(c, grads), cf.Stage(c, grads)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    outs = [torch.zeros(1, dtype=torch.float64, device=dev) for _ in range(2)]
    torch.cuda.synchronize()
    for rep in range(20):
        for h, s, o in zip(handles, streams, outs):
            cf.cf_stage_grad_sqnorm(c, [h], o, s)
    torch.cuda.synchronize()
    assert outs[0].item() == outs[1].item()
    assert abs(outs[0].item() - ref) <= 1e-12 * ref
    assert c.read_flags() == 0


def test_hot_calls_from_several_host_threads(dev):
    """Four host threads, each with its own stream, context and handles, run whole recoveries at the same
    time; every result must be the one a single thread gets."""
    import threading
    n_threads = 4
    wls = [workloads.make_workload(1, device=dev, shape=workloads.StageShape(128, 352, 2), seed=700 + i)
           for i in range(n_threads)]
    wants = []
    for wl in wls:
        refs = [oracle.stage_grad_sqnorm(np_stage(wl.grads[s])) for s in (0, 2)]
        wants.append((refs, oracle.recover_stage_weighted_avg(np_stage(wl.weights[0]), np_stage(wl.weights[2]), *refs)))
    torch.cuda.synchronize()
    errors, omegas = [], [None] * n_threads

    def work(i):
        try:
            torch.cuda.set_device(dev)
            wl = wls[i]
            s = torch.cuda.Stream()
            with torch.cuda.stream(s):
                c = cf.Context(0, stream=s)
                for rep in range(10):
                    prev, nxt, lost = (cf.Stage(c, wl.weights[k], stream=s) for k in (0, 2, 1))
                    gp, gn = cf.Stage(c, wl.grads[0], stream=s), cf.Stage(c, wl.grads[2], stream=s)
                    om = cf.cf_stage_grad_sqnorm(c, [gp, gn], stream=s)
                    cf.cf_recover_stage_weighted_avg(c, prev, nxt, om[0:1], om[1:2], lost, stream=s)
                    s.synchronize()
                    for h in (prev, nxt, lost, gp, gn):
                        h.close()
                omegas[i] = om.cpu().numpy()
                assert c.read_flags(stream=s) == 0
        except Exception as e:                       # reported by the main thread
            errors.append((i, repr(e)))

    threads = [threading.Thread(target=work, args=(i,)) for i in range(n_threads)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    torch.cuda.synchronize()
    for i, (wl, (refs, want)) in enumerate(zip(wls, wants)):
        for k in range(2):
            assert abs(omegas[i][k] - refs[k]) <= 1e-12 * refs[k]
        for g, x in zip(np_stage(wl.weights[1]), want):
            assert int(em.ulp_distance(g.reshape(-1), x.reshape(-1)).max()) <= 2
