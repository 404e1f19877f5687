"""CPU-side checks of the boundary: the library loads and exports every symbol
the header declares; host-only logic (chunk planning, status strings, argument
validation that needs no device)."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_2506_15461_amd as cf

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(cf.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return cf.load_library()


def test_header_and_binding_agree_on_exports(lib):
    header = open(os.path.join(ROOT, "include", "checkfree.h")).read()
    declared = set(re.findall(r"CF_API[^;(]*?\b(cf_[a-z_0-9]+)\s*\(", header))
    assert declared == set(cf.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    for required in ("cf_stage_grad_sqnorm", "cf_recover_stage_weighted_avg", "cf_copy_stage"):
        assert required in declared


def test_no_internal_symbols_leak(lib):
    import subprocess
    out = subprocess.run(["nm", "-D", "--defined-only", cf.LIB_PATH], capture_output=True, text=True).stdout
    syms = [l.split()[-1] for l in out.splitlines() if " T " in l]
    assert sorted(s for s in syms if s.startswith("cf_")) == sorted(cf.EXPORTS)
    assert not [s for s in syms if "cf_launch" in s]


def test_status_strings(lib):
    assert cf.status_string(cf.CF_OK) == "CF_OK"
    for code in range(-9, 0):
        assert cf.status_string(code).startswith("CF_ERR_")
    assert "unknown" in cf.status_string(-99)


def test_default_tuning(lib):
    t = cf.default_tuning()
    assert t["chunk_bytes"] >= 4096 and t["chunk_bytes"] & (t["chunk_bytes"] - 1) == 0


def test_chunk_plan_covers_every_element_once(lib):
    numels = [1, 0, 2047, 2048, 2049, 70000, 5, 32768 * 3]
    chunk = 4096
    plan = cf.plan_chunks(numels, chunk * 4)        # fp32: 16 KiB chunks hold 4096 elements
    seen = {t: [] for t in range(len(numels))}
    for t, first, length in plan:
        assert 0 < length <= chunk
        seen[t].append((first, length))
    for t, n in enumerate(numels):
        pos = 0
        for first, length in seen[t]:          # in order, contiguous, no overlap
            assert first == pos
            assert first % chunk == 0
            pos += length
        assert pos == n
    assert len(plan) == sum((n + chunk - 1) // chunk for n in numels)
    # chunks are listed in tensor order
    assert [t for t, _, _ in plan] == sorted(t for t, _, _ in plan)


def test_chunk_plan_model_shape(lib):
    import workloads
    shape = workloads.SPECS[3].shape
    numels = [int(np.prod(s)) for s in shape.tensor_shapes()]
    assert sum(numels) == 205_537_280 and len(numels) == 36
    plan = cf.plan_chunks(numels, 128 << 10)
    assert sum(l for _, _, l in plan) == sum(numels)
    assert len(plan) == 6280
    # bf16 chunks hold twice the elements in the same bytes
    plan16 = cf.plan_chunks(numels, 128 << 10, cf.CF_BF16)
    assert sum(l for _, _, l in plan16) == sum(numels) and max(l for _, _, l in plan16) == 65536


def test_plan_argument_errors(lib):
    arr = (cf.CfTensor * 1)()
    arr[0].numel = 10
    arr[0].numel = 3000
    assert lib.cf_plan_num_chunks(arr, 1, 0) == 2 ** 64 - 1
    assert lib.cf_plan_num_chunks(arr, 1, 5000) == 2 ** 64 - 1          # not a power of two
    assert lib.cf_plan_num_chunks(arr, 1, 2048) == 2 ** 64 - 1          # below one tile
    assert lib.cf_plan_num_chunks(None, 1, 4096) == 2 ** 64 - 1
    assert lib.cf_plan_num_chunks(None, 0, 4096) == 0
    assert lib.cf_plan_num_chunks(arr, 1, 4096) == 3
    ct = (ctypes.c_uint32 * 1)()
    cfirst = (ctypes.c_uint64 * 1)()
    cl = (ctypes.c_uint32 * 1)()
    assert lib.cf_plan_chunks(arr, 1, 4096, ct, cfirst, cl, 1) == cf.CF_ERR_LIMIT      # needs 3 slots
    assert lib.cf_plan_chunks(arr, 1, 4096, None, cfirst, cl, 8) == cf.CF_ERR_NULL
    arr[0].dtype = 7
    assert lib.cf_plan_num_chunks(arr, 1, 4096) == 2 ** 64 - 1


def test_null_and_bad_arguments_without_a_device(lib):
    assert lib.cf_ctx_create(0, None, None) == cf.CF_ERR_NULL
    bad = cf.CfTuning(chunk_bytes=1000)
    h = ctypes.c_void_p()
    assert lib.cf_ctx_create(0, ctypes.byref(bad), ctypes.byref(h)) == cf.CF_ERR_LIMIT
    assert lib.cf_ctx_destroy(None) == cf.CF_OK
    assert lib.cf_stage_destroy(None) == cf.CF_OK
    assert lib.cf_stage_create(None, None, 0, ctypes.byref(h)) == cf.CF_ERR_NULL
    assert lib.cf_stage_grad_sqnorm(None, None, 0, None, None) == cf.CF_ERR_NULL
    assert lib.cf_recover_stage_weighted_avg(None, None, None, None, None, None, None) == cf.CF_ERR_NULL
    assert lib.cf_copy_stage(None, None, None, None) == cf.CF_ERR_NULL
    assert lib.cf_read_flags(None, None, None, 0) == cf.CF_ERR_NULL
    assert lib.cf_stage_numel(None) == 0 and lib.cf_stage_num_chunks(None) == 0


def test_context_creation_fails_cleanly_without_a_gpu(lib):
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(cf.CheckFreeError) as e:
        cf.Context(0)
    assert e.value.status == cf.CF_ERR_HIP


def test_recovered_learning_rate(lib):
    # Algorithm 1, third step: lambda_i <- 1.1 lambda_i
    assert cf.cf_recovered_learning_rate(1.0) == 1.1
    assert cf.cf_recovered_learning_rate(3e-4) == 1.1 * 3e-4
    assert cf.cf_recovered_learning_rate(0.0) == 0.0
    assert lib.cf_recover_stage_with_weights(None, None, None, 1.0, 1.0, None, None) == cf.CF_ERR_NULL


def test_recovery_plan_matches_the_oracle_on_every_subset(lib):
    # Algorithm 1 / CheckFree+ / "consecutive stages: no": the library's plan against the oracle's,
    # for every set of lost stages of pipelines of 2..6 stages, in two orders of the lost list
    import itertools
    import oracle
    kinds = {"average": cf.CF_RECOVER_WEIGHTED_AVG, "copy": cf.CF_RECOVER_COPY}
    for s in range(2, 7):
        for n in range(s + 1):
            for lost in itertools.combinations(range(s), n):
                for order in (lost, lost[::-1]):
                    for plus in (False, True):
                        try:
                            want = oracle.recovery_plan(s, order, plus)
                        except ValueError:
                            with pytest.raises(cf.CheckFreeError) as e:
                                cf.cf_plan_recovery(s, order, plus)
                            assert e.value.status == cf.CF_ERR_VALUE
                            continue
                        got = cf.cf_plan_recovery(s, order, plus)
                        assert [g[0] for g in got] == list(order)
                        for g, w in zip(got, want):
                            assert g[1] == kinds[w[0]] and g[2] == w[1] and g[3] == w[-1]


def test_recovery_plan_errors_write_nothing(lib):
    u32 = ctypes.c_uint32
    steps = (cf.CfRecoveryStep * 3)()
    for st in steps:
        st.lost = st.prev = st.next = 777
    def call(s, lost, plus):
        arr = (u32 * max(1, len(lost)))(*lost)
        return lib.cf_plan_recovery(s, arr, len(lost), plus, steps)
    assert call(8, [3, 4], 1) == cf.CF_ERR_VALUE           # neighbours lost together
    assert call(8, [2, 0], 0) == cf.CF_ERR_VALUE           # the first stage, without CheckFree+
    assert call(8, [2, 8], 1) == cf.CF_ERR_LIMIT           # no such stage
    assert call(8, [2, 5, 2], 1) == cf.CF_ERR_LIMIT        # named twice
    assert call(1, [0], 1) == cf.CF_ERR_LIMIT              # a single stage has no neighbour
    assert call(0, [0], 1) == cf.CF_ERR_LIMIT
    assert all(st.lost == 777 and st.prev == 777 and st.next == 777 for st in steps)
    assert lib.cf_plan_recovery(8, None, 2, 1, steps) == cf.CF_ERR_NULL
    assert lib.cf_plan_recovery(8, (u32 * 1)(3), 1, 1, None) == cf.CF_ERR_NULL
    assert lib.cf_plan_recovery(8, None, 0, 1, None) == cf.CF_OK
    assert call(8, [7, 3, 0], 1) == cf.CF_OK
    assert [(st.lost, st.kind, st.prev, st.next) for st in steps] == [
        (7, cf.CF_RECOVER_COPY, 6, 6), (3, cf.CF_RECOVER_WEIGHTED_AVG, 2, 4), (0, cf.CF_RECOVER_COPY, 1, 1)]


def test_plus_stage_order_matches_the_oracle(lib):
    import oracle
    for s in range(4, 12):
        for mb in (0, 1, 2, 3, 10, 11, 2 ** 40, 2 ** 40 + 1):
            assert cf.cf_plus_stage_order(s, mb) == oracle.plus_stage_order(s, mb)
    order = (ctypes.c_uint32 * 4)(9, 9, 9, 9)
    for s in (0, 1, 2, 3):
        assert lib.cf_plus_stage_order(s, 1, order) == cf.CF_ERR_LIMIT
    assert list(order) == [9, 9, 9, 9]
    assert lib.cf_plus_stage_order(4, 1, None) == cf.CF_ERR_NULL


def test_stage_pair_check_shapes_and_dtypes(lib):
    F, H = cf.CF_F32, cf.CF_BF16
    A = [(0x1000, 100, F), (0x2000, 7, H), (0, 0, F)]
    B = [(0x9000, 100, F), (0xA000, 7, H), (0, 0, F)]
    assert cf.check_stage_pair(A, B) == cf.CF_OK
    assert cf.check_stage_pair(A, B[:2]) == cf.CF_ERR_SHAPE_MISMATCH
    assert cf.check_stage_pair(A, [(0x9000, 101, F)] + B[1:]) == cf.CF_ERR_SHAPE_MISMATCH
    assert cf.check_stage_pair(A, [(0x9000, 100, H)] + B[1:]) == cf.CF_ERR_SHAPE_MISMATCH
    assert cf.check_stage_pair(A, [(0x9000, 100, 5)] + B[1:]) == cf.CF_ERR_DTYPE
    assert cf.check_stage_pair([(0x1002, 4, F)], [(0x9000, 4, F)]) == cf.CF_ERR_ALIGN      # fp32 at 2 mod 4
    assert cf.check_stage_pair([(0x1001, 4, H)], [(0x9000, 4, H)]) == cf.CF_ERR_ALIGN
    assert cf.check_stage_pair([(0x1002, 4, H)], [(0x9000, 4, H)]) == cf.CF_OK
    assert cf.check_stage_pair([(0, 4, F)], [(0x9000, 4, F)]) == cf.CF_ERR_NULL
    assert cf.check_stage_pair([], []) == cf.CF_OK


def test_stage_pair_check_aliasing(lib):
    F = cf.CF_F32
    # identical memory, tensor for tensor: allowed (in-place recovery)
    A = [(0x1000, 100, F), (0x2000, 50, F)]
    assert cf.check_stage_pair(A, A) == cf.CF_OK
    # same addresses but crossed over between tensors of equal size: output 0 overwrites input 1
    assert cf.check_stage_pair([(0x1000, 100, F), (0x2000, 100, F)], [(0x2000, 100, F), (0x1000, 100, F)]) == cf.CF_ERR_ALIAS
    # shifted overlap with its own counterpart
    assert cf.check_stage_pair([(0x1000, 100, F)], [(0x1004, 100, F)]) == cf.CF_ERR_ALIAS
    # touching but not overlapping: [0x1000, 0x1190) then 0x1190
    assert cf.check_stage_pair([(0x1000, 100, F)], [(0x1190, 100, F)]) == cf.CF_OK
    assert cf.check_stage_pair([(0x1000, 100, F)], [(0x118C, 100, F)]) == cf.CF_ERR_ALIAS   # last dword shared
    # output inside a much larger input that starts far below it
    big = [(0x10000, 1 << 20, F), (0x900000, 10, F)]
    out = [(0xA00000, 1 << 20, F), (0x10000 + 4 * 5000, 10, F)]
    assert cf.check_stage_pair(big, out) == cf.CF_ERR_ALIAS
    # many small inputs after a large one: the sweep must still see the large one
    ins = [(0x10000, 1 << 20, F)] + [(0x800000 + 0x100 * k, 8, F) for k in range(20)]
    outs = [(0x2000000, 1 << 20, F)] + [(0x3000000 + 0x100 * k, 8, F) for k in range(19)] + [(0x10000 + 0x3FFF00, 8, F)]
    assert cf.check_stage_pair(ins, outs) == cf.CF_ERR_ALIAS
    outs[-1] = (0x10000 + 0x400000, 8, F)                      # first byte after the large input
    assert cf.check_stage_pair(ins, outs) == cf.CF_OK
    # two output tensors overlapping each other
    assert cf.check_stage_pair([(0x1000, 10, F), (0x2000, 10, F)], [(0x9000, 10, F), (0x9020, 10, F)]) == cf.CF_ERR_ALIAS
    assert cf.check_stage_pair([(0x1000, 10, F), (0x2000, 10, F)], [(0x9000, 10, F), (0x9028, 10, F)]) == cf.CF_OK
    # empty tensors never alias
    assert cf.check_stage_pair([(0x1000, 0, F), (0x1000, 4, F)], [(0x1000, 0, F), (0x1000, 4, F)]) == cf.CF_OK


def test_stage_pair_check_against_brute_force(lib):
    rng = np.random.default_rng(0)
    F = cf.CF_F32
    for trial in range(300):
        n = int(rng.integers(1, 6))
        sizes = rng.integers(1, 12, n)
        ins = [(0x1000 + 4 * int(rng.integers(0, 60)), int(s), F) for s in sizes]
        outs = [(0x1000 + 4 * int(rng.integers(0, 120)), int(s), F) for s in sizes]
        if rng.random() < 0.3:
            k = int(rng.integers(0, n))
            outs[k] = ins[k]
        def rng_of(t):
            return range(t[0], t[0] + 4 * t[1])
        bad = False
        for i, o in enumerate(outs):
            so = set(rng_of(o))
            for j, a in enumerate(ins):
                if so & set(rng_of(a)) and not (i == j and a[0] == o[0]):
                    bad = True
            for j, o2 in enumerate(outs):
                if j != i and so & set(rng_of(o2)):
                    bad = True
        want = cf.CF_ERR_ALIAS if bad else cf.CF_OK
        assert cf.check_stage_pair(ins, outs) == want, (ins, outs)


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0
    assert "one GPU" in r.stderr and r.stdout.strip() == ""


def test_plain_c_client_host_only(lib):
    """A C99 program (gcc -pedantic -Werror) includes the header, links the library and calls the
    host-only entry points."""
    import subprocess
    from paper_2506_15461_amd import build as hip_build
    if not os.path.exists(hip_build.C_SMOKE_BIN):
        hip_build.build_c_smoke(verbose=False)
    r = subprocess.run([hip_build.C_SMOKE_BIN, "--host-only"], capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
    assert "host-only ok" in r.stdout
