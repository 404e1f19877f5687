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
    for code in range(-8, 0):
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
