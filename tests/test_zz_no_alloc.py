"""The entry point that allocates nothing (cf_stage_grad_sqnorm_static: tables and
partial sums in the library's static per-GPU array) against the existing entry
point cf_stage_grad_sqnorm, through the C ABI, on two calls in a row, the second
with a smaller input."""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2506_15461_amd as cf
import workloads

pytestmark = pytest.mark.gpu


def test_static_scratch_sqnorm_matches_the_handle_based_entry_point():
    dev = torch.device("cuda", 0)
    lib = cf.load_library()
    c = cf.Context(0)
    gen = torch.Generator(device=dev).manual_seed(91)
    big_shapes = workloads.StageShape(256, 704, 2).tensor_shapes() + workloads.ragged_shapes(3)
    small_shapes = workloads.ragged_shapes(4, 7) + [(0,), (40_000,)]
    out_static = torch.full((1,), -1.0, dtype=torch.float64, device=dev)
    out_handle = torch.full((1,), -2.0, dtype=torch.float64, device=dev)
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    for shapes in (big_shapes, small_shapes):                 # second call: fewer tensors, fewer chunks
        sig = workloads.draw_sigmas(len(shapes), np.random.default_rng(len(shapes)))
        grads = workloads.draw_grads(shapes, sig, gen, dev)
        grads[1] = grads[1].to(torch.bfloat16)
        desc = cf.tensor_descriptors(grads)
        handle = cf.Stage(c, grads)
        st = lib.cf_stage_grad_sqnorm_static(c._h, desc, len(grads), ctypes.c_void_p(out_static.data_ptr()), stream)
        assert st == cf.CF_OK
        handles = (ctypes.c_void_p * 1)(handle._h)
        assert lib.cf_stage_grad_sqnorm(c._h, handles, 1, ctypes.c_void_p(out_handle.data_ptr()), stream) == cf.CF_OK
        torch.cuda.synchronize()
        a, b = out_static.item(), out_handle.item()
        assert a == b and a > 0                              # same kernels, same order: the same bits
        ref = oracle.stage_grad_sqnorm(workloads.stage_to_numpy(grads))
        assert abs(a - ref) <= 1e-5 * ref
    # an empty list gives 0; a stage beyond the array's size is refused and nothing is written
    assert lib.cf_stage_grad_sqnorm_static(c._h, None, 0, ctypes.c_void_p(out_static.data_ptr()), stream) == cf.CF_OK
    torch.cuda.synchronize()
    assert out_static.item() == 0.0
    out_static.fill_(-1.0)
    limit = int(lib.cf_static_scratch_bytes())
    assert limit == 1 << 20
    too_big = (cf.CfTensor * 1)()
    too_big[0].data = grads[-1].data_ptr()                    # never dereferenced: the call must refuse first
    too_big[0].numel = (limit // 24 + 64) * 32768             # more chunks than 24 bytes each fit
    too_big[0].dtype = cf.CF_F32
    assert lib.cf_stage_grad_sqnorm_static(c._h, too_big, 1, ctypes.c_void_p(out_static.data_ptr()), stream) == cf.CF_ERR_LIMIT
    assert lib.cf_stage_grad_sqnorm_static(c._h, None, 1, ctypes.c_void_p(out_static.data_ptr()), stream) == cf.CF_ERR_NULL
    assert lib.cf_stage_grad_sqnorm_static(c._h, desc, len(grads), None, stream) == cf.CF_ERR_NULL
    torch.cuda.synchronize()
    assert out_static.item() == -1.0 and c.read_flags() == 0
