"""The synthetic-input recipe: shapes, element counts and seeding (CPU only)."""
import numpy as np
import torch

import workloads


def test_stage_shapes_and_element_counts():
    want = {1: (18, 14_158_848), 2: (36, 51_388_416), 3: (36, 205_537_280), 4: (36, 205_537_280), 5: (27, 154_152_960)}
    for cid, (n_tensors, numel) in want.items():
        shape = workloads.SPECS[cid].shape
        assert len(shape.tensor_shapes()) == n_tensors
        assert shape.numel() == numel
    extra = workloads.SPECS[4].extra_copy_shapes
    assert extra == [(32000, 2048), (2048, 32000), (2048,)]
    assert workloads.SPECS[4].shape.numel() + sum(int(np.prod(s)) for s in extra) == 336_611_328
    assert workloads.SPECS[5].n_stages == 8 and workloads.SPECS[2].param_dtype == "bf16"
    d, f = 2048, 5632
    per_layer = workloads.StageShape(d, f, 1).tensor_shapes()
    assert per_layer == [(d, d)] * 4 + [(d, f), (d, f), (f, d), (d,), (d,)]


def test_same_seed_same_bits_and_distributions():
    shape = workloads.StageShape(64, 176, 2)
    a = workloads.make_workload(2, shape=shape)
    b = workloads.make_workload(2, shape=shape)
    c = workloads.make_workload(2, shape=shape, seed=99)
    for s in range(3):
        for x, y, z in zip(a.weights[s], b.weights[s], c.weights[s]):
            assert x.dtype == torch.bfloat16 and torch.equal(x.view(torch.int16), y.view(torch.int16))
            assert not torch.equal(x.view(torch.int16), z.view(torch.int16)) or x.numel() < 4
        for x, y in zip(a.grads[s], b.grads[s]):
            assert x.dtype == torch.float32 and torch.equal(x, y)
    assert np.array_equal(a.sigmas, b.sigmas)
    assert np.all(a.sigmas >= 1e-5) and np.all(a.sigmas <= 1e-2)
    w = torch.cat([t.float().reshape(-1) for t in a.weights[0]])
    assert abs(float(w.std()) - 0.02) < 0.002 and abs(float(w.mean())) < 0.002
    g = a.grads[1][4]
    assert abs(float(g.std()) / a.sigmas[1, 4] - 1) < 0.1


def test_pipeline_workload_loses_an_intermediate_stage():
    shape = workloads.StageShape(32, 88, 1)
    seen = set()
    for seed in range(40):
        wl = workloads.make_workload(5, shape=shape, seed=seed)
        assert 1 <= wl.lost <= 6                      # never the first or the last stage
        seen.add(wl.lost)
        for s in range(8):
            assert len(wl.grads[s]) == 9
            assert (len(wl.weights[s]) == 9) == (abs(s - wl.lost) <= 1)
    assert len(seen) >= 4
    assert workloads.make_workload(5, shape=shape).lost == workloads.make_workload(5, shape=shape).lost


def test_numpy_views_keep_the_bits():
    t = torch.tensor([1.0, -2.5, 3.140625], dtype=torch.bfloat16)
    v = workloads.to_numpy(t)
    assert v.dtype == np.uint16 and v.tolist() == [0x3F80, 0xC020, 0x4049]
    f = torch.tensor([1.5, float("nan")])
    assert workloads.to_numpy(f).dtype == np.float32
