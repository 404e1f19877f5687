"""Seeded synthetic inputs: LLaMa-shaped pipeline stages (weights and gradients).

This module only *draws inputs*; it contains none of the recovery arithmetic
and is the one piece of code that the oracle's tests and the HIP path's tests
and benchmark both use.  The values stand in for the weights and gradients of
the paper's LLaMa models (appendix table "Model hyperparameters": dim 1024 and
2048, 24 layers in 6 stages = 4 decoder layers per stage), which cannot be
trained here; the cost of the path does not depend on the values.

Recipe
  * decoder layer (d, ffn): Wq, Wk, Wv, Wo [d,d]; gate, up [d,ffn]; down [ffn,d];
    attention-norm and ffn-norm vectors [d]  -- 9 tensors, in that order;
  * weights ~ N(0, 0.02) (norm vectors included), fp32, or bf16 = the fp32 draw
    rounded to nearest-even;
  * gradients fp32 ~ N(0, sigma_t), one sigma_t = 10^U(-5,-2) per tensor;
  * one seed per workload.  The sigmas (and the lost-stage index of the
    pipeline workload) come from a host generator seeded with `seed`; the
    tensor values from a generator on the target device seeded with `seed + 1`,
    drawn stage by stage, per stage all weights first (list order), then all
    gradients.
"""
from dataclasses import dataclass, field
from typing import List, Optional

import numpy as np
import torch

PARAM_STD = 0.02
SIGMA_LOG10_RANGE = (-5.0, -2.0)
BASE_SEED = 154610


@dataclass
class StageShape:
    d: int
    ffn: int
    layers: int

    def tensor_shapes(self):
        d, f = self.d, self.ffn
        per_layer = [(d, d), (d, d), (d, d), (d, d), (d, f), (d, f), (f, d), (d,), (d,)]
        return [s for _ in range(self.layers) for s in per_layer]

    def numel(self):
        return sum(int(np.prod(s)) for s in self.tensor_shapes())


@dataclass
class WorkloadSpec:
    name: str
    shape: StageShape
    param_dtype: str = "f32"          # "f32" | "bf16"
    n_stages: int = 3                 # stages that exist in the workload
    seed: int = BASE_SEED
    extra_copy_shapes: list = field(default_factory=list)   # CheckFree+ (de)embedding payload


# The five workloads (1-based ids).
SPECS = {
    1: WorkloadSpec("llama124m-shape-2layer-fp32", StageShape(768, 2048, 2), "f32", 3, BASE_SEED + 1),
    2: WorkloadSpec("llama500m-shape-4layer-bf16w-fp32g", StageShape(1024, 2816, 4), "bf16", 3,
                    BASE_SEED + 2),
    3: WorkloadSpec("llama1.5b-shape-4layer-fp32", StageShape(2048, 5632, 4), "f32", 3, BASE_SEED + 3),
    4: WorkloadSpec("checkfreeplus-copy-1.5b-shape-fp32", StageShape(2048, 5632, 4), "f32", 1,
                    BASE_SEED + 4, [(32000, 2048), (2048, 32000), (2048,)]),
    5: WorkloadSpec("pipeline8x3layer-1.5b-shape-fp32", StageShape(2048, 5632, 3), "f32", 8,
                    BASE_SEED + 5),
}


def _torch_dtype(name):
    return {"f32": torch.float32, "bf16": torch.bfloat16}[name]


def draw_sigmas(n: int, host_rng: np.random.Generator) -> np.ndarray:
    lo, hi = SIGMA_LOG10_RANGE
    return 10.0 ** host_rng.uniform(lo, hi, size=n)


def draw_weights(shapes, dtype_name, gen, device) -> List[torch.Tensor]:
    out = []
    for s in shapes:
        w = torch.empty(s, dtype=torch.float32, device=device).normal_(0.0, PARAM_STD, generator=gen)
        out.append(w.to(_torch_dtype(dtype_name)) if dtype_name != "f32" else w)
    return out


def draw_grads(shapes, sigmas, gen, device) -> List[torch.Tensor]:
    return [torch.empty(s, dtype=torch.float32, device=device).normal_(0.0, float(sig), generator=gen)
            for s, sig in zip(shapes, sigmas)]


@dataclass
class Workload:
    spec: WorkloadSpec
    weights: List[List[torch.Tensor]]        # [stage][tensor]
    grads: List[List[torch.Tensor]]          # [stage][tensor], fp32
    sigmas: np.ndarray                        # [stage, tensor]
    lost: Optional[int] = None                # 0-based index of the lost stage
    extra: List[torch.Tensor] = field(default_factory=list)


def make_workload(config_id: int, device="cpu", shape: Optional[StageShape] = None,
                  seed: Optional[int] = None, with_grads: bool = True) -> Workload:
    """Draw workload `config_id` (1..5).  `shape` overrides the stage shape (for
    reduced-size test cases that keep the structure)."""
    spec = SPECS[config_id]
    if shape is not None:
        spec = WorkloadSpec(spec.name + "-reduced", shape, spec.param_dtype, spec.n_stages, spec.seed,
                            spec.extra_copy_shapes)
    if seed is not None:
        spec = WorkloadSpec(spec.name, spec.shape, spec.param_dtype, spec.n_stages, seed,
                            spec.extra_copy_shapes)
    host_rng = np.random.default_rng(spec.seed)
    gen = torch.Generator(device=device)
    gen.manual_seed(spec.seed + 1)
    shapes = spec.shape.tensor_shapes()
    sigmas = draw_sigmas(spec.n_stages * len(shapes), host_rng).reshape(spec.n_stages, len(shapes))
    lost = None
    if spec.n_stages == 3:
        lost = 1
    elif spec.n_stages > 3:
        lost = int(host_rng.integers(1, spec.n_stages - 1))     # an intermediate stage
    weights, grads = [], []
    for s in range(spec.n_stages):
        # In the pipeline workload only the lost stage and its two neighbours need weights.
        need_w = spec.n_stages <= 3 or abs(s - lost) <= 1
        weights.append(draw_weights(shapes, spec.param_dtype, gen, device) if need_w else [])
        grads.append(draw_grads(shapes, sigmas[s], gen, device) if with_grads else [])
    extra = draw_weights(spec.extra_copy_shapes, "f32", gen, device) if spec.extra_copy_shapes else []
    return Workload(spec, weights, grads, sigmas, lost, extra)


def ragged_shapes(seed: int, n_tensors: int = 11, max_numel: int = 70000):
    """A small stage with awkward tensor sizes (1 element, primes, just above and
    below powers of two) for parity cases that span several tiles and a ragged
    tail."""
    rng = np.random.default_rng(seed)
    fixed = [1, 2, 3, 5, 255, 257, 1023, 4099, 16384, 32771, 65537]
    sizes = fixed[:n_tensors]
    while len(sizes) < n_tensors:
        sizes.append(int(rng.integers(1, max_numel)))
    return [(int(n),) for n in sizes]


def to_numpy(t: torch.Tensor) -> np.ndarray:
    """Host numpy view of a tensor's values: fp32 as float32, bf16 as uint16 bit
    patterns."""
    t = t.detach().contiguous().cpu()
    if t.dtype == torch.bfloat16:
        return t.view(torch.int16).numpy().view(np.uint16)
    return t.numpy()


def stage_to_numpy(stage):
    return [to_numpy(t) for t in stage]
