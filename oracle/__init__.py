"""CheckFree recovery -- CPU oracle (numpy front end of oracle/cf_oracle.c).

TEST INFRASTRUCTURE, NOT A PRODUCT PATH: imported only by tests/, by the smoke
check and by the benchmark's CPU-baseline leg.  It imports nothing from the HIP
package and the HIP package imports nothing from here.

A *stage* is an ordered list of numpy arrays, one per weight (or gradient)
tensor: a stage's weights are the weight tensors of its layers taken together
(section "Problem Statement", paragraph "Distributed Training").
dtype float32 is fp32; dtype uint16 holds bfloat16 bit patterns.

Functions (paper: section "CheckFree: Memoryless Recovery", its display
equation and Algorithm 1; section "CheckFree+: First and Last Stage Recovery"):

  stage_grad_sqnorm(grads)                    omega_i = ||grad W^S_i||^2
  effective_omega(w_prev, w_next)             weights used, incl. the degenerate rule
  recover_stage_weighted_avg(prev, next, ..)  W^S_i = (w_{i-1} W_{i-1} + w_{i+1} W_{i+1}) / (w_{i-1} + w_{i+1})
  blend_unrounded(prev, next, ..)             the same value in binary64, not narrowed
  copy_stage(src)                             bytewise copy (CheckFree+)
  copy_stage_ranges(src, dst, ranges)         slices of that copy (keeping a replica current piece by piece)
  adam_step_with_sqnorm(w, m, v, g, ...)      one Adam step of a stage (the paper's optimizer) and omega of the
                                              gradient it consumed, in the same pass
  recovery_plan(num_stages, lost, plus)       which stages rebuild each lost stage, or why none can
  plus_stage_order(num_stages, microbatch)    CheckFree+ order of the stages for one microbatch
"""
import ctypes
import os

import numpy as np

from . import build_oracle

_LIB = None


def _lib():
    global _LIB
    if _LIB is None:
        # CF_ORACLE_LIB: a differently built copy of the oracle; used only by the mutation
        # tests, which check that the pins reject deliberately broken oracles.
        path = os.environ.get("CF_ORACLE_LIB") or build_oracle.build(force=False)
        lib = ctypes.CDLL(path)
        c_dp = ctypes.POINTER(ctypes.c_double)
        lib.cfo_sqnorm_f32.restype = ctypes.c_double
        lib.cfo_sqnorm_f32.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
        lib.cfo_sqnorm_bf16.restype = ctypes.c_double
        lib.cfo_sqnorm_bf16.argtypes = [ctypes.c_void_p, ctypes.c_uint64]
        lib.cfo_stage_sqnorm_f32.restype = ctypes.c_double
        lib.cfo_stage_sqnorm_f32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32]
        lib.cfo_stage_sqnorm_f32_mt.restype = ctypes.c_double
        lib.cfo_stage_sqnorm_f32_mt.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint32,
                                                ctypes.c_int]
        lib.cfo_effective_omega.restype = ctypes.c_int
        lib.cfo_effective_omega.argtypes = [ctypes.c_double, ctypes.c_double, c_dp, c_dp]
        for name in ("cfo_blend_f32", "cfo_blend_bf16"):
            fn = getattr(lib, name)
            fn.restype = None
            fn.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_void_p, ctypes.c_void_p,
                           ctypes.c_void_p, ctypes.c_uint64, ctypes.c_int]
        lib.cfo_blend_f64.restype = None
        lib.cfo_blend_f64.argtypes = [ctypes.c_double, ctypes.c_double, ctypes.c_void_p,
                                      ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64]
        lib.cfo_copy_bytes.restype = None
        lib.cfo_copy_bytes.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64,
                                       ctypes.c_int]
        lib.cfo_copy_range.restype = None
        lib.cfo_copy_range.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                       ctypes.c_uint32]
        lib.cfo_common_scale.restype = None
        lib.cfo_common_scale.argtypes = [c_dp, c_dp]
        lib.cfo_adam_step_f32.restype = ctypes.c_double
        lib.cfo_adam_step_f32.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                          ctypes.c_uint64, ctypes.c_double, ctypes.c_double, ctypes.c_double,
                                          ctypes.c_double, ctypes.c_uint64]
        lib.cfo_bf16_to_f64.restype = ctypes.c_double
        lib.cfo_bf16_to_f64.argtypes = [ctypes.c_uint16]
        lib.cfo_f64_to_bf16.restype = ctypes.c_uint16
        lib.cfo_f64_to_bf16.argtypes = [ctypes.c_double]
        lib.cfo_max_threads.restype = ctypes.c_int
        lib.cfo_max_threads.argtypes = []
        _LIB = lib
    return _LIB


def max_threads() -> int:
    """Threads OpenMP would use by default on this host."""
    return int(_lib().cfo_max_threads())


def _flat(a, dtype):
    a = np.ascontiguousarray(a)
    if a.dtype != dtype:
        raise TypeError(f"expected {np.dtype(dtype)}, got {a.dtype}")
    return a.reshape(-1)


def stage_grad_sqnorm(grads, threads: int = 1) -> float:
    """omega of one stage: sum over its tensors (list order) of the sum of
    squares of every gradient element, accumulated in binary64.  Gradients are
    fp32 in every workload; a stage holding bf16 gradients (uint16 bit
    patterns) is summed tensor by tensor in the same way."""
    if any(np.asarray(g).dtype == np.uint16 for g in grads):
        omega = 0.0
        for g in grads:
            g = np.ascontiguousarray(g)
            if g.dtype == np.uint16:
                omega += float(_lib().cfo_sqnorm_bf16(g.ctypes.data, g.size))
            else:
                g = _flat(g, np.float32)
                omega += float(_lib().cfo_sqnorm_f32(g.ctypes.data, g.size))
        return omega
    arrs = [_flat(g, np.float32) for g in grads]
    n = len(arrs)
    ptrs = (ctypes.c_void_p * max(n, 1))(*[a.ctypes.data for a in arrs])
    lens = (ctypes.c_uint64 * max(n, 1))(*[a.size for a in arrs])
    if threads <= 1:
        return float(_lib().cfo_stage_sqnorm_f32(ptrs, lens, n))
    return float(_lib().cfo_stage_sqnorm_f32_mt(ptrs, lens, n, int(threads)))


def tensor_grad_sqnorms(grads):
    """The squared norm of each tensor of a stage, in list order; omega is their sum."""
    return [stage_grad_sqnorm([g]) for g in grads]


def effective_omega(omega_prev: float, omega_next: float):
    """(w_prev, w_next, degenerate): the weights the blend really uses."""
    ep, en = ctypes.c_double(), ctypes.c_double()
    flag = _lib().cfo_effective_omega(float(omega_prev), float(omega_next),
                                      ctypes.byref(ep), ctypes.byref(en))
    return ep.value, en.value, bool(flag)


def common_scale(omega_prev: float, omega_next: float):
    """Both weights times the power of two that brings their sum into [1, 2): the
    form in which the blend uses them (the equation is unchanged by a common factor)."""
    wp, wn = ctypes.c_double(float(omega_prev)), ctypes.c_double(float(omega_next))
    _lib().cfo_common_scale(ctypes.byref(wp), ctypes.byref(wn))
    return wp.value, wn.value


def recover_stage_weighted_avg(prev, next, omega_prev: float, omega_next: float,
                               threads: int = 1):
    """The lost stage: for every tensor pair of the two neighbouring stages the
    elementwise weighted average with weights omega_prev, omega_next, computed
    in binary64 and rounded once to the tensors' own type."""
    if len(prev) != len(next):
        raise ValueError("neighbouring stages differ in tensor count")
    out = []
    for a, b in zip(prev, next):
        a = np.ascontiguousarray(a)
        b = np.ascontiguousarray(b)
        if a.shape != b.shape or a.dtype != b.dtype:
            raise ValueError("neighbouring stages are not congruent")
        o = np.empty_like(a)
        if a.dtype == np.float32:
            fn = _lib().cfo_blend_f32
        elif a.dtype == np.uint16:
            fn = _lib().cfo_blend_bf16
        else:
            raise TypeError(f"unsupported weight dtype {a.dtype}")
        fn(float(omega_prev), float(omega_next), a.ctypes.data, b.ctypes.data, o.ctypes.data,
           a.size, int(threads))
        out.append(o)
    return out


def blend_unrounded(prev, next, omega_prev: float, omega_next: float):
    """Binary64 value of the display equation for binary64 inputs, one array."""
    a = _flat(prev, np.float64)
    b = _flat(next, np.float64)
    o = np.empty_like(a)
    _lib().cfo_blend_f64(float(omega_prev), float(omega_next), a.ctypes.data, b.ctypes.data,
                         o.ctypes.data, a.size)
    return o.reshape(np.shape(prev))


def copy_stage(src, threads: int = 1):
    """CheckFree+ recovery of an end stage or of the (de)embedding: every tensor
    reproduced bit for bit."""
    out = []
    for s in src:
        s = np.ascontiguousarray(s)
        d = np.empty_like(s)
        _lib().cfo_copy_bytes(d.ctypes.data, s.ctypes.data, s.nbytes, int(threads))
        out.append(d)
    return out


def copy_stage_ranges(src, dst, ranges):
    """Slices of a stage copy: for every (tensor index, first element, element
    count) in `ranges` those elements of src's tensor are carried into dst's,
    in place; everything else in dst is left alone.  Returns dst."""
    for t, first, count in ranges:
        s, d = src[t], dst[t]
        if s.shape != d.shape or s.dtype != d.dtype or not (s.flags.c_contiguous and d.flags.c_contiguous):
            raise ValueError("source and destination tensors are not congruent contiguous arrays")
        if first < 0 or count < 0 or first + count > s.size:
            raise ValueError("range outside the tensor")
        _lib().cfo_copy_range(d.ctypes.data, s.ctypes.data, int(first), int(count), s.itemsize)
    return dst


def adam_step_with_sqnorm(weights, exp_avg, exp_avg_sq, grads, lr: float, beta1: float = 0.9,
                          beta2: float = 0.999, eps: float = 1e-8, step: int = 1):
    """One Adam step (no weight decay) over every tensor of a stage, IN PLACE on
    the fp32 arrays of `weights`, `exp_avg` (m) and `exp_avg_sq` (v); `step` is t,
    counted from 1.  Returns omega of the stage: the squared norm of `grads`,
    tensors added in list order."""
    if not (len(weights) == len(exp_avg) == len(exp_avg_sq) == len(grads)):
        raise ValueError("the four tensor lists differ in length")
    if step < 1:
        raise ValueError("Adam counts its steps from 1")
    omega = 0.0
    for w, m, v, g in zip(weights, exp_avg, exp_avg_sq, grads):
        for a in (w, m, v, g):
            if a.dtype != np.float32 or not a.flags.c_contiguous or a.shape != w.shape:
                raise ValueError("Adam step takes congruent contiguous float32 arrays")
        omega += float(_lib().cfo_adam_step_f32(w.ctypes.data, m.ctypes.data, v.ctypes.data, g.ctypes.data,
                                                w.size, float(lr), float(beta1), float(beta2), float(eps),
                                                int(step)))
    return omega


def bf16_to_f64(bits: int) -> float:
    return float(_lib().cfo_bf16_to_f64(int(bits)))


def f64_to_bf16(x: float) -> int:
    return int(_lib().cfo_f64_to_bf16(float(x)))


def recovery_plan(num_stages: int, lost, plus: bool = False):
    """For every lost stage (0-based; the (de)embedding layers are not stages),
    ("average", i - 1, i + 1) or ("copy", j), or raises ValueError.

    Algorithm 1 rebuilds stage i from W_{i-1} and W_{i+1}: it exists only for a
    stage with two neighbours (section "CheckFree: Memoryless Recovery", last
    paragraph: no second neighbour to average with at the two ends).  Section
    "CheckFree+: First and Last Stage Recovery": the first stage is copied from
    the second, the last from the second to last.  Both need their sources
    alive: neighbouring stages lost together are beyond either method (the
    comparison table's row for consecutive stages; the limitations paragraph)."""
    lost = list(lost)
    if len(set(lost)) != len(lost) or any(not 0 <= i < num_stages for i in lost):
        raise IndexError("lost stages must be distinct indices below num_stages")
    plan = []
    for i in lost:
        if num_stages < 2:
            raise IndexError("a pipeline of one stage has no neighbour")
        if 0 < i < num_stages - 1:
            step = ("average", i - 1, i + 1)
        elif not plus:
            raise ValueError("CheckFree cannot rebuild the first or the last stage")
        elif i == 0:
            step = ("copy", 1)
        else:
            step = ("copy", num_stages - 2)
        if any(src in lost for src in step[1:]):
            raise ValueError("a neighbouring stage is lost as well")
        plan.append(step)
    return plan


def plus_stage_order(num_stages: int, microbatch: int):
    """The stage at each pipeline position for one microbatch under CheckFree+
    (its section's two printed sequences: S_1, S_2, ..., S_{s-1}, S_s for half
    of the microbatches and S_2, S_1, ..., S_s, S_{s-1} for the other half).
    Which half is which is not said: even microbatches take the first
    sequence here.  The two exchanged pairs have to be distinct."""
    if num_stages < 4:
        raise IndexError("the first two and the last two stages must be four different stages")
    standard = list(range(num_stages))
    if microbatch % 2 == 0:
        return standard
    return [standard[1], standard[0]] + standard[2:-2] + [standard[-1], standard[-2]]
