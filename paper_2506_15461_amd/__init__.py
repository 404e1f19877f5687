"""CheckFree stage recovery on MI355X: thin Python binding of libcheckfree.so.

Argument marshalling only -- every step of the path (squared gradient norms,
norm-to-weight scaling, weighted-average blend, copy) runs in the HIP kernels
behind the C ABI of include/checkfree.h.  PyTorch supplies device memory and
streams.  There is no CPU fallback: without the built library every call here
raises.

Paper: "All is Not Lost: LLM Recovery without Checkpoints", sections "CheckFree:
Memoryless Recovery" (omega_i = ||grad W^S_i||^2, the weighted-average display
equation, Algorithm 1) and "CheckFree+: First and Last Stage Recovery".

    ctx   = Context(0)
    prev  = Stage(ctx, prev_weights);  nxt = Stage(ctx, next_weights);  lost = Stage(ctx, lost_weights)
    gp    = Stage(ctx, prev_grads);    gn  = Stage(ctx, next_grads)
    omega = cf_stage_grad_sqnorm(ctx, [gp, gn])            # float64[2], stays on the device
    cf_recover_stage_weighted_avg(ctx, prev, nxt, omega[0:1], omega[1:2], lost)
    cf_copy_stage(ctx, src, dst)                           # CheckFree+
"""
import ctypes
import os
import weakref

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libcheckfree.so")

CF_OK = 0
CF_ERR_NULL, CF_ERR_SHAPE_MISMATCH, CF_ERR_DTYPE, CF_ERR_ALIGN = -1, -2, -3, -4
CF_ERR_LIMIT, CF_ERR_HIP, CF_ERR_ALIAS, CF_ERR_CONTEXT, CF_ERR_VALUE = -5, -6, -7, -8, -9
CF_F32, CF_BF16 = 0, 1
CF_FLAG_DEGENERATE_OMEGA, CF_FLAG_NONFINITE_OMEGA = 1, 2
CF_RECOVER_WEIGHTED_AVG, CF_RECOVER_COPY = 0, 1

# Every symbol include/checkfree.h declares.
EXPORTS = (
    "cf_ctx_create", "cf_ctx_destroy", "cf_stage_create", "cf_stage_destroy",
    "cf_stage_num_tensors", "cf_stage_numel", "cf_stage_nbytes", "cf_stage_num_chunks",
    "cf_stage_grad_sqnorm", "cf_recover_stage_weighted_avg", "cf_copy_stage", "cf_read_flags",
    "cf_plan_num_chunks", "cf_plan_chunks", "cf_default_tuning", "cf_status_string",
    "cf_recover_stage_with_weights", "cf_recovered_learning_rate", "cf_check_stage_pair",
    "cf_stage_grad_sqnorm_per_tensor",
    "cf_workspace_bytes", "cf_ctx_create_in", "cf_stage_table_bytes", "cf_stage_create_in",
    "cf_copy_stage_range", "cf_stage_grad_sqnorm_static", "cf_static_scratch_bytes",
    "cf_adam_scratch_bytes", "cf_adam_step_with_sqnorm",
    "cf_plan_recovery", "cf_plus_stage_order",
)


class CfTensor(ctypes.Structure):
    _fields_ = [("data", ctypes.c_void_p), ("numel", ctypes.c_uint64),
                ("dtype", ctypes.c_int32), ("reserved", ctypes.c_int32)]


class CfAdamParams(ctypes.Structure):
    _fields_ = [("learning_rate", ctypes.c_double), ("beta1", ctypes.c_double), ("beta2", ctypes.c_double),
                ("epsilon", ctypes.c_double), ("step", ctypes.c_uint64)]


class CfRecoveryStep(ctypes.Structure):
    _fields_ = [("lost", ctypes.c_uint32), ("kind", ctypes.c_int32), ("prev", ctypes.c_uint32),
                ("next", ctypes.c_uint32)]


class CfTuning(ctypes.Structure):
    _fields_ = [("chunk_bytes", ctypes.c_uint32), ("sqnorm_blocks_per_cu", ctypes.c_uint32),
                ("reserved0", ctypes.c_uint32), ("reserved1", ctypes.c_uint32)]


class CheckFreeError(RuntimeError):
    def __init__(self, status, what):
        self.status = status
        super().__init__(f"{what}: {status_string(status)} ({status})")


_lib = None


def load_library():
    """Loads libcheckfree.so (once).  PyTorch is imported first so that the
    library binds to the HIP runtime PyTorch already carries."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(
            f"{LIB_PATH} is not built; run `python -c 'import __graft_entry__ as g; g.build()'` "
            "(or `python paper_2506_15461_amd/build.py`).  There is no fallback path.")
    try:
        import torch  # noqa: F401  (brings in libamdhip64)
    except Exception:
        pass
    lib = ctypes.CDLL(LIB_PATH)
    vp, u32, u64, i32 = ctypes.c_void_p, ctypes.c_uint32, ctypes.c_uint64, ctypes.c_int32
    lib.cf_ctx_create.restype = i32
    lib.cf_ctx_create.argtypes = [ctypes.c_int, ctypes.POINTER(CfTuning), ctypes.POINTER(vp)]
    lib.cf_workspace_bytes.restype = u64
    lib.cf_workspace_bytes.argtypes = []
    lib.cf_ctx_create_in.restype = i32
    lib.cf_ctx_create_in.argtypes = [ctypes.c_int, ctypes.POINTER(CfTuning), vp, u64, vp, ctypes.POINTER(vp)]
    lib.cf_stage_table_bytes.restype = u64
    lib.cf_stage_table_bytes.argtypes = [vp, ctypes.POINTER(CfTensor), u32]
    lib.cf_stage_create_in.restype = i32
    lib.cf_stage_create_in.argtypes = [vp, ctypes.POINTER(CfTensor), u32, vp, u64, vp, ctypes.POINTER(vp)]
    lib.cf_copy_stage_range.restype = i32
    lib.cf_copy_stage_range.argtypes = [vp, vp, vp, u32, u32, vp]
    lib.cf_stage_grad_sqnorm_static.restype = i32
    lib.cf_stage_grad_sqnorm_static.argtypes = [vp, ctypes.POINTER(CfTensor), u32, vp, vp]
    lib.cf_static_scratch_bytes.restype = u64
    lib.cf_static_scratch_bytes.argtypes = []
    lib.cf_adam_scratch_bytes.restype = u64
    lib.cf_adam_scratch_bytes.argtypes = [vp]
    lib.cf_adam_step_with_sqnorm.restype = i32
    lib.cf_adam_step_with_sqnorm.argtypes = [vp, vp, vp, vp, vp, ctypes.POINTER(CfAdamParams), vp, u64, vp, vp]
    lib.cf_ctx_destroy.restype = i32
    lib.cf_ctx_destroy.argtypes = [vp]
    lib.cf_stage_create.restype = i32
    lib.cf_stage_create.argtypes = [vp, ctypes.POINTER(CfTensor), u32, ctypes.POINTER(vp)]
    lib.cf_stage_destroy.restype = i32
    lib.cf_stage_destroy.argtypes = [vp]
    lib.cf_stage_num_tensors.restype = u32
    lib.cf_stage_num_tensors.argtypes = [vp]
    lib.cf_stage_numel.restype = u64
    lib.cf_stage_numel.argtypes = [vp]
    lib.cf_stage_nbytes.restype = u64
    lib.cf_stage_nbytes.argtypes = [vp]
    lib.cf_stage_num_chunks.restype = u32
    lib.cf_stage_num_chunks.argtypes = [vp]
    lib.cf_stage_grad_sqnorm.restype = i32
    lib.cf_stage_grad_sqnorm.argtypes = [vp, ctypes.POINTER(vp), u32, vp, vp]
    lib.cf_stage_grad_sqnorm_per_tensor.restype = i32
    lib.cf_stage_grad_sqnorm_per_tensor.argtypes = [vp, vp, vp, vp, vp]
    lib.cf_recover_stage_weighted_avg.restype = i32
    lib.cf_recover_stage_weighted_avg.argtypes = [vp, vp, vp, vp, vp, vp, vp]
    lib.cf_recover_stage_with_weights.restype = i32
    lib.cf_recover_stage_with_weights.argtypes = [vp, vp, vp, ctypes.c_double, ctypes.c_double, vp, vp]
    lib.cf_recovered_learning_rate.restype = ctypes.c_double
    lib.cf_recovered_learning_rate.argtypes = [ctypes.c_double]
    lib.cf_plan_recovery.restype = i32
    lib.cf_plan_recovery.argtypes = [u32, ctypes.POINTER(u32), u32, ctypes.c_int, ctypes.POINTER(CfRecoveryStep)]
    lib.cf_plus_stage_order.restype = i32
    lib.cf_plus_stage_order.argtypes = [u32, u64, ctypes.POINTER(u32)]
    lib.cf_copy_stage.restype = i32
    lib.cf_copy_stage.argtypes = [vp, vp, vp, vp]
    lib.cf_read_flags.restype = i32
    lib.cf_read_flags.argtypes = [vp, vp, ctypes.POINTER(u32), ctypes.c_int]
    lib.cf_plan_num_chunks.restype = u64
    lib.cf_plan_num_chunks.argtypes = [ctypes.POINTER(CfTensor), u32, u32]
    lib.cf_plan_chunks.restype = i32
    lib.cf_plan_chunks.argtypes = [ctypes.POINTER(CfTensor), u32, u32, ctypes.POINTER(u32),
                                   ctypes.POINTER(u64), ctypes.POINTER(u32), u64]
    lib.cf_check_stage_pair.restype = i32
    lib.cf_check_stage_pair.argtypes = [ctypes.POINTER(CfTensor), u32, ctypes.POINTER(CfTensor), u32]
    lib.cf_default_tuning.restype = None
    lib.cf_default_tuning.argtypes = [ctypes.POINTER(CfTuning)]
    lib.cf_status_string.restype = ctypes.c_char_p
    lib.cf_status_string.argtypes = [i32]
    _lib = lib
    return lib


def status_string(status: int) -> str:
    return load_library().cf_status_string(int(status)).decode()


def _check(status, what):
    if status != CF_OK:
        raise CheckFreeError(status, what)


def default_tuning() -> dict:
    t = CfTuning()
    load_library().cf_default_tuning(ctypes.byref(t))
    return {name: getattr(t, name) for name, _ in CfTuning._fields_}


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _dtype_code(t):
    import torch
    if t.dtype == torch.float32:
        return CF_F32
    if t.dtype == torch.bfloat16:
        return CF_BF16
    raise CheckFreeError(CF_ERR_DTYPE, f"tensor dtype {t.dtype}")


def tensor_descriptors(tensors):
    """ctypes array of cf_tensor for a list of contiguous torch tensors."""
    arr = (CfTensor * max(len(tensors), 1))()
    for i, t in enumerate(tensors):
        if not t.is_contiguous():
            raise ValueError("stage tensors must be contiguous")
        arr[i].data = t.data_ptr() if t.numel() else None
        arr[i].numel = t.numel()
        arr[i].dtype = _dtype_code(t)
        arr[i].reserved = 0
    return arr


class Context:
    """cf_ctx: per-device bookkeeping (launch shape, sticky flag word).

    By default the context's device word block is a torch allocation handed to
    cf_ctx_create_in (nothing is allocated by the library, nothing waited for;
    the block is cleared by a kernel on `stream`).  owned=True lets the library
    allocate it (cf_ctx_create)."""

    def __init__(self, device=0, owned=False, stream=None, **tuning):
        import torch
        self._h = ctypes.c_void_p()
        self.device = torch.device("cuda", device) if isinstance(device, int) else torch.device(device)
        index = self.device.index if self.device.index is not None else torch.cuda.current_device()
        self.device = torch.device("cuda", index)
        self._stages = weakref.WeakSet()
        t = CfTuning(**{k: int(v) for k, v in tuning.items()}) if tuning else None
        tp = ctypes.byref(t) if t is not None else None
        lib = load_library()
        self.workspace = None
        if owned or not torch.cuda.is_available():
            _check(lib.cf_ctx_create(index, tp, ctypes.byref(self._h)), "cf_ctx_create")
        else:
            nbytes = int(lib.cf_workspace_bytes())
            self.workspace = torch.empty(nbytes, dtype=torch.uint8, device=self.device)
            _check(lib.cf_ctx_create_in(index, tp, ctypes.c_void_p(self.workspace.data_ptr()), nbytes,
                                        _stream_ptr(stream), ctypes.byref(self._h)), "cf_ctx_create_in")

    def read_flags(self, clear=False, stream=None) -> int:
        out = ctypes.c_uint32(0)
        _check(load_library().cf_read_flags(self._h, _stream_ptr(stream), ctypes.byref(out), int(bool(clear))),
               "cf_read_flags")
        return int(out.value)

    def close(self):
        """Destroys the context and, first, every stage still alive on it."""
        if self._h:
            for st in list(self._stages):
                st.close()
            load_library().cf_ctx_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


class Stage:
    """cf_stage: the tensor list of one pipeline stage (weights or gradients).
    Keeps the tensors alive; the library only borrows their memory.

    By default the stage's device tables live in a torch allocation handed to
    cf_stage_create_in: creating the handle allocates nothing in the library,
    copies nothing and waits for nothing; the tables are written by a small
    kernel on `stream` (default: the current stream), and work that uses the
    stage must be ordered after it.  `table` is an existing uint8 device
    tensor of at least stage_table_bytes(ctx, tensors) bytes to use instead of a
    new one.  owned=True lets the library allocate the tables and wait
    (cf_stage_create)."""

    def __init__(self, ctx: Context, tensors, owned=False, stream=None, table=None):
        import torch
        self.ctx = ctx
        self.tensors = list(tensors)
        for t in self.tensors:
            if t.device != ctx.device:
                raise ValueError(f"tensor on {t.device}, context on {ctx.device}")
        self._h = ctypes.c_void_p()
        self.table = None
        desc = tensor_descriptors(self.tensors)
        lib = load_library()
        if owned:
            _check(lib.cf_stage_create(ctx._h, desc, len(self.tensors), ctypes.byref(self._h)), "cf_stage_create")
        else:
            nbytes = int(lib.cf_stage_table_bytes(ctx._h, desc, len(self.tensors)))
            if nbytes == 2 ** 64 - 1:
                nbytes = 0          # an invalid list: cf_stage_create_in names the reason
            if table is None:
                table = torch.empty(nbytes, dtype=torch.uint8, device=ctx.device)
            elif table.dtype != torch.uint8 or not table.is_contiguous() or table.device != ctx.device:
                raise ValueError("table must be a contiguous uint8 tensor on the context's device")
            self.table = table
            _check(lib.cf_stage_create_in(ctx._h, desc, len(self.tensors),
                                          ctypes.c_void_p(table.data_ptr() if table.numel() else None), table.numel(),
                                          _stream_ptr(stream), ctypes.byref(self._h)), "cf_stage_create_in")
        ctx._stages.add(self)

    def __repr__(self):
        return f"Stage({len(self.tensors)} tensors, {self.numel} elements, {self.nbytes} bytes, {self.num_chunks} chunks)"

    @property
    def numel(self):
        return int(load_library().cf_stage_numel(self._h))

    @property
    def nbytes(self):
        return int(load_library().cf_stage_nbytes(self._h))

    @property
    def num_chunks(self):
        return int(load_library().cf_stage_num_chunks(self._h))

    def close(self):
        if self._h:
            load_library().cf_stage_destroy(self._h)
            self._h = ctypes.c_void_p()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def stage_table_bytes(ctx: Context, tensors) -> int:
    """Bytes of device memory cf_stage_create_in needs for a stage of these tensors."""
    desc = tensor_descriptors(list(tensors))
    n = int(load_library().cf_stage_table_bytes(ctx._h, desc, len(tensors)))
    if n == 2 ** 64 - 1:
        raise CheckFreeError(CF_ERR_LIMIT, "cf_stage_table_bytes")
    return n


def cf_stage_grad_sqnorm(ctx: Context, grad_stages, out=None, stream=None):
    """omega_s = ||grad W^S_s||^2 for every stage of `grad_stages`, one launch.
    Returns a float64 device tensor of len(grad_stages) (written into `out` if
    given).  Asynchronous on the stream."""
    import torch
    n = len(grad_stages)
    if out is None:
        out = torch.empty(n, dtype=torch.float64, device=ctx.device)
    if out.dtype != torch.float64 or out.numel() < n or not out.is_contiguous() or out.device != ctx.device:
        raise ValueError("out must be a contiguous float64 device tensor with one element per stage")
    handles = (ctypes.c_void_p * max(n, 1))(*[s._h for s in grad_stages])
    _check(load_library().cf_stage_grad_sqnorm(ctx._h, handles, n, ctypes.c_void_p(out.data_ptr()),
                                               _stream_ptr(stream)), "cf_stage_grad_sqnorm")
    return out


def cf_stage_grad_sqnorm_static(ctx: Context, grads, out, stream=None):
    """omega of one stage given as a list of gradient tensors, written into the
    one-element float64 device tensor `out`; the library's tables live in its
    static per-GPU array, so nothing is allocated anywhere on the way."""
    desc = tensor_descriptors(list(grads))
    _check(load_library().cf_stage_grad_sqnorm_static(ctx._h, desc, len(grads), _omega_ptr(ctx, out),
                                                      _stream_ptr(stream)), "cf_stage_grad_sqnorm_static")
    return out


def adam_scratch_bytes(grads: Stage) -> int:
    return int(load_library().cf_adam_scratch_bytes(grads._h))


def cf_adam_step_with_sqnorm(ctx: Context, weights: Stage, exp_avg: Stage, exp_avg_sq: Stage, grads: Stage,
                             lr: float, beta1: float = 0.9, beta2: float = 0.999, eps: float = 1e-8, step: int = 1,
                             scratch=None, out=None, stream=None):
    """One Adam step of a stage (weights, exp_avg, exp_avg_sq updated in place) and,
    from the same pass over `grads`, omega of the stage as a one-element float64
    device tensor.  `scratch` is a uint8 device tensor of adam_scratch_bytes(grads)
    bytes (allocated here if not given).  Asynchronous on the stream."""
    import torch
    need = adam_scratch_bytes(grads)
    if scratch is None:
        scratch = torch.empty(need, dtype=torch.uint8, device=ctx.device)
    if out is None:
        out = torch.empty(1, dtype=torch.float64, device=ctx.device)
    params = CfAdamParams(float(lr), float(beta1), float(beta2), float(eps), int(step))
    _check(load_library().cf_adam_step_with_sqnorm(
        ctx._h, weights._h, exp_avg._h, exp_avg_sq._h, grads._h, ctypes.byref(params),
        ctypes.c_void_p(scratch.data_ptr() if scratch.numel() else None), scratch.numel(), _omega_ptr(ctx, out),
        _stream_ptr(stream)), "cf_adam_step_with_sqnorm")
    return out


def cf_stage_grad_sqnorm_per_tensor(ctx: Context, grad_stage: Stage, stream=None):
    """(omega, per-tensor squared norms) of one stage as float64 device tensors
    of 1 and len(tensors) elements.  Asynchronous on the stream."""
    import torch
    n = len(grad_stage.tensors)
    omega = torch.empty(1, dtype=torch.float64, device=ctx.device)
    per_tensor = torch.empty(n, dtype=torch.float64, device=ctx.device)
    _check(load_library().cf_stage_grad_sqnorm_per_tensor(
        ctx._h, grad_stage._h, ctypes.c_void_p(per_tensor.data_ptr() if n else None),
        ctypes.c_void_p(omega.data_ptr()), _stream_ptr(stream)), "cf_stage_grad_sqnorm_per_tensor")
    return omega, per_tensor


def _omega_ptr(ctx, w):
    import torch
    if w.dtype != torch.float64 or w.numel() != 1 or w.device != ctx.device:
        raise ValueError("omega must be a one-element float64 device tensor (e.g. omega[i:i+1])")
    return ctypes.c_void_p(w.data_ptr())


def cf_recover_stage_weighted_avg(ctx: Context, prev: Stage, next: Stage, omega_prev, omega_next,
                                  lost: Stage, stream=None):
    """lost <- (omega_prev * prev + omega_next * next) / (omega_prev + omega_next),
    the omegas read from device memory by the kernel.  Asynchronous."""
    _check(load_library().cf_recover_stage_weighted_avg(
        ctx._h, prev._h, next._h, _omega_ptr(ctx, omega_prev), _omega_ptr(ctx, omega_next), lost._h,
        _stream_ptr(stream)), "cf_recover_stage_weighted_avg")
    return lost


def cf_recover_stage_with_weights(ctx: Context, prev: Stage, next: Stage, omega_prev: float, omega_next: float,
                                  lost: Stage, stream=None):
    """The recovery with host-supplied weights (uniform average: equal weights;
    copy of one neighbour: zero weight on the other).  Asynchronous."""
    _check(load_library().cf_recover_stage_with_weights(
        ctx._h, prev._h, next._h, float(omega_prev), float(omega_next), lost._h, _stream_ptr(stream)),
        "cf_recover_stage_with_weights")
    return lost


def cf_recovered_learning_rate(learning_rate: float) -> float:
    """1.1 x the stage's current learning rate (Algorithm 1, third step)."""
    return float(load_library().cf_recovered_learning_rate(float(learning_rate)))


def cf_plan_recovery(num_stages: int, lost, checkfree_plus: bool = False):
    """[(lost, kind, prev, next), ...] for the lost stages (0-based), kind being
    CF_RECOVER_WEIGHTED_AVG or CF_RECOVER_COPY; raises CheckFreeError when a stage
    cannot be rebuilt (an end stage without CheckFree+, neighbouring stages lost
    together).  Host logic only."""
    lost = [int(i) for i in lost]
    arr = (ctypes.c_uint32 * max(1, len(lost)))(*lost)
    steps = (CfRecoveryStep * max(1, len(lost)))()
    _check(load_library().cf_plan_recovery(int(num_stages), arr, len(lost), int(bool(checkfree_plus)), steps),
           "cf_plan_recovery")
    return [(s.lost, s.kind, s.prev, s.next) for s in steps[:len(lost)]]


def cf_plus_stage_order(num_stages: int, microbatch: int):
    """The stage that runs at each pipeline position for this microbatch under
    CheckFree+ (first two and last two stages exchanged on odd microbatches)."""
    order = (ctypes.c_uint32 * max(1, int(num_stages)))()
    _check(load_library().cf_plus_stage_order(int(num_stages), int(microbatch), order), "cf_plus_stage_order")
    return list(order[:int(num_stages)])


def cf_copy_stage(ctx: Context, src: Stage, dst: Stage, stream=None):
    """dst <- src bit for bit (CheckFree+ end-stage / (de)embedding recovery)."""
    _check(load_library().cf_copy_stage(ctx._h, src._h, dst._h, _stream_ptr(stream)), "cf_copy_stage")
    return dst


def cf_copy_stage_range(ctx: Context, src: Stage, dst: Stage, first_chunk: int, n_chunks: int, stream=None):
    """dst <- src for chunks first_chunk .. first_chunk + n_chunks - 1 only (a slice of
    a replica refresh); the rest of dst is left as it is."""
    _check(load_library().cf_copy_stage_range(ctx._h, src._h, dst._h, int(first_chunk), int(n_chunks),
                                              _stream_ptr(stream)), "cf_copy_stage_range")
    return dst


def check_stage_pair(inputs, outputs) -> int:
    """Host-only: status of the (input, output) congruence and aliasing check for
    descriptor lists given as (address, numel, dtype) triples."""
    def pack(items):
        arr = (CfTensor * max(len(items), 1))()
        for i, (addr, numel, dtype) in enumerate(items):
            arr[i].data = addr or None
            arr[i].numel = int(numel)
            arr[i].dtype = int(dtype)
        return arr
    return int(load_library().cf_check_stage_pair(pack(inputs), len(inputs), pack(outputs), len(outputs)))


def plan_chunks(numels, chunk_bytes, dtype=CF_F32):
    """Host-only: the chunk plan (tensor index, first element, length) the
    library would use for tensors of the given element counts."""
    n = len(numels)
    arr = (CfTensor * max(n, 1))()
    for i, m in enumerate(numels):
        arr[i].data = None
        arr[i].numel = int(m)
        arr[i].dtype = dtype
    lib = load_library()
    total = lib.cf_plan_num_chunks(arr, n, int(chunk_bytes))
    if total == 2 ** 64 - 1:
        raise CheckFreeError(CF_ERR_LIMIT, "cf_plan_num_chunks")
    cap = max(int(total), 1)
    ct = (ctypes.c_uint32 * cap)()
    cf = (ctypes.c_uint64 * cap)()
    cl = (ctypes.c_uint32 * cap)()
    _check(lib.cf_plan_chunks(arr, n, int(chunk_bytes), ct, cf, cl, int(total)), "cf_plan_chunks")
    return [(ct[i], cf[i], cl[i]) for i in range(int(total))]
