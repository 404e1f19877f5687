/*
 * checkfree.h -- C ABI of the CheckFree stage-recovery hot path on AMD CDNA4
 * (gfx950), hand-written HIP behind plain C entry points.
 *
 * Paper: "All is Not Lost: LLM Recovery without Checkpoints" (CheckFree /
 * CheckFree+).  A pipeline *stage* S_i holds a consecutive block of layers; its
 * weights W^S_i are all the weight tensors of those layers taken together
 * (section "Problem Statement", paragraph "Distributed Training").  Here a stage
 * is an ordered list of contiguous device tensors.
 *
 * The three operations:
 *
 *   cf_stage_grad_sqnorm           omega_i = || grad W^S_i ||^2
 *       (section "CheckFree: Memoryless Recovery": every stage keeps the squared
 *       norm of its last gradient, one scalar, ready for a newcomer)
 *
 *   cf_recover_stage_weighted_avg  W^S_i = (omega_{i-1} W^S_{i-1} + omega_{i+1} W^S_{i+1})
 *                                          / (omega_{i-1} + omega_{i+1})
 *       (display equation of that section; Algorithm 1, third step)
 *
 *   cf_copy_stage                  W^S_dst = W^S_src, bit for bit
 *       (section "CheckFree+: First and Last Stage Recovery": a first/last stage
 *       is restored from its neighbour, embedding and de-embedding without any
 *       loss from the replicas kept on the neighbouring stages)
 *
 * General rules
 *   - Every function returns a cf_status (0 = CF_OK, negative = error) and never
 *     throws, aborts or exits.  Nothing is launched when an error is returned.
 *   - Pointers named d_* and every cf_tensor.data are DEVICE pointers; everything
 *     else is a HOST pointer.
 *   - The library never allocates, frees or keeps alive tensor memory.  A handle
 *     needs a small device block (a context 256 bytes; a stage 24 bytes per
 *     chunk and 4 per tensor: about 150 KB for a 1.5B-parameter-model stage).
 *     With cf_ctx_create_in / cf_stage_create_in that block is the caller's
 *     (sized by cf_workspace_bytes / cf_stage_table_bytes) and creating a
 *     handle allocates no device memory, copies nothing between host and
 *     device and waits for nothing: it enqueues one small kernel per 128
 *     tensors on the caller's stream.  cf_ctx_create / cf_stage_create are the
 *     same calls on a block the library allocates itself, followed by a wait.
 *   - The hot calls allocate nothing, copy nothing between host and device,
 *     and do not synchronise: they enqueue work on the caller's stream and
 *     return.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *   - Calls may be issued on any streams.  A stage handle made by
 *     cf_stage_create_in is usable by work that is ordered after the stream it
 *     was created on (the same stream, or after a wait on it).  The only shared
 *     device state is the context's flag word (updated atomically) and, per
 *     stage handle, the scratch of cf_stage_grad_sqnorm inside the stage's
 *     block: the same gradient-stage handle must not be in two
 *     cf_stage_grad_sqnorm calls that may run at the same time.
 *   - Entry points may be called from several host threads; a handle must not be
 *     destroyed while another thread still uses it.
 *   - Data-dependent conditions cannot be returned synchronously; they raise
 *     sticky bits in a device flag word read by cf_read_flags.
 */
#ifndef CHECKFREE_H
#define CHECKFREE_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#if defined(__GNUC__) || defined(__clang__)
#define CF_API __attribute__((visibility("default")))
#else
#define CF_API
#endif

typedef int32_t cf_status;

enum {
    CF_OK = 0,
    CF_ERR_NULL = -1,            /* a required pointer argument is NULL */
    CF_ERR_SHAPE_MISMATCH = -2,  /* stages differ in tensor count, numel or dtype */
    CF_ERR_DTYPE = -3,           /* unknown dtype, or a dtype the operation does not take */
    CF_ERR_ALIGN = -4,           /* tensor data not aligned to its element size */
    CF_ERR_LIMIT = -5,           /* a size exceeds what the library supports */
    CF_ERR_HIP = -6,             /* a HIP runtime call failed (no device, bad stream, ...) */
    CF_ERR_ALIAS = -7,           /* output tensors overlap inputs other than element for element */
    CF_ERR_CONTEXT = -8,         /* handles belong to different contexts */
    CF_ERR_VALUE = -9            /* a scalar argument outside its domain */
};

/* Element types of stage tensors. */
enum {
    CF_F32 = 0,   /* IEEE binary32 */
    CF_BF16 = 1   /* bfloat16 (upper half of a binary32) */
};

/* Sticky device flags (cf_read_flags). */
enum {
    CF_FLAG_DEGENERATE_OMEGA = 1u,  /* a recovery saw an unusable omega pair and used the uniform average */
    CF_FLAG_NONFINITE_OMEGA = 2u    /* a squared norm came out Inf or NaN */
};

/* One contiguous tensor in device memory.  `data` must be aligned to the element
 * size; nothing more is required.  Every kernel moves 16 bytes per lane, with
 * the vector body placed on the 128-byte boundaries of the tensor it writes and
 * the tensors it reads read at whatever alignment they have: views into flat
 * buffers at odd offsets run within a few per cent of tensors that came from
 * an allocator.  numel may be 0 (then data may be NULL). */
typedef struct cf_tensor {
    void *data;      /* device pointer */
    uint64_t numel;  /* number of elements */
    int32_t dtype;   /* CF_F32 or CF_BF16 */
    int32_t reserved;
} cf_tensor;

/* Launch shape knobs.  Zero in any field keeps the default. */
typedef struct cf_tuning {
    uint32_t chunk_bytes;          /* bytes per work chunk: a power of two, 4 KiB .. 4 MiB (default 128 KiB);
                                      results of the norm differ between chunk sizes only in the last bits */
    uint32_t sqnorm_blocks_per_cu; /* grid of the norm's first pass: 1..64 = at most that many workgroups per
                                      compute unit, every workgroup with the same number of chunks; 65 = one
                                      workgroup per chunk; default 0 = 2 per compute unit (the measured best
                                      from 100 MB to several GB).  Never changes a result bit. */
    uint32_t reserved0;
    uint32_t reserved1;
} cf_tuning;

typedef struct cf_ctx cf_ctx;      /* opaque: per-device bookkeeping */
typedef struct cf_stage cf_stage;  /* opaque: a stage's tensor list, uploaded once */

/* ---- set-up in caller-provided device memory: allocates no device memory,
 *      copies nothing, never synchronises ---- */

/* Bytes of device memory a context needs (its word block: sticky flags). */
CF_API uint64_t cf_workspace_bytes(void);

/* Creates a context on HIP device `device` whose word block is the caller's
 * DEVICE memory `d_workspace` (at least cf_workspace_bytes() bytes, 16-byte
 * aligned, alive and untouched by others until cf_ctx_destroy).  One small
 * kernel on `stream` clears it; work that uses the context must be ordered
 * after that.  `tuning` may be NULL.
 * Errors: CF_ERR_NULL, CF_ERR_ALIGN, CF_ERR_LIMIT (workspace too small, bad
 * tuning value), CF_ERR_HIP. */
CF_API cf_status cf_ctx_create_in(int device, const cf_tuning *tuning, void *d_workspace,
                                  uint64_t workspace_bytes, void *stream, cf_ctx **out);

/* Bytes of device memory the tables of a stage with these tensors need under
 * `ctx`'s chunk size (0 for a stage without tensors).  UINT64_MAX if the list
 * would be refused by cf_stage_create_in. */
CF_API uint64_t cf_stage_table_bytes(const cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors);

/* Describes a stage (paper, section "Problem Statement": a stage's weights are
 * the weight tensors of its layers; Algorithm 1, the two "Receive" steps, is
 * where a joining node first holds its neighbours' stages and needs handles
 * for them): `tensors` is a HOST array of `num_tensors` descriptors, borrowed
 * only for the duration of this call.  The tensors' memory is borrowed for as
 * long as the stage handle is used; the caller keeps it alive and at the same
 * addresses.  The stage's tables are written into the caller's DEVICE memory
 * `d_table` (at least cf_stage_table_bytes() bytes, 16-byte aligned, alive and
 * untouched by others until cf_stage_destroy; may be NULL when that size is 0)
 * by small kernels enqueued on `stream`, fed from their argument blocks (128
 * tensors per launch).  num_tensors may be 0.
 * Errors: CF_ERR_NULL, CF_ERR_DTYPE, CF_ERR_ALIGN, CF_ERR_LIMIT (table_bytes
 * too small, a tensor above 2^40 elements, or a stage above 2^31 - 1 one-KiB
 * tiles, about 2 TiB), CF_ERR_HIP. */
CF_API cf_status cf_stage_create_in(cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, void *d_table,
                                    uint64_t table_bytes, void *stream, cf_stage **out);

/* ---- the same set-up on memory the library allocates (convenience; these two
 *      call hipMalloc and wait for the set-up kernels) ---- */

/* cf_ctx_create_in on a block of cf_workspace_bytes() bytes from hipMalloc,
 * ready on return.  Errors: CF_ERR_NULL, CF_ERR_HIP, CF_ERR_LIMIT (bad tuning
 * value). */
CF_API cf_status cf_ctx_create(int device, const cf_tuning *tuning, cf_ctx **out);

/* Destroys the context (and frees its word block if the library allocated it).
 * Stages created from it must be destroyed first: while any is alive this
 * returns CF_ERR_CONTEXT and frees nothing.  NULL is accepted. */
CF_API cf_status cf_ctx_destroy(cf_ctx *ctx);

/* cf_stage_create_in on a block of cf_stage_table_bytes() bytes from hipMalloc,
 * on the default stream, ready for use on any stream on return.  Errors as for
 * cf_stage_create_in. */
CF_API cf_status cf_stage_create(cf_ctx *ctx, const cf_tensor *tensors, uint32_t num_tensors, cf_stage **out);

/* Destroys the handle (never the tensors; the tables only if the library
 * allocated them).  Work that uses the handle must have finished.  NULL is
 * accepted. */
CF_API cf_status cf_stage_destroy(cf_stage *stage);

/* Introspection; 0 for a NULL handle. */
CF_API uint32_t cf_stage_num_tensors(const cf_stage *stage);
CF_API uint64_t cf_stage_numel(const cf_stage *stage);   /* elements over all tensors */
CF_API uint64_t cf_stage_nbytes(const cf_stage *stage);  /* bytes over all tensors */
CF_API uint32_t cf_stage_num_chunks(const cf_stage *stage);

/* ---- the hot path ---- */

/* omega_s = sum over every tensor of grad_stages[s] of the sum of squares of its
 * elements, for s = 0 .. n_stages-1, in ONE multi-tensor streaming launch over
 * all stages (groups of at most 64 stages per launch) plus its second pass.  Paper: section "CheckFree: Memoryless Recovery",
 * omega_i = ||grad W^S_i||^2; Algorithm 1, the two "Receive" steps.
 *
 *   grad_stages  HOST array of n_stages stage handles (tensors CF_F32 or CF_BF16)
 *   d_omega_out  DEVICE array of n_stages doubles, written by the kernel
 *
 * Every element is widened to binary64, squared and accumulated there per
 * lane, reduced per wavefront (cross-lane moves) and then per workgroup
 * (through LDS) to one binary64 partial per chunk at a fixed slot, and the
 * partials of a stage are summed in a fixed order by a second, tiny kernel
 * enqueued right behind the first: the result is bit-identical from run to run
 * and does not depend on the grid size.  Squares of binary32 values neither
 * underflow nor overflow in binary64, and the relative error of omega is below
 * 1e-10 for every stage size and every accepted tuning (all terms are
 * non-negative, so it is at most the length of the longest chain of additions,
 * at most 2^19, times 2^-53; about 1e-14 for a 1.5B-parameter-model stage).  An
 * empty stage gives 0.  A non-finite result (a NaN or Inf gradient) raises
 * CF_FLAG_NONFINITE_OMEGA.  The same stage handle must not appear in two
 * sqnorm calls that run concurrently (each handle's block holds its
 * partial-sum scratch, 8 bytes per chunk).
 * Errors: CF_ERR_NULL, CF_ERR_CONTEXT, CF_ERR_LIMIT, CF_ERR_HIP. */
CF_API cf_status cf_stage_grad_sqnorm(cf_ctx *ctx, const cf_stage *const *grad_stages, uint32_t n_stages,
                               double *d_omega_out, void *stream);

/* omega of ONE stage and, alongside, the squared norm of each of its tensors
 * (what a gradient-clipping or monitoring pass wants from the same read of the
 * gradients): the streaming pass of cf_stage_grad_sqnorm runs once, then two
 * independent second passes add its per-chunk partials per stage and per tensor.
 *
 *   d_tensor_sqnorm  DEVICE array of cf_stage_num_tensors(grad_stage) doubles
 *   d_omega_out      DEVICE, one double; bit-identical to what
 *                    cf_stage_grad_sqnorm writes for the same stage
 *
 * The per-tensor values are each a fixed-order binary64 sum of that tensor's
 * partials; their sum equals omega up to binary64 rounding, not bit for bit.
 * Errors: CF_ERR_NULL, CF_ERR_CONTEXT, CF_ERR_LIMIT, CF_ERR_HIP. */
CF_API cf_status cf_stage_grad_sqnorm_per_tensor(cf_ctx *ctx, const cf_stage *grad_stage,
                                                 double *d_tensor_sqnorm, double *d_omega_out, void *stream);

/* For callers that cannot allocate device memory at all -- code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc: omega of ONE
 * stage given as a bare tensor list (HOST array, borrowed for the call), as
 * cf_stage_grad_sqnorm computes it and with the same bits, but with the chunk
 * table and the partial sums in a fixed array inside the library's device image
 * instead of in a stage handle's block.  Calls no hipMalloc / hipFree and no
 * allocating routine, copies nothing between host and device, does not wait.
 *
 *   d_omega_out  DEVICE, one double
 *
 * The array is cf_static_scratch_bytes() bytes (1 MiB) per GPU, held from the
 * first context created on that GPU until the process ends.  A stage needs 24
 * bytes per chunk and 4 per tensor of it (rounded up to 256-byte sections): with
 * the default 128 KiB chunk that is room for about 5.7 GB of gradients; a larger
 * stage is refused with CF_ERR_LIMIT and nothing is launched.  All calls on one
 * GPU share that GPU's array, whatever their context or stream: two calls that
 * may run at the same time on one GPU race, and the caller must order them.
 * Nothing in the array has to be cleared between calls.
 * Errors: CF_ERR_NULL, CF_ERR_DTYPE, CF_ERR_ALIGN, CF_ERR_LIMIT, CF_ERR_HIP. */
CF_API cf_status cf_stage_grad_sqnorm_static(cf_ctx *ctx, const cf_tensor *grads, uint32_t num_tensors,
                                             double *d_omega_out, void *stream);

/* Size in bytes of the per-GPU array cf_stage_grad_sqnorm_static works in. */
CF_API uint64_t cf_static_scratch_bytes(void);

/* ---- omega at no extra memory traffic: as a by-product of the optimizer step ---- */

/* Scalars of one Adam step.  The paper trains with Adam, no weight decay, betas
 * (0.9, 0.999) (appendix "Optimizers"); it names no epsilon (1e-8 is the value of
 * the algorithm's authors). */
typedef struct cf_adam_params {
    double learning_rate;   /* finite */
    double beta1, beta2;    /* in [0, 1) */
    double epsilon;         /* >= 0, finite */
    uint64_t step;          /* t of this step, counted from 1 */
} cf_adam_params;

/* Bytes of DEVICE scratch cf_adam_step_with_sqnorm needs for this gradient stage
 * (8 bytes per KiB of gradients: one partial sum per tile).  0 for NULL. */
CF_API uint64_t cf_adam_scratch_bytes(const cf_stage *grads);

/* One Adam step over a whole stage AND omega of the gradient it consumed, in one
 * pass over the gradients.  Paper: section "CheckFree: Memoryless Recovery" (every
 * stage keeps omega = ||grad W^S||^2 of its last gradient, ready for a newcomer)
 * and appendix "Optimizers" (Adam): the optimizer step reads every gradient
 * element anyway, so omega leaves it as a by-product and keeping it current
 * costs no memory traffic of its own.
 *
 * For every element (Kingma & Ba, Algorithm 1; t = params->step):
 *   m <- beta1 m + (1 - beta1) g          v <- beta2 v + (1 - beta2) g^2
 *   w <- w - lr (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps)
 * in binary64; m and v are rounded once to binary32 when stored and the weight
 * update uses the stored values; w is rounded once; eps is outside the root.
 * The two bias corrections are applied as multiplications by their binary64
 * reciprocals.
 *
 *   weights, exp_avg (m), exp_avg_sq (v)   updated in place; CF_F32 tensors only
 *   grads                                   read only; CF_F32; its handle's scratch
 *                                           is used as by cf_stage_grad_sqnorm
 *   d_scratch                               DEVICE, cf_adam_scratch_bytes(grads)
 *                                           bytes, 8-byte aligned, caller's
 *   d_omega_out                             DEVICE, one double: the sum of g^2 over
 *                                           the stage, bit-reproducible; the same
 *                                           terms as cf_stage_grad_sqnorm adds, in
 *                                           another fixed order, so equal to it to
 *                                           within rounding (relative 1e-14), not
 *                                           bit for bit
 *
 * The four stages must agree tensor by tensor in numel (CF_ERR_SHAPE_MISMATCH);
 * none of weights, exp_avg, exp_avg_sq may overlap another of the four other
 * than element for element (CF_ERR_ALIAS).  Enqueues three kernels on `stream`;
 * allocates nothing, copies nothing, does not wait.  A non-finite omega raises
 * CF_FLAG_NONFINITE_OMEGA.
 * Errors: CF_ERR_NULL, CF_ERR_CONTEXT, CF_ERR_SHAPE_MISMATCH, CF_ERR_DTYPE,
 * CF_ERR_ALIAS, CF_ERR_VALUE (a parameter outside its domain), CF_ERR_LIMIT
 * (scratch too small), CF_ERR_ALIGN, CF_ERR_HIP. */
CF_API cf_status cf_adam_step_with_sqnorm(cf_ctx *ctx, cf_stage *weights, cf_stage *exp_avg, cf_stage *exp_avg_sq,
                                          const cf_stage *grads, const cf_adam_params *params, void *d_scratch,
                                          uint64_t scratch_bytes, double *d_omega_out, void *stream);

/* Rebuilds a lost intermediate stage from its two neighbours:
 *   lost[t][k] = (w_p * prev[t][k] + w_n * next[t][k]) / (w_p + w_n)
 * for every tensor t and element k, with w_p = *d_omega_prev, w_n = *d_omega_next
 * read from DEVICE memory by the kernel (so the norms never visit the host).
 * Paper: display equation of section "CheckFree: Memoryless Recovery"; Algorithm
 * 1's third step prints omega_{i-1} on both terms, which contradicts the
 * section's own special cases; the display equation is followed.
 *
 * Arithmetic per element: both products and their sum in binary64, each rounded
 * separately (no fused multiply-add), times the binary64 reciprocal of
 * (w_p + w_n), one rounding (nearest even) to the tensor's dtype.  Subnormals are
 * kept.  Before that both weights are multiplied by the power of two that brings
 * their sum into [1, 2) (exact, and the equation does not change under a common
 * factor), so no product leaves the binary64 range however large or small the
 * omegas are.
 *
 * If the pair is unusable -- either omega negative, NaN or Inf, or their sum not
 * a positive normal binary64 number -- both weights are replaced by 1 (the
 * uniform average) and CF_FLAG_DEGENERATE_OMEGA is raised.
 *
 * prev, next and lost must agree tensor by tensor in numel and dtype
 * (CF_ERR_SHAPE_MISMATCH).  A tensor of `lost` may be the very same memory as the
 * corresponding tensor of prev or next; any other overlap is CF_ERR_ALIAS.
 * Errors: CF_ERR_NULL, CF_ERR_SHAPE_MISMATCH, CF_ERR_ALIAS, CF_ERR_CONTEXT,
 * CF_ERR_HIP. */
CF_API cf_status cf_recover_stage_weighted_avg(cf_ctx *ctx, const cf_stage *prev, const cf_stage *next,
                                        const double *d_omega_prev, const double *d_omega_next,
                                        cf_stage *lost, void *stream);

/* The same recovery with the two weights given by the HOST, for the strategies
 * the paper compares the gradient-norm weighting with (section "Motivation",
 * the re-initialisation figure; section "CheckFree: Memoryless Recovery"):
 *   omega_prev = omega_next (any positive value)   uniform average of the neighbours
 *   omega_next = 0, omega_prev > 0                 copy of the previous stage
 *   omega_prev = 0, omega_next > 0                 copy of the next stage
 * and for callers that keep their omegas on the host.  Arithmetic, degenerate
 * rule, flags, aliasing rules and errors as for cf_recover_stage_weighted_avg. */
CF_API cf_status cf_recover_stage_with_weights(cf_ctx *ctx, const cf_stage *prev, const cf_stage *next,
                                               double omega_prev, double omega_next, cf_stage *lost,
                                               void *stream);

/* Copies every tensor of src into the corresponding tensor of dst, bit for bit
 * (NaN payloads, signed zeros and subnormals included); bytes outside dst's
 * tensors are not touched.  Paper: section "CheckFree+: First and Last Stage
 * Recovery" (first/last stage from its neighbour; embedding, de-embedding from
 * their replicas).  src and dst must agree in numel and dtype per tensor
 * (CF_ERR_SHAPE_MISMATCH) and must not overlap unless identical (CF_ERR_ALIAS).
 * Errors: CF_ERR_NULL, CF_ERR_SHAPE_MISMATCH, CF_ERR_ALIAS, CF_ERR_CONTEXT,
 * CF_ERR_HIP. */
CF_API cf_status cf_copy_stage(cf_ctx *ctx, const cf_stage *src, cf_stage *dst, void *stream);

/* The same copy for the chunks first_chunk .. first_chunk + n_chunks - 1 of the
 * stage only (chunks as cf_plan_chunks lists them for the context's chunk size;
 * cf_stage_num_chunks of them in all); every other byte of dst is left as it
 * is.  Paper: section "CheckFree+: First and Last Stage Recovery", last
 * paragraph: the embedding and de-embedding layers are kept as replicas on the
 * neighbouring stages so that they can be restored without loss; keeping such a
 * replica current means copying it again every iteration, and this call lets
 * that copy be issued in slices, on a side stream, between the compute-bound
 * kernels of a training step instead of as one bandwidth-bound block.
 * Errors: as cf_copy_stage, and CF_ERR_LIMIT if the range reaches past the
 * stage's last chunk. */
CF_API cf_status cf_copy_stage_range(cf_ctx *ctx, const cf_stage *src, cf_stage *dst, uint32_t first_chunk,
                                     uint32_t n_chunks, void *stream);

/* ---- after the fact ---- */

/* Enqueues a one-thread kernel on `stream` that reads the context's sticky flag
 * word and, if `clear` is non-zero, resets it to 0 in the same atomic
 * operation (a flag raised meanwhile by work on another stream is either
 * reported now or kept for the next read); waits for `stream`; stores the value
 * in *flags (HOST).  One cf_read_flags at a time per context.
 * Errors: CF_ERR_NULL, CF_ERR_HIP. */
CF_API cf_status cf_read_flags(cf_ctx *ctx, void *stream, uint32_t *flags, int clear);

/* ---- host-only helpers (no device needed) ---- */

/* Number of work chunks a tensor list is cut into with `chunk_bytes` bytes per
 * chunk (every tensor starts a new chunk; an empty tensor has none).  Only numel
 * and dtype of the descriptors are read.  Returns UINT64_MAX on a NULL list with
 * num_tensors > 0, an unknown dtype or an invalid chunk_bytes. */
CF_API uint64_t cf_plan_num_chunks(const cf_tensor *tensors, uint32_t num_tensors, uint32_t chunk_bytes);

/* Writes the chunk plan into HOST arrays of capacity `cap` chunks: the tensor
 * each chunk belongs to, its first element and its length in elements.  Returns
 * CF_ERR_LIMIT if cap is too small. */
CF_API cf_status cf_plan_chunks(const cf_tensor *tensors, uint32_t num_tensors, uint32_t chunk_bytes,
                         uint32_t *chunk_tensor, uint64_t *chunk_first, uint32_t *chunk_len, uint64_t cap);

/* The check cf_recover_stage_* and cf_copy_stage apply to an (input stage, output
 * stage) pair, on bare descriptors: every descriptor valid (CF_ERR_DTYPE,
 * CF_ERR_NULL, CF_ERR_ALIGN, CF_ERR_LIMIT), same tensor count, numel and dtype
 * tensor by tensor (CF_ERR_SHAPE_MISMATCH), no output tensor sharing a byte with
 * any input tensor except its own counterpart at exactly the same address, and
 * no two output tensors sharing a byte (CF_ERR_ALIAS).  Pointers are compared,
 * never dereferenced. */
CF_API cf_status cf_check_stage_pair(const cf_tensor *in, uint32_t num_in, const cf_tensor *out,
                                     uint32_t num_out);

/* Learning rate of a stage that has just been recovered: the paper scales the
 * stage's current rate up by 1.1 (Algorithm 1, third step; the scheduler then
 * carries on from there).  Pure host arithmetic. */
#define CF_RECOVERY_LR_FACTOR 1.1
CF_API double cf_recovered_learning_rate(double learning_rate);

/* How one lost stage is rebuilt, and from which live stages (0-based indices
 * into the pipeline's stages, the embedding and de-embedding layers not
 * counted). */
enum {
    CF_RECOVER_WEIGHTED_AVG = 0,  /* cf_recover_stage_weighted_avg(prev, next, their omegas) */
    CF_RECOVER_COPY = 1           /* cf_copy_stage(prev); next == prev */
};

typedef struct cf_recovery_step {
    uint32_t lost;   /* the stage to rebuild */
    int32_t kind;    /* CF_RECOVER_WEIGHTED_AVG or CF_RECOVER_COPY */
    uint32_t prev;   /* source stage(s) */
    uint32_t next;
} cf_recovery_step;

/* Which operation restores each of the `n_lost` stages in `lost` (HOST array,
 * any order, no repeats) of a pipeline of `num_stages` stages; steps[k] answers
 * lost[k] (HOST array of n_lost entries, written only on CF_OK).
 *   - An intermediate stage i is the weighted average of stages i-1 and i+1
 *     (Algorithm 1: it receives W_{i-1}, omega_{i-1}, W_{i+1}, omega_{i+1}).
 *   - The first and the last stage have a single neighbour.  Plain CheckFree
 *     (checkfree_plus == 0) cannot rebuild them: CF_ERR_VALUE.  CheckFree+
 *     (section "CheckFree+: First and Last Stage Recovery") copies the second
 *     stage into the first and the second to last into the last, which the
 *     swapped execution order has trained to stand in for them.
 *   - A source stage must be alive: two neighbouring stages lost together
 *     cannot be rebuilt by either method (the paper's comparison table and its
 *     limitations paragraph): CF_ERR_VALUE.
 * CF_ERR_LIMIT: a stage index >= num_stages, a repeated index, or fewer than 3
 * stages (2 for a copy).  n_lost == 0 is CF_OK.  Pure host logic. */
CF_API cf_status cf_plan_recovery(uint32_t num_stages, const uint32_t *lost, uint32_t n_lost, int checkfree_plus,
                                  cf_recovery_step *steps);

/* CheckFree+ execution order of the stages for one microbatch (same section):
 * half of the microbatches run the stages in their standard order, the other
 * half with the first two stages exchanged and the last two exchanged, so that
 * the second stage learns the first one's role and the second to last the
 * last one's.  order[p] (HOST array of num_stages entries) is the stage that
 * runs at position p.  The paper does not say which half is which: here the
 * even-numbered microbatches keep the standard order and the odd-numbered ones
 * are exchanged.  The two exchanged pairs must be distinct: num_stages >= 4,
 * else CF_ERR_LIMIT.  Pure host logic. */
CF_API cf_status cf_plus_stage_order(uint32_t num_stages, uint64_t microbatch, uint32_t *order);

/* The tuning values in effect when `tuning` is NULL or holds zeros. */
CF_API void cf_default_tuning(cf_tuning *out);

/* A static, human-readable name for a status code. */
CF_API const char *cf_status_string(cf_status status);

#ifdef __cplusplus
}
#endif
#endif /* CHECKFREE_H */
