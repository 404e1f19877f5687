// Internal interface between the C ABI (host side) and the gfx950 kernels.
// Not installed; the public contract is include/checkfree.h.
#ifndef CF_KERNELS_H
#define CF_KERNELS_H

#include <hip/hip_runtime_api.h>
#include <stdint.h>

// One unit of work: a contiguous run of elements of one tensor.  A stage's
// chunk table is an array of these in device memory, in tensor order; stages
// that agree in numel and dtype per tensor have tables that agree in everything
// but the addresses, so entry c of three congruent stages names the same
// elements of corresponding tensors.
struct CfChunk {
    uint64_t addr;   // device address of the chunk's first element
    uint32_t len;    // elements
    uint32_t dtype;  // CF_F32 / CF_BF16
};

constexpr int CF_THREADS = 256;          // workgroup size of the norm's first pass: 4 wavefronts
constexpr int CF_WAVES = CF_THREADS / 64;
constexpr int CF_FINALIZE_THREADS = 1024;   // workgroup size of the norm's second pass
constexpr int CF_MAX_SEG = 64;           // stages per sqnorm launch
constexpr int CF_TILE_THREADS = 64;      // blend/copy: one wavefront per workgroup
constexpr uint32_t CF_TILE_BYTES = CF_TILE_THREADS * 16u;   // one 16-byte vector per lane: the blend/copy work unit

// Device word block of a context (CF_CTX_WORDS 32-bit words).
constexpr int CF_CTX_WORDS = 64;
constexpr int CF_WORD_FLAGS = 1;         // sticky CF_FLAG_* bits
constexpr int CF_WORD_FLAGS_READ = 2;    // what the last read-flags kernel saw

struct CfSqnormSeg {
    const CfChunk *chunks;   // the stage's chunk table
    double *partials;        // one slot per chunk
    uint32_t chunk_begin;    // index of the stage's first chunk in the launch
    uint32_t n_chunks;
};

struct CfSqnormArgs {
    CfSqnormSeg seg[CF_MAX_SEG];
    uint32_t n_seg;
    uint32_t total_chunks;
    double *omega_out;       // n_seg doubles
    uint32_t *words;         // context word block
};

// A stage's tensor list as it travels to the table-building kernel: in the
// kernel argument block, CF_TABLE_BATCH tensors per launch, so that describing a
// stage needs no host-to-device copy and no staging buffer.
constexpr int CF_TABLE_BATCH = 128;

struct CfTableTensor {
    uint64_t addr;
    uint64_t numel;
    uint32_t dtype;
    uint32_t first_chunk;    // index of the tensor's first chunk in the stage's table
};

struct CfTableArgs {
    CfTableTensor tensor[CF_TABLE_BATCH];
    CfChunk *chunks;          // the stage's chunk table (device)
    uint32_t *tensor_first;   // num_tensors + 1 entries (device)
    uint32_t n;               // tensors in this launch
    uint32_t tensor_base;     // index of tensor[0] in the stage
    uint32_t chunk_bytes;
    uint32_t end_chunk;       // total chunks of the stage, written behind the last tensor when `last`
    uint32_t last;            // this launch holds the stage's last tensor
};

// The file-scope device array behind the entry point that allocates nothing: its size, and its
// address in the memory of `device` (which must be the current device).  Every GPU holds its own
// copy of the array at its own address; the address is looked up once per device and kept.
constexpr uint64_t CF_STATIC_SCRATCH_BYTES = 1ull << 20;
hipError_t cf_static_scratch_address(int device, void **ptr);

// Writes the chunk table entries and first-chunk indices of the tensors in `args`.
hipError_t cf_launch_build_table(const CfTableArgs &args, hipStream_t stream);

// Sets the CF_CTX_WORDS words of a context's word block to zero.
hipError_t cf_launch_clear_words(uint32_t *words, hipStream_t stream);

// words[CF_WORD_FLAGS_READ] <- words[CF_WORD_FLAGS], atomically exchanged with 0 when `clear`.
hipError_t cf_launch_read_flags(uint32_t *words, int clear, hipStream_t stream);

// First pass over `grid` workgroups, then the fixed-order second pass (one workgroup per stage).
hipError_t cf_launch_sqnorm(const CfSqnormArgs &args, uint32_t grid, hipStream_t stream);

// Per-tensor second pass over a stage's partials (after cf_launch_sqnorm on the same stream):
// tensor t owns chunks tensor_first_chunk[t] .. tensor_first_chunk[t+1]-1.
hipError_t cf_launch_sqnorm_tensors(const double *partials, const uint32_t *tensor_first_chunk, uint32_t num_tensors,
                                    double *d_tensor_out, hipStream_t stream);

// One workgroup per tile; a chunk holds at most 2^tile_shift tiles of CF_TILE_BYTES.
// The weights are read from d_omega_* when those are non-null, else taken from h_omega_*.
// hold_stores: every wavefront holds its vector store back a little (fp32 tensors; pays on large stages only).
hipError_t cf_launch_blend(const CfChunk *prev, const CfChunk *next, const CfChunk *lost, uint32_t n_chunks,
                           uint32_t tile_shift, const double *d_omega_prev, const double *d_omega_next,
                           double h_omega_prev, double h_omega_next, uint32_t *words, bool hold_stores,
                           hipStream_t stream);

// Sizes from which holding the stores back pays (bytes of the written stage, or of the copied range).
constexpr uint64_t CF_BLEND_HOLD_MIN_BYTES = 448ull << 20;
constexpr uint64_t CF_COPY_HOLD_MIN_BYTES = 64ull << 20;

// Scalars of one Adam step, prepared by the host: the bias corrections enter as reciprocals.
struct CfAdamArgs {
    double beta1, one_minus_beta1;
    double beta2, one_minus_beta2;
    double rcp_correction1, rcp_correction2;   // 1 / (1 - beta^t)
    double lr, eps;
};

// One Adam step over four congruent fp32 stages, one workgroup per tile; every tile's sum of
// squared gradients goes to tile_partials[(chunk << tile_shift) + tile], and a second kernel adds a
// chunk's tiles into partials[chunk] (the slots the norm's second pass reads).
hipError_t cf_launch_adam_sqnorm(const CfChunk *weights, const CfChunk *exp_avg, const CfChunk *exp_avg_sq,
                                 const CfChunk *grads, uint32_t n_chunks, uint32_t tile_shift, const CfAdamArgs &p,
                                 double *tile_partials, double *partials, hipStream_t stream);

// The norm's second pass alone (one workgroup per stage of `args`), for partials that are already there.
hipError_t cf_launch_sqnorm_finalize(const CfSqnormArgs &args, hipStream_t stream);

// Chunks first_chunk .. first_chunk + n_chunks - 1 of the two tables.
hipError_t cf_launch_copy(const CfChunk *src, const CfChunk *dst, uint32_t first_chunk, uint32_t n_chunks,
                          uint32_t tile_shift, bool hold_stores, hipStream_t stream);

#endif
