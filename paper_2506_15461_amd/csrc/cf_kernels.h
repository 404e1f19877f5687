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

// Device word block owned by a context.
constexpr int CF_WORD_FLAGS = 1;         // sticky CF_FLAG_* bits

struct CfSqnormSeg {
    const CfChunk *chunks;   // the stage's chunk table
    float *partials;         // one slot per chunk
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

// First pass over `grid` workgroups, then the fixed-order second pass (one workgroup per stage).
hipError_t cf_launch_sqnorm(const CfSqnormArgs &args, uint32_t grid, hipStream_t stream);

// Per-tensor second pass over a stage's partials (after cf_launch_sqnorm on the same stream):
// tensor t owns chunks tensor_first_chunk[t] .. tensor_first_chunk[t+1]-1.
hipError_t cf_launch_sqnorm_tensors(const float *partials, const uint32_t *tensor_first_chunk, uint32_t num_tensors,
                                    double *d_tensor_out, hipStream_t stream);

// One workgroup per tile; a chunk holds at most 2^tile_shift tiles of CF_TILE_BYTES.
// The weights are read from d_omega_* when those are non-null, else taken from h_omega_*.
hipError_t cf_launch_blend(const CfChunk *prev, const CfChunk *next, const CfChunk *lost, uint32_t n_chunks,
                           uint32_t tile_shift, const double *d_omega_prev, const double *d_omega_next,
                           double h_omega_prev, double h_omega_next, uint32_t *words, hipStream_t stream);

hipError_t cf_launch_copy(const CfChunk *src, const CfChunk *dst, uint32_t n_chunks, uint32_t tile_shift,
                          hipStream_t stream);

#endif
