// Device-side helpers shared by the kernel files: address-space-qualified
// pointer types, the fixed-order wavefront and workgroup sums, and the one-element
// step of the squared norm.  Header-only; included by .hip files only.
#ifndef CF_DEVICE_H
#define CF_DEVICE_H

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// Tensor data is always device (global) memory; saying so keeps the compiler
// from emitting generic-address (flat) memory instructions.
#define CF_GLOBAL __attribute__((address_space(1)))
typedef CF_GLOBAL const float *gcf32;
typedef CF_GLOBAL float *gf32;
typedef CF_GLOBAL const f32x4 *gcf32x4;
typedef CF_GLOBAL f32x4 *gf32x4;
typedef CF_GLOBAL const u32x4 *gcu32x4;
typedef CF_GLOBAL u32x4 *gu32x4;
typedef CF_GLOBAL const uint16_t *gcu16;
typedef CF_GLOBAL uint16_t *gu16;
typedef CF_GLOBAL const uint32_t *gcu32;
typedef CF_GLOBAL uint32_t *gu32;
typedef CF_GLOBAL const unsigned char *gcu8;
typedef CF_GLOBAL unsigned char *gu8;

// Sixteen-byte vectors that are only known to be aligned to their element (4 or
// 2 bytes).  The vector body of a kernel is laid on the 128-byte boundaries of
// the tensor it writes; the tensors it reads may sit differently inside their
// lines, and are then read with the same one-instruction 16-byte loads at
// whatever alignment they have (global memory accesses need no more than that
// on this platform).
typedef f32x4 f32x4_e4 __attribute__((aligned(4)));
typedef u32x4 u32x4_e4 __attribute__((aligned(4)));
typedef u32x4 u32x4_e2 __attribute__((aligned(2)));
typedef CF_GLOBAL const f32x4_e4 *gcf32x4_e4;
typedef CF_GLOBAL f32x4_e4 *gf32x4_e4;
typedef CF_GLOBAL const u32x4_e4 *gcu32x4_e4;
typedef CF_GLOBAL const u32x4_e2 *gcu32x4_e2;

constexpr uint32_t kFlagDegenerateOmega = 1u;
constexpr uint32_t kFlagNonfiniteOmega = 2u;
constexpr uint32_t kDtypeF32 = 0u;

// ---------------------------------------------------------------------------
// Wavefront reduction on the DPP cross-lane path (no LDS traffic).
// ---------------------------------------------------------------------------

template <int kCtrl>
__device__ __forceinline__ double dpp_permute(double v)
{
    const int lo = __builtin_amdgcn_update_dpp(0, __double2loint(v), kCtrl, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, __double2hiint(v), kCtrl, 0xF, 0xF, true);
    return __hiloint2double(hi, lo);
}

__device__ __forceinline__ double read_lane(double v, int lane)
{
    return __hiloint2double(__builtin_amdgcn_readlane(__double2hiint(v), lane),
                            __builtin_amdgcn_readlane(__double2loint(v), lane));
}

// Sum of v over the 64 lanes, same value in a fixed association on every run:
// butterfly inside each row of 16 lanes (quad_perm [1,0,3,2], quad_perm
// [2,3,0,1], row_half_mirror, row_mirror; a binary64 value moves as its two
// halves), then the four row sums as (r0 + r1) + (r2 + r3).
__device__ __forceinline__ double wave_sum(double v)
{
    v += dpp_permute<0xB1>(v);
    v += dpp_permute<0x4E>(v);
    v += dpp_permute<0x141>(v);
    v += dpp_permute<0x140>(v);
    return (read_lane(v, 0) + read_lane(v, 16)) + (read_lane(v, 32) + read_lane(v, 48));
}

// Elements before the first 128-byte boundary at or after `addr`.  The vector
// body of every streaming kernel starts there, so that the 1 KiB a wavefront
// moves per memory instruction covers eight whole cache lines: on this chip a
// body that is only 16-byte aligned (a tensor that is a view into a flat buffer,
// say) costs a two-read-one-write stream 17 % of its bandwidth, because every
// wavefront then writes two partial lines.
constexpr uint32_t kBodyAlign = 128;

__device__ __forceinline__ uint32_t head_elems(uint64_t addr, uint32_t elem_bytes, uint32_t len)
{
    uint32_t h = (uint32_t)((kBodyAlign - (uint32_t)(addr & (kBodyAlign - 1u))) & (kBodyAlign - 1u)) / elem_bytes;
    return h < len ? h : len;
}

// Sum over a workgroup of kThreads threads in a fixed order: the wavefront
// butterfly, then the wavefront sums added one after the other by thread 0 (one
// barrier).  The result is valid in thread 0 only.
template <int kThreads>
__device__ __forceinline__ double block_sum_fixed_order(double v, double *wave_sums)
{
    const uint32_t tid = threadIdx.x;
    const double w = wave_sum(v);
    if ((tid & 63u) == 0) wave_sums[tid >> 6] = w;
    __syncthreads();
    double total = 0.0;
    if (tid == 0) {
#pragma unroll
        for (int k = 0; k < kThreads / 64; ++k) total += wave_sums[k];
    }
    return total;
}

// One element's share of a squared norm: widened to binary64 (exact), squared
// and added there.
__device__ __forceinline__ void sq_acc(double &acc, float v)
{
    const double x = (double)v;
    acc = __builtin_fma(x, x, acc);
}

}  // namespace

#endif
