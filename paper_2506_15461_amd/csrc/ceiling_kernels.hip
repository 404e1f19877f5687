// Two trivial streaming kernels over ONE flat buffer -- no chunk table, no tensor list, no reduction
// beyond a dummy -- used only by the benchmark to measure what this GPU's memory system sustains for a
// read-only stream and for a copy, independently of the library's own kernels.  Built into its own
// small library (libcf_ceiling.so); nothing in libcheckfree.so uses it.
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
#define CFC_GLOBAL __attribute__((address_space(1)))

// Grid-stride read of n16 sixteen-byte vectors; the sum only keeps the loads alive.
__global__ __launch_bounds__(256) void cfc_read_kernel(const CFC_GLOBAL u32x4 *src, uint64_t n16, uint32_t *sink)
{
    uint32_t acc = 0;
    const uint64_t stride = (uint64_t)gridDim.x * 256u;
    for (uint64_t i = (uint64_t)blockIdx.x * 256u + threadIdx.x; i < n16; i += stride) {
        const u32x4 v = __builtin_nontemporal_load(src + i);
        acc += v.x ^ v.y ^ v.z ^ v.w;
    }
    if (acc == 0x9E3779B9u) *sink = acc;   // practically never: the store exists so the loop is not removed
}

// One vector per thread, one 1 KiB tile per 64-thread workgroup, in address order.
__global__ __launch_bounds__(64) void cfc_copy_kernel(const CFC_GLOBAL u32x4 *src, CFC_GLOBAL u32x4 *dst, uint64_t n16)
{
    const uint64_t i = (uint64_t)blockIdx.x * 64u + threadIdx.x;
    if (i < n16) __builtin_nontemporal_store(__builtin_nontemporal_load(src + i), dst + i);
}

extern "C" {

// Reads `bytes` (a multiple of 16, 16-byte aligned) from device memory on `stream` with
// `workgroups` workgroups of 256 threads.  `d_sink` is 4 bytes of device memory.  Returns a hipError_t.
__attribute__((visibility("default"))) int cfc_read(const void *d_src, uint64_t bytes, void *d_sink,
                                                    uint32_t workgroups, void *stream)
{
    if (!d_src || !d_sink || bytes % 16 || !workgroups) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(cfc_read_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       (const CFC_GLOBAL u32x4 *)d_src, bytes / 16, static_cast<uint32_t *>(d_sink));
    return (int)hipGetLastError();
}

// Copies `bytes` (a multiple of 16, below 2^31 KiB, both pointers 16-byte aligned) on `stream`.
__attribute__((visibility("default"))) int cfc_copy(const void *d_src, void *d_dst, uint64_t bytes, void *stream)
{
    const uint64_t n16 = bytes / 16;
    const uint64_t grid = (n16 + 63) / 64;
    if (!d_src || !d_dst || bytes % 16 || grid == 0 || grid > 0x7FFFFFFFull) return (int)hipErrorInvalidValue;
    hipLaunchKernelGGL(cfc_copy_kernel, dim3((uint32_t)grid), dim3(64), 0, static_cast<hipStream_t>(stream),
                       (const CFC_GLOBAL u32x4 *)d_src, (CFC_GLOBAL u32x4 *)d_dst, n16);
    return (int)hipGetLastError();
}

}  // extern "C"
