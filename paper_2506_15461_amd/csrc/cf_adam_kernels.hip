// omega as a by-product of the optimizer step (gfx950).
//
// Paper: every stage keeps omega = ||grad W^S||^2 of its last gradient (section
// "CheckFree: Memoryless Recovery"), and training uses Adam without weight decay
// (appendix "Optimizers").  The optimizer step is the one pass of an iteration
// that reads every gradient element anyway; here it also squares it, so keeping
// omega current costs no HBM traffic of its own.
//
// The step is a four-read-three-write stream (g, m, v, w in; m, v, w out; 28 bytes
// per element), and on this chip such mixed streams run fastest as tiny work
// units dispatched in address order: one single-wavefront workgroup per 1 KiB
// tile, one 16-byte vector per lane and stream, exactly the walk of the blend and
// copy kernels.  Each tile leaves one binary64 partial sum of squares; a second
// kernel adds the tiles of every chunk in a fixed order into the stage's
// per-chunk partial slots, and the norm's own second pass finishes omega.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "cf_device.h"
#include "cf_kernels.h"

// Every binary64 operation below is rounded on its own, as the update rule is
// written; the only fused multiply-add is the explicit one of the squared norm,
// whose product is exact anyway.
#pragma clang fp contract(off)

namespace {

// One element of Adam (Kingma & Ba, Algorithm 1) in binary64 with binary32
// storage: the moments are rounded once when stored and the weight update uses
// the stored values; eps sits beside the square root.  Dividing by the bias
// corrections is done as a multiplication by their binary64 reciprocals.
__device__ __forceinline__ void adam_element(const CfAdamArgs &p, float g, float &m, float &v, float &w, double &sq)
{
    const double grad = (double)g;
    sq = __builtin_fma(grad, grad, sq);
    const double m_new = p.beta1 * (double)m + p.one_minus_beta1 * grad;
    const double v_new = p.beta2 * (double)v + p.one_minus_beta2 * (grad * grad);
    m = (float)m_new;
    v = (float)v_new;
    const double m_hat = (double)m * p.rcp_correction1;
    const double v_hat = (double)v * p.rcp_correction2;
    w = (float)((double)w - (p.lr * m_hat) / (__builtin_sqrt(v_hat) + p.eps));
}

// Workgroup index -> (chunk, tile of the chunk), as in the blend.  The tile's
// sum of squares goes to tile_partials[blockIdx.x]; a tile past a chunk's end
// finds no element and writes 0 there (the adding kernel does not read it).
//
// At most three wavefronts per SIMD: with four streams read and three written
// per wavefront, more of them in flight than that only get in each other's way
// in the memory system.  Measured on this chip (µs per step, 57 / 196 / 784 MiB
// per stream): 8 per SIMD 70.2 / 240.3 / 949.8, 4: 68.4 / 230.0 / 911.2,
// 3: 67.5 / 224.7 / 897.1, 2: 75.8 / 254.7 / 1029.9.
__global__ __launch_bounds__(CF_TILE_THREADS) __attribute__((amdgpu_waves_per_eu(1, 3))) void cf_adam_sqnorm_kernel(const CfChunk *weights, const CfChunk *exp_avg,
                                                                        const CfChunk *exp_avg_sq, const CfChunk *grads,
                                                                        uint32_t tile_shift, CfAdamArgs p,
                                                                        double *tile_partials)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t c = blockIdx.x >> tile_shift;
    const uint32_t tile = blockIdx.x & ((1u << tile_shift) - 1u);
    const CfChunk cg = grads[c];
    const uint32_t len = cg.len;   // a tile past the end of a short chunk finds no vector below and adds 0
    const CfChunk cw = weights[c];
    const CfChunk cm = exp_avg[c];
    const CfChunk cv = exp_avg_sq[c];
    gcf32 pg = (gcf32)cg.addr;
    gf32 pm = (gf32)cm.addr;
    gf32 pv = (gf32)cv.addr;
    gf32 pw = (gf32)cw.addr;

    // The vector body lies on the 128-byte boundaries of the weights; gradient and moments are
    // read, and the moments written, at whatever alignment they have.
    double sq = 0.0;
    const uint32_t head = head_elems(cw.addr, 4u, len);   // whole lines for the streams that are written
    const uint32_t rem = len - head;
    const uint32_t n4 = rem >> 2;
    const uint32_t vi = tile * CF_TILE_THREADS + tid;
    if (vi < n4) {
        const f32x4 g = __builtin_nontemporal_load((gcf32x4_e4)(pg + head) + vi);
        f32x4 m = __builtin_nontemporal_load((gcf32x4_e4)(pm + head) + vi);
        f32x4 v = __builtin_nontemporal_load((gcf32x4_e4)(pv + head) + vi);
        f32x4 w = __builtin_nontemporal_load((gcf32x4)(pw + head) + vi);
        float m0 = m.x, m1 = m.y, m2 = m.z, m3 = m.w;
        float v0 = v.x, v1 = v.y, v2 = v.z, v3 = v.w;
        float w0 = w.x, w1 = w.y, w2 = w.z, w3 = w.w;
        double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
        adam_element(p, g.x, m0, v0, w0, s0);
        adam_element(p, g.y, m1, v1, w1, s1);
        adam_element(p, g.z, m2, v2, w2, s2);
        adam_element(p, g.w, m3, v3, w3, s3);
        sq = (s0 + s1) + (s2 + s3);
        m.x = m0, m.y = m1, m.z = m2, m.w = m3;
        v.x = v0, v.y = v1, v.z = v2, v.w = v3;
        w.x = w0, w.y = w1, w.z = w2, w.w = w3;
        __builtin_nontemporal_store(m, (gf32x4_e4)(pm + head) + vi);
        __builtin_nontemporal_store(v, (gf32x4_e4)(pv + head) + vi);
        __builtin_nontemporal_store(w, (gf32x4)(pw + head) + vi);
    }
    if (tile == 0) {
        // the few elements before and after the 128-byte aligned body
        const uint32_t tail = rem & 3u;
        const uint32_t tbase = head + (n4 << 2);
        uint32_t i = len;   // none
        if (tid < head) i = tid;
        else if (tid - head < tail) i = tbase + (tid - head);
        if (i < len) {
            float m = pm[i], v = pv[i], w = pw[i];
            adam_element(p, pg[i], m, v, w, sq);
            pm[i] = m;
            pv[i] = v;
            pw[i] = w;
        }
    }
    const double t = wave_sum(sq);
    if (tid == 0) tile_partials[blockIdx.x] = t;
}

// One wavefront per chunk adds the chunk's tile partials in a fixed order
// (lane-strided, then the wavefront butterfly) into the stage's per-chunk slot.
__global__ __launch_bounds__(CF_TILE_THREADS) void cf_tile_partials_kernel(const CfChunk *grads, uint32_t tile_shift,
                                                                          const double *tile_partials, double *partials)
{
    const uint32_t c = blockIdx.x;
    const uint64_t nbytes = (uint64_t)grads[c].len * 4u;
    uint32_t tiles = (uint32_t)((nbytes + CF_TILE_BYTES - 1) / CF_TILE_BYTES);
    if (tiles == 0) tiles = 1;
    const double *src = tile_partials + ((uint64_t)c << tile_shift);
    double acc = 0.0;
    for (uint32_t j = threadIdx.x; j < tiles; j += CF_TILE_THREADS) acc += src[j];
    const double total = wave_sum(acc);
    if (threadIdx.x == 0) partials[c] = total;
}

}  // namespace

hipError_t cf_launch_adam_sqnorm(const CfChunk *weights, const CfChunk *exp_avg, const CfChunk *exp_avg_sq,
                                 const CfChunk *grads, uint32_t n_chunks, uint32_t tile_shift, const CfAdamArgs &p,
                                 double *tile_partials, double *partials, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_adam_sqnorm_kernel, dim3(n_chunks << tile_shift), dim3(CF_TILE_THREADS), 0, stream, weights,
                       exp_avg, exp_avg_sq, grads, tile_shift, p, tile_partials);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cf_tile_partials_kernel, dim3(n_chunks), dim3(CF_TILE_THREADS), 0, stream, grads, tile_shift,
                       tile_partials, partials);
    return hipGetLastError();
}
