// gfx950 kernels of the CheckFree recovery hot path.
//
// All three are HBM-streaming kernels: a grid of 256-thread workgroups walks a
// device-side chunk table (one multi-tensor launch per operation), every lane
// moves 16 bytes per memory instruction with the streaming (non-temporal) cache
// policy, and there is no reuse, so nothing is staged through LDS on the
// streaming side (LDS carries only the fixed-order second pass of the norm).
// Nothing here is a contraction, so no MFMA.
//
// Paper: "CheckFree: Memoryless Recovery" (omega = squared gradient norm of a
// stage; the weighted-average display equation; Algorithm 1) and "CheckFree+:
// First and Last Stage Recovery" (exact copies).
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <mutex>

#include "cf_device.h"
#include "cf_kernels.h"

// Device memory for callers that cannot allocate (code under graph capture, tight serving loops):
// cf_stage_grad_sqnorm_static puts its chunk table and partial sums here instead of in a block the
// caller or the library allocated.  One copy per GPU, held until the process ends.  In host code
// the name below is only a stand-in for the symbol, never a device address: the address comes from
// cf_static_scratch_address() and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[CF_STATIC_SCRATCH_BYTES];

// Every binary64 operation of the blend is rounded on its own, as the formula
// is written; fused multiply-adds are only the explicit ones below.
#pragma clang fp contract(off)

namespace {

// ---------------------------------------------------------------------------
// omega = ||grad W^S||^2, all stages of a launch in one grid.
// ---------------------------------------------------------------------------

// Sum of squares of this lane's share of one fp32 chunk.  Lane t of the
// workgroup takes the 16-byte vectors t, t+256, t+512, ... of the chunk's
// aligned body; kUnroll of them are in flight at a time.  Every element is
// widened to binary64 (exact) and squared and accumulated there: one
// conversion and one fused multiply-add per element, far below what the
// memory stream leaves room for, so the squares of binary32 values can neither
// underflow nor overflow and the rounding error of omega does not depend on how
// long a lane's chain is.
template <int kUnroll>
__device__ __forceinline__ double chunk_sqsum_f32(gcf32 p, uint32_t len, uint32_t tid)
{
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    const uint32_t head = head_elems((uint64_t)p, 4u, len);
    if (tid < head) sq_acc(a0, p[tid]);
    gcf32x4 q = (gcf32x4)(p + head);
    const uint32_t rem = len - head;
    const uint32_t n4 = rem >> 2;
    uint32_t i = tid;
    for (; i + (kUnroll - 1) * CF_THREADS < n4; i += kUnroll * CF_THREADS) {
        f32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(q + i + u * CF_THREADS);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            sq_acc(a0, v[u].x);
            sq_acc(a1, v[u].y);
            sq_acc(a2, v[u].z);
            sq_acc(a3, v[u].w);
        }
    }
    if (i < n4) {
        // The last, partial round keeps its loads in flight together too: a lane whose vector lies
        // past the chunk's end takes zeros instead, and adding the square of zero changes no accumulator.
        f32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t j = i + u * CF_THREADS;
            v[u] = (j < n4) ? __builtin_nontemporal_load(q + j) : (f32x4)(0.f);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            sq_acc(a0, v[u].x);
            sq_acc(a1, v[u].y);
            sq_acc(a2, v[u].z);
            sq_acc(a3, v[u].w);
        }
    }
    const uint32_t tail = rem & 3u;
    if (tid < tail) sq_acc(a0, p[head + (n4 << 2) + tid]);
    return (a0 + a1) + (a2 + a3);
}

// The same for a bfloat16 chunk: eight elements per 16-byte vector, each
// widened to binary32 and on to binary64 (both exact).
__device__ __forceinline__ void sq_acc_bf16_word(double &lo_acc, double &hi_acc, uint32_t word)
{
    sq_acc(lo_acc, __uint_as_float(word << 16));
    sq_acc(hi_acc, __uint_as_float(word & 0xFFFF0000u));
}

template <int kUnroll>
__device__ __forceinline__ double chunk_sqsum_bf16(gcu16 p, uint32_t len, uint32_t tid)
{
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    const uint32_t head = head_elems((uint64_t)p, 2u, len);
    if (tid < head) sq_acc(a0, __uint_as_float((uint32_t)p[tid] << 16));
    gcu32x4 q = (gcu32x4)(p + head);
    const uint32_t rem = len - head;
    const uint32_t n8 = rem >> 3;
    uint32_t i = tid;
    for (; i + (kUnroll - 1) * CF_THREADS < n8; i += kUnroll * CF_THREADS) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) v[u] = __builtin_nontemporal_load(q + i + u * CF_THREADS);
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            sq_acc_bf16_word(a0, a1, v[u].x);
            sq_acc_bf16_word(a2, a3, v[u].y);
            sq_acc_bf16_word(a0, a1, v[u].z);
            sq_acc_bf16_word(a2, a3, v[u].w);
        }
    }
    if (i < n8) {
        u32x4 v[kUnroll];
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            const uint32_t j = i + u * CF_THREADS;
            v[u] = (j < n8) ? __builtin_nontemporal_load(q + j) : (u32x4)(0u);
        }
#pragma unroll
        for (int u = 0; u < kUnroll; ++u) {
            sq_acc_bf16_word(a0, a1, v[u].x);
            sq_acc_bf16_word(a2, a3, v[u].y);
            sq_acc_bf16_word(a0, a1, v[u].z);
            sq_acc_bf16_word(a2, a3, v[u].w);
        }
    }
    const uint32_t tail = rem & 7u;
    if (tid < tail) sq_acc(a0, __uint_as_float((uint32_t)p[head + (n8 << 3) + tid] << 16));
    return (a0 + a1) + (a2 + a3);
}

// First pass.  Workgroup b takes chunks b, b + grid, b + 2 grid, ... (by default
// the grid has one workgroup per chunk).  The four wavefront sums of a chunk
// meet in LDS and leave as ONE binary64 partial at slot `chunk` of the owning
// stage's partial array, so the partials do not depend on the grid size.  There
// is no fence and no atomic on this streaming pass: on this chip an agent-scope
// release per workgroup (an L2 write-back) cuts a read-only stream to under
// 40 % of what it reaches without, and even a capped grid whose last-arriving
// workgroup adds the partials up is slower than the second launch below.
__global__ __launch_bounds__(CF_THREADS) void cf_sqnorm_partials_kernel(CfSqnormArgs args)
{
    __shared__ double wave_part[2][CF_WAVES];
    const uint32_t tid = threadIdx.x;
    const uint32_t wave = tid >> 6;
    const uint32_t lane = tid & 63u;

    uint32_t s = 0;
    uint32_t parity = 0;
    for (uint32_t c = blockIdx.x; c < args.total_chunks; c += gridDim.x) {
        while (s + 1 < args.n_seg && c >= args.seg[s + 1].chunk_begin) ++s;
        const uint32_t local = c - args.seg[s].chunk_begin;
        const CfChunk ch = args.seg[s].chunks[local];
        const double t = (ch.dtype == kDtypeF32) ? chunk_sqsum_f32<8>((gcf32)ch.addr, ch.len, tid)
                                                 : chunk_sqsum_bf16<8>((gcu16)ch.addr, ch.len, tid);
        const double w = wave_sum(t);
        // Two LDS rows used alternately: one barrier per chunk is enough, because a
        // row is rewritten only after the barrier of the chunk in between.
        if (lane == 0) wave_part[parity][wave] = w;
        __syncthreads();
        if (tid == 0)
            args.seg[s].partials[local] =
                (wave_part[parity][0] + wave_part[parity][1]) + (wave_part[parity][2] + wave_part[parity][3]);
        parity ^= 1u;
    }
}

// Second pass, stream-ordered after the first: workgroup k adds the partials of
// stage k in a fixed order (lane-strided serial sums, then the fixed-order
// workgroup sum) and writes omega_k.
__global__ __launch_bounds__(CF_FINALIZE_THREADS) void cf_sqnorm_finalize_kernel(CfSqnormArgs args)
{
    __shared__ double wave_sums[CF_FINALIZE_THREADS / 64];
    const uint32_t tid = threadIdx.x;
    const uint32_t k = blockIdx.x;
    const double *part = args.seg[k].partials;
    const uint64_t np = args.seg[k].n_chunks;
    double acc = 0.0;
    for (uint64_t i = tid; i < np; i += CF_FINALIZE_THREADS) acc += part[i];
    const double omega = block_sum_fixed_order<CF_FINALIZE_THREADS>(acc, wave_sums);
    if (tid == 0) {
        args.omega_out[k] = omega;
        if (!(omega - omega == 0.0)) atomicOr(&args.words[CF_WORD_FLAGS], kFlagNonfiniteOmega);
    }
}

// Second pass, per tensor: workgroup t adds the partials of the chunks of tensor
// t (chunks first[t] .. first[t+1]-1 of the stage) in a fixed order.
__global__ __launch_bounds__(CF_THREADS) void cf_sqnorm_finalize_tensors_kernel(const double *partials,
                                                                               const uint32_t *first,
                                                                               double *tensor_out)
{
    __shared__ double wave_sums[CF_WAVES];
    const uint32_t tid = threadIdx.x;
    const uint32_t lo = first[blockIdx.x];
    const uint32_t hi = first[blockIdx.x + 1];
    double acc = 0.0;
    for (uint32_t i = lo + tid; i < hi; i += CF_THREADS) acc += partials[i];
    const double total = block_sum_fixed_order<CF_THREADS>(acc, wave_sums);
    if (tid == 0) tensor_out[blockIdx.x] = total;
}

// ---------------------------------------------------------------------------
// W_lost = (w_p W_prev + w_n W_next) / (w_p + w_n)
// ---------------------------------------------------------------------------

struct BlendWeights {
    double wp, wn, rcp;   // rcp = 1 / (wp + wn)
};

// Numerator as written, each operation rounded in binary64; then the reciprocal
// of the denominator; one narrowing.
__device__ __forceinline__ double blend_f64(const BlendWeights &w, double a, double b)
{
    double pa = w.wp * a;
    double pb = w.wn * b;
    double num = pa + pb;
    return num * w.rcp;
}

__device__ __forceinline__ float blend_to_f32(const BlendWeights &w, float a, float b)
{
    return (float)blend_f64(w, (double)a, (double)b);
}

// binary64 -> bfloat16 bits in ONE rounding to nearest even.  Narrowing to
// binary32 first and cutting that to its upper 16 bits gives the same result
// as the direct rounding unless the binary32 value lands exactly on a bfloat16
// tie (low half 0x8000) that x itself is not on: every bfloat16 rounding
// boundary is a binary32 number and rounding is monotone, so only then can the
// first rounding have moved x onto the boundary.  In that rare case the
// binary32 value is nudged one ulp back toward x before the cut.
__device__ __forceinline__ uint32_t f64_to_bf16_bits(double x)
{
    const float f = (float)x;
    uint32_t u = __float_as_uint(f);
    if ((u & 0xFFFFu) == 0x8000u) {
        const double back = __builtin_fabs((double)f);
        const double ax = __builtin_fabs(x);
        if (back > ax) u -= 1u;
        else if (back < ax) u += 1u;
    }
    u += 0x7FFFu + ((u >> 16) & 1u);
    return (x != x) ? 0x7FC0u : (u >> 16);
}

__device__ __forceinline__ double bf16_bits_to_f64(uint32_t h)
{
    return (double)__uint_as_float(h << 16);
}

__device__ __forceinline__ uint32_t blend_bf16_pair(const BlendWeights &w, uint32_t a, uint32_t b)
{
    uint32_t lo = f64_to_bf16_bits(blend_f64(w, bf16_bits_to_f64(a & 0xFFFFu), bf16_bits_to_f64(b & 0xFFFFu)));
    uint32_t hi = f64_to_bf16_bits(blend_f64(w, bf16_bits_to_f64(a >> 16), bf16_bits_to_f64(b >> 16)));
    return lo | (hi << 16);
}

// A wavefront's vector store held back for about 64 * kCycles64 cycles after the
// values it stores are there (the asm takes them as inputs, so it cannot move
// ahead of the arithmetic, and nothing with side effects moves across it).
// Why: the tensors of a blend or a copy are usually placed alike, so the line a
// wavefront writes lies in the same memory banks as the lines it has just read,
// and its neighbours are still streaming from those banks; a store that arrives
// right behind the loads breaks into that.  Measured on this chip: holding the
// store back wins 2.5-3 % on fp32 blends of 0.5 GiB per tensor stream and more
// and 1-2 % on copies from 64 MiB on; it costs 1.5-3 % on small launches, which
// live on how fast wavefront slots turn over.  So the host asks for it by size.
template <int kCycles64>
__device__ __forceinline__ void hold_store_f32(const f32x4 &o)
{
    asm volatile("s_sleep %4" ::"v"(o.x), "v"(o.y), "v"(o.z), "v"(o.w), "n"(kCycles64) : "memory");
}

template <int kCycles64>
__device__ __forceinline__ void hold_store_u32(const u32x4 &o)
{
    asm volatile("s_sleep %4" ::"v"(o.x), "v"(o.y), "v"(o.z), "v"(o.w), "n"(kCycles64) : "memory");
}

constexpr int kBlendHold = 32;   // fp32 blend: 2048 cycles (the bf16 blend's own arithmetic already takes that long)
constexpr int kCopyHold = 8;     // copy: 512 cycles

// The two omegas as they arrive (device memory or host-given) and what the
// blend needs of them.  make_weights() holds the norm-to-weight scaling: the
// usable-pair rule, the common power of two, the one binary64 division.
__device__ __forceinline__ BlendWeights make_weights(double wp, double wn, uint32_t *words, bool reporter)
{
    BlendWeights w;
    w.wp = wp;
    w.wn = wn;
    double den = w.wp + w.wn;
    // Usable pair: both finite and non-negative, sum a positive normal number.
    const bool usable = (w.wp - w.wp == 0.0) && (w.wn - w.wn == 0.0) && w.wp >= 0.0 && w.wn >= 0.0 &&
                        (den - den == 0.0) && den >= 2.2250738585072014e-308;
    if (!usable) {
        w.wp = 1.0;
        w.wn = 1.0;
        den = 2.0;
        if (reporter) atomicOr(&words[CF_WORD_FLAGS], kFlagDegenerateOmega);
    }
    // The equation does not change when both weights are multiplied by one
    // number: scale them by the power of two that brings their sum into [1, 2)
    // (exact), so that no product weight x value leaves the binary64 range
    // whatever the magnitude of the omegas.
    const int scale = 1023 - (int)((uint64_t)__double_as_longlong(den) >> 52);
    w.wp = __builtin_ldexp(w.wp, scale);
    w.wn = __builtin_ldexp(w.wn, scale);
    w.rcp = 1.0 / (w.wp + w.wn);
    return w;
}

// One single-wavefront workgroup blends one *tile*: 64 sixteen-byte vectors of
// each of the three streams, one vector per lane.  Workgroups are dispatched in
// tile order, so at any moment the chip reads two narrow moving windows and
// writes a third, and a compute unit takes a new tile whenever one wavefront
// slot frees up; on this memory system that sustains about a quarter more
// bandwidth for a two-read-one-write stream than a resident grid of 256-thread
// workgroups striding over large chunks.  Tile 0 of a chunk also takes the few
// elements before and after the body.  The body is laid on the 128-byte
// boundaries of the written tensor; the two tensors that are read may sit
// differently inside their lines and are read at whatever alignment they have.
// The tile's loads are issued first and the weights are derived while they are
// in flight: a wavefront lives for one load-compute-store round, so the
// division must not stand between its start and its loads.
__device__ __forceinline__ void blend_tile_f32(double wp, double wn, uint32_t *words, bool reporter, gcf32 pa, gcf32 pb,
                                               gf32 po, uint32_t len, uint32_t tile, uint32_t tid, bool hold)
{
    const uint32_t head = head_elems((uint64_t)po, 4u, len);   // whole lines for the stream that is written
    const uint32_t rem = len - head;
    const uint32_t n4 = rem >> 2;
    const uint32_t v = tile * CF_TILE_THREADS + tid;
    const uint32_t tail = rem & 3u;
    const uint32_t tbase = head + (n4 << 2);
    // an extra element of tile 0: lane t < head takes element t, lane head <= t < head + tail a tail element
    uint32_t extra = len;
    if (tile == 0) {
        if (tid < head) extra = tid;
        else if (tid - head < tail) extra = tbase + (tid - head);
    }
    f32x4 a = (f32x4)(0.f), b = (f32x4)(0.f);
    float ea = 0.f, eb = 0.f;
    if (v < n4) {
        a = __builtin_nontemporal_load((gcf32x4_e4)(pa + head) + v);
        b = __builtin_nontemporal_load((gcf32x4_e4)(pb + head) + v);
    }
    if (extra < len) {
        ea = pa[extra];
        eb = pb[extra];
    }
    const BlendWeights w = make_weights(wp, wn, words, reporter);
    if (v < n4) {
        f32x4 o;
        o.x = blend_to_f32(w, a.x, b.x);
        o.y = blend_to_f32(w, a.y, b.y);
        o.z = blend_to_f32(w, a.z, b.z);
        o.w = blend_to_f32(w, a.w, b.w);
        if (hold) hold_store_f32<kBlendHold>(o);
        __builtin_nontemporal_store(o, (gf32x4)(po + head) + v);
    }
    if (extra < len) po[extra] = blend_to_f32(w, ea, eb);
}

__device__ __forceinline__ uint16_t blend_to_bf16(const BlendWeights &w, uint16_t a, uint16_t b)
{
    return (uint16_t)f64_to_bf16_bits(blend_f64(w, bf16_bits_to_f64(a), bf16_bits_to_f64(b)));
}

__device__ __forceinline__ void blend_tile_bf16(double wp, double wn, uint32_t *words, bool reporter, gcu16 pa, gcu16 pb,
                                                gu16 po, uint32_t len, uint32_t tile, uint32_t tid)
{
    const uint32_t head = head_elems((uint64_t)po, 2u, len);   // whole lines for the stream that is written
    const uint32_t rem = len - head;
    const uint32_t n8 = rem >> 3;
    const uint32_t v = tile * CF_TILE_THREADS + tid;
    const uint32_t tail = rem & 7u;
    const uint32_t tbase = head + (n8 << 3);
    // extra elements of tile 0: up to 63 before the body (lane t takes element t) and up to 7 behind it
    const bool has_head = tile == 0 && tid < head;
    const bool has_tail = tile == 0 && tid < tail;
    u32x4 a = (u32x4)(0u), b = (u32x4)(0u);
    uint16_t ha = 0, hb = 0, ta = 0, tb = 0;
    if (v < n8) {
        a = __builtin_nontemporal_load((gcu32x4_e2)(pa + head) + v);
        b = __builtin_nontemporal_load((gcu32x4_e2)(pb + head) + v);
    }
    if (has_head) {
        ha = pa[tid];
        hb = pb[tid];
    }
    if (has_tail) {
        ta = pa[tbase + tid];
        tb = pb[tbase + tid];
    }
    const BlendWeights w = make_weights(wp, wn, words, reporter);
    if (v < n8) {
        u32x4 o;
        o.x = blend_bf16_pair(w, a.x, b.x);
        o.y = blend_bf16_pair(w, a.y, b.y);
        o.z = blend_bf16_pair(w, a.z, b.z);
        o.w = blend_bf16_pair(w, a.w, b.w);
        __builtin_nontemporal_store(o, (gu32x4)(po + head) + v);
    }
    if (has_head) po[tid] = blend_to_bf16(w, ha, hb);
    if (has_tail) po[tbase + tid] = blend_to_bf16(w, ta, tb);
}

// Workgroup index -> (chunk, tile of the chunk).  A chunk holds at most
// 2^tile_shift tiles; a workgroup whose tile lies past the chunk's end finds
// no vector of its own and does nothing.  The norm-to-weight scaling belongs
// to this kernel: every workgroup reads the two binary64 omegas from device
// memory and derives identical weights (make_weights, called by the tile
// functions once their loads are out).
//
// The omegas come from device memory (d_omega_* non-null: the norms never visit
// the host) or, for the ablation variants with explicit weights, by value.
__global__ __launch_bounds__(CF_TILE_THREADS) void cf_blend_kernel(const CfChunk *prev, const CfChunk *next,
                                                              const CfChunk *lost, uint32_t tile_shift,
                                                              const double *d_omega_prev,
                                                              const double *d_omega_next, double h_omega_prev,
                                                              double h_omega_next, uint32_t *words, uint32_t hold)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t c = blockIdx.x >> tile_shift;
    const uint32_t tile = blockIdx.x & ((1u << tile_shift) - 1u);
    // Everything the wavefront needs from memory before its tile is asked for at once: the three
    // chunk entries and the two omegas are independent loads.
    const CfChunk co = lost[c];
    const CfChunk ca = prev[c];
    const CfChunk cb = next[c];
    const double wp = d_omega_prev ? *d_omega_prev : h_omega_prev;
    const double wn = d_omega_next ? *d_omega_next : h_omega_next;
    // A tile past the end of a short chunk finds no vector of its own below and does nothing; it is
    // not sent home earlier, since a branch here would hold the address loads back behind it.
    const bool reporter = blockIdx.x == 0 && tid == 0;
    if (co.dtype == kDtypeF32)
        blend_tile_f32(wp, wn, words, reporter, (gcf32)ca.addr, (gcf32)cb.addr, (gf32)co.addr, co.len, tile, tid, hold != 0);
    else
        blend_tile_bf16(wp, wn, words, reporter, (gcu16)ca.addr, (gcu16)cb.addr, (gu16)co.addr, co.len, tile, tid);
}

// ---------------------------------------------------------------------------
// Bit-exact multi-tensor copy (CheckFree+): same tile-per-workgroup walk.
// ---------------------------------------------------------------------------

__global__ __launch_bounds__(CF_TILE_THREADS) void cf_copy_kernel(const CfChunk *src, const CfChunk *dst,
                                                             uint32_t first_chunk, uint32_t tile_shift, uint32_t hold)
{
    const uint32_t tid = threadIdx.x;
    const uint32_t c = first_chunk + (blockIdx.x >> tile_shift);
    const uint32_t tile = blockIdx.x & ((1u << tile_shift) - 1u);
    const CfChunk cd = dst[c];
    const CfChunk cs = src[c];
    const uint32_t esize = (cd.dtype == kDtypeF32) ? 4u : 2u;
    const uint32_t nbytes = cd.len * esize;   // a tile past the end of a short chunk finds no vector below
    gcu8 ps = (gcu8)cs.addr;
    gu8 pd = (gu8)cd.addr;
    const uint32_t head = head_elems((uint64_t)pd, 1u, nbytes);   // whole lines for the stream that is written
    const uint32_t rem = nbytes - head;
    const uint32_t n16 = rem >> 4;
    const uint32_t v = tile * CF_TILE_THREADS + tid;
    if (v < n16) {
        // the source may sit differently inside its lines: read at element alignment
        const u32x4 x = (esize == 4u) ? __builtin_nontemporal_load((gcu32x4_e4)(ps + head) + v)
                                      : __builtin_nontemporal_load((gcu32x4_e2)(ps + head) + v);
        if (hold) hold_store_u32<kCopyHold>(x);
        __builtin_nontemporal_store(x, (gu32x4)(pd + head) + v);
    }
    if (tile == 0) {
        // Up to 127 bytes before the body and 15 behind it, moved as whole elements (both are
        // multiples of the element size, and the tensors are aligned to it).
        const uint32_t tail = rem & 15u;
        const uint32_t tbase = head + (n16 << 4);
        if (esize == 4u) {
            if (tid < (head >> 2)) ((gu32)pd)[tid] = ((gcu32)ps)[tid];
            if (tid < (tail >> 2)) ((gu32)(pd + tbase))[tid] = ((gcu32)(ps + tbase))[tid];
        } else {
            if (tid < (head >> 1)) ((gu16)pd)[tid] = ((gcu16)ps)[tid];
            if (tid < (tail >> 1)) ((gu16)(pd + tbase))[tid] = ((gcu16)(ps + tbase))[tid];
        }
    }
}

// ---------------------------------------------------------------------------
// Set-up kernels: nothing here touches tensor data.
// ---------------------------------------------------------------------------

// Workgroup b writes the chunk table entries of tensor b of the launch, whose
// description arrived in the kernel argument block: a stage is described to
// the device without a host-to-device copy, asynchronously on the caller's
// stream.
__global__ __launch_bounds__(CF_THREADS) void cf_build_table_kernel(CfTableArgs args)
{
    const uint32_t b = blockIdx.x;
    const CfTableTensor t = args.tensor[b];
    const uint32_t esize = (t.dtype == kDtypeF32) ? 4u : 2u;
    const uint64_t chunk_elems = args.chunk_bytes / esize;
    const uint64_t n = (t.numel + chunk_elems - 1) / chunk_elems;
    for (uint64_t j = threadIdx.x; j < n; j += CF_THREADS) {
        const uint64_t first = j * chunk_elems;
        const uint64_t left = t.numel - first;
        CfChunk c;
        c.addr = t.addr + first * esize;
        c.len = (uint32_t)(left < chunk_elems ? left : chunk_elems);
        c.dtype = t.dtype;
        args.chunks[t.first_chunk + j] = c;
    }
    if (threadIdx.x == 0) {
        args.tensor_first[args.tensor_base + b] = t.first_chunk;
        if (args.last && b + 1 == args.n) args.tensor_first[args.tensor_base + args.n] = args.end_chunk;
    }
}

__global__ __launch_bounds__(CF_CTX_WORDS) void cf_clear_words_kernel(uint32_t *words) { words[threadIdx.x] = 0u; }

// The sticky flags are read, and cleared if asked, in one atomic step, so a
// flag raised by a kernel on another stream is either seen by this read or
// still there for the next.
__global__ __launch_bounds__(64) void cf_read_flags_kernel(uint32_t *words, int clear)
{
    words[CF_WORD_FLAGS_READ] = clear ? atomicExch(&words[CF_WORD_FLAGS], 0u) : atomicOr(&words[CF_WORD_FLAGS], 0u);
}

}  // namespace

hipError_t cf_static_scratch_address(int device, void **ptr)
{
    constexpr int kMaxDevices = 64;
    static std::mutex mutex;
    static void *address[kMaxDevices] = {};
    if (!ptr || device < 0 || device >= kMaxDevices) return hipErrorInvalidValue;
    std::lock_guard<std::mutex> lock(mutex);
    if (!address[device]) {
        void *p = nullptr;
        const hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess) return e;
        if (!p) return hipErrorInvalidSymbol;
        address[device] = p;
    }
    *ptr = address[device];
    return hipSuccess;
}

hipError_t cf_launch_sqnorm_finalize(const CfSqnormArgs &args, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_sqnorm_finalize_kernel, dim3(args.n_seg), dim3(CF_FINALIZE_THREADS), 0, stream, args);
    return hipGetLastError();
}

hipError_t cf_launch_sqnorm(const CfSqnormArgs &args, uint32_t grid, hipStream_t stream)
{
    if (args.total_chunks != 0) {
        hipLaunchKernelGGL(cf_sqnorm_partials_kernel, dim3(grid), dim3(CF_THREADS), 0, stream, args);
        hipError_t e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    return cf_launch_sqnorm_finalize(args, stream);
}

hipError_t cf_launch_sqnorm_tensors(const double *partials, const uint32_t *tensor_first_chunk, uint32_t num_tensors,
                                    double *d_tensor_out, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_sqnorm_finalize_tensors_kernel, dim3(num_tensors), dim3(CF_THREADS), 0, stream, partials,
                       tensor_first_chunk, d_tensor_out);
    return hipGetLastError();
}

hipError_t cf_launch_blend(const CfChunk *prev, const CfChunk *next, const CfChunk *lost, uint32_t n_chunks,
                           uint32_t tile_shift, const double *d_omega_prev, const double *d_omega_next,
                           double h_omega_prev, double h_omega_next, uint32_t *words, bool hold_stores,
                           hipStream_t stream)
{
    hipLaunchKernelGGL(cf_blend_kernel, dim3(n_chunks << tile_shift), dim3(CF_TILE_THREADS), 0, stream, prev, next, lost,
                       tile_shift, d_omega_prev, d_omega_next, h_omega_prev, h_omega_next, words, hold_stores ? 1u : 0u);
    return hipGetLastError();
}

hipError_t cf_launch_copy(const CfChunk *src, const CfChunk *dst, uint32_t first_chunk, uint32_t n_chunks,
                          uint32_t tile_shift, bool hold_stores, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_copy_kernel, dim3(n_chunks << tile_shift), dim3(CF_TILE_THREADS), 0, stream, src, dst,
                       first_chunk, tile_shift, hold_stores ? 1u : 0u);
    return hipGetLastError();
}

hipError_t cf_launch_build_table(const CfTableArgs &args, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_build_table_kernel, dim3(args.n), dim3(CF_THREADS), 0, stream, args);
    return hipGetLastError();
}

hipError_t cf_launch_clear_words(uint32_t *words, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_clear_words_kernel, dim3(1), dim3(CF_CTX_WORDS), 0, stream, words);
    return hipGetLastError();
}

hipError_t cf_launch_read_flags(uint32_t *words, int clear, hipStream_t stream)
{
    hipLaunchKernelGGL(cf_read_flags_kernel, dim3(1), dim3(1), 0, stream, words, clear);
    return hipGetLastError();
}
