// Device-side helpers shared by the kernels: one-workgroup scans and sub-wavefront reductions.
// gfx950 only (64-lane wavefronts).
//
// No kernel here passes data between workgroups of one launch: on this multi-die GPU that needs a
// device-scope release/acquire per workgroup, i.e. an L2 write-back each, which costs far more than
// the extra kernel launch that a grid-wide dependency is turned into instead.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stx {

// Exclusive prefix sum of one value per thread across a 256-thread workgroup; *total (shared or
// register, may be null) receives the sum.  All 256 threads must call it.
__device__ inline int32_t block_exclusive_scan(int32_t v, int32_t *total)
{
    __shared__ int32_t s_scan[256];
    const int tid = threadIdx.x;
    __syncthreads();   // protect s_scan against a previous use
    s_scan[tid] = v;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        int32_t a = tid >= off ? s_scan[tid - off] : 0;
        __syncthreads();
        s_scan[tid] += a;
        __syncthreads();
    }
    if (total) *total = s_scan[255];
    return s_scan[tid] - v;
}

// The lanes of the wavefront (among those with `valid`) whose digit equals this lane's: one ballot per bit of the
// digit, and per lane an exclusive-nor of the ballot with the lane's own bit spread over a word.
__device__ inline uint64_t digit_class_mask(int dgt, bool valid, int bits)
{
    const uint64_t v = __ballot(valid);
    uint32_t lo = (uint32_t)v, hi = (uint32_t)(v >> 32);
#pragma unroll
    for (int bit = 0; bit < 8; ++bit) {
        if (bit < bits) {   // uniform
            const uint32_t x = (uint32_t)(-(int32_t)((dgt >> bit) & 1));   // all ones when the lane's bit is set
            const uint64_t bm = __ballot(x != 0u);
            lo &= ~((uint32_t)bm ^ x);
            hi &= ~((uint32_t)(bm >> 32) ^ x);
        }
    }
    return (uint64_t)hi << 32 | lo;
}

// Sum over the LPR consecutive lanes that share a row (LPR a power of two <= 64, groups aligned).
// Butterfly: every lane of the group ends with the same bits.
template <int LPR>
__device__ inline float group_sum(float v)
{
#pragma unroll
    for (int m = LPR / 2; m >= 1; m >>= 1) v += __shfl_xor(v, m, LPR);
    return v;
}

// Streaming variants: data that is read or written once and not needed in cache afterwards.
typedef float stx_f4 __attribute__((ext_vector_type(4)));
__device__ inline float4 ld4_stream(const float *p)
{
    stx_f4 t = __builtin_nontemporal_load(reinterpret_cast<const stx_f4 *>(p));
    return make_float4(t.x, t.y, t.z, t.w);
}
__device__ inline void st4_stream(float *p, float4 v)
{
    stx_f4 t = {v.x, v.y, v.z, v.w};
    __builtin_nontemporal_store(t, reinterpret_cast<stx_f4 *>(p));
}
__device__ inline float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }

}  // namespace stx
