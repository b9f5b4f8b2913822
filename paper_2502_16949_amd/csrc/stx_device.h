// Device-side helpers shared by the kernels: the "last workgroup finishes the job" handshake,
// a one-workgroup exclusive scan, and sub-wavefront reductions.  gfx950 only (64-lane wavefronts).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace stx {

// Every workgroup of a grid calls this once after writing its share of a global array.  Exactly one
// workgroup (the last to arrive) gets `true`, after which it may read what all the others wrote.
// Nothing waits on anything: the counter is a ticket, not a lock.  The caller resets *ticket to 0 when
// it is done so the next launch starts clean.
__device__ inline bool last_block_arrives(int32_t *ticket)
{
    __shared__ int s_is_last;
    __threadfence();   // release: this thread's global writes are visible device-wide
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = atomicAdd(ticket, 1);
        s_is_last = (t == (int)gridDim.x - 1);
    }
    __syncthreads();
    bool last = s_is_last != 0;
    if (last) __threadfence();   // acquire: drop stale cached lines before reading the others' data
    return last;
}

// In-place exclusive prefix sum of data[0..n) by one 256-thread workgroup; returns the total in
// *total (if non-null).  Each thread owns a contiguous slice.
__device__ inline void block_exclusive_scan_inplace(int32_t *data, int n, int32_t *total)
{
    __shared__ int32_t s_scan[256];
    const int tid = threadIdx.x;
    const int per = (n + 255) / 256;
    const int lo = min(tid * per, n), hi = min(lo + per, n);
    int32_t s = 0;
    for (int i = lo; i < hi; ++i) s += data[i];
    s_scan[tid] = s;
    __syncthreads();
    for (int off = 1; off < 256; off <<= 1) {
        int32_t v = tid >= off ? s_scan[tid - off] : 0;
        __syncthreads();
        s_scan[tid] += v;
        __syncthreads();
    }
    int32_t run = s_scan[tid] - s;
    for (int i = lo; i < hi; ++i) {
        int32_t v = data[i];
        data[i] = run;
        run += v;
    }
    if (total && tid == 255) *total = s_scan[255];
    __syncthreads();
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

__device__ inline float4 ld4(const float *p) { return *reinterpret_cast<const float4 *>(p); }
__device__ inline void st4(float *p, float4 v) { *reinterpret_cast<float4 *>(p) = v; }

}  // namespace stx
