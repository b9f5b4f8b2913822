// Device-side body of the first kernel of the incidence build (see stx_build.hip): one thread per entry of A
// writes the CSR arrays, the sort keys and the tile histogram of the first digit; optionally draws the
// negatives, fills the presence bitmap of the columns, counts rows per relation.  In a header so that it
// can also run in a launch shared with another kernel.
#pragma once

#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

// SplitMix64 (Steele, Lea, Flood, OOPSLA 2014) used as a counter-based generator: output number `ctr`
// of the sequence started at `seed`.
__device__ inline uint64_t splitmix64_at(uint64_t seed, uint64_t ctr)
{
    uint64_t z = seed + (ctr + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

// `block` of `nblocks`: the index of the workgroup among those of the emit (the launch may hold others).
// ARENA: the body's LDS arrays live in the emit_lds(MAP, RC) bytes at `lds` instead of arrays of its own.
template <int ITEMS, bool MAP, bool SAMPLE, bool RC, bool ARENA = false>
__device__ inline void emit_body(const int block, const int nblocks, const EmitArgs &a, unsigned char *lds = nullptr)
{
    const BatchPtrs &bp = a.bp;
    const int32_t n_ent = a.n_ent, n_rel = a.n_rel, nnz = a.nnz;
    int32_t *__restrict__ rowptr = a.rowptr;
    int32_t *__restrict__ colidx = a.colidx;
    float *__restrict__ vals = a.vals;
    int32_t *__restrict__ keys = a.keys;
    const int radix = a.radix;
    int32_t *__restrict__ table = a.table;
    int32_t *__restrict__ ctrl = a.ctrl;
    const ColMap &map = a.map;
    const RelCnt &rc = a.rc;
    int32_t *s_hist, *s_rc;
    uint32_t *s_map;
    if constexpr (ARENA) {
        s_hist = reinterpret_cast<int32_t *>(lds);
        s_map = reinterpret_cast<uint32_t *>(lds) + 256;
        s_rc = s_hist + 256 + (MAP ? kMapMaxWords : 4);
    } else {
        __shared__ int32_t o_hist[256];
        __shared__ uint32_t o_map[MAP ? kMapMaxWords : 1];
        __shared__ int32_t o_rc[RC ? kRelCntMax : 1];
        s_hist = o_hist; s_map = o_map; s_rc = o_rc;
    }
    const int tid = threadIdx.x;
    s_hist[tid] = 0;
    if (RC) {
        for (int r = tid; r < rc.n_rel; r += kThreads) s_rc[r] = 0;
        for (int r = block * kThreads + tid; r < rc.n_rel; r += nblocks * kThreads) rc.other[r] = 0;
    }
    if (MAP) {
        for (int w = tid; w < map.words; w += kThreads) s_map[w] = 0u;
        for (int w = block * kThreads + tid; w < map.words; w += nblocks * kThreads) map.other[w] = 0u;
    }
    __syncthreads();
    const int32_t base = block * (kThreads * ITEMS);
    // First every index of the thread's entries is fetched (the loads of all items are in flight together:
    // a store in between would order them one after the other), then the entries are written.
    int32_t raw[ITEMS];
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int32_t e = base + it * kThreads + tid;
        raw[it] = 0;
        if (e < nnz) {
            const int32_t row = e / 3, slot = e - 3 * row;
            if (row < bp.b) {
                raw[it] = slot == 0 ? bp.h[row] : (slot == 1 ? bp.r[row] : bp.t[row]);
            } else if (SAMPLE) {   // the positive's side that a negative may keep; the draw decides below
                const int32_t i = (row - bp.b) / bp.k;
                raw[it] = slot == 0 ? bp.h[i] : (slot == 1 ? bp.r[i] : bp.t[i]);
            } else {
                const int32_t j = row - bp.b;
                raw[it] = slot == 0 ? bp.nh[j] : (slot == 1 ? bp.r[j / bp.k] : bp.nt[j]);
            }
        }
    }
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        int32_t e = base + it * kThreads + tid;
        if (e < nnz) {
            int32_t row = e / 3, slot = e - 3 * row;
            int32_t idx = raw[it];
            if (SAMPLE && row >= bp.b && slot != 1) {
                // the three threads of a row draw the same number; slots 0 and 2 store their side
                const int32_t j = row - bp.b;
                const uint64_t u = splitmix64_at(bp.seed, bp.base_ctr + (uint64_t)j);
                const int32_t ent = (int32_t)(((u & 0xFFFFFFFFull) * (uint64_t)n_ent) >> 32);
                const bool head = (u >> 63) != 0;
                if (slot == 0) { idx = head ? ent : idx; bp.nh_out[j] = idx; }
                else           { idx = head ? idx : ent; bp.nt_out[j] = idx; }
            }
            int32_t lim = slot == 1 ? n_rel : n_ent;
            if (idx < 0 || idx >= lim) {           // clamp so nothing downstream reads outside a table
                atomicAdd(&ctrl[CTRL_BAD_INDEX], 1);
                idx = idx < 0 ? 0 : lim - 1;
            }
            int32_t col = slot == 1 ? n_ent + idx : idx;
            colidx[e] = col;
            if (a.colidx2) a.colidx2[e] = col;
            vals[e] = slot == 2 ? -1.0f : 1.0f;
            if (slot == 0) rowptr[row] = e;
            if (e == nnz - 1) rowptr[row + 1] = nnz;
            if (keys) keys[e] = col;           // (null: the first pass of the sort reads colidx instead)
            atomicAdd(&s_hist[col & (radix - 1)], 1);
            if (MAP) atomicOr(&s_map[col >> 5], 1u << (col & 31));
            if (RC && slot == 1) atomicAdd(&s_rc[idx], 1);
        }
    }
    __syncthreads();
    if (tid < radix) table[block * radix + tid] = s_hist[tid];
    if (MAP) {
        for (int w = tid; w < map.words; w += kThreads) {
            const uint32_t v = s_map[w];
            if (v) atomicOr(&map.cur[w], v);
        }
    }
    if (RC) {
        for (int r = tid; r < rc.n_rel; r += kThreads) {
            const int32_t v = s_rc[r];
            if (v) atomicAdd(&rc.cur[r], v);
        }
    }
}

}  // namespace stx
