// The last kernel of a build as a device function: from the sorted keys (columns) and payloads (positions
// 3*row + slot in A) to the segment arrays of A^T.  k_seg_write runs it alone; the fused transposed product of
// stx_train_step can take it along in its own launch, because it reads the sorted keys itself and only the
// fix-up kernel after it needs the segment arrays.
#pragma once
#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

// Per sorted entry: its segment, row, sign and packed form; per segment: its column and first entry.
// Thread t of a tile owns the 8 consecutive entries base + 8t .. base + 8t + 7.
// MAP: the segment of an entry is the rank of its column in the presence bitmap (every workgroup counts the
// bits of the map itself: a prefix per thread's share of the words in LDS, the words in between read again
// from the cached map); otherwise it is counted from the heads of the earlier tiles (k_seg_count).
// ARENA: the body's LDS arrays live in the kSegWriteLds bytes at `lds` instead of arrays of its own.
template <bool MAP, bool ARENA = false>
__device__ inline void seg_write_body(const int block, const int nblocks, const SegWriteArgs &a,
                                      unsigned char *lds = nullptr)
{
    const int32_t *__restrict__ keys = a.keys;
    const int32_t *__restrict__ pay = a.pay;
    const int32_t nnz = a.nnz;
    int32_t *s_base_p, *s_chunk;
    if constexpr (ARENA) {
        s_chunk = reinterpret_cast<int32_t *>(lds);
        s_base_p = s_chunk + kThreads;
    } else {
        __shared__ int32_t o_base;
        __shared__ int32_t o_chunk[MAP ? kThreads : 1];
        s_base_p = &o_base; s_chunk = o_chunk;
    }
    int32_t &s_base = *s_base_p;
    const int tid = threadIdx.x;
    if (tid == 0) s_base = 0;
    __syncthreads();
    int32_t map_total = 0;
    constexpr int WPT = kMapMaxWords / kThreads;
    const int wpt = MAP ? (a.map.words + kThreads - 1) / kThreads : 1;   // words per thread, <= WPT
    if (MAP) {   // thread t owns words [t*wpt, (t+1)*wpt): set bits below its first word
        int32_t mine = 0;
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int w = tid * wpt + q;
            if (q < wpt && w < a.map.words) mine += __popc(a.map.cur[w]);
        }
        s_chunk[tid] = block_exclusive_scan(mine, &map_total);
        __syncthreads();
    } else {   // segments that start in earlier tiles
        int32_t h = 0;
        for (int t = tid; t < block; t += kThreads) h += a.tile_heads[t];
        for (int m = 32; m >= 1; m >>= 1) h += __shfl_xor(h, m, 64);   // one LDS atomic per wavefront
        if ((tid & 63) == 0 && h) atomicAdd(&s_base, h);
    }
    const int32_t e0 = block * kSegWTile + tid * kSegWItems;
    int32_t kk[kSegWItems + 1];
    kk[0] = (e0 > 0 && e0 - 1 < nnz) ? keys[e0 - 1] : -1;
    if (e0 + kSegWItems <= nnz) {
        const int4 x = *reinterpret_cast<const int4 *>(keys + e0), y = *reinterpret_cast<const int4 *>(keys + e0 + 4);
        kk[1] = x.x; kk[2] = x.y; kk[3] = x.z; kk[4] = x.w; kk[5] = y.x; kk[6] = y.y; kk[7] = y.z; kk[8] = y.w;
    } else {
#pragma unroll
        for (int i = 0; i < kSegWItems; ++i) kk[i + 1] = e0 + i < nnz ? keys[e0 + i] : -1;
    }
    int32_t cnt = 0;
#pragma unroll
    for (int i = 0; i < kSegWItems; ++i)
        if (e0 + i < nnz && kk[i + 1] != kk[i]) ++cnt;
    int32_t seg;
    if (MAP) {
        const int32_t c0 = kk[0];                                        // column of the entry before e0 (-1: none)
        seg = -1;
        if (c0 >= 0) {
            const int w = c0 >> 5, owner = w / wpt;
            seg = s_chunk[owner] + __popc(a.map.cur[w] & ((1u << (c0 & 31)) - 1u));
#pragma unroll
            for (int q = 0; q < WPT - 1; ++q) {
                const int v = owner * wpt + q;
                if (v < w) seg += __popc(a.map.cur[v]);
            }
        }
        if (block == nblocks - 1 && tid == 0) {
            a.n_touched[0] = map_total;
            a.seg_ptr[map_total] = nnz;
        }
    } else {
        int32_t tile_total;
        const int32_t before = block_exclusive_scan(cnt, &tile_total);   // its barriers also publish s_base
        seg = s_base + before - 1;                                       // segment of the entry before e0
        if (block == nblocks - 1 && tid == 0) {
            a.n_touched[0] = s_base + tile_total;
            a.seg_ptr[s_base + tile_total] = nnz;
        }
    }
    int32_t o_seg[kSegWItems], o_row[kSegWItems], o_pk[kSegWItems];
    int8_t o_sign[kSegWItems];
    const bool whole = e0 + kSegWItems <= nnz;   // e0 is a multiple of 8: 32-byte vector accesses are aligned
    int32_t pp[kSegWItems];
    if (whole) {
        const int4 x = *reinterpret_cast<const int4 *>(pay + e0), y = *reinterpret_cast<const int4 *>(pay + e0 + 4);
        pp[0] = x.x; pp[1] = x.y; pp[2] = x.z; pp[3] = x.w; pp[4] = y.x; pp[5] = y.y; pp[6] = y.z; pp[7] = y.w;
    } else {
#pragma unroll
        for (int i = 0; i < kSegWItems; ++i) pp[i] = e0 + i < nnz ? pay[e0 + i] : 0;
    }
#pragma unroll
    for (int i = 0; i < kSegWItems; ++i) {
        int32_t e = e0 + i;
        bool head = e < nnz && kk[i + 1] != kk[i];   // e == 0: kk[0] = -1 differs from every column id
        if (head) {
            ++seg;
            a.touched_cols[seg] = kk[i + 1];
            a.seg_ptr[seg] = e;
        }
        int32_t row = pp[i] / 3;
        int32_t neg = (pp[i] - 3 * row) == 2 ? 1 : 0;
        o_seg[i] = seg;
        o_row[i] = row;
        o_sign[i] = neg ? (int8_t)-1 : (int8_t)1;
        o_pk[i] = (row << 2) | (head ? 2 : 0) | neg;
    }
    if (whole) {
        static_assert(kSegWItems == 8, "vector stores below assume 8 entries per thread");
        *reinterpret_cast<int4 *>(a.seg_id + e0) = make_int4(o_seg[0], o_seg[1], o_seg[2], o_seg[3]);
        *reinterpret_cast<int4 *>(a.seg_id + e0 + 4) = make_int4(o_seg[4], o_seg[5], o_seg[6], o_seg[7]);
        *reinterpret_cast<int4 *>(a.row_idx + e0) = make_int4(o_row[0], o_row[1], o_row[2], o_row[3]);
        *reinterpret_cast<int4 *>(a.row_idx + e0 + 4) = make_int4(o_row[4], o_row[5], o_row[6], o_row[7]);
        *reinterpret_cast<int4 *>(a.packed + e0) = make_int4(o_pk[0], o_pk[1], o_pk[2], o_pk[3]);
        *reinterpret_cast<int4 *>(a.packed + e0 + 4) = make_int4(o_pk[4], o_pk[5], o_pk[6], o_pk[7]);
        uint32_t s0 = 0, s1 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s0 |= (uint32_t)(uint8_t)o_sign[i] << (8 * i);
            s1 |= (uint32_t)(uint8_t)o_sign[4 + i] << (8 * i);
        }
        *reinterpret_cast<uint2 *>(a.sign + e0) = make_uint2(s0, s1);
    } else {
#pragma unroll
        for (int i = 0; i < kSegWItems; ++i) {
            int32_t e = e0 + i;
            if (e < nnz) { a.seg_id[e] = o_seg[i]; a.row_idx[e] = o_row[i]; a.sign[e] = o_sign[i]; a.packed[e] = o_pk[i]; }
        }
    }
}

}  // namespace stx
