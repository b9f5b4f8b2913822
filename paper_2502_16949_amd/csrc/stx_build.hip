// Negative sampling and construction of the incidence matrix A (CSR) and of A^T sorted by column.
//
// A is the `hrt` incidence matrix of SparseTransX Sec. 4.2.2: one row per triplet, +1 at the head
// column, +1 at column n_ent + relation, -1 at the tail column (the `ht` form of Sec. 4.2.1 is slots 0
// and 2 of each row).  Appendix G needs A^T for the backward product; it is produced here by a stable
// least-significant-digit radix sort of the 3*rows column ids, so that every column's entries are
// contiguous and in a unique order, which is what lets the backward product run without atomics.
//
// Launch sequence for one batch (P = number of digit passes, 1..4):
//   k_emit            keys + CSR arrays + tile histograms of digit 0 (+ the negatives, when they are drawn
//                     here; + a presence bitmap of the columns when the table has few enough of them;
//                     + rows per relation for TransR)
//   k_scatter  x P    stable scatter by digit p
//   k_hist     x P-1  tile histograms of digit p (between scatters)
//   k_seg_count       segment heads per tile (only without the presence bitmap)
//   k_seg_write       touched_cols, seg_ptr, row_idx, sign, seg_id, packed, U
// stx_train_step lets independent work of the step share the launches of the first scatter pass and of
// the following histogram pass (stx_step.hip, stx_transr.hip).
// The tile histograms (tile-major table[tile][digit]) must become global offsets before a scatter.
// With few tiles every scatter workgroup derives its own offsets from the raw table (a few coalesced
// reads per thread); with many tiles a small k_super_sums first adds the histograms up in groups of tiles.
#include "stx_emit_body.h"
#include "stx_sort_body.h"

namespace stx {

__global__ __launch_bounds__(kThreads) void k_sample(const int32_t *__restrict__ h, const int32_t *__restrict__ t,
                                                     int64_t total, int32_t k, uint64_t n_ent, uint64_t seed,
                                                     uint64_t base_ctr, int32_t *__restrict__ nh,
                                                     int32_t *__restrict__ nt)
{
    int64_t idx = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (idx >= total) return;
    int64_t i = idx / k;
    uint64_t u = splitmix64_at(seed, base_ctr + (uint64_t)idx);
    int32_t e = (int32_t)(((u & 0xFFFFFFFFull) * n_ent) >> 32);
    bool head = (u >> 63) != 0;
    nh[idx] = head ? e : h[i];
    nt[idx] = head ? t[i] : e;
}

__global__ void k_clear_ctrl(int32_t *ctrl)
{
    if (threadIdx.x < CTRL_WORDS) ctrl[threadIdx.x] = 0;
}

__global__ __launch_bounds__(kThreads) void k_clear_words(uint32_t *p, int n)
{
    for (int i = (int)blockIdx.x * kThreads + threadIdx.x; i < n; i += (int)gridDim.x * kThreads) p[i] = 0u;
}

// Empty batch: A has no rows and A^T no segments.
__global__ void k_empty_incidence(int32_t *rowptr, int32_t *seg_ptr, int32_t *n_touched)
{
    if (threadIdx.x == 0) { rowptr[0] = 0; seg_ptr[0] = 0; n_touched[0] = 0; }
}

template <int ITEMS, bool MAP, bool SAMPLE, bool RC>
__global__ __launch_bounds__(kThreads) void k_emit(EmitArgs a)
{
    emit_body<ITEMS, MAP, SAMPLE, RC>((int)blockIdx.x, (int)gridDim.x, a);
}

template <int ITEMS>
__global__ __launch_bounds__(kThreads) void k_hist(const int32_t *__restrict__ keys, int32_t nnz, int shift,
                                                   int radix, int32_t *__restrict__ table)
{
    hist_body<ITEMS>((int)blockIdx.x, keys, nnz, shift, radix, table);
}

// With many tiles the scatter workgroups cannot each read the whole table.  This kernel adds the tile
// histograms up in groups of kSuperTile tiles: super[g][digit] = sum over the tiles of group g.  A
// scatter workgroup then needs its group's earlier tiles plus one row per group.
__global__ __launch_bounds__(kThreads) void k_super_sums(const int32_t *__restrict__ table, int radix, int ntiles,
                                                         int32_t *__restrict__ super)
{
    const int tid = threadIdx.x, t0 = blockIdx.x * kSuperTile, t1 = min(t0 + kSuperTile, ntiles);
    if (tid >= radix) return;
    int32_t a = 0;
#pragma unroll 8
    for (int t = t0; t < t1; ++t) a += table[t * radix + tid];
    super[blockIdx.x * radix + tid] = a;
}

template <bool FIRST, bool TWO_LEVEL, int ITEMS>
__global__ __launch_bounds__(kThreads) void k_scatter(ScatterArgs a)
{
    scatter_body<FIRST, TWO_LEVEL, ITEMS>((int)blockIdx.x, a);
}

// Number of segment heads (first entry of a column's run) in each tile of the sorted keys.
__global__ __launch_bounds__(kThreads) void k_seg_count(const int32_t *__restrict__ keys, int32_t nnz,
                                                        int32_t *__restrict__ tile_heads)
{
    __shared__ int32_t s_cnt;
    const int tid = threadIdx.x;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    const int32_t base = blockIdx.x * kSegWTile;
    int32_t c = 0;
#pragma unroll
    for (int it = 0; it < kSegWItems; ++it) {
        int32_t e = base + it * kThreads + tid;
        if (e < nnz) c += (e == 0 || keys[e] != keys[e - 1]) ? 1 : 0;
    }
    if (c) atomicAdd(&s_cnt, c);
    __syncthreads();
    if (tid == 0) tile_heads[blockIdx.x] = s_cnt;
}

// Per sorted entry: its segment, row, sign and packed form; per segment: its column and first entry.
// Thread t of a tile owns the 8 consecutive entries base + 8t .. base + 8t + 7.
// MAP: the segment of an entry is the rank of its column in the presence bitmap (every workgroup scans
// the map itself); otherwise it is counted from the heads of the earlier tiles (k_seg_count).
template <bool MAP>
__global__ __launch_bounds__(kThreads) void k_seg_write(const int32_t *__restrict__ keys,
                                                        const int32_t *__restrict__ pay, int32_t nnz,
                                                        const int32_t *__restrict__ tile_heads,
                                                        int32_t *__restrict__ n_touched,
                                                        int32_t *__restrict__ touched_cols,
                                                        int32_t *__restrict__ seg_ptr, int32_t *__restrict__ row_idx,
                                                        int8_t *__restrict__ sign, int32_t *__restrict__ seg_id,
                                                        int32_t *__restrict__ packed, ColMap map)
{
    __shared__ int32_t s_base;
    __shared__ uint32_t s_word[MAP ? kMapMaxWords : 1];
    __shared__ int32_t s_pref[MAP ? kMapMaxWords : 1];
    const int tid = threadIdx.x;
    if (tid == 0) s_base = 0;
    __syncthreads();
    int32_t map_total = 0;
    if (MAP) {   // thread t owns words [t*wpt, (t+1)*wpt): set bits below each word
        constexpr int WPT = kMapMaxWords / kThreads;
        const int wpt = (map.words + kThreads - 1) / kThreads;
        uint32_t wv[WPT];
        int32_t mine = 0;
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int w = tid * wpt + q;
            wv[q] = (q < wpt && w < map.words) ? map.cur[w] : 0u;
            mine += __popc(wv[q]);
        }
        int32_t run = block_exclusive_scan(mine, &map_total);
#pragma unroll
        for (int q = 0; q < WPT; ++q) {
            const int w = tid * wpt + q;
            if (q < wpt && w < map.words) { s_word[w] = wv[q]; s_pref[w] = run; run += __popc(wv[q]); }
        }
        __syncthreads();
    } else {   // segments that start in earlier tiles
        int32_t a = 0;
        for (int t = tid; t < (int)blockIdx.x; t += kThreads) a += tile_heads[t];
        if (a) atomicAdd(&s_base, a);
    }
    const int32_t e0 = blockIdx.x * kSegWTile + tid * kSegWItems;
    int32_t kk[kSegWItems + 1];
    kk[0] = (e0 > 0 && e0 - 1 < nnz) ? keys[e0 - 1] : -1;
    if (e0 + kSegWItems <= nnz) {
        const int4 a = *reinterpret_cast<const int4 *>(keys + e0), b = *reinterpret_cast<const int4 *>(keys + e0 + 4);
        kk[1] = a.x; kk[2] = a.y; kk[3] = a.z; kk[4] = a.w; kk[5] = b.x; kk[6] = b.y; kk[7] = b.z; kk[8] = b.w;
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
        seg = c0 < 0 ? -1 : s_pref[c0 >> 5] + __popc(s_word[c0 >> 5] & ((1u << (c0 & 31)) - 1u));
        if (blockIdx.x == gridDim.x - 1 && tid == 0) {
            n_touched[0] = map_total;
            seg_ptr[map_total] = nnz;
        }
    } else {
        int32_t tile_total;
        const int32_t before = block_exclusive_scan(cnt, &tile_total);   // its barriers also publish s_base
        seg = s_base + before - 1;                                       // segment of the entry before e0
        if (blockIdx.x == gridDim.x - 1 && tid == 0) {
            n_touched[0] = s_base + tile_total;
            seg_ptr[s_base + tile_total] = nnz;
        }
    }
    int32_t o_seg[kSegWItems], o_row[kSegWItems], o_pk[kSegWItems];
    int8_t o_sign[kSegWItems];
    const bool whole = e0 + kSegWItems <= nnz;   // e0 is a multiple of 8: 32-byte vector accesses are aligned
    int32_t pp[kSegWItems];
    if (whole) {
        const int4 a = *reinterpret_cast<const int4 *>(pay + e0), b = *reinterpret_cast<const int4 *>(pay + e0 + 4);
        pp[0] = a.x; pp[1] = a.y; pp[2] = a.z; pp[3] = a.w; pp[4] = b.x; pp[5] = b.y; pp[6] = b.z; pp[7] = b.w;
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
            touched_cols[seg] = kk[i + 1];
            seg_ptr[seg] = e;
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
        *reinterpret_cast<int4 *>(seg_id + e0) = make_int4(o_seg[0], o_seg[1], o_seg[2], o_seg[3]);
        *reinterpret_cast<int4 *>(seg_id + e0 + 4) = make_int4(o_seg[4], o_seg[5], o_seg[6], o_seg[7]);
        *reinterpret_cast<int4 *>(row_idx + e0) = make_int4(o_row[0], o_row[1], o_row[2], o_row[3]);
        *reinterpret_cast<int4 *>(row_idx + e0 + 4) = make_int4(o_row[4], o_row[5], o_row[6], o_row[7]);
        *reinterpret_cast<int4 *>(packed + e0) = make_int4(o_pk[0], o_pk[1], o_pk[2], o_pk[3]);
        *reinterpret_cast<int4 *>(packed + e0 + 4) = make_int4(o_pk[4], o_pk[5], o_pk[6], o_pk[7]);
        uint32_t s0 = 0, s1 = 0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            s0 |= (uint32_t)(uint8_t)o_sign[i] << (8 * i);
            s1 |= (uint32_t)(uint8_t)o_sign[4 + i] << (8 * i);
        }
        *reinterpret_cast<uint2 *>(sign + e0) = make_uint2(s0, s1);
    } else {
#pragma unroll
        for (int i = 0; i < kSegWItems; ++i) {
            int32_t e = e0 + i;
            if (e < nnz) { seg_id[e] = o_seg[i]; row_idx[e] = o_row[i]; sign[e] = o_sign[i]; packed[e] = o_pk[i]; }
        }
    }
}

// ---------------------------------------------------------------------------------------------------
stx_status launch_clear_ctrl(stx_ctx *c)
{
    hipLaunchKernelGGL(k_clear_ctrl, dim3(1), dim3(64), 0, c->stream, c->ctrl);
    return hip_ok(hipGetLastError());
}

stx_status launch_clear_maps(stx_ctx *c)
{
    if (c->map_words == 0) return STX_OK;
    // the two maps are adjacent in the workspace
    hipLaunchKernelGGL(k_clear_words, dim3(8), dim3(kThreads), 0, c->stream, c->colmap[0], 2 * c->map_words);
    c->map_cur = 0;
    return hip_ok(hipGetLastError());
}

stx_status launch_clear_rel_counts(stx_ctx *c)
{
    if (!c->rel_cnt[0]) return STX_OK;
    hipLaunchKernelGGL(k_clear_words, dim3(8), dim3(kThreads), 0, c->stream, (uint32_t *)c->rel_cnt[0],
                       (int)(2 * c->cfg.n_rel));
    c->cnt_cur = 0;
    return hip_ok(hipGetLastError());
}

stx_status launch_sample(stx_ctx *c, const int32_t *h, const int32_t *t, int64_t m, int32_t k, uint64_t seed,
                         uint64_t base_ctr, int32_t *nh, int32_t *nt)
{
    int64_t total = m * k;
    if (total == 0) return STX_OK;
    int64_t blocks = (total + kThreads - 1) / kThreads;
    ProfScope prof(c, "k_sample");
    hipLaunchKernelGGL(k_sample, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, h, t, total, k,
                       (uint64_t)c->cfg.n_ent, seed, base_ctr, nh, nt);
    return hip_ok(hipGetLastError());
}

bool prepare_emit_ahead(stx_ctx *c, const stx_batch *next, stx_incidence *inc)
{
    c->ahead.armed = c->ahead.done = false;
    c->ahead.scatter_armed = c->ahead.scatter_done = false;
    if (!next || next->b <= 0 || next->k < 0 || next->b > c->cfg.max_batch || next->k > c->cfg.max_neg) return false;
    if (!next->h || !next->r || !next->t || (next->k > 0 && (!next->neg_h || !next->neg_t))) return false;
    if (next->m_total < 0 || next->global_offset < 0) return false;
    if (c->map_words <= 0 || c->rel_cnt[0] != nullptr) return false;   // needs the bitmap path, no relation counts
    const int64_t nnz = 3 * (int64_t)next->b * (1 + next->k);
    if (nnz > (1 << 19)) return false;                                  // the small-sort shape of the first kernel only
    const int ntiles = (int)((nnz + kThreads * kSortItems - 1) / (kThreads * kSortItems));
    const int bits0 = c->sort_bits < c->digit_bits ? c->sort_bits : c->digit_bits;
    const uint64_t base_ctr = (next->epoch * (uint64_t)next->m_total + (uint64_t)next->global_offset) * (uint64_t)next->k;
    const BatchPtrs bp{next->h, next->r, next->t, nullptr, nullptr, next->b, next->k > 0 ? next->k : 1,
                       next->neg_h, next->neg_t, next->seed, base_ctr};
    const ColMap map{c->colmap[c->map_cur], c->colmap[c->map_cur ^ 1], c->map_words};
    c->map_cur ^= 1;
    c->ahead.args = EmitArgs{bp, (int32_t)c->cfg.n_ent, (int32_t)c->cfg.n_rel, (int32_t)nnz, inc->a_rowptr, inc->a_colidx,
                             inc->a_vals, c->keys[2], 1 << bits0, ntiles, c->table, c->ctrl, map,
                             RelCnt{nullptr, nullptr, 0}};
    c->ahead.ntiles = ntiles;
    c->ahead.inc = inc;
    c->ahead.armed = true;
    // the first scatter pass (keys[2] -> keys[1], payload = position) can follow in the next launch when its
    // workgroups derive their offsets from the raw histograms themselves
    if (ntiles <= kSelfScanTiles) {
        c->ahead.sargs = ScatterArgs{c->keys[2], c->pay[0], c->keys[1], c->pay[1], (int32_t)nnz, 0, bits0, ntiles, c->table,
                                     c->super};
        c->ahead.scatter_armed = true;
    }
    return true;
}

stx_status launch_build(stx_ctx *c, const int32_t *h, const int32_t *r, const int32_t *t, const int32_t *nh,
                        const int32_t *nt, int32_t b, int32_t k, stx_incidence *inc, const SampleArgs *sample,
                        StepFusion *fusion)
{
    hipStream_t s = c->stream;
    c->sorted_inc = nullptr;
    c->sorted_keys = nullptr;
    c->cnt_inc = nullptr;
    c->cnt_ptr = nullptr;
    c->prep_inc = nullptr;
    // the first kernel may already have run, in the launch of the previous step's transposed product
    const bool ahead_done = c->ahead.done, ahead_scattered = c->ahead.scatter_done;
    c->ahead.armed = c->ahead.done = false;
    c->ahead.scatter_armed = c->ahead.scatter_done = false;
    if (b == 0) {
        hipLaunchKernelGGL(k_empty_incidence, dim3(1), dim3(64), 0, s, inc->a_rowptr, inc->at_seg_ptr,
                           inc->n_touched);
        return hip_ok(hipGetLastError());
    }
    const int32_t nnz = (int32_t)inc->nnz;
    // keys per thread: few when the sort is small (more workgroups, shorter serial ranking per workgroup),
    // more when it is large (fewer tiles, smaller histogram table)
    const int items = nnz <= (1 << 19) ? kSortItems : 2 * kSortItems;
    const int ntiles = (nnz + kThreads * items - 1) / (kThreads * items);
    const int n_ent = (int)c->cfg.n_ent, n_rel = (int)c->cfg.n_rel;
    BatchPtrs bp{h, r, t, nh, nt, b, k > 0 ? k : 1, nullptr, nullptr, 0, 0};
    if (sample) { bp.nh_out = sample->neg_h; bp.nt_out = sample->neg_t; bp.seed = sample->seed; bp.base_ctr = sample->base_ctr; }
    const bool use_map = c->map_words > 0;
    const EmitArgs &pa = c->ahead.args;
    const bool emitted = ahead_done && sample && use_map && c->ahead.inc == inc && pa.bp.h == h && pa.bp.r == r &&
                         pa.bp.t == t && pa.bp.b == b && pa.bp.k == bp.k && pa.nnz == nnz &&
                         pa.bp.nh_out == bp.nh_out && pa.bp.nt_out == bp.nt_out && pa.bp.seed == bp.seed &&
                         pa.bp.base_ctr == bp.base_ctr;
    const bool scattered0 = emitted && ahead_scattered;   // ... and the first scatter pass as well
    ColMap map{nullptr, nullptr, 0};
    if (emitted) {
        map = pa.map;                    // (the maps changed roles when it was prepared)
    } else if (use_map) {
        map = ColMap{c->colmap[c->map_cur], c->colmap[c->map_cur ^ 1], c->map_words};
        c->map_cur ^= 1;
    }

    int bits0 = c->sort_bits < c->digit_bits ? c->sort_bits : c->digit_bits;
    const bool use_rc = c->rel_cnt[0] != nullptr;
    RelCnt rc{nullptr, nullptr, 0};
    if (use_rc) {
        rc = RelCnt{c->rel_cnt[c->cnt_cur], c->rel_cnt[c->cnt_cur ^ 1], n_rel};
        c->cnt_ptr = rc.cur;
        c->cnt_inc = inc;
        c->cnt_cur ^= 1;
    }
    // keys[2] receives the unsorted keys: the sorted keys of the previous batch (in keys[0] or keys[1]) stay
    // readable while this batch's first kernel runs
    const EmitArgs ea{bp, n_ent, n_rel, nnz, inc->a_rowptr, inc->a_colidx, inc->a_vals, c->keys[2], 1 << bits0, ntiles,
                      c->table, c->ctrl, map, rc};
    if (!emitted) {
    ProfScope prof(c, "k_emit");
#define STX_EMIT(I, M, S, R) hipLaunchKernelGGL((k_emit<I, M, S, R>), dim3(ntiles), dim3(kThreads), 0, s, ea)
#define STX_EMIT3(I, M, S) do { if (use_rc) STX_EMIT(I, M, S, true); else STX_EMIT(I, M, S, false); } while (0)
#define STX_EMIT2(I, M) do { if (sample) STX_EMIT3(I, M, true); else STX_EMIT3(I, M, false); } while (0)
    if (items == kSortItems) { if (use_map) STX_EMIT2(kSortItems, true); else STX_EMIT2(kSortItems, false); }
    else                     { if (use_map) STX_EMIT2(2 * kSortItems, true); else STX_EMIT2(2 * kSortItems, false); }
#undef STX_EMIT2
#undef STX_EMIT3
#undef STX_EMIT
    }
    const bool two_level = ntiles > kSelfScanTiles;
    const int ngroups = (ntiles + kSuperTile - 1) / kSuperTile;
    int cur = 0;
    for (int p = 0; p < c->sort_passes; ++p) {
        int shift = p * c->digit_bits;
        int bits = c->sort_bits - shift < c->digit_bits ? c->sort_bits - shift : c->digit_bits;
        if (p == 0 && scattered0) {   // ran in the launch of the previous step's fix-up kernel
            cur ^= 1;
            continue;
        }
        if (p == 1 && scattered0 && fusion && !fusion->forward_done && !two_level && items == kSortItems &&
            launch_fwd_hist(c, inc, fusion, c->keys[cur], nnz, shift, 1 << bits, ntiles)) {
            // the forward pass, which could not share the first scatter pass's launch, shares this histogram's
        } else if (p > 0 && fusion && fusion->forward_done && !fusion->finish_done && items == kSortItems) {
            launch_hist_finish(c, fusion, c->keys[cur], nnz, shift, 1 << bits, ntiles);
        } else if (p > 0) {
            ProfScope prof(c, "k_hist");
            if (items == kSortItems)
                hipLaunchKernelGGL(k_hist<kSortItems>, dim3(ntiles), dim3(kThreads), 0, s, c->keys[cur], nnz, shift,
                                   1 << bits, c->table);
            else
                hipLaunchKernelGGL(k_hist<2 * kSortItems>, dim3(ntiles), dim3(kThreads), 0, s, c->keys[cur], nnz, shift,
                                   1 << bits, c->table);
        }
        if (two_level) {
            ProfScope prof(c, "k_super_sums");
            hipLaunchKernelGGL(k_super_sums, dim3(ngroups), dim3(kThreads), 0, s, c->table, 1 << bits, ntiles,
                               c->super);
        }
        const ScatterArgs sa{p == 0 ? c->keys[2] : c->keys[cur], c->pay[cur], c->keys[cur ^ 1], c->pay[cur ^ 1], nnz, shift,
                             bits, ntiles, c->table, c->super};
#define STX_SCATTER(F, S, I)                                                                                  \
    hipLaunchKernelGGL((k_scatter<F, S, I>), dim3(ntiles), dim3(kThreads), 0, s, sa)
#define STX_SCATTER2(F, S) do { if (items == kSortItems) STX_SCATTER(F, S, kSortItems); else STX_SCATTER(F, S, 2 * kSortItems); } while (0)
        if (p == 0 && fusion && !two_level && items == kSortItems && launch_fwd_scatter(c, inc, fusion, sa)) {
            // the forward pass ran in the same launch
        } else if (p == 0 && fusion && !two_level && items == kSortItems && launch_prep_scatter(c, inc, fusion->p, sa)) {
            // TransR: the item lists and the bf16 copies of M_r were made in the same launch
        } else if (p > 0 && scattered0 && fusion && fusion->forward_done && !fusion->finish_done && !two_level &&
                   items == kSortItems) {
            launch_scatter_finish(c, fusion, sa);   // the sum of the loss rides here
        } else {
            ProfScope prof(c, "k_scatter");
            if (p == 0) { if (two_level) STX_SCATTER2(true, true); else STX_SCATTER2(true, false); }
            else        { if (two_level) STX_SCATTER2(false, true); else STX_SCATTER2(false, false); }
        }
#undef STX_SCATTER2
#undef STX_SCATTER
        cur ^= 1;
    }
    const int nseg = (nnz + kSegWTile - 1) / kSegWTile;
    if (!use_map) {
        ProfScope prof(c, "k_seg_count");
        hipLaunchKernelGGL(k_seg_count, dim3(nseg), dim3(kThreads), 0, s, c->keys[cur], nnz, c->tile_heads);
    }
    ProfScope prof(c, "k_seg_write");
    if (use_map)
        hipLaunchKernelGGL(k_seg_write<true>, dim3(nseg), dim3(kThreads), 0, s, c->keys[cur], c->pay[cur], nnz,
                           c->tile_heads, inc->n_touched, inc->at_touched_cols, inc->at_seg_ptr, inc->at_row_idx,
                           inc->at_sign, inc->at_seg_id, inc->at_packed, map);
    else
        hipLaunchKernelGGL(k_seg_write<false>, dim3(nseg), dim3(kThreads), 0, s, c->keys[cur], c->pay[cur], nnz,
                           c->tile_heads, inc->n_touched, inc->at_touched_cols, inc->at_seg_ptr, inc->at_row_idx,
                           inc->at_sign, inc->at_seg_id, inc->at_packed, map);
    c->sorted_inc = inc;
    c->sorted_keys = c->keys[cur];
    return hip_ok(hipGetLastError());
}

}  // namespace stx
