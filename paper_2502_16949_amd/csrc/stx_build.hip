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
// stx_train_step lets independent work of the step share the launches of the scatter and histogram passes
// (stx_step.hip, stx_transr.hip), leaves k_seg_write to the launch of the fused transposed product
// (stx_backward.hip), and, when a call names the batch of the next call, runs k_emit, the first scatter pass
// and the second histogram pass of that batch inside this step's launches (prepare_emit_ahead, take_*_ahead).
// Histograms of digit 0 and of the later digits live in two tables, so that the next batch's k_emit can run
// beside a later pass of this batch.
// The tile histograms (tile-major table[tile][digit]) must become global offsets before a scatter.
// With few tiles every scatter workgroup derives its own offsets from the raw table (a few coalesced
// reads per thread); with many tiles a small k_super_sums first adds the histograms up in groups of tiles.
#include "stx_emit_body.h"
#include "stx_segw_body.h"
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
    for (int m = 32; m >= 1; m >>= 1) c += __shfl_xor(c, m, 64);   // one LDS atomic per wavefront, not per thread
    if ((tid & 63) == 0 && c) atomicAdd(&s_cnt, c);
    __syncthreads();
    if (tid == 0) tile_heads[blockIdx.x] = s_cnt;
}

template <bool MAP>
__global__ __launch_bounds__(kThreads) void k_seg_write(SegWriteArgs a)
{
    seg_write_body<MAP>((int)blockIdx.x, (int)gridDim.x, a);
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
    hipLaunchKernelGGL(k_clear_words, dim3(8), dim3(kThreads), 0, c->stream, c->colmap[0], 3 * c->map_words);
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

static void clear_ahead(stx_ctx *c)
{
    c->ahead.armed = false;
    c->ahead.emit_done = c->ahead.scatter_done = c->ahead.hist_done = false;
    c->ahead.scatter_ok = c->ahead.hist_ok = false;
    c->ahead.late_only = false;
}

bool prepare_emit_ahead(stx_ctx *c, const stx_batch *next, stx_incidence *inc)
{
    clear_ahead(c);
    if (!next || next->b <= 0 || next->k < 0 || next->b > c->cfg.max_batch || next->k > c->cfg.max_neg) return false;
    if (!next->h || !next->r || !next->t || (next->k > 0 && (!next->neg_h || !next->neg_t))) return false;
    if (next->m_total < 0 || next->global_offset < 0) return false;
    const int64_t nnz = 3 * (int64_t)next->b * (1 + next->k);
    if (nnz > (1 << 19)) {
        // A large sort: its first kernel (no bitmap, no row counts: the shapes of the large benchmark) can run in the
        // fix-up launch that ends this step, whose own workgroups mostly wait for memory.
        if (c->map_words > 0 || c->rel_cnt[0] || c->cfg.model == STX_TRANSR) return false;
        const int ntiles = (int)((nnz + kThreads * kBigSortItems - 1) / (kThreads * kBigSortItems));
        const int bits0 = c->sort_bits < c->digit_bits ? c->sort_bits : c->digit_bits;
        const uint64_t base_ctr = (next->epoch * (uint64_t)next->m_total + (uint64_t)next->global_offset) * (uint64_t)next->k;
        const BatchPtrs bp{next->h, next->r, next->t, nullptr, nullptr, next->b, next->k > 0 ? next->k : 1,
                           next->neg_h, next->neg_t, next->seed, base_ctr};
        c->ahead.args = EmitArgs{bp, (int32_t)c->cfg.n_ent, (int32_t)c->cfg.n_rel, (int32_t)nnz, inc->a_rowptr, inc->a_colidx,
                                 inc->a_vals, nullptr, 1 << bits0, ntiles, c->table, c->ctrl, ColMap{nullptr, nullptr, 0},
                                 RelCnt{nullptr, nullptr, 0}, nullptr};
        c->ahead.ntiles = ntiles;
        c->ahead.inc = inc;
        c->ahead.armed = true;
        c->ahead.late_only = true;
        return true;
    }
    if (c->map_words <= 0) return false;                               // small sorts: needs the bitmap path
    if (c->cfg.model == STX_TRANSR && !c->rel_cnt[0]) return false;     // TransR: its work items must come from counts
    const int ntiles = (int)((nnz + kThreads * kSortItems - 1) / (kThreads * kSortItems));
    const int bits0 = c->sort_bits < c->digit_bits ? c->sort_bits : c->digit_bits;
    const uint64_t base_ctr = (next->epoch * (uint64_t)next->m_total + (uint64_t)next->global_offset) * (uint64_t)next->k;
    const BatchPtrs bp{next->h, next->r, next->t, nullptr, nullptr, next->b, next->k > 0 ? next->k : 1,
                       next->neg_h, next->neg_t, next->seed, base_ctr};
    const ColMap map{c->colmap[c->map_cur], c->colmap[(c->map_cur + 1) % 3], c->map_words};
    c->map_cur = (c->map_cur + 1) % 3;
    RelCnt rc{nullptr, nullptr, 0};
    if (c->rel_cnt[0]) {   // TransR: the rows per relation are counted on the way (the two buffers alternate)
        rc = RelCnt{c->rel_cnt[c->cnt_cur], c->rel_cnt[c->cnt_cur ^ 1], (int)c->cfg.n_rel};
        c->cnt_cur ^= 1;
    }
    c->ahead.args = EmitArgs{bp, (int32_t)c->cfg.n_ent, (int32_t)c->cfg.n_rel, (int32_t)nnz, inc->a_rowptr, inc->a_colidx,
                             inc->a_vals, c->keys[2], 1 << bits0, ntiles, c->table, c->ctrl, map, rc,
                             c->cix[c->cix_cur]};
    c->cix_cur ^= 1;
    c->ahead.ntiles = ntiles;
    c->ahead.inc = inc;
    c->ahead.armed = true;
    // the first scatter pass (keys[2] -> keys[1], payload = position) can follow in the next launch when its
    // workgroups derive their offsets from the raw histograms themselves, and the histograms of the second
    // digit in the launch after that
    if (ntiles <= kSelfScanTiles) {
        c->ahead.sargs = ScatterArgs{c->keys[2], c->pay[0], c->keys[1], c->pay[1], (int32_t)nnz, 0, bits0, ntiles, c->table,
                                     c->super};
        c->ahead.scatter_ok = true;
        if (c->sort_passes >= 2) {
            const int left = c->sort_bits - c->digit_bits;
            c->ahead.hargs = HistArgs{c->keys[1], (int32_t)nnz, c->digit_bits, 1 << (left < c->digit_bits ? left : c->digit_bits),
                                      c->table1, ntiles};
            c->ahead.hist_ok = true;
        }
    }
    return true;
}

// The stages of the next build in their order; a launch that asks gets the stage that is due, at most one per
// launch because every stage reads what the whole of the one before it wrote.
EmitAhead take_emit_ahead(stx_ctx *c, bool fixup_launch)
{
    if (!c->ahead.armed || c->ahead.emit_done || c->ahead.late_only != fixup_launch) return EmitAhead{};
    c->ahead.emit_done = true;
    return EmitAhead{c->ahead.args, c->ahead.ntiles};
}

ScatterAhead take_scatter_ahead(stx_ctx *c)
{
    if (!c->ahead.armed || !c->ahead.emit_done || !c->ahead.scatter_ok || c->ahead.scatter_done) return ScatterAhead{};
    c->ahead.scatter_done = true;
    if (c->ahead.sargs.keys_out == c->sorted_keys) {   // the last build's sorted keys are about to be overwritten
        c->sorted_inc = nullptr;
        c->sorted_keys = nullptr;
    }
    return ScatterAhead{c->ahead.sargs, c->ahead.ntiles};
}

HistAhead take_hist_ahead(stx_ctx *c)
{
    if (!c->ahead.armed || !c->ahead.scatter_done || !c->ahead.hist_ok || c->ahead.hist_done) return HistAhead{};
    c->ahead.hist_done = true;
    return HistAhead{c->ahead.hargs, c->ahead.ntiles};
}

stx_status launch_build(stx_ctx *c, const int32_t *h, const int32_t *r, const int32_t *t, const int32_t *nh,
                        const int32_t *nt, int32_t b, int32_t k, stx_incidence *inc, const SampleArgs *sample,
                        StepFusion *fusion)
{
    hipStream_t s = c->stream;
    if (c->segw.armed) launch_seg_write_late(c);   // (a build whose last kernel nobody took along)
    c->sorted_inc = nullptr;
    c->sorted_keys = nullptr;
    c->sampled_inc = sample ? inc : nullptr;   // negatives drawn here keep the relation and one entity of their positive
    c->cnt_inc = nullptr;
    c->cnt_ptr = nullptr;
    c->prep_inc = nullptr;
    c->tr_fused_inc = nullptr;
    // the first kernels may already have run, in launches of the previous step
    const EmitAheadState prev = c->ahead;
    clear_ahead(c);
    if (b == 0) {
        hipLaunchKernelGGL(k_empty_incidence, dim3(1), dim3(64), 0, s, inc->a_rowptr, inc->at_seg_ptr,
                           inc->n_touched);
        return hip_ok(hipGetLastError());
    }
    const int32_t nnz = (int32_t)inc->nnz;
    // keys per thread: few when the sort is small (more workgroups, shorter serial ranking per workgroup),
    // more when it is large (fewer tiles, smaller histogram table)
    const int items = nnz <= (1 << 19) ? kSortItems : kBigSortItems;
    const int ntiles = (nnz + kThreads * items - 1) / (kThreads * items);
    const int n_ent = (int)c->cfg.n_ent, n_rel = (int)c->cfg.n_rel;
    BatchPtrs bp{h, r, t, nh, nt, b, k > 0 ? k : 1, nullptr, nullptr, 0, 0};
    if (sample) { bp.nh_out = sample->neg_h; bp.nt_out = sample->neg_t; bp.seed = sample->seed; bp.base_ctr = sample->base_ctr; }
    const bool use_map = c->map_words > 0;
    const EmitArgs &pa = prev.args;
    const bool emitted = prev.armed && prev.emit_done && sample && (use_map || prev.late_only) && prev.inc == inc && pa.bp.h == h && pa.bp.r == r &&
                         pa.bp.t == t && pa.bp.b == b && pa.bp.k == bp.k && pa.nnz == nnz &&
                         pa.bp.nh_out == bp.nh_out && pa.bp.nt_out == bp.nt_out && pa.bp.seed == bp.seed &&
                         pa.bp.base_ctr == bp.base_ctr;
    const bool scattered0 = emitted && prev.scatter_done;   // ... and the first scatter pass as well
    const bool counted1 = scattered0 && prev.hist_done;     // ... and the histograms of the second digit
    ColMap map{nullptr, nullptr, 0};
    int32_t *colidx2 = nullptr;
    if (emitted) {
        map = pa.map;                    // (the maps changed roles when it was prepared)
        colidx2 = pa.colidx2;
    } else {
        if (use_map) {
            map = ColMap{c->colmap[c->map_cur], c->colmap[(c->map_cur + 1) % 3], c->map_words};
            c->map_cur = (c->map_cur + 1) % 3;
        }
        // (no copy of the column ids: only a batch that was prepared ahead runs its forward pass in a launch
        // that takes the next batch's first kernel along)
    }
    if (fusion) fusion->colidx = colidx2;
    c->step_colidx = fusion ? colidx2 : nullptr;
    c->step_colidx_inc = inc;

    int bits0 = c->sort_bits < c->digit_bits ? c->sort_bits : c->digit_bits;
    const bool use_rc = c->rel_cnt[0] != nullptr;
    RelCnt rc{nullptr, nullptr, 0};
    if (use_rc && emitted) {   // counted when the first kernel ran ahead
        c->cnt_ptr = pa.rc.cur;
        c->cnt_inc = inc;
    } else if (use_rc) {
        rc = RelCnt{c->rel_cnt[c->cnt_cur], c->rel_cnt[c->cnt_cur ^ 1], n_rel};
        c->cnt_ptr = rc.cur;
        c->cnt_inc = inc;
        c->cnt_cur ^= 1;
    }
    // this batch has its map, its counts and its copy of the column ids: the next batch's first kernels can be
    // prepared (the rotating buffers go to the batches in their order), for the launches below and those of the
    // backward pass to take along
    if (fusion && fusion->next) prepare_emit_ahead(c, fusion->next, inc);
    // keys[2] receives the unsorted keys: the sorted keys of the previous batch (in keys[0] or keys[1]) stay
    // readable while this batch's first kernel runs
    // (a large sort reads its unsorted keys, which are the column ids, from A itself: 4 bytes per entry less to write)
    const bool keys_in_a = items == kBigSortItems;
    const EmitArgs ea{bp, n_ent, n_rel, nnz, inc->a_rowptr, inc->a_colidx, inc->a_vals, keys_in_a ? nullptr : c->keys[2],
                      1 << bits0, ntiles, c->table, c->ctrl, map, rc, colidx2};
    if (!emitted) {
    ProfScope prof(c, "k_emit");
#define STX_EMIT(I, M, S, R) hipLaunchKernelGGL((k_emit<I, M, S, R>), dim3(ntiles), dim3(kThreads), 0, s, ea)
#define STX_EMIT3(I, M, S) do { if (use_rc) STX_EMIT(I, M, S, true); else STX_EMIT(I, M, S, false); } while (0)
#define STX_EMIT2(I, M) do { if (sample) STX_EMIT3(I, M, true); else STX_EMIT3(I, M, false); } while (0)
    if (items == kSortItems) { if (use_map) STX_EMIT2(kSortItems, true); else STX_EMIT2(kSortItems, false); }
    else                     { if (use_map) STX_EMIT2(kBigSortItems, true); else STX_EMIT2(kBigSortItems, false); }
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
        // (histograms of the later digits go to the second table: the first one may be receiving the next batch's)
        if (p == 1 && counted1) {
            // the histograms of this digit are there already
        } else if (p == 1 && scattered0 && fusion && !fusion->forward_done && !two_level && items == kSortItems &&
            launch_fwd_hist(c, inc, fusion, c->keys[cur], nnz, shift, 1 << bits, ntiles)) {
            // the forward pass, which could not share the first scatter pass's launch, shares this histogram's
        } else if (p > 0 && fusion && fusion->forward_done && !fusion->finish_done && items == kSortItems) {
            launch_hist_finish(c, fusion, c->keys[cur], nnz, shift, 1 << bits, ntiles);
        } else if (p > 0) {
            ProfScope prof(c, "k_hist");
            if (items == kSortItems)
                hipLaunchKernelGGL(k_hist<kSortItems>, dim3(ntiles), dim3(kThreads), 0, s, c->keys[cur], nnz, shift,
                                   1 << bits, c->table1);
            else
                hipLaunchKernelGGL(k_hist<kBigSortItems>, dim3(ntiles), dim3(kThreads), 0, s, c->keys[cur], nnz, shift,
                                   1 << bits, c->table1);
        }
        if (two_level) {
            ProfScope prof(c, "k_super_sums");
            hipLaunchKernelGGL(k_super_sums, dim3(ngroups), dim3(kThreads), 0, s, p == 0 ? c->table : c->table1, 1 << bits,
                               ntiles, c->super);
        }
        const ScatterArgs sa{p == 0 ? (keys_in_a ? inc->a_colidx : c->keys[2]) : c->keys[cur], c->pay[cur], c->keys[cur ^ 1],
                             c->pay[cur ^ 1], nnz, shift,
                             bits, ntiles, p == 0 ? c->table : c->table1, c->super};
#define STX_SCATTER(F, S, I)                                                                                  \
    hipLaunchKernelGGL((k_scatter<F, S, I>), dim3(ntiles), dim3(kThreads), 0, s, sa)
#define STX_SCATTER2(F, S) do { if (items == kSortItems) STX_SCATTER(F, S, kSortItems); else STX_SCATTER(F, S, kBigSortItems); } while (0)
        if (p == 0 && fusion && !two_level && items == kSortItems && launch_fwd_scatter(c, inc, fusion, sa, true)) {
            // the forward pass ran in the same launch
        } else if (p == 1 && counted1 && fusion && !fusion->forward_done && !two_level && items == kSortItems &&
                   launch_fwd_scatter(c, inc, fusion, sa, false)) {
            // the forward pass shares the launch of the sort's last pass
        } else if (fusion && !two_level && items == kSortItems && (p == 0 || (p == 1 && scattered0)) &&
                   launch_prep_scatter(c, inc, fusion->p, sa, p == 0)) {
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
    c->segw.args = SegWriteArgs{c->keys[cur], c->pay[cur], nnz, c->tile_heads, inc->n_touched, inc->at_touched_cols,
                                inc->at_seg_ptr, inc->at_row_idx, inc->at_sign, inc->at_seg_id, inc->at_packed, map};
    c->segw.ntiles = nseg;
    c->segw.use_map = use_map;
    c->segw.armed = true;
    c->sorted_inc = inc;
    c->sorted_keys = c->keys[cur];
    if (c->segw.allowed) return hip_ok(hipGetLastError());   // the transposed product takes it along
    return launch_seg_write_late(c);
}

// The last kernel of the build that is waiting, if one is.
stx_status launch_seg_write_late(stx_ctx *c)
{
    if (!c->segw.armed) return STX_OK;
    c->segw.armed = false;
    ProfScope prof(c, "k_seg_write");
    if (c->segw.use_map)
        hipLaunchKernelGGL(k_seg_write<true>, dim3(c->segw.ntiles), dim3(kThreads), 0, c->stream, c->segw.args);
    else
        hipLaunchKernelGGL(k_seg_write<false>, dim3(c->segw.ntiles), dim3(kThreads), 0, c->stream, c->segw.args);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
