// Transposed product A^T.G without atomics, and the sparse SGD update.
//
// SparseTransX Appendix G: for C = A.X the gradient is dL/dX = A^T.dL/dC, itself a sparse-dense
// product.  A^T arrives sorted by column (see stx_build.hip), so the gradient row of column c is the
// signed sum of the G rows named by one contiguous run ("segment") of sorted entries.  Power-law graphs
// make segment lengths wildly uneven (one entity can own >10% of all entries), so work is split by
// entries, not by segments:
//
//   k_seg_reduce   each workgroup owns a tile of consecutive sorted entries, each of its lane groups a
//                  chunk of LPR of them.  A group walks its chunk in order, adding signed G rows into
//                  registers and closing a run whenever an entry is flagged as a segment head.  Runs that
//                  lie inside the chunk are stored to the output directly.  A chunk's first / last run
//                  may continue in a neighbouring chunk; those go to LDS, are stitched in chunk order by
//                  one group, and the (at most two) runs that cross the workgroup's own borders are
//                  stored as partial rows.
//   k_seg_fixup    the workgroup in which a border-crossing run ends adds up that run's partial rows,
//                  in tile order, and stores the result.
//
// Every output row is written exactly once and every sum has a fixed association order, so results are
// bitwise reproducible from run to run.
//
// FUSED variants of both kernels apply the SGD update in place of the store: wherever a gradient row
// would be written they write table[column] - lr * gradient (and wrap it for TorusE) instead, with the
// same two roundings as k_sgd_rows, so the gradient rows never travel to memory and back.  The table
// row of a run is fetched together with the run's first source row, so closing a run costs no extra
// memory round trip.
//
// In stx_train_step the launches of both kernels carry more (template parameter RIDE): the product reads the
// sorted keys and payloads of the build itself, so that the build's last kernel and the sum of the loss run
// as extra workgroups of its launch, and one stage of the next batch's build rides in each launch; with TransR
// the dL/dM_r product (stx_transr_dm_body.h) rides in the product's launch and the sums of its partial matrices
// in the fix-up's.  All parts of a launch share one block of LDS.
#include "stx_emit_body.h"
#include "stx_forward_body.h"
#include "stx_rowops.h"
#include "stx_segw_body.h"
#include "stx_sort_body.h"
#include "stx_transr_dm_body.h"

namespace stx {

// Work that rides in the launches of the transposed product, as workgroups with the low block indices: the last
// kernel of this batch's build and the sum of the loss (SegWriteRide), and one stage of the next batch's build
// per launch (EmitAhead, ScatterAhead, HistAhead).
struct SegWriteRide {
    SegWriteArgs args;
    int ntiles;
    int use_map;
    // a final sum of the loss that waits for a launch (fin_n > 0: one more workgroup)
    const float *fin_partials;
    int fin_n;
    float fin_scale;
    float *fin_loss;
};

enum { HAS_FIRST = 1, FIRST_CONT = 2, HAS_LAST = 4 };

template <int ITERS>
struct Acc {
    float4 v[ITERS];
    __device__ inline void zero()
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
    }
    __device__ inline void add(const Acc &o)
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            v[it].x += o.v[it].x; v[it].y += o.v[it].y; v[it].z += o.v[it].z; v[it].w += o.v[it].w;
        }
    }
};

template <int LPR, int ITERS>
__device__ inline void load_row(const float *__restrict__ p, int d4, int lig, Acc<ITERS> &a)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        a.v[it] = j < d4 ? ld4(p + 4 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
// ... of a table far larger than the caches, read once and rewritten: fetched past them
template <int LPR, int ITERS>
__device__ inline void load_row_stream(const float *__restrict__ p, int d4, int lig, Acc<ITERS> &a)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        a.v[it] = j < d4 ? ld4_stream(p + 4 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
template <int LPR, int ITERS>
__device__ inline void store_row_stream(float *__restrict__ p, int d4, int lig, const Acc<ITERS> &a)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) st4_stream(p + 4 * j, a.v[it]);
    }
}
template <int LPR, int ITERS>
__device__ inline void store_row(float *__restrict__ p, int d4, int lig, const Acc<ITERS> &a)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) st4(p + 4 * j, a.v[it]);
    }
}

struct FusedArgs {             // the update that replaces the store of a gradient row (FUSED kernels)
    float *table;              // rows of 4*d4 floats: row c for column c < n_split
    float *table_b;            // ... and row c - n_split of this one for the other columns
    int32_t n_split;
    const int32_t *touched_cols;
    const int32_t *cols_sorted;  // column of every sorted entry, or null: then it is looked up through the segment
    float lr;
    int mode;                  // 0 plain, 1 keep the fractional part (TorusE, Sec. 4.6), 2 rescale to unit length
    int stream;                // tables far larger than the caches: updated rows bypass them on the way out
};
__device__ inline float *fused_row(const FusedArgs &fu, int32_t col, int ld_tab)
{
    // (unsigned 32 x 32 -> 64 bit product: one instruction, where signed 64-bit operands take six)
    const bool first = col < fu.n_split;
    const uint32_t r = (uint32_t)(first ? col : col - fu.n_split);
    return (first ? fu.table : fu.table_b) + (uint64_t)r * (uint32_t)ld_tab;
}

// A second, independent transposed product that shares the launch (TransH: the sums of gw over the
// relation columns beside the sums of gx / gy over all columns).  Workgroups from `first_block` on work
// on it; all of its entries read `src`.
struct SegSecond {
    int first_block;           // INT_MAX: no second product
    int32_t e_begin, e_end;
    const float *src;
    float *out_rows, *partials;
    float *fused_table;        // FUSED: its columns all lie at or above n_split and update this table ...
    int fused_mode;            // ... in this mode
};

// table row <- x - lr * g, each product and difference rounded once, as in k_sgd_rows.
template <int LPR, int ITERS>
__device__ inline void apply_update(float *__restrict__ row, int d4, int lig, const Acc<ITERS> &x, const Acc<ITERS> &g,
                                    float lr, int mode, int stream)
{
    Acc<ITERS> o;
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const float *xv = &x.v[it].x, *gv = &g.v[it].x;
        float *ov = &o.v[it].x;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float step = lr * gv[q];
            float nv = xv[q] - step;
            if (mode == 1) {
                nv = nv - floorf(nv);
                if (nv >= 1.0f) nv = 0.0f;
            }
            ov[q] = nv;
            ss += nv * nv;
        }
    }
    if (mode == 2) {   // all lanes of the group are here together
        ss = group_sum<LPR>(ss);
        if (ss > 0.f) {
            const float inv = 1.0f / sqrtf(ss);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                o.v[it].x *= inv; o.v[it].y *= inv; o.v[it].z *= inv; o.v[it].w *= inv;
            }
        }
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int j = lig + it * LPR;
        if (j < d4) {
            if (stream) st4_stream(row + 4 * j, o.v[it]);
            else st4(row + 4 * j, o.v[it]);   // a small table is read again by the next step's forward pass
        }
    }
}

// PACKED: the source rows are records of ld_src bytes at src_a (dim/4 sign bytes) with their coefficients in
// src_b, as the forward pass of an L1-kind distance stores them; values and summation order are the same as with
// dense rows, so both forms give the same bits.
// RAW: `packed` and `seg_id` are the sorted payloads and keys of the build instead (a lane derives its entry's
// row, sign, column and whether it heads a segment from them), and the first sw.ntiles workgroups run the
// build's last kernel, whose arrays nothing reads before the fix-up launch.
// RIDE: 0 none of this; 1 RAW; 2 RAW, and the first kernel of the next batch's build comes along; 3 RAW, and the
// first scatter pass of the next batch's sort comes along; 4 as 2, and that kernel counts the rows per relation;
// 5 as 3, and TransR's dL/dM_r product comes along (its 128 registers still leave four workgroups on a CU, more
// than such a batch gives this product).
template <int LPR, int ITERS, bool PACKED, int CHUNK, bool FUSED, int RIDE>
__global__ __launch_bounds__(kThreads, RIDE == 5 ? 4 : (ITERS == 1 && PACKED && FUSED && RIDE != 4) ? 8 : 1) void k_seg_reduce(const int32_t *__restrict__ packed,
                                                         const int32_t *__restrict__ seg_id, int32_t e_begin,
                                                         int32_t e_end, const float *__restrict__ src_a,
                                                         const float *__restrict__ src_b, int32_t split,
                                                         int ld_src, int tail_off, int d4, float *__restrict__ out_rows,
                                                         int ld_out, float *__restrict__ partials, FusedArgs fu,
                                                         SegSecond sec, SegWriteRide sw, EmitAhead ea,
                                                         ScatterAhead sca, DmRide dm)
{
    constexpr bool RAW = RIDE != 0;
    // One block of LDS for whichever part a workgroup plays (the parts' own arrays would add up and cost the
    // launch wavefronts per CU): the product's arrays below, or those of a body that rides.
    constexpr int GROUPS_ = kThreads / LPR, ROWF_ = ITERS * LPR * 4;
    constexpr int OWN_LDS = (GROUPS_ * 2 * ROWF_ + (FUSED ? GROUPS_ * ROWF_ : 4) + 5 * GROUPS_) * 4;
    constexpr int RIDE_LDS = RIDE == 0 ? 0
                             : (RIDE == 3 || RIDE == 5) ? kScatterLds
                             : (RIDE == 2 || RIDE == 4) ? emit_lds(true, RIDE == 4)
                                                         : (kFinishLds > kSegWriteLds ? kFinishLds : kSegWriteLds);
    constexpr int ARENA_LDS = OWN_LDS > RIDE_LDS ? OWN_LDS : RIDE_LDS;
    static_assert(kFinishLds <= OWN_LDS || RIDE == 0 || kFinishLds <= RIDE_LDS, "the loss sum fits the block");
    __shared__ __align__(16) unsigned char s_arena[ARENA_LDS];
    int block = (int)blockIdx.x;
    if constexpr (RAW) {
        static_assert(FUSED, "the segment of an entry is not known here");
        static_assert(kSegWriteLds <= ARENA_LDS && kFinishLds <= ARENA_LDS, "riders fit the block of LDS");
        if (block < sw.ntiles) {      // uniform in the workgroup
            if (sw.use_map) seg_write_body<true, true>(block, sw.ntiles, sw.args, s_arena);
            else seg_write_body<false, true>(block, sw.ntiles, sw.args, s_arena);
            return;
        }
        block -= sw.ntiles;
        if (sw.fin_n > 0) {
            if (block == 0) {
                finish_loss_body<true>(sw.fin_partials, sw.fin_n, sw.fin_scale, sw.fin_loss, s_arena);
                return;
            }
            --block;
        }
    }
    if constexpr (RIDE == 2 || RIDE == 4) {
        if (block < ea.ntiles) {      // uniform in the workgroup
            emit_body<kSortItems, true, true, RIDE == 4, true>(block, ea.ntiles, ea.args, s_arena);
            return;
        }
        block -= ea.ntiles;
    }
    if constexpr (RIDE == 5) {
        if (block < dm.blocks) {      // uniform in the workgroup
            transr_dm_body(block, 0, dm.args);
            return;
        }
        block -= dm.blocks;
    }
    if constexpr (RIDE == 3 || RIDE == 5) {
        if (block < sca.ntiles) {
            scatter_body<true, false, kSortItems, true>(block, sca.args, s_arena);
            return;
        }
        block -= sca.ntiles;
    }
    if (block >= sec.first_block) {   // uniform in the workgroup
        block -= sec.first_block;
        e_begin = sec.e_begin; e_end = sec.e_end;
        src_a = src_b = sec.src; split = sec.e_end;
        out_rows = sec.out_rows; partials = sec.partials;
        fu.table_b = sec.fused_table; fu.mode = sec.fused_mode;
    }
    // A row wider than the lanes of a group cover at once can be cut into slices of LPR float4, one per
    // blockIdx.y: every pointer moves to the slice's first column and the width shrinks to the slice.
    const int ld_tab = d4 * 4;                             // floats per table row (fused update)
    int pk_off = 0;                                        // packed records: sign byte of the slice's first float4
    if (gridDim.y > 1) {
        const int c4 = (int)blockIdx.y * LPR;
        d4 = min(LPR, d4 - c4);
        if (PACKED) pk_off = c4;
        else { src_a += 4 * c4; src_b += 4 * c4; }
        if (out_rows) out_rows += 4 * c4;
        partials += 4 * c4;
        if (fu.table) fu.table += 4 * c4;
        if (fu.table_b) fu.table_b += 4 * c4;
    }
    constexpr int GROUPS = kThreads / LPR;
    // rows in flight per lane: dense rows cost 4*ITERS registers each; packed rows are a byte and a float,
    // so a whole chunk is fetched at once and the kernel pays one memory latency per chunk
    constexpr int UNROLL = PACKED ? (FUSED ? 4 : (CHUNK < 8 ? CHUNK : 8)) : (ITERS == 1 ? (FUSED ? 4 : 8) : (ITERS == 2 ? 4 : 2));
    constexpr int TILE = GROUPS * CHUNK;    // sorted entries per workgroup
    static_assert(CHUNK <= LPR && CHUNK % UNROLL == 0, "one entry per lane per chunk");
    constexpr int VROWS = PACKED ? 1 : UNROLL;
    constexpr int ROWF = ITERS * LPR * 4;   // floats per staged row in LDS
    static_assert(GROUPS == GROUPS_ && ROWF == ROWF_, "sizes of the block of LDS");
    float (*s_part)[2][ROWF] = reinterpret_cast<float (*)[2][ROWF]>(s_arena);
    // FUSED: table row and column of the run that leaves each chunk to the right; which chunk's they are for
    // the stitched run that closes in a chunk (-1: none closes there)
    float (*s_x)[FUSED ? ROWF : 4] = reinterpret_cast<float (*)[FUSED ? ROWF : 4]>(s_arena + GROUPS * 2 * ROWF * 4);
    int32_t *s_small = reinterpret_cast<int32_t *>(s_arena + (GROUPS * 2 * ROWF + (FUSED ? GROUPS * ROWF : 4)) * 4);
    int32_t *s_info = s_small, *s_seg_first = s_small + GROUPS, *s_seg_last = s_small + 2 * GROUPS;
    int32_t *s_col_last = s_small + 3 * GROUPS, *s_fin_src = s_small + 4 * GROUPS;

    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int pk_sh = PACKED ? 31 - __clz(ld_src) : 0;
    const uint8_t *pk_lane = reinterpret_cast<const uint8_t *>(src_a) + pk_off + lig;
    const int32_t tile0 = e_begin + block * TILE;
    const int32_t ec0 = tile0 + grp * CHUNK;
    const int32_t ec1 = min(ec0 + CHUNK, e_end);

    int info = 0;
    if (ec0 < e_end) {
        const int n = ec1 - ec0;
        int32_t meta = 0;                                  // 0: row 0, a safe address
        int32_t colv = 0;                                  // FUSED: the column of this lane's entry
        bool right_head = true;                            // the entry after the chunk heads a segment
        if constexpr (RAW) {
            if (lig < CHUNK && ec0 + lig < ec1) {
                const int32_t e = ec0 + lig;
                const int32_t pos = packed[e], kc = seg_id[e], kp = e > 0 ? seg_id[e - 1] : -1;
                const int32_t row = pos / 3;
                meta = (row << 2) | (kc != kp ? 2 : 0) | (pos - 3 * row == 2 ? 1 : 0);
                colv = kc;
            }
            if (ec1 < e_end) right_head = seg_id[ec1] != seg_id[ec1 - 1];
        } else {
            if (lig < CHUNK && ec0 + lig < ec1) meta = packed[ec0 + lig];
            if (FUSED && lig < CHUNK && ec0 + lig < ec1)
                colv = fu.cols_sorted ? fu.cols_sorted[ec0 + lig] : fu.touched_cols[seg_id[ec0 + lig]];
            if (ec1 < e_end) right_head = (packed[ec1] & 2) != 0;
        }
        Acc<ITERS> xcur;                                   // FUSED: table row of the run that is being summed
        int32_t colcur = 0;
        xcur.zero();
        const int32_t meta0 = __shfl(meta, 0, LPR);
        const bool first_open = (ec0 > e_begin) && !(meta0 & 2);
        const bool right_open = (ec1 < e_end) && !right_head;
        int32_t cur_seg = RAW ? 0 : seg_id[ec0];
        int nflush = 0;
        Acc<ITERS> acc;
        acc.zero();

        auto flush = [&](bool last_run) {
            const bool open_left = (nflush == 0) && first_open;
            const bool open_right = last_run && right_open;
            if (!open_left && !open_right) {
                if constexpr (FUSED)
                    apply_update<LPR, ITERS>(fused_row(fu, colcur, ld_tab), d4, lig, xcur, acc, fu.lr, fu.mode, fu.stream);
                else
                    store_row_stream<LPR, ITERS>(out_rows + (int64_t)cur_seg * ld_out, d4, lig, acc);
            } else {
                const int slot = open_left ? 0 : 1;
#pragma unroll
                for (int it = 0; it < ITERS; ++it)
                    st4(&s_part[grp][slot][(lig + it * LPR) * 4], acc.v[it]);
                if (open_left) {
                    info |= HAS_FIRST | (open_right ? FIRST_CONT : 0);
                    if (lig == 0) s_seg_first[grp] = cur_seg;
                } else {
                    info |= HAS_LAST;
                    if (lig == 0) s_seg_last[grp] = cur_seg;
                    if constexpr (FUSED) {   // the run began in this chunk: its table row is already here
#pragma unroll
                        for (int it = 0; it < ITERS; ++it) st4(&s_x[grp][(lig + it * LPR) * 4], xcur.v[it]);
                        if (lig == 0) s_col_last[grp] = colcur;
                    }
                }
            }
            ++nflush;
        };

        for (int j0 = 0; j0 < n; j0 += UNROLL) {
            Acc<ITERS> v[VROWS];
            Acc<ITERS> xr[FUSED ? UNROLL : 1];
            int32_t mu[UNROLL], cu[UNROLL];
            uint8_t sb[UNROLL][ITERS];
            float cf[UNROLL];
            // every lane learns the batch's entries first (shuffles back to back, one wait), then all row
            // loads go out unconditionally: entries past the end of the chunk carry meta 0, i.e. row 0
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) mu[u] = __shfl(meta, (j0 + u) & (LPR - 1), LPR);
            if constexpr (FUSED) {
#pragma unroll
                for (int u = 0; u < UNROLL; ++u) cu[u] = __shfl(colv, (j0 + u) & (LPR - 1), LPR);
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const uint32_t row = (uint32_t)mu[u] >> 2;
                if constexpr (FUSED) {   // a run begins here: its table row comes along with its first source row
                    if (mu[u] & 2) {   // (a row of a table beyond the caches is read once here and rewritten: past them)
                        if (fu.stream) load_row_stream<LPR, ITERS>(fused_row(fu, cu[u], ld_tab), d4, lig, xr[u]);
                        else load_row<LPR, ITERS>(fused_row(fu, cu[u], ld_tab), d4, lig, xr[u]);
                    }
                }
                if constexpr (PACKED) {
                    // (records of 1 << pk_sh bytes: a shift and an add give the address)
                    const uint8_t *pb = pk_lane + ((uint64_t)row << pk_sh);
#pragma unroll
                    for (int it = 0; it < ITERS; ++it) {
                        const int j = lig + it * LPR;
                        sb[u][it] = j < d4 ? pb[it * LPR] : (uint8_t)0;
                    }
                    cf[u] = src_b[row];
                } else {   // entries before `split` read src_a, the rest src_b (entity vs relation columns)
                    // (tail_off: where the rows that tail entries read sit, relative to the head entries' rows)
                    load_row<LPR, ITERS>((ec0 + j0 + u < split ? src_a : src_b) + (uint64_t)row * (uint32_t)ld_src + ((mu[u] & 1) ? tail_off : 0),
                                         d4, lig, v[u]);
                }
            }
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                const int jj = j0 + u;
                if (jj < n) {
                    if (mu[u] & 2) {
                        if (jj > 0) {
                            flush(false);
                            ++cur_seg;
                            acc.zero();
                        }
                        if constexpr (FUSED) { xcur = xr[u]; colcur = cu[u]; }
                    }
                    if constexpr (PACKED) {
                        // the dense row the forward pass would have stored is +c, -c or 0 per element, and a tail
                        // entry subtracts it: one fused multiply-add per element with the element's sign
                        const float c = (mu[u] & 1) ? -cf[u] : cf[u];
#pragma unroll
                        for (int it = 0; it < ITERS; ++it) {
                            const unsigned b = sb[u][it];   // (shift up, arithmetic shift down: sign-extends two bits)
                            acc.v[it].x = __builtin_fmaf(c, (float)((int)(b << 30) >> 30), acc.v[it].x);
                            acc.v[it].y = __builtin_fmaf(c, (float)((int)(b << 28) >> 30), acc.v[it].y);
                            acc.v[it].z = __builtin_fmaf(c, (float)((int)(b << 26) >> 30), acc.v[it].z);
                            acc.v[it].w = __builtin_fmaf(c, (float)((int)(b << 24) >> 30), acc.v[it].w);
                        }
                    } else {
                        Acc<ITERS> &vu = v[u];
                        if (mu[u] & 1) {
#pragma unroll
                            for (int it = 0; it < ITERS; ++it) {
                                acc.v[it].x -= vu.v[it].x; acc.v[it].y -= vu.v[it].y;
                                acc.v[it].z -= vu.v[it].z; acc.v[it].w -= vu.v[it].w;
                            }
                        } else {
                            acc.add(vu);
                        }
                    }
                }
            }
        }
        flush(true);
    }
    if (lig == 0) { s_info[grp] = info; s_fin_src[grp] = -1; }
    __syncthreads();

    // Stitch the chunk-crossing runs in chunk order (group 0 only; lanes keep their float4 slices).
    if (grp == 0) {
        bool have = false, started_in = false;
        int32_t cur_seg = 0;
        int cur_src = 0;                                   // chunk in which the current run began
        Acc<ITERS> cur;
        cur.zero();
        float *my_part = partials + (int64_t)block * 2 * ld_out;
        for (int g = 0; g < GROUPS; ++g) {
            const int inf = s_info[g];
            if (inf & HAS_FIRST) {
                Acc<ITERS> p;
#pragma unroll
                for (int it = 0; it < ITERS; ++it) p.v[it] = ld4(&s_part[g][0][(lig + it * LPR) * 4]);
                if (!have) {
                    have = true; started_in = false; cur = p; cur_seg = s_seg_first[g];
                } else {
                    cur.add(p);
                }
                if (!(inf & FIRST_CONT)) {   // the run ends inside chunk g
                    if (!started_in) {
                        store_row<LPR, ITERS>(my_part, d4, lig, cur);   // began in an earlier workgroup
                    } else if constexpr (FUSED) {   // left in chunk g's consumed slot; group g applies it below
#pragma unroll
                        for (int it = 0; it < ITERS; ++it) st4(&s_part[g][0][(lig + it * LPR) * 4], cur.v[it]);
                        if (lig == 0) s_fin_src[g] = cur_src;
                    } else {
                        store_row<LPR, ITERS>(out_rows + (int64_t)cur_seg * ld_out, d4, lig, cur);
                    }
                    have = false;
                }
            }
            if (inf & HAS_LAST) {
                have = true; started_in = true; cur_seg = s_seg_last[g]; cur_src = g;
#pragma unroll
                for (int it = 0; it < ITERS; ++it) cur.v[it] = ld4(&s_part[g][1][(lig + it * LPR) * 4]);
            }
        }
        if (have) store_row<LPR, ITERS>(my_part + (started_in ? ld_out : 0), d4, lig, cur);   // runs on into the next tile
    }
    if constexpr (FUSED) {   // the stitched runs that closed inside the tile: one per group at most, applied in parallel
        __syncthreads();
        const int src = s_fin_src[grp];
        if (src >= 0) {
            Acc<ITERS> x, g;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                x.v[it] = ld4(&s_x[src][(lig + it * LPR) * 4]);
                g.v[it] = ld4(&s_part[grp][0][(lig + it * LPR) * 4]);
            }
            apply_update<LPR, ITERS>(fused_row(fu, s_col_last[src], ld_tab), d4, lig, x, g, fu.lr, fu.mode, fu.stream);
        }
    }
}

// RIDE: 1 the first scatter pass of the next batch's sort comes along, 2 its histogram pass of the second digit,
// 3 as 2, and the sums of TransR's partial dL/dM_r matrices come along, 4 the first kernel of the next batch's
// build when that sort is a large one (nothing after this launch reads the A arrays it overwrites).
template <int LPR, int ITERS, int CHUNK, bool FUSED, int RIDE>
__global__ __launch_bounds__(kThreads) void k_seg_fixup(const int32_t *__restrict__ packed,
                                                        const int32_t *__restrict__ seg_id,
                                                        const int32_t *__restrict__ seg_ptr, int32_t e_begin,
                                                        int32_t e_end, int d4, float *__restrict__ out_rows,
                                                        int ld_out, const float *__restrict__ partials, FusedArgs fu,
                                                        SegSecond sec, ScatterAhead sa, HistAhead ha, DmRide dm,
                                                        EmitAhead ea)
{
    int block = (int)blockIdx.x;
    if constexpr (RIDE == 4) {
        if (block < ea.ntiles) {      // uniform in the workgroup
            emit_body<kBigSortItems, false, true, false>(block, ea.ntiles, ea.args);
            return;
        }
        block -= ea.ntiles;
    }
    if constexpr (RIDE == 3) {
        if (block < dm.blocks) {      // uniform in the workgroup
            const int slices = (dm.args.k * dm.args.d + kDmFixupSlice - 1) / kDmFixupSlice;
            transr_dm_fixup_body(block / slices, block % slices, dm.args);
            return;
        }
        block -= dm.blocks;
    }
    if constexpr (RIDE == 1) {
        if (block < sa.ntiles) {      // uniform in the workgroup
            scatter_body<true, false, kSortItems>(block, sa.args);
            return;
        }
        block -= sa.ntiles;
    }
    if constexpr (RIDE == 2 || RIDE == 3) {
        if (block < ha.ntiles) {
            hist_body<kSortItems>(block, ha.args.keys, ha.args.nnz, ha.args.shift, ha.args.radix, ha.args.table);
            return;
        }
        block -= ha.ntiles;
    }
    // The tiles are taken from the last one down: the relation columns sort last and own the longest runs (one
    // relation has a fifth of a batch's rows), whose closing workgroups add up the most partial rows; started
    // last, after the other workgroups have come and gone, their chains would set the time of the launch.
    block = ((int)gridDim.x - (RIDE == 1 ? sa.ntiles : RIDE == 2 ? ha.ntiles : RIDE == 3 ? ha.ntiles + dm.blocks
                               : RIDE == 4 ? ea.ntiles : 0)) - 1 - block;
    if (block >= sec.first_block) {   // uniform in the workgroup
        block -= sec.first_block;
        e_begin = sec.e_begin; e_end = sec.e_end;
        out_rows = sec.out_rows; partials = sec.partials;
        fu.table_b = sec.fused_table; fu.mode = sec.fused_mode;
    }
    const int ld_tab = d4 * 4;
    if (gridDim.y > 1) {                                   // column slices, as in k_seg_reduce
        const int c4 = (int)blockIdx.y * LPR;
        d4 = min(LPR, d4 - c4);
        if (out_rows) out_rows += 4 * c4;
        partials += 4 * c4;
        if (fu.table) fu.table += 4 * c4;
        if (fu.table_b) fu.table_b += 4 * c4;
    }
    constexpr int GROUPS = kThreads / LPR;
    constexpr int ROWF = ITERS * LPR * 4;
    constexpr int TILE = GROUPS * CHUNK;
    static_assert(TILE <= kThreads, "one thread per entry of the tile in the head search");
    __shared__ float s_sum[GROUPS][ROWF];
    const int32_t j = block;
    if (j == 0) return;                                         // tile 0 never ends a crossing run
    const int32_t tile0 = e_begin + j * TILE;
    if (tile0 >= e_end) return;
    const int32_t tile1 = min(tile0 + TILE, e_end);
    const int32_t e = tile0 + (int32_t)threadIdx.x;
    // everything the decision needs is fetched in one round trip
    const int32_t m_first = packed[tile0];
    const int32_t m_mine = (e > tile0 && e < tile1) ? packed[e] : 0;
    const int32_t m_next = tile1 < e_end ? packed[tile1] : 2;
    const int32_t seg = seg_id[tile0];
    if (m_first & 2) return;                                    // the tile starts a new segment: nothing crosses in
    const int any_head = __syncthreads_or((m_mine >> 1) & 1);
    const bool closes = any_head || (m_next & 2);
    if (!closes) return;                                        // the run goes on; a later tile finishes it

    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int32_t col = FUSED ? fu.touched_cols[seg] : 0;
    const int32_t j0 = (seg_ptr[seg] - e_begin) / TILE;         // tile in which the run began
    const int n = j - j0 + 1;                                   // partial rows: (j0, slot 1), (j0+1 .. j, slot 0)
    Acc<ITERS> xrow;                                            // FUSED: the table row, fetched beside the partial rows
    xrow.zero();
    if (FUSED && grp == 0) {
        if (fu.stream) load_row_stream<LPR, ITERS>(fused_row(fu, col, ld_tab), d4, lig, xrow);
        else load_row<LPR, ITERS>(fused_row(fu, col, ld_tab), d4, lig, xrow);
    }
    const int per = (n + GROUPS - 1) / GROUPS;
    const int lo = min(grp * per, n), hi = min(lo + per, n);
    Acc<ITERS> acc;
    acc.zero();
    constexpr int FU = ITERS == 1 ? 8 : 2;
    int q = lo;
    for (; q + FU <= hi; q += FU) {   // FU partial rows in flight, added in tile order
        Acc<ITERS> v[FU];
#pragma unroll
        for (int u = 0; u < FU; ++u)
            load_row<LPR, ITERS>(partials + ((int64_t)(j0 + q + u) * 2 + (q + u == 0 ? 1 : 0)) * ld_out, d4, lig, v[u]);
#pragma unroll
        for (int u = 0; u < FU; ++u) acc.add(v[u]);
    }
    for (; q < hi; ++q) {
        Acc<ITERS> v;
        load_row<LPR, ITERS>(partials + ((int64_t)(j0 + q) * 2 + (q == 0 ? 1 : 0)) * ld_out, d4, lig, v);
        acc.add(v);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) st4(&s_sum[grp][(lig + it * LPR) * 4], acc.v[it]);
    __syncthreads();
    if (grp == 0) {
        const int used = (n + per - 1) / per;                   // groups that had at least one row
        for (int g = 1; g < used; ++g) {
            Acc<ITERS> v;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) v.v[it] = ld4(&s_sum[g][(lig + it * LPR) * 4]);
            acc.add(v);
        }
        if constexpr (FUSED) apply_update<LPR, ITERS>(fused_row(fu, col, ld_tab), d4, lig, xrow, acc, fu.lr, fu.mode, fu.stream);
        else store_row<LPR, ITERS>(out_rows + (int64_t)seg * ld_out, d4, lig, acc);
    }
}

// Row update for every segment s (column c = touched_cols[s]):
//   c <  n_split : table_a row c            -= lr * grad_rows[s]   (width 4*d4_a, mode_a)
//   c >= n_split : table_b row c - n_split  -= lr * grad_rows[s]   (width 4*d4_b, mode 0), if table_b
//                  table_w row c - n_split  -= lr * w_rows[s]      (width 4*d4_a, mode_w), if table_w
// Each product and each difference is rounded once.  mode 1: then keep the fractional part (TorusE,
// Sec. 4.6).  mode 2: then rescale the row to unit length (TransH normals).
template <int LPR, int ITERS>
__device__ inline void sgd_row(float *__restrict__ row, const float *__restrict__ grad, int d4, int lig, float lr,
                               int mode)
{
    Acc<ITERS> x, g;
    load_row<LPR, ITERS>(row, d4, lig, x);
    load_row<LPR, ITERS>(grad, d4, lig, g);
    float ss = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        float *xv = &x.v[it].x;
        const float *gv = &g.v[it].x;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            float step = lr * gv[q];
            float nv = xv[q] - step;
            if (mode == 1) {
                nv = nv - floorf(nv);
                if (nv >= 1.0f) nv = 0.0f;
            }
            xv[q] = nv;
            ss += nv * nv;
        }
    }
    if (mode == 2) {
        ss = group_sum<LPR>(ss);
        if (ss > 0.f) {
            const float inv = 1.0f / sqrtf(ss);
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                x.v[it].x *= inv; x.v[it].y *= inv; x.v[it].z *= inv; x.v[it].w *= inv;
            }
        }
    }
    store_row<LPR, ITERS>(row, d4, lig, x);
}

template <int LPR, int ITERS>
__global__ __launch_bounds__(kThreads) void k_sgd_rows(const int32_t *__restrict__ touched_cols,
                                                       const int32_t *__restrict__ n_touched,
                                                       float *__restrict__ table_a, int d4_a, int mode_a,
                                                       int32_t n_split, float *__restrict__ table_b, int d4_b,
                                                       float *__restrict__ table_w, int mode_w,
                                                       const float *__restrict__ grad_rows,
                                                       const float *__restrict__ w_rows, int ld, float lr, int stream)
{
    constexpr int GROUPS = kThreads / LPR;
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int32_t U = n_touched[0];
    if (!table_b && !table_w) {
        // One table (TransE / TorusE): a group takes four consecutive segments per turn so that the four
        // column ids, then the eight rows (table + gradient), are in flight together.
        constexpr int UB = ITERS <= 2 ? 4 : 2;
        for (int64_t s0 = ((int64_t)blockIdx.x * GROUPS + grp) * UB; s0 < U; s0 += (int64_t)gridDim.x * GROUPS * UB) {
            int32_t col[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) col[u] = touched_cols[min(s0 + u, (int64_t)U - 1)];
            Acc<ITERS> x[UB], g[UB];
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                if (stream) load_row_stream<LPR, ITERS>(table_a + (int64_t)col[u] * d4_a * 4, d4_a, lig, x[u]);
                else load_row<LPR, ITERS>(table_a + (int64_t)col[u] * d4_a * 4, d4_a, lig, x[u]);
                const float *pg = grad_rows + min(s0 + u, (int64_t)U - 1) * ld;
#pragma unroll
                for (int it = 0; it < ITERS; ++it) {
                    const int j = lig + it * LPR;
                    g[u].v[it] = j < d4_a ? ld4_stream(pg + 4 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
                }
            }
#pragma unroll
            for (int u = 0; u < UB; ++u) {
                if (s0 + u < U && col[u] < n_split) {
#pragma unroll
                    for (int it = 0; it < ITERS; ++it) {
                        float *xv = &x[u].v[it].x;
                        const float *gv = &g[u].v[it].x;
#pragma unroll
                        for (int q = 0; q < 4; ++q) {
                            float step = lr * gv[q];
                            float nv = xv[q] - step;
                            if (mode_a == 1) {
                                nv = nv - floorf(nv);
                                if (nv >= 1.0f) nv = 0.0f;
                            }
                            xv[q] = nv;
                        }
                    }
                    float *pr = table_a + (int64_t)col[u] * d4_a * 4;
#pragma unroll
                    for (int it = 0; it < ITERS; ++it) {
                        const int j = lig + it * LPR;
                        if (j < d4_a) {
                            if (stream) st4_stream(pr + 4 * j, x[u].v[it]);
                            else st4(pr + 4 * j, x[u].v[it]);
                        }
                    }
                }
            }
        }
        return;
    }
    for (int64_t s = (int64_t)blockIdx.x * GROUPS + grp; s < U; s += (int64_t)gridDim.x * GROUPS) {
        const int32_t col = touched_cols[s];
        if (col < n_split) {
            sgd_row<LPR, ITERS>(table_a + (int64_t)col * d4_a * 4, grad_rows + s * ld, d4_a, lig, lr, mode_a);
        } else {
            const int64_t r = col - n_split;
            if (table_b) sgd_row<LPR, ITERS>(table_b + r * d4_b * 4, grad_rows + s * ld, d4_b, lig, lr, 0);
            if (table_w) sgd_row<LPR, ITERS>(table_w + r * d4_a * 4, w_rows + s * ld, d4_a, lig, lr, mode_w);
        }
    }
}

// ---- dispatch --------------------------------------------------------------------------------------
template <int LPR, int ITERS>
static void seg_go(stx_ctx *c, const stx_incidence *inc, int32_t e_begin, int32_t e_end, const float *src_a,
                   const float *src_b, int32_t split, int ld_src, int width, float *out_rows, int ld_out,
                   bool packed_src, const FusedArgs *fused, const SegSecondHost *second, int tail_off)
{
    // Entries per lane group: short chunks shorten every group's serial walk when the whole product is
    // small (latency bound); long ones mean fewer partial rows when it is large (bandwidth bound).
    constexpr int CH_LONG = LPR == 64 ? 64 : (LPR < 32 ? LPR : 32), CH_SHORT = LPR < 16 ? LPR : 16;
    constexpr int GROUPS = kThreads / LPR;
    const bool small = (e_end - e_begin) <= (1 << 20);
    const int tile = GROUPS * (small ? CH_SHORT : CH_LONG);
    const int ntiles1 = (e_end - e_begin + tile - 1) / tile;
    SegSecond sec{0x7fffffff, 0, 0, nullptr, nullptr, nullptr, nullptr, 0};
    int ntiles = ntiles1;
    if (second && second->e_end > second->e_begin) {
        sec = SegSecond{ntiles1, second->e_begin, second->e_end, second->src, second->out_rows,
                        c->partials + (int64_t)ntiles1 * 2 * ld_out, second->fused_table, second->fused_mode};
        ntiles += (second->e_end - second->e_begin + tile - 1) / tile;
    }
    const FusedArgs fu = fused ? *fused : FusedArgs{nullptr, nullptr, 0, nullptr, nullptr, 0.f, 0, 0};
    // The last kernel of this batch's build, when it was left waiting (stx_train_step), runs in the launch of a
    // fused product of one float4 per lane, and so does the sum of the loss; a product that cannot take them runs
    // after them.  The stages of the next batch's build that are due ride too, one per launch.
    const bool raw_now = fused && ITERS == 1 && c->segw.armed && c->sorted_inc == inc;
    if (c->segw.armed && !raw_now) launch_seg_write_late(c);
    const SegWriteRide no_segw{};
    const SegWriteRide segw = raw_now ? SegWriteRide{c->segw.args, c->segw.ntiles, c->segw.use_map ? 1 : 0,
                                                     c->loss_partials, c->fin_n, c->fin_scale, c->fin_loss}
                                      : no_segw;
    const int segw_blocks = segw.ntiles + (segw.fin_n > 0 ? 1 : 0);
    if (raw_now) { c->segw.armed = false; c->fin_n = 0; }
    EmitAhead r_emit{};
    ScatterAhead r_scat{}, f_scat{};
    HistAhead f_hist{};
    if (raw_now) {
        // (the scatter pass writes one of the sort's buffers: not in this launch if that is the one this product
        // reads, as after a sort of one or three passes; the fix-up launch reads neither)
        if (!c->ahead.scatter_ok || c->ahead.sargs.keys_out != segw.args.keys) r_scat = take_scatter_ahead(c);
        if (r_scat.ntiles == 0) r_emit = take_emit_ahead(c);
        if (ntiles > 1) {   // a fix-up launch follows
            f_hist = take_hist_ahead(c);
            if (f_hist.ntiles == 0) f_scat = take_scatter_ahead(c);
        }
    }
    // TransR's dL/dM_r product, left by the backward pass: along with the launch that also takes the scatter pass
    // (the steady state of stx_train_step), its sums along with the fix-up launch; ahead of any other launch.
    DmRide r_dm{}, f_dm{};
    bool dm_fixup_after = false;
    if (c->dm_ride.armed) {
        if (raw_now && r_scat.ntiles && !packed_src && LPR <= 32) {
            c->dm_ride.armed = false;
            r_dm = DmRide{c->dm_ride.args, c->dm_ride.items};
            if (c->dm_ride.fixup) {
                const DmArgs &da = c->dm_ride.args;
                if (ntiles > 1 && f_hist.ntiles)
                    f_dm = DmRide{da, da.n_fix * ((da.k * da.d + kDmFixupSlice - 1) / kDmFixupSlice)};
                else
                    dm_fixup_after = true;
            }
        } else {
            launch_transr_dm_late(c);
        }
    }
    // the first kernel of a large next build: in the fix-up launch, the last one of the step
    EmitAhead f_emit{};
    if (fused && ITERS == 1 && ntiles > 1 && c->ahead.armed && c->ahead.late_only) f_emit = take_emit_ahead(c, true);
    const int r_blocks = r_emit.ntiles + r_scat.ntiles + r_dm.blocks,
              f_blocks = f_scat.ntiles + f_hist.ntiles + f_dm.blocks + f_emit.ntiles;
    // Wide rows (more than one float4 per lane) run as column slices of the one-float4 kernels: more rows in
    // flight per lane and ITERS times the workgroups.  The unit-length rescale needs whole rows.
    const bool whole_rows = fused && (fu.mode == 2 || sec.fused_mode == 2);
    if (ITERS > 1 && !whole_rows) {
        const dim3 grid((unsigned)ntiles, (unsigned)ITERS);
#define STX_SLICED(P, CH, F)                                                                                    \
    do {                                                                                                        \
        {                                                                                                       \
            ProfScope prof(c, "k_seg_reduce");                                                                  \
            hipLaunchKernelGGL((k_seg_reduce<LPR, 1, P, CH, F, 0>), grid, dim3(kThreads), 0, c->stream,         \
                               inc->at_packed, inc->at_seg_id, e_begin, e_end, src_a, src_b, split, ld_src,     \
                               tail_off, width / 4, out_rows, ld_out, c->partials, fu, sec, no_segw, r_emit,    \
                               r_scat, r_dm);                                                                   \
        }                                                                                                       \
        if (ntiles > 1) {                                                                                       \
            ProfScope prof(c, "k_seg_fixup");                                                                   \
            hipLaunchKernelGGL((k_seg_fixup<LPR, 1, CH, F, 0>), grid, dim3(kThreads), 0, c->stream,             \
                               inc->at_packed, inc->at_seg_id, inc->at_seg_ptr, e_begin, e_end, width / 4,      \
                               out_rows, ld_out, c->partials, fu, sec, f_scat, f_hist, f_dm, f_emit);           \
        }                                                                                                       \
    } while (0)
#define STX_SLICED2(P, CH) do { if (fused) STX_SLICED(P, CH, true); else STX_SLICED(P, CH, false); } while (0)
        if (packed_src) { if (small) STX_SLICED2(true, CH_SHORT); else STX_SLICED2(true, CH_LONG); }
        else            { if (small) STX_SLICED2(false, CH_SHORT); else STX_SLICED2(false, CH_LONG); }
#undef STX_SLICED2
#undef STX_SLICED
        return;
    }
#define STX_SEG_R(P, CH, F, R)                                                                                  \
    hipLaunchKernelGGL((k_seg_reduce<LPR, ITERS, P, CH, F, (F && ITERS == 1 && !(R == 5 && (P || LPR > 32))) ? R : 0>), \
                       dim3(ntiles + segw_blocks + r_blocks), dim3(kThreads), 0, c->stream, segw.args.pay,      \
                       segw.args.keys, e_begin, e_end, src_a, src_b, split, ld_src, tail_off, width / 4,        \
                       out_rows, ld_out, c->partials, fu, sec, segw, r_emit, r_scat, r_dm)
#define STX_SEG_F(CH, F, R)                                                                                     \
    hipLaunchKernelGGL((k_seg_fixup<LPR, ITERS, CH, F, (F && ITERS == 1 && !(R == 3 && LPR > 32)) ? R : 0>), dim3(ntiles + f_blocks), \
                       dim3(kThreads), 0, c->stream, inc->at_packed, inc->at_seg_id, inc->at_seg_ptr, e_begin,  \
                       e_end, width / 4, out_rows, ld_out, c->partials, fu, sec, f_scat, f_hist, f_dm, f_emit)
#define STX_SEG(P, CH, F)                                                                                       \
    do {                                                                                                        \
        {                                                                                                       \
            ProfScope prof(c, "k_seg_reduce");                                                                  \
            if (F && ITERS == 1 && raw_now && r_scat.ntiles && r_dm.blocks) STX_SEG_R(P, CH, F, 5);             \
            else if (F && ITERS == 1 && raw_now && r_scat.ntiles) STX_SEG_R(P, CH, F, 3);                       \
            else if (F && ITERS == 1 && raw_now && r_emit.ntiles && r_emit.args.rc.cur) STX_SEG_R(P, CH, F, 4); \
            else if (F && ITERS == 1 && raw_now && r_emit.ntiles) STX_SEG_R(P, CH, F, 2);                       \
            else if (F && ITERS == 1 && raw_now) STX_SEG_R(P, CH, F, 1);                                        \
            else                                                                                                \
                hipLaunchKernelGGL((k_seg_reduce<LPR, ITERS, P, CH, F, 0>), dim3(ntiles), dim3(kThreads), 0,    \
                                   c->stream, inc->at_packed, inc->at_seg_id, e_begin, e_end, src_a, src_b,     \
                                   split, ld_src, tail_off, width / 4, out_rows, ld_out, c->partials, fu, sec,  \
                                   no_segw, r_emit, r_scat, r_dm);                                              \
        }                                                                                                       \
        if (ntiles > 1) {                                                                                       \
            ProfScope prof(c, "k_seg_fixup");                                                                   \
            if (F && ITERS == 1 && f_hist.ntiles && f_dm.blocks) STX_SEG_F(CH, F, 3);                           \
            else if (F && ITERS == 1 && f_hist.ntiles) STX_SEG_F(CH, F, 2);                                     \
            else if (F && ITERS == 1 && f_scat.ntiles) STX_SEG_F(CH, F, 1);                                     \
            else if (F && ITERS == 1 && f_emit.ntiles) STX_SEG_F(CH, F, 4);                                     \
            else STX_SEG_F(CH, F, 0);                                                                           \
        }                                                                                                       \
    } while (0)
#define STX_SEG2(P, CH) do { if (fused) STX_SEG(P, CH, true); else STX_SEG(P, CH, false); } while (0)
    if (packed_src) { if (small) STX_SEG2(true, CH_SHORT); else STX_SEG2(true, CH_LONG); }
    else            { if (small) STX_SEG2(false, CH_SHORT); else STX_SEG2(false, CH_LONG); }
    if (dm_fixup_after) launch_transr_dm_fixup_late(c);
#undef STX_SEG2
#undef STX_SEG
#undef STX_SEG_F
#undef STX_SEG_R
}

template <int LPR, int ITERS>
static void sgd_go(stx_ctx *c, const stx_incidence *inc, const SgdTables &T, const float *grad_rows,
                   const float *w_rows, float lr)
{
    constexpr int GROUPS = kThreads / LPR;
    int64_t cap = inc->nnz < c->cfg.n_ent + c->cfg.n_rel ? inc->nnz : c->cfg.n_ent + c->cfg.n_rel;
    int64_t blocks = (cap + GROUPS - 1) / GROUPS;
    if (!T.table_b && !T.table_w) blocks = (blocks + 3) / 4;   // that path takes four segments per group and turn
    if (blocks > 8192) blocks = 8192;   // grid-stride beyond this (measured faster than one segment per group)
    if (blocks < 1) blocks = 1;
    ProfScope prof(c, "k_sgd_rows");
    hipLaunchKernelGGL((k_sgd_rows<LPR, ITERS>), dim3((unsigned)blocks), dim3(kThreads), 0, c->stream,
                       inc->at_touched_cols, inc->n_touched, T.table_a, T.width_a / 4, T.mode_a, (int32_t)T.n_split,
                       T.table_b, T.width_b / 4, T.table_w, T.mode_w, grad_rows, w_rows, c->ld, lr, big_tables(c));
}

stx_status launch_seg_reduce(stx_ctx *c, const stx_incidence *inc, int64_t e_begin, int64_t e_end,
                             const float *src_a, const float *src_b, int64_t split, int ld_src, int width,
                             float *out_rows, int ld_out, bool packed_src, const SegFusedHost *fh,
                             const SegSecondHost *second, int tail_off)
{
    if (e_end <= e_begin) return STX_OK;
    Launch L = row_launch(width);
    // the sorted keys of the last build on this context are the columns of the sorted entries
    FusedArgs fu{nullptr, nullptr, 0, inc->at_touched_cols, c->sorted_inc == inc ? c->sorted_keys : nullptr, 0.f, 0,
                 big_tables(c)};
    if (fh) { fu.table = fh->table; fu.table_b = fh->table_b; fu.n_split = fh->n_split; fu.lr = fh->lr; fu.mode = fh->mode; }
    const FusedArgs *fused = fh ? &fu : nullptr;
    STX_DISPATCH_ROW(L, seg_go, c, inc, (int32_t)e_begin, (int32_t)e_end, src_a, src_b, (int32_t)split, ld_src, width,
                     out_rows, ld_out, packed_src, fused, second, packed_src ? 0 : tail_off);
    return hip_ok(hipGetLastError());
}

stx_status launch_sgd_rows(stx_ctx *c, const stx_incidence *inc, const SgdTables &T, const float *grad_rows,
                           const float *w_rows, float lr)
{
    if (inc->n_rows == 0) return STX_OK;
    Launch L = row_launch(T.width_a > T.width_b ? T.width_a : T.width_b);
    STX_DISPATCH_ROW(L, sgd_go, c, inc, T, grad_rows, w_rows, lr);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
