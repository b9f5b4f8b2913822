// TransR: the per-relation projection products on the matrix cores.
//
// SparseTransX Sec. 4.4 rearranges M_r h + r - M_r t into M_r (h - t) + r, so the `ht` incidence
// product (Sec. 4.2.1) feeds one projection per row.  Rows with the same relation share M_r, and the
// relation columns of the sorted A^T (stx_build.hip) already list every relation's rows contiguously,
// so the projections are dense products over runs of that list:
//
//   forward   Y_g  = X_g . M_r^T + r        (n_g x d)(d x k)      k_transr_rows<false>
//   backward  GX_g = GY_g . M_r             (n_g x k)(k x d)      k_transr_rows<true>
//             dM_r = GY_g^T . X_g           (k x n_g)(n_g x d)    k_transr_dm (+ k_transr_dm_fixup); bodies in stx_transr_dm_body.h
//
// Operands are bfloat16 (round to nearest even), products accumulate in fp32 in
// v_mfma_f32_32x32x16_bf16; x = h - t is formed in fp32 first.
//
// Work items.  Group sizes are power-law distributed, so the list of every relation is cut into
// items of at most 64 entries (the two row products) and 256 entries (the dM product); an item never
// spans two relations, so a workgroup loads one M_r and runs dense tiles.  k_transr_prepare builds
// the item lists (and the list of relations whose several dM items leave partial matrices to add up)
// with one scan over the relation segments, and the kernels are launched with the largest possible
// item count; workgroups past the real count leave at once.
//
// Operand order.  The 32x32x16 MFMA wants, from lane l of 64, row (l % 32) of its operand and the
// eight consecutive reduction elements 8*(l / 32) .. of that row, for A and B alike; accumulator
// register v holds row 8*(v / 4) + 4*(l / 32) + v % 4 of column l % 32.  Every bfloat16 operand that
// is read from global memory is therefore stored as a sequence of fragments of 32 rows x 16 reduction
// elements, fragment (reduction step ks, row tile rt) at ((ks * row_tiles + rt) * 64 + lane) * 8
// elements: a wavefront fetches one fragment as one contiguous kilobyte, 16 bytes per lane.  That
// holds for the two copies of M_r made by k_transr_prepare (rows = output columns of the forward
// product, reduction over d; rows = output columns of GX, reduction over k) and for the transposed
// tiles X^T and GY^T (rows = columns of x / gy, reduction over the 64 entries of an item) which the
// row kernels leave behind for the dM product while they have the tile in LDS anyway.
#include "stx_emit_body.h"
#include "stx_forward_body.h"
#include "stx_sort_body.h"
#include "stx_transr_dm_body.h"

namespace stx {

constexpr int kMaxNT = kMaxProjDim / 32 / 2;   // 32-column tiles per wavefront (two wavefronts share the columns)
constexpr int kLdsPad = 8;                      // halfwords added to every LDS row: 16-byte reads stay conflict-free

struct PrepArgs {
    const int32_t *touched_cols, *n_touched, *seg_ptr, *seg_id;
    int32_t n_ent, e_begin;
    const float *M;
    uint16_t *m16, *m16t;
    int4 *items, *dm_items, *fix_items;
    int32_t *counts;
    int d, k;
    // Rows per relation in the batch, counted while A was written (null: not available).  With them
    // neither the item lists nor the choice of the M_r to convert need the sorted A^T, so the whole
    // preparation can run beside the sort instead of after it.
    const int32_t *rel_cnt;
    int32_t n_rel;
    int nplan;                   // workgroups that build the item lists (the others convert one M_r each)
    int whole_lists;             // row items name their relation's whole list and their index in it (k_transr_fused)
};

// Item lists of the relation segments (one workgroup).  Row item: {relation, first sorted entry,
// entries (<= 64), 0}.  dM item: {relation, first row item, entries (<= 256), slot}; slot is -1 when the
// segment has a single dM item, which then writes dL/dM_r itself.  Fix-up item, one per segment with
// several dM items: {relation, first slot of the segment, its number of slots, 0}.
// Workgroup `block` of the planners handles relations (or touched segments) 256*block .. and first adds
// up what the lists before them need, so the planners do not wait for each other.
template <bool FROM_COUNTS>
__device__ inline void transr_plan(const int block, const PrepArgs &p)
{
    __shared__ int32_t s_o64[kThreads + 1], s_o256[kThreads + 1], s_op[kThreads], s_beg[kThreads], s_len[kThreads],
        s_rel[kThreads], s_wave[kThreads / 64][5];
    const int tid = threadIdx.x;
    // the relations' lists, in the order of the sorted A^T: by touched segment, or by relation id with the
    // counted rows (an absent relation has no rows and gets no item)
    const int32_t first = FROM_COUNTS ? 0 : p.seg_id[p.e_begin], last = FROM_COUNTS ? p.n_rel : p.n_touched[0];
    const int32_t sb = first + block * kThreads;
    if (sb >= last) return;
    int32_t base64 = 0, base256 = 0, basep = 0, base_len = 0, basef = 0;
    {   // items, slots, entries and fix-up items of the lists before this workgroup's
        int32_t pre[5] = {0, 0, 0, 0, 0};
        for (int32_t s = first + tid; s < sb; s += kThreads) {
            const int32_t len = FROM_COUNTS ? p.rel_cnt[s] : p.seg_ptr[s + 1] - p.seg_ptr[s];
            const int32_t n256 = (len + 255) >> 8;
            pre[0] += (len + 63) >> 6; pre[1] += n256; pre[2] += n256 > 1 ? n256 : 0; pre[3] += len; pre[4] += n256 > 1 ? 1 : 0;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) {
#pragma unroll
            for (int q = 0; q < 5; ++q) pre[q] += __shfl_xor(pre[q], off);
        }
        if ((tid & 63) == 0) {
#pragma unroll
            for (int q = 0; q < 5; ++q) s_wave[tid >> 6][q] = pre[q];
        }
        __syncthreads();
#pragma unroll
        for (int ww = 0; ww < kThreads / 64; ++ww) {
            base64 += s_wave[ww][0]; base256 += s_wave[ww][1]; basep += s_wave[ww][2]; base_len += s_wave[ww][3];
            basef += s_wave[ww][4];
        }
        __syncthreads();
    }
    {
        const int32_t s = sb + tid;
        int32_t beg = 0, len = 0, rel = 0;
        if (s < last) {
            if (FROM_COUNTS) {
                len = p.rel_cnt[s];
                rel = s;
            } else {
                beg = p.seg_ptr[s];
                len = p.seg_ptr[s + 1] - beg;
                rel = p.touched_cols[s] - p.n_ent;
            }
        }
        const int32_t n64 = (len + 63) >> 6, n256 = (len + 255) >> 8;
        // five exclusive scans across the workgroup at once: shuffles inside a wavefront, LDS across the four
        int32_t inc3[5] = {n64, n256, n256 > 1 ? n256 : 0, len, n256 > 1 ? 1 : 0};
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                const int32_t up = __shfl_up(inc3[q], off);
                if ((tid & 63) >= off) inc3[q] += up;
            }
        }
        if ((tid & 63) == 63) {
#pragma unroll
            for (int q = 0; q < 5; ++q) s_wave[tid >> 6][q] = inc3[q];
        }
        __syncthreads();
        int32_t before[5] = {0, 0, 0, 0, 0}, tot[5] = {0, 0, 0, 0, 0};
#pragma unroll
        for (int ww = 0; ww < kThreads / 64; ++ww) {
#pragma unroll
            for (int q = 0; q < 5; ++q) {
                if (ww < (tid >> 6)) before[q] += s_wave[ww][q];
                tot[q] += s_wave[ww][q];
            }
        }
        const int32_t o64 = before[0] + inc3[0] - n64, o256 = before[1] + inc3[1] - n256,
                      op = before[2] + inc3[2] - (n256 > 1 ? n256 : 0);
        const int32_t t64 = tot[0], t256 = tot[1], tp = tot[2];
        if (FROM_COUNTS) beg = p.e_begin + base_len + before[3] + inc3[3] - len;   // relation lists follow each other
        s_o64[tid] = o64; s_o256[tid] = o256; s_op[tid] = op;
        s_beg[tid] = beg; s_len[tid] = len; s_rel[tid] = rel;
        if (tid == 0) { s_o64[kThreads] = t64; s_o256[kThreads] = t256; }
        __syncthreads();
        for (int32_t w = tid; w < t64; w += kThreads) {
            int lo = 0, hi = kThreads;                     // last segment whose first item is <= w
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_o64[mid] <= w) lo = mid; else hi = mid;
            }
            const int32_t li = w - s_o64[lo];
            p.items[base64 + w] = p.whole_lists ? make_int4(s_rel[lo], s_beg[lo], s_len[lo], li)
                                                : make_int4(s_rel[lo], s_beg[lo] + 64 * li, min(64, s_len[lo] - 64 * li), 0);
        }
        for (int32_t w = tid; w < t256; w += kThreads) {
            int lo = 0, hi = kThreads;
            while (hi - lo > 1) {
                const int mid = (lo + hi) >> 1;
                if (s_o256[mid] <= w) lo = mid; else hi = mid;
            }
            const int32_t li = w - s_o256[lo], parts = (s_len[lo] + 255) >> 8, first = basep + s_op[lo];
            p.dm_items[base256 + w] = make_int4(s_rel[lo], base64 + s_o64[lo] + 4 * li,
                                                min(256, s_len[lo] - 256 * li), parts > 1 ? first + li : -1);
        }
        if (n256 > 1)   // this thread's segment has several dM items: its partial matrices are summed afterwards
            p.fix_items[basef + before[4] + inc3[4] - 1] = make_int4(rel, basep + op, n256, 0);
        // the planner of the last lists knows the totals
        if (sb + kThreads >= last && tid == 0) {
            p.counts[0] = base64 + t64; p.counts[1] = base256 + t256; p.counts[2] = basef + tot[4];
        }
        (void)tp;
    }
}

// The first nplan workgroups build the item lists; each of the others writes the two bfloat16 operand-order
// copies of kPrepRows rows of one M_r (k / kPrepRows workgroups per relation) if that relation occurs in the
// batch (known from the counted rows, else it looks its column up in the sorted touched list).
constexpr int kPrepRows = 32;
template <bool FROM_COUNTS>
__device__ inline void transr_prepare_body(const int block, const PrepArgs &p)
{
    if (block < p.nplan) { transr_plan<FROM_COUNTS>(block, p); return; }
    const int tid = threadIdx.x;
    const int nsplit = p.k / kPrepRows;
    const int32_t r = (block - p.nplan) / nsplit;
    const int a0 = ((block - p.nplan) - r * nsplit) * kPrepRows;
    if (FROM_COUNTS) {
        if (p.rel_cnt[r] == 0) return;
    } else {
        const int32_t target = p.n_ent + r;
        const int32_t n_seg = p.n_touched[0];
        int32_t lo = p.seg_id[p.e_begin], hi = n_seg;     // relation columns sort after all entity columns
        while (lo < hi) {                                 // first position with touched_cols[pos] >= target
            const int32_t mid = (lo + hi) >> 1;
            if (p.touched_cols[mid] < target) lo = mid + 1; else hi = mid;
        }
        if (lo >= n_seg || p.touched_cols[lo] != target) return;
    }
    // The rows go through LDS as bfloat16: the fp32 rows are read with whole-row float4 accesses, and both
    // operand-order copies are written 16 bytes per thread, contiguous across threads.
    __shared__ __attribute__((aligned(16))) uint16_t s_m[kPrepRows * (kMaxProjDim + kLdsPad)];
    const int64_t kd = (int64_t)p.k * p.d;
    const float *__restrict__ M = p.M + r * kd;
    uint16_t *__restrict__ fwd = p.m16 + r * kd;          // rows a, reduction over j
    uint16_t *__restrict__ gx = p.m16t + r * kd;          // rows j, reduction over a
    const int stride = p.d + kLdsPad, q4 = p.d >> 2;
    const int rt_f = p.k >> 5, rt_g = p.d >> 5, ks_d = p.d >> 4;
    {
        constexpr int rows = kPrepRows;
        for (int g0 = tid; g0 < rows * q4; g0 += 8 * kThreads) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int g = g0 + u * kThreads;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (g < rows * q4) { const int i = g / q4; v[u] = ld4(M + (int64_t)(a0 + i) * p.d + 4 * (g - i * q4)); }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int g = g0 + u * kThreads;
                if (g < rows * q4) {
                    const int i = g / q4, c4 = 4 * (g - i * q4);
                    *reinterpret_cast<uint2 *>(s_m + i * stride + c4) = make_uint2(pack2(v[u].x, v[u].y), pack2(v[u].z, v[u].w));
                }
            }
        }
        __syncthreads();
        {   // forward operand: the row tiles of these rows, every reduction step over j
            const int nt_n = rows >> 5, pieces = ks_d * nt_n * 64;
            for (int pc = tid; pc < pieces; pc += kThreads) {
                const int l = pc & 63, blk = pc >> 6, ks = blk / nt_n, ntl = blk - ks * nt_n;
                const uint4 o = *reinterpret_cast<const uint4 *>(s_m + (32 * ntl + (l & 31)) * stride + 16 * ks + 8 * (l >> 5));
                *reinterpret_cast<uint4 *>(fwd + ((int64_t)(ks * rt_f + (a0 >> 5) + ntl) * 64 + l) * 8) = o;
            }
        }
        {   // GX operand: every row tile over j, the reduction steps that these rows of M_r cover
            const int ks_n = rows >> 4, pieces = ks_n * rt_g * 64;
            for (int pc = tid; pc < pieces; pc += kThreads) {
                const int l = pc & 63, blk = pc >> 6, ksl = blk / rt_g, nt = blk - ksl * rt_g;
                const uint16_t *src = s_m + (16 * ksl + 8 * (l >> 5)) * stride + 32 * nt + (l & 31);
                uint4 o;
                o.x = (uint32_t)src[0] | (uint32_t)src[stride] << 16;
                o.y = (uint32_t)src[2 * stride] | (uint32_t)src[3 * stride] << 16;
                o.z = (uint32_t)src[4 * stride] | (uint32_t)src[5 * stride] << 16;
                o.w = (uint32_t)src[6 * stride] | (uint32_t)src[7 * stride] << 16;
                *reinterpret_cast<uint4 *>(gx + ((int64_t)(((a0 >> 4) + ksl) * rt_g + nt) * 64 + l) * 8) = o;
            }
        }
    }
}

template <bool FROM_COUNTS>
__global__ __launch_bounds__(kThreads) void k_transr_prepare(PrepArgs p)
{
    transr_prepare_body<FROM_COUNTS>((int)blockIdx.x, p);
}

// stx_train_step: with the rows per relation counted while A was written, the preparation depends on
// nothing the sort produces and shares the launch of its first scatter pass (whose workgroups come first).
// (FIRST false: a later pass, when the first one ran ahead of time in a launch of the previous step)
template <bool FIRST>
__global__ __launch_bounds__(kThreads) void k_prep_scatter(PrepArgs p, ScatterArgs sa)
{
    if ((int)blockIdx.x < sa.ntiles) scatter_body<FIRST, false, kSortItems>((int)blockIdx.x, sa);
    else transr_prepare_body<true>((int)blockIdx.x - sa.ntiles, p);
}

struct RowsArgs {
    const int4 *items;
    const int32_t *counts;       // [0] = number of row items
    const int32_t *colidx, *packed;
    const int32_t *pay;          // the sort's payloads (3*row + slot) in place of `packed`, or null
    const float *E, *Rv;
    const uint16_t *Mb;          // operand-order copies of M_r: n_out rows, reduction n_red
    uint16_t *tiles;             // per item: the 64-entry operand tile transposed, n_red rows in operand order
    int n_red, n_out;
    // a deferred final sum of the loss that the launch's last workgroup takes along (fin_n == 0: none)
    const float *fin_partials;
    int fin_n;
    float fin_scale;
    float *fin_loss;
};

// One workgroup per row item.  The item's operand rows are staged in LDS as bfloat16 (forward:
// x = E[h] - E[t]; GX: the rows of dL/dy), stored once more, transposed, for the dM product, and
// multiplied by M_r's fragments fetched straight from the operand-order copy.
// Wavefront w: rows 32*(w/2).., column tiles w%2, w%2+2, ..
// GX = false: Y[row]  = x . M_r^T + r_vec     (out width k, reduction over d)
// GX = true : GX[row] = gy . M_r              (out width d, reduction over k)
// SMALL (both widths <= 128): all of the wavefront's M_r fragments are requested before the operand rows
// are staged, so that their latency is hidden behind the gather instead of following it.
template <bool GX, bool SMALL>
__global__ __launch_bounds__(kThreads) void k_transr_rows(RowsArgs p, const float *__restrict__ gy,
                                                          float *__restrict__ out)
{
    __shared__ __attribute__((aligned(16))) uint16_t s_a[64 * (kMaxProjDim + kLdsPad)];
    __shared__ int32_t s_row[64], s_h[64], s_t[64];
    const int tid = threadIdx.x;
    if (p.fin_n > 0 && blockIdx.x == gridDim.x - 1) {     // the extra workgroup of the launch
        finish_loss_body(p.fin_partials, p.fin_n, p.fin_scale, p.fin_loss);
        return;
    }
    const int4 item = p.items[blockIdx.x];                // the list is allocated for the launch bound: any index is readable
    if ((int32_t)blockIdx.x >= p.counts[0]) return;
    const int rel = item.x, begin = item.y, count = item.z;
    const int l = tid & 63, w = tid >> 6, wr = w >> 1, wc = w & 1, l31 = l & 31, kg = l >> 5;
    const int ntl = p.n_out >> 5, ntw = (ntl - wc + 1) >> 1, KS = p.n_red >> 4;
    const uint16_t *Mb = p.Mb + (int64_t)rel * p.n_out * p.n_red;
    uint4 bpre[SMALL ? 8 : 1][SMALL ? 2 : 1];
    if (SMALL && 32 * wr < count) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (ks < KS && q < ntw) bpre[ks][q] = ld16(Mb + ((int64_t)(ks * ntl + wc + 2 * q) * 64 + l) * 8);
        }
    }
    if (tid < 64) {
        int32_t row = -1, hh = 0, tt = 0;
        if (tid < count) {
            row = p.pay ? p.pay[begin + tid] / 3 : p.packed[begin + tid] >> 2;
            if (!GX) { hh = p.colidx[3 * row]; tt = p.colidx[3 * row + 2]; }
        }
        s_row[tid] = row; s_h[tid] = hh; s_t[tid] = tt;
    }
    __syncthreads();

    // stage the tile: rows past `count` are zero
    const int stride = p.n_red + kLdsPad, q4 = p.n_red >> 2, total = 64 * q4;
    for (int g0 = tid; g0 < total; g0 += 8 * kThreads) {
        float4 v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int g = g0 + u * kThreads;
            v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
            if (g < total) {
                const int i = g / q4, c4 = 4 * (g - i * q4);
                if (i < count) {
                    if (GX) v[u] = ld4(gy + (int64_t)s_row[i] * p.n_red + c4);
                    else v[u] = sub4(ld4(p.E + (int64_t)s_h[i] * p.n_red + c4), ld4(p.E + (int64_t)s_t[i] * p.n_red + c4));
                }
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const int g = g0 + u * kThreads;
            if (g < total) {
                const int i = g / q4, c4 = 4 * (g - i * q4);
                *reinterpret_cast<uint2 *>(s_a + i * stride + c4) = make_uint2(pack2(v[u].x, v[u].y), pack2(v[u].z, v[u].w));
            }
        }
    }
    __syncthreads();

    {   // the transposed tile, in operand order, for the dM product (reduction steps past `count` are never read)
        const int rt = p.n_red >> 5, pieces = ((count + 15) >> 4) * rt * 64;
        uint16_t *tile = p.tiles + (int64_t)blockIdx.x * 64 * p.n_red;
        for (int pc = tid; pc < pieces; pc += kThreads) {
            const int l = pc & 63, blk = pc >> 6, ks = blk / rt, mt = blk - ks * rt;
            const uint16_t *s = s_a + (16 * ks + 8 * (l >> 5)) * stride + 32 * mt + (l & 31);
            uint4 o;
            o.x = (uint32_t)s[0] | (uint32_t)s[stride] << 16;
            o.y = (uint32_t)s[2 * stride] | (uint32_t)s[3 * stride] << 16;
            o.z = (uint32_t)s[4 * stride] | (uint32_t)s[5 * stride] << 16;
            o.w = (uint32_t)s[6 * stride] | (uint32_t)s[7 * stride] << 16;
            *reinterpret_cast<uint4 *>(tile + (int64_t)pc * 8) = o;
        }
    }

    if (32 * wr >= count) return;                          // no barrier below
    const uint16_t *arow = s_a + (32 * wr + l31) * stride + 8 * kg;
    floatx16 acc[kMaxNT];
#pragma unroll
    for (int q = 0; q < kMaxNT; ++q) acc[q] = zero16();
    if constexpr (SMALL) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks < KS) {
                const uint4 a = *reinterpret_cast<const uint4 *>(arow + 16 * ks);
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (q < ntw)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a), as_frag(bpre[ks][q]), acc[q], 0, 0, 0);
            }
        }
    } else
    for (int ks0 = 0; ks0 < KS; ks0 += 4) {
        uint4 a[4], b[4][kMaxNT];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (ks0 + u < KS) {
#pragma unroll
                for (int q = 0; q < kMaxNT; ++q)
                    if (q < ntw) b[u][q] = ld16(Mb + ((int64_t)((ks0 + u) * ntl + wc + 2 * q) * 64 + l) * 8);
                a[u] = *reinterpret_cast<const uint4 *>(arow + 16 * (ks0 + u));
            }
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            if (ks0 + u < KS) {
#pragma unroll
                for (int q = 0; q < kMaxNT; ++q)
                    if (q < ntw)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a[u]), as_frag(b[u][q]), acc[q], 0, 0, 0);
            }
        }
    }
#pragma unroll
    for (int q = 0; q < kMaxNT; ++q) {
        if (q < ntw) {
            const int n = (wc + 2 * q) * 32 + l31;
            const float add = GX ? 0.f : p.Rv[(int64_t)rel * p.n_out + n];
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int32_t row_m = s_row[32 * wr + 8 * (v >> 2) + 4 * kg + (v & 3)];
                if (row_m >= 0) out[(int64_t)row_m * p.n_out + n] = acc[q][v] + add;
            }
        }
    }
}

struct FusedArgs {
    const int4 *items;
    const int32_t *counts;       // [0] = number of row items
    const int32_t *colidx, *packed;
    const int32_t *pay;          // the sort's payloads (3*row + slot) in place of `packed`, or null
    const float *E, *Rv;
    const uint16_t *Mf, *Mg;     // operand-order copies of M_r: forward (rows a, reduction over j), GX (rows j, reduction over a)
    uint16_t *xt, *gyt;          // per item: the transposed 64-entry tiles of x and of dL/dy for the dM product
    float *gy, *gx;              // rows x k: dL/dy;  rows x d: dL/dx
    float *scores, *loss_partials;
    int d, k;
    int32_t kneg;                // negatives per positive; 1 + kneg divides 64
    float margin, scale;
};

// TransR, both widths <= 128 and 1 + kneg a divisor of 64: the whole of a row's way through the model in one
// kernel (Sec. 4.4 forward, the distance and hinge of Sec. 5.3, and the first backward product).  A work item is up
// to 64 / (1 + kneg) positives of one relation TOGETHER WITH their negatives, which keep the relation and
// therefore sit in the same list of the sorted A^T (positives first, in row order, then their negatives in the
// same order), so the hinge of every pair is decided inside the workgroup:
//   x = E[h] - E[t] staged as bfloat16, stored transposed for the dM product;  Y = X M_r^T + r on the matrix cores;
//   distances of the 64 rows of Y from LDS;  hinge, coefficients, scores, the item's share of the loss;
//   dL/dy to memory (dL/dr sums it per relation) and, as bfloat16, back into LDS and transposed to memory;
//   dL/dx = dL/dy M_r on the matrix cores, to memory for the transposed product over the entity columns.
// Tile slots: positives 0 .. P'-1, then negative kk of positive i at P' + i*kneg + kk.
// The first workgroups of the launch may run the first kernel of the next batch's build (ea.ntiles > 0), which
// overwrites the caller's A arrays: the launcher lets it ride only when p.colidx is the context's own copy of this
// batch's column ids.
template <int DIST>
__global__ __launch_bounds__(kThreads, 3) void k_transr_fused(FusedArgs p, EmitAhead ea)
{
    constexpr int kW = 128;
    __shared__ __attribute__((aligned(16))) uint16_t s_a[64 * (kW + kLdsPad)];
    __shared__ __attribute__((aligned(16))) float s_y[64 * (kW + 4)];
    __shared__ int32_t s_row[64], s_h[64], s_t[64];
    __shared__ float s_dist[64], s_cs[64];
    static_assert(sizeof(float) * 64 * (kW + 4) >= (size_t)emit_lds(true, true), "the rider's arrays fit the tile of y");
    const int tid = threadIdx.x;
    int block = (int)blockIdx.x;
    if (block < ea.ntiles) {
        emit_body<kSortItems, true, true, true, true>(block, ea.ntiles, ea.args, reinterpret_cast<unsigned char *>(s_y));
        return;
    }
    block -= ea.ntiles;
    const int4 item = p.items[block];                     // the list is allocated for the launch bound
    if (block >= p.counts[0]) {
        if (tid == 0) p.loss_partials[block] = 0.f;
        return;
    }
    const int rel = item.x, seg_begin = item.y, len = item.z, li = item.w;
    const int rpp = 1 + p.kneg, P = 64 / rpp, n_pos = len / rpp, p0 = li * P;
    const int Pn = min(P, n_pos - p0), count = Pn * rpp;
    const int l = tid & 63, w = tid >> 6, wr = w >> 1, wc = w & 1, l31 = l & 31, kg = l >> 5;
    const int d = p.d, k = p.k;
    // ---- forward fragments of M_r, requested before the gather so that their latency hides behind it
    const int ntl_f = k >> 5, ntw_f = (ntl_f - wc + 1) >> 1, KS_f = d >> 4;
    const uint16_t *Mf = p.Mf + (int64_t)rel * d * k;
    uint4 bpre[8][2];
    if (32 * wr < count) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (ks < KS_f && q < ntw_f) bpre[ks][q] = ld16(Mf + ((int64_t)(ks * ntl_f + wc + 2 * q) * 64 + l) * 8);
        }
    }
    if (tid < 64) {
        int32_t row = -1, hh = 0, tt = 0;
        if (tid < count) {
            const int e = tid < Pn ? seg_begin + p0 + tid
                                   : seg_begin + n_pos + (p0 + (tid - Pn) / p.kneg) * p.kneg + (tid - Pn) % p.kneg;
            row = p.pay ? p.pay[e] / 3 : p.packed[e] >> 2;
            hh = p.colidx[3 * row]; tt = p.colidx[3 * row + 2];
        }
        s_row[tid] = row; s_h[tid] = hh; s_t[tid] = tt;
    }
    __syncthreads();
    // ---- x = E[h] - E[t] of the 64 slots as bfloat16 (slots past `count` are zero)
    {
        const int stride = d + kLdsPad, q4 = d >> 2, total = 64 * q4;
        for (int g0 = tid; g0 < total; g0 += 8 * kThreads) {
            float4 v[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int g = g0 + u * kThreads;
                v[u] = make_float4(0.f, 0.f, 0.f, 0.f);
                if (g < total) {
                    const int i = g / q4, c4 = 4 * (g - i * q4);
                    if (i < count) v[u] = sub4(ld4(p.E + (int64_t)s_h[i] * d + c4), ld4(p.E + (int64_t)s_t[i] * d + c4));
                }
            }
#pragma unroll
            for (int u = 0; u < 8; ++u) {
                const int g = g0 + u * kThreads;
                if (g < total) {
                    const int i = g / q4, c4 = 4 * (g - i * q4);
                    *reinterpret_cast<uint2 *>(s_a + i * stride + c4) = make_uint2(pack2(v[u].x, v[u].y), pack2(v[u].z, v[u].w));
                }
            }
        }
    }
    __syncthreads();
    // ---- a tile of 64 slots, transposed into operand order for the dM product
    auto put_transposed = [&](uint16_t *tiles, int width) {
        const int stride = width + kLdsPad, rt = width >> 5, pieces = ((count + 15) >> 4) * rt * 64;
        uint16_t *tile = tiles + (int64_t)block * 64 * width;
        for (int pc = tid; pc < pieces; pc += kThreads) {
            const int ll = pc & 63, blk = pc >> 6, ks = blk / rt, mt = blk - ks * rt;
            const uint16_t *src = s_a + (16 * ks + 8 * (ll >> 5)) * stride + 32 * mt + (ll & 31);
            uint4 o;
            o.x = (uint32_t)src[0] | (uint32_t)src[stride] << 16;
            o.y = (uint32_t)src[2 * stride] | (uint32_t)src[3 * stride] << 16;
            o.z = (uint32_t)src[4 * stride] | (uint32_t)src[5 * stride] << 16;
            o.w = (uint32_t)src[6 * stride] | (uint32_t)src[7 * stride] << 16;
            *reinterpret_cast<uint4 *>(tile + (int64_t)pc * 8) = o;
        }
    };
    put_transposed(p.xt, d);
    // ---- Y = X M_r^T + r: wavefront w takes rows 32*(w/2).. and the column tiles w%2, w%2 + 2
    constexpr int kYS = kW + 4;                            // floats per row of the tile of y
    if (32 * wr < count) {
        const uint16_t *arow = s_a + (32 * wr + l31) * (d + kLdsPad) + 8 * kg;
        floatx16 acc[2] = {zero16(), zero16()};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks < KS_f) {
                const uint4 a = *reinterpret_cast<const uint4 *>(arow + 16 * ks);
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (q < ntw_f)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a), as_frag(bpre[ks][q]), acc[q], 0, 0, 0);
            }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (q < ntw_f) {
                const int n = (wc + 2 * q) * 32 + l31;
                const float add = p.Rv[(int64_t)rel * k + n];
#pragma unroll
                for (int v = 0; v < 16; ++v) s_y[(32 * wr + 8 * (v >> 2) + 4 * kg + (v & 3)) * kYS + n] = acc[q][v] + add;
            }
        }
    }
    __syncthreads();
    // ---- the GX fragments of M_r: requested now, used after the distances and the hinge
    const int ntl_g = d >> 5, ntw_g = (ntl_g - wc + 1) >> 1, KS_g = k >> 4;
    const uint16_t *Mg = p.Mg + (int64_t)rel * d * k;
    if (32 * wr < count) {
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
#pragma unroll
            for (int q = 0; q < 2; ++q)
                if (ks < KS_g && q < ntw_g) bpre[ks][q] = ld16(Mg + ((int64_t)(ks * ntl_g + wc + 2 * q) * 64 + l) * 8);
        }
    }
    // ---- distances: four lanes per slot, each over every fourth element, added across the four
    {
        const int slot = tid >> 2, c = tid & 3;
        float acc = 0.f;
        if (slot < count)
            for (int n = c; n < k; n += 4) acc += term<DIST>(s_y[slot * kYS + n]);
        acc += __shfl_xor(acc, 1);
        acc += __shfl_xor(acc, 2);
        if (c == 0) s_dist[slot] = slot < count ? finish<DIST>(acc) : 0.f;
    }
    __syncthreads();
    // ---- hinge of every (positive, negative) pair of the item; coefficient of every slot; scores; loss share
    if (tid < 64) {
        float hs = 0.f;
        if (tid < Pn) {
            const float dpos = s_dist[tid];
            int n_active = 0;
            for (int kk = 0; kk < p.kneg; ++kk) {
                const int ns = Pn + tid * p.kneg + kk;
                const float dneg = s_dist[ns];
                const float arg = (p.margin + dpos) - dneg;
                const bool active = arg > 0.f;
                if (active) { hs += arg; ++n_active; }
                s_cs[ns] = coef_scale<DIST>(active ? -p.scale : 0.f, dneg);
                p.scores[s_row[ns]] = dneg;
            }
            s_cs[tid] = coef_scale<DIST>((float)n_active * p.scale, dpos);
            p.scores[s_row[tid]] = dpos;
        } else if (tid >= count) {
            s_cs[tid] = 0.f;
        }
#pragma unroll
        for (int off = 32; off >= 1; off >>= 1) hs += __shfl_xor(hs, off);
        if (tid == 0) p.loss_partials[block] = hs;
    }
    __syncthreads();
    // ---- dL/dy: to memory in fp32, and as bfloat16 into the operand tile (the products over x are done with it)
    {
        const int stride = k + kLdsPad, q4 = k >> 2, total = 64 * q4;
        for (int g = tid; g < total; g += kThreads) {
            const int i = g / q4, c4 = 4 * (g - i * q4);
            float4 gy = make_float4(0.f, 0.f, 0.f, 0.f);
            if (i < count) {
                const float4 y = *reinterpret_cast<const float4 *>(s_y + i * kYS + c4);
                const float cs = s_cs[i];
                gy = make_float4(dterm<DIST>(y.x, cs), dterm<DIST>(y.y, cs), dterm<DIST>(y.z, cs), dterm<DIST>(y.w, cs));
                st4(p.gy + (int64_t)s_row[i] * k + c4, gy);
            }
            *reinterpret_cast<uint2 *>(s_a + i * stride + c4) = make_uint2(pack2(gy.x, gy.y), pack2(gy.z, gy.w));
        }
    }
    __syncthreads();
    put_transposed(p.gyt, k);
    // ---- dL/dx = dL/dy M_r
    if (32 * wr < count) {
        const uint16_t *arow = s_a + (32 * wr + l31) * (k + kLdsPad) + 8 * kg;
        floatx16 acc[2] = {zero16(), zero16()};
#pragma unroll
        for (int ks = 0; ks < 8; ++ks) {
            if (ks < KS_g) {
                const uint4 a = *reinterpret_cast<const uint4 *>(arow + 16 * ks);
#pragma unroll
                for (int q = 0; q < 2; ++q)
                    if (q < ntw_g)
                        acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a), as_frag(bpre[ks][q]), acc[q], 0, 0, 0);
            }
        }
#pragma unroll
        for (int q = 0; q < 2; ++q) {
            if (q < ntw_g) {
                const int n = (wc + 2 * q) * 32 + l31;
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int32_t row_m = s_row[32 * wr + 8 * (v >> 2) + 4 * kg + (v & 3)];
                    if (row_m >= 0) p.gx[(int64_t)row_m * d + n] = acc[q][v];
                }
            }
        }
    }
}

// dL/dM_r (transr_dm_body): one workgroup per dM item and per 128 x 128 block of the matrix (blockIdx.y); one
// more workgroup may follow the items and take a deferred final sum of the loss along.
__global__ __launch_bounds__(kThreads, 4) void k_transr_dm(DmArgs p)
{
    if ((int)blockIdx.x >= p.n_items) {
        if (blockIdx.y == 0 && p.fin_n > 0) finish_loss_body(p.fin_partials, p.fin_n, p.fin_scale, p.fin_loss);
        return;
    }
    transr_dm_body((int)blockIdx.x, (int)blockIdx.y, p);
}

// The sums of the partial matrices (transr_dm_fixup_body): blockIdx.y slices the matrix.
__global__ __launch_bounds__(kThreads) void k_transr_dm_fixup(DmArgs p)
{
    transr_dm_fixup_body((int)blockIdx.x, (int)blockIdx.y, p);
}

// M_r <- M_r - lr * dL/dM_r for every relation present in the batch: workgroup (r, y) looks relation r's
// column up in the sorted touched list, leaves if it is absent, and updates slice y of the matrix
// (four float4 per thread).
constexpr int kProjSlice = kThreads * 16;
__global__ __launch_bounds__(kThreads) void k_sgd_proj(const int32_t *__restrict__ touched_cols,
                                                       const int32_t *__restrict__ n_touched,
                                                       const int32_t *__restrict__ first_rel_seg, int32_t n_ent,
                                                       int64_t kd, float *__restrict__ M,
                                                       const float *__restrict__ g_proj, float lr)
{
    const int32_t target = n_ent + (int32_t)blockIdx.x;
    int32_t lo = first_rel_seg[0], hi = n_touched[0];     // relation columns sort after all entity columns
    while (lo < hi) {                                     // first position with touched_cols[pos] >= target
        const int32_t mid = (lo + hi) >> 1;
        if (touched_cols[mid] < target) lo = mid + 1; else hi = mid;
    }
    if (lo >= n_touched[0] || touched_cols[lo] != target) return;
    float *m = M + (int64_t)blockIdx.x * kd;
    const float *g = g_proj + (int64_t)blockIdx.x * kd;
    const int64_t base = (int64_t)blockIdx.y * kProjSlice + (int64_t)threadIdx.x * 4;
    float4 x[4], gg[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t idx = base + (int64_t)u * kThreads * 4;
        if (idx < kd) { x[u] = ld4(m + idx); gg[u] = ld4_stream(g + idx); }
    }
#pragma unroll
    for (int u = 0; u < 4; ++u) {
        const int64_t idx = base + (int64_t)u * kThreads * 4;
        if (idx < kd) {
            const float s0 = lr * gg[u].x, s1 = lr * gg[u].y, s2 = lr * gg[u].z, s3 = lr * gg[u].w;
            st4(m + idx, make_float4(x[u].x - s0, x[u].y - s1, x[u].z - s2, x[u].w - s3));
        }
    }
}

// ---------------------------------------------------------------------------------------------------
static RowsArgs rows_args(stx_ctx *c, const stx_incidence *inc, const stx_params *p, bool gx)
{
    RowsArgs a;
    a.items = (const int4 *)c->tr_items;
    a.counts = c->tr_counts;
    a.colidx = inc->a_colidx; a.packed = inc->at_packed;
    // (stx_train_step may have left the last kernel of the build, which writes `packed`, to a later launch)
    a.pay = (c->segw.armed && c->sorted_inc == inc) ? c->segw.args.pay : nullptr;
    a.E = p->ent; a.Rv = p->rel;
    a.Mb = gx ? c->tr_m16t : c->tr_m16;
    a.tiles = gx ? c->tr_gyt : c->tr_xt;
    a.n_red = gx ? c->cfg.rel_dim : c->cfg.dim;
    a.n_out = gx ? c->cfg.dim : c->cfg.rel_dim;
    a.fin_partials = nullptr; a.fin_n = 0; a.fin_scale = 1.0f; a.fin_loss = nullptr;
    return a;
}

// Most row items / dM items a batch of `rows` rows can have: every relation segment adds at most one
// item that is not full.
static int64_t max_segments(const stx_ctx *c, int64_t rows) { return rows < c->cfg.n_rel ? rows : c->cfg.n_rel; }
static unsigned row_items_max(const stx_ctx *c, int64_t rows) { return (unsigned)(rows / 64 + max_segments(c, rows)); }
static unsigned dm_items_max(const stx_ctx *c, int64_t rows) { return (unsigned)(rows / 256 + max_segments(c, rows)); }
// (a segment with several dM items has more than 256 rows)
static unsigned fix_items_max(int64_t rows) { return (unsigned)(rows / (kProjRowsDm + 1)); }

static PrepArgs prep_args(stx_ctx *c, const stx_incidence *inc, const stx_params *p)
{
    PrepArgs a;
    a.touched_cols = inc->at_touched_cols; a.n_touched = inc->n_touched;
    a.seg_ptr = inc->at_seg_ptr; a.seg_id = inc->at_seg_id;
    a.n_ent = (int32_t)c->cfg.n_ent;
    a.e_begin = (int32_t)(2 * inc->n_rows);               // relation columns follow the entity columns
    a.M = p->proj; a.m16 = c->tr_m16; a.m16t = c->tr_m16t;
    a.items = (int4 *)c->tr_items; a.dm_items = (int4 *)c->tr_dm_items; a.fix_items = (int4 *)c->tr_fix_items;
    a.counts = c->tr_counts;
    a.d = c->cfg.dim; a.k = c->cfg.rel_dim;
    a.rel_cnt = c->cnt_inc == inc ? c->cnt_ptr : nullptr;  // the counts of the last build, if that was this incidence
    a.n_rel = (int32_t)c->cfg.n_rel;
    const int64_t lists = inc->n_rows < c->cfg.n_rel ? inc->n_rows : c->cfg.n_rel;   // most touched relations
    a.nplan = (int)(((a.rel_cnt ? c->cfg.n_rel : lists) + kThreads - 1) / kThreads);
    a.whole_lists = 0;
    return a;
}

// workgroups of the preparation: the planners, then k / kPrepRows per relation
static unsigned prep_blocks(const stx_ctx *c, const PrepArgs &a)
{
    return (unsigned)(a.nplan + c->cfg.n_rel * (c->cfg.rel_dim / kPrepRows));
}

bool launch_prep_scatter(stx_ctx *c, const stx_incidence *inc, const stx_params *p, const ScatterArgs &sa, bool first)
{
    if (c->cfg.model != STX_TRANSR || inc->n_rows == 0) return false;
    PrepArgs a = prep_args(c, inc, p);
    if (!a.rel_cnt) return false;
    a.whole_lists = transr_fused_ok(c, inc) ? 1 : 0;      // (stx_train_step runs the forward pass this prepares)
    ProfScope prof(c, "k_prep_scatter");
    const dim3 grid((unsigned)(sa.ntiles + prep_blocks(c, a)));
    if (first) hipLaunchKernelGGL(k_prep_scatter<true>, grid, dim3(kThreads), 0, c->stream, a, sa);
    else hipLaunchKernelGGL(k_prep_scatter<false>, grid, dim3(kThreads), 0, c->stream, a, sa);
    c->prep_inc = inc;
    c->prep_whole = a.whole_lists;
    return true;
}

stx_status launch_transr_project(stx_ctx *c, const stx_incidence *inc, const stx_params *p)
{
    if (inc->n_rows == 0) return STX_OK;
    if (c->prep_inc != inc || c->prep_whole != 0) {   // not yet prepared beside the sort
        launch_seg_write_late(c);   // (the segment lists may be needed)
        const PrepArgs a = prep_args(c, inc, p);
        ProfScope prof(c, "k_transr_prepare");
        if (a.rel_cnt)
            hipLaunchKernelGGL(k_transr_prepare<true>, dim3(prep_blocks(c, a)), dim3(kThreads), 0, c->stream, a);
        else
            hipLaunchKernelGGL(k_transr_prepare<false>, dim3(prep_blocks(c, a)), dim3(kThreads), 0, c->stream, a);
    }
    c->prep_inc = nullptr;      // the copies of M_r are good for this forward pass only: the update changes M_r
    ProfScope prof(c, "k_transr_project");
    if (c->cfg.dim <= 128 && c->cfg.rel_dim <= 128)
        hipLaunchKernelGGL((k_transr_rows<false, true>), dim3(row_items_max(c, inc->n_rows)), dim3(kThreads), 0,
                           c->stream, rows_args(c, inc, p, false), (const float *)nullptr, c->gbuf[0]);
    else
        hipLaunchKernelGGL((k_transr_rows<false, false>), dim3(row_items_max(c, inc->n_rows)), dim3(kThreads), 0,
                           c->stream, rows_args(c, inc, p, false), (const float *)nullptr, c->gbuf[0]);
    return hip_ok(hipGetLastError());
}

// Which batches k_transr_fused takes: both widths at most 128 and whole positives with their negatives per 64-slot tile.
bool transr_fused_ok(const stx_ctx *c, const stx_incidence *inc)
{
    return c->cfg.model == STX_TRANSR && c->cfg.dim <= 128 && c->cfg.rel_dim <= 128 && inc->k < 64 && 64 % (1 + inc->k) == 0;
}

stx_status launch_transr_fused(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores, float *loss)
{
    float scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    if (c->prep_inc != inc || c->prep_whole != 1) {   // not yet prepared beside the sort
        launch_seg_write_late(c);   // (the segment lists may be needed)
        PrepArgs a = prep_args(c, inc, p);
        a.whole_lists = 1;
        ProfScope prof(c, "k_transr_prepare");
        if (a.rel_cnt)
            hipLaunchKernelGGL(k_transr_prepare<true>, dim3(prep_blocks(c, a)), dim3(kThreads), 0, c->stream, a);
        else
            hipLaunchKernelGGL(k_transr_prepare<false>, dim3(prep_blocks(c, a)), dim3(kThreads), 0, c->stream, a);
    }
    c->prep_inc = nullptr;      // the copies of M_r are good for this forward pass only: the update changes M_r
    FusedArgs a;
    a.items = (const int4 *)c->tr_items; a.counts = c->tr_counts;
    const bool own_ids = c->step_colidx && c->step_colidx_inc == inc;
    a.colidx = own_ids ? c->step_colidx : inc->a_colidx;
    a.packed = inc->at_packed;
    a.pay = (c->segw.armed && c->sorted_inc == inc) ? c->segw.args.pay : nullptr;
    a.E = p->ent; a.Rv = p->rel; a.Mf = c->tr_m16; a.Mg = c->tr_m16t;
    a.xt = c->tr_xt; a.gyt = c->tr_gyt;
    a.gy = c->gbuf[0]; a.gx = c->gbuf[1];
    a.scores = scores; a.loss_partials = c->loss_partials;
    a.d = c->cfg.dim; a.k = c->cfg.rel_dim; a.kneg = inc->k;
    a.margin = c->cfg.margin; a.scale = scale;
    EmitAhead ea{};
    if (own_ids && c->ahead.armed && !c->ahead.emit_done && c->ahead.args.rc.cur) ea = take_emit_ahead(c);
    const unsigned items = row_items_max(c, inc->n_rows);
    const dim3 grid(items + (unsigned)ea.ntiles);
    {
        ProfScope prof(c, "k_transr_fused");
        switch (c->cfg.dist) {
        case STX_L1: hipLaunchKernelGGL(k_transr_fused<STX_L1>, grid, dim3(kThreads), 0, c->stream, a, ea); break;
        case STX_L2: hipLaunchKernelGGL(k_transr_fused<STX_L2>, grid, dim3(kThreads), 0, c->stream, a, ea); break;
        case STX_TORUS_L1: hipLaunchKernelGGL(k_transr_fused<STX_TORUS_L1>, grid, dim3(kThreads), 0, c->stream, a, ea); break;
        case STX_L2_SQ: hipLaunchKernelGGL(k_transr_fused<STX_L2_SQ>, grid, dim3(kThreads), 0, c->stream, a, ea); break;
        default: hipLaunchKernelGGL(k_transr_fused<STX_TORUS_L2>, grid, dim3(kThreads), 0, c->stream, a, ea); break;
        }
    }
    c->tr_fused_inc = inc;
    if (c->defer_finish) { c->fin_n = (int)items; c->fin_scale = scale; c->fin_loss = loss; return hip_ok(hipGetLastError()); }
    return launch_finish_loss(c, (int)items, scale, loss);
}

stx_status launch_transr_backward(stx_ctx *c, const stx_incidence *inc, const stx_params *p, stx_grads *g,
                                  const float *fused_lr)
{
    if (inc->n_rows == 0) return STX_OK;
    const bool fused_rows = c->tr_fused_inc == inc;       // the forward kernel already formed dL/dx and the tiles
    if (!fused_rows) {
        RowsArgs ra = rows_args(c, inc, p, true);
        unsigned blocks = row_items_max(c, inc->n_rows);
        if (c->fin_n > 0) {
            ra.fin_partials = c->loss_partials; ra.fin_n = c->fin_n; ra.fin_scale = c->fin_scale; ra.fin_loss = c->fin_loss;
            c->fin_n = 0;
            ++blocks;
        }
        ProfScope prof(c, "k_transr_gx");
        if (c->cfg.dim <= 128 && c->cfg.rel_dim <= 128)
            hipLaunchKernelGGL((k_transr_rows<true, true>), dim3(blocks), dim3(kThreads), 0, c->stream, ra, c->gbuf[0],
                               c->gbuf[1]);
        else
            hipLaunchKernelGGL((k_transr_rows<true, false>), dim3(blocks), dim3(kThreads), 0, c->stream, ra, c->gbuf[0],
                               c->gbuf[1]);
    }
    DmArgs a;
    a.dm_items = (const int4 *)c->tr_dm_items; a.fix_items = (const int4 *)c->tr_fix_items; a.counts = c->tr_counts;
    a.n_fix = (int)fix_items_max(inc->n_rows);
    a.gyt = c->tr_gyt; a.xt = c->tr_xt;
    a.g_proj = fused_lr ? nullptr : g->proj; a.partials = c->gbuf[2];
    a.d = c->cfg.dim; a.k = c->cfg.rel_dim;
    a.M = p->proj; a.lr = fused_lr ? *fused_lr : 0.f; a.fused = fused_lr ? 1 : 0;
    a.n_items = (int)dm_items_max(c, inc->n_rows);
    a.fin_partials = nullptr; a.fin_n = 0; a.fin_scale = 1.0f; a.fin_loss = nullptr;
    // Left for the launches of the transposed incidence product, which follow at once; in stx_train_step they take
    // this along (one workgroup per dM item: both widths at most 128), otherwise they launch it first.
    c->dm_ride = DmRideState{true, a.n_fix > 0 /* else no relation can have two items */, a, a.n_items};
    if (!(fused_lr && fused_rows && a.d <= 128 && a.k <= 128 && c->segw.armed && c->sorted_inc == inc))
        return launch_transr_dm_late(c);
    return hip_ok(hipGetLastError());
}

static void launch_dm_fixup(stx_ctx *c, const DmArgs &a)
{
    ProfScope prof(c, "k_transr_dm_fixup");
    hipLaunchKernelGGL(k_transr_dm_fixup,
                       dim3((unsigned)a.n_fix, (unsigned)(((int64_t)a.k * a.d + kDmFixupSlice - 1) / kDmFixupSlice)),
                       dim3(kThreads), 0, c->stream, a);
}

stx_status launch_transr_dm_late(stx_ctx *c)
{
    if (!c->dm_ride.armed) return STX_OK;
    c->dm_ride.armed = false;
    DmArgs a = c->dm_ride.args;
    if (c->fin_n > 0) {   // a deferred sum of the loss: one more workgroup
        a.fin_partials = c->loss_partials; a.fin_n = c->fin_n; a.fin_scale = c->fin_scale; a.fin_loss = c->fin_loss;
        c->fin_n = 0;
    }
    {
        ProfScope prof(c, "k_transr_dm");
        hipLaunchKernelGGL(k_transr_dm, dim3((unsigned)a.n_items + (a.fin_n > 0 ? 1u : 0u),
                                             (unsigned)(((a.k + 127) / 128) * ((a.d + 127) / 128))),
                           dim3(kThreads), 0, c->stream, a);
    }
    if (c->dm_ride.fixup) launch_dm_fixup(c, a);
    return hip_ok(hipGetLastError());
}

// The sum of the partial matrices alone, after a launch that took the product along but not the sum.
stx_status launch_transr_dm_fixup_late(stx_ctx *c)
{
    launch_dm_fixup(c, c->dm_ride.args);
    return hip_ok(hipGetLastError());
}

stx_status launch_transr_sgd_proj(stx_ctx *c, const stx_incidence *inc, stx_params *p, const stx_grads *g, float lr)
{
    if (inc->n_rows == 0) return STX_OK;
    ProfScope prof(c, "k_sgd_proj");
    const int64_t kd = (int64_t)c->cfg.rel_dim * c->cfg.dim;
    hipLaunchKernelGGL(k_sgd_proj, dim3((unsigned)c->cfg.n_rel, (unsigned)((kd + kProjSlice - 1) / kProjSlice)),
                       dim3(kThreads), 0, c->stream, inc->at_touched_cols, inc->n_touched,
                       inc->at_seg_id + 2 * inc->n_rows, (int32_t)c->cfg.n_ent, kd,
                       p->proj, g->proj, lr);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
