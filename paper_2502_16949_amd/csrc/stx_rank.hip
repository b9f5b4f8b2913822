// Link prediction by exhaustive scoring: how many entities score below (and exactly like) the true entity
// of each test triplet.  TransE / TorusE first; TransH and TransR, further down, reuse the same sweep.
//
// SparseTransX Sec. 4.7 lists link prediction among the framework's functions and Sec. 6.1 measures
// accuracy as Hits@10, the share of test triplets whose true entity is among the ten best candidates.
// For the translational score of Sec. 4.3 / 4.6 that is a nearest-neighbour count around a query point:
//   tail side  q = h + r,  score(e) = dist(q - e);     head side  q = t - r,  score(e) = dist(e - q).
//
// The work is nq x n_ent x dim subtract-and-accumulate steps on tables that fit the caches: plain vector
// arithmetic, no memory bound and (for the L1 kinds) no product to give to the matrix cores.  It is tiled
// like a matrix product: a workgroup owns 128 queries, walks the candidates 128 at a time and the row in
// chunks of 32 floats staged (transposed) in LDS; a thread keeps an 8 x 8 block of partial distances in
// registers, so every value fetched from LDS feeds eight steps.  Sums run over the row in index order in
// one thread; the true entity's own sum is formed the same way, so it compares equal to itself.
// Counts are integers: candidate slices of one query block add theirs with atomics, in any order.
#include <new>

#include "stx_rowops.h"

namespace stx {

constexpr int kRankQ = 128;            // queries per workgroup
constexpr int kRankE = 128;            // candidates per tile
constexpr int kRankJ = 32;             // floats of a row per staged chunk
constexpr int kRankLd = kRankQ + 4;    // floats per LDS row: keeps float4 alignment, shifts banks by 4 per row

// One step of the distance sum (Sec. 4.3, 4.6), index order.  The L2 kinds use a fused multiply-add.
template <int DIST>
__device__ inline float rank_step(float acc, float y)
{
    if (DIST == STX_L1) return acc + fabsf(y);
    if (DIST == STX_L2 || DIST == STX_L2_SQ) return __builtin_fmaf(y, y, acc);
    const float f = __builtin_amdgcn_fractf(y);            // fractional part, always below 1
    const float m = fminf(f, 1.0f - f);
    return DIST == STX_TORUS_L1 ? acc + m : __builtin_fmaf(m, m, acc);
}

struct RankArgs {
    const float *X;                    // TransE / TorusE: [E;R]; TransH: E.  Rows of dim floats
    const float *D, *W;                // TransH: d_r and w_r, n_rel rows each
    const int32_t *h, *r, *t;          // [nq]; r may be null: every query has relation 0
    int64_t nq;
    int32_t n_ent, n_rel;
    int dim;
    int32_t slice;                     // candidates per blockIdx.y, a multiple of kRankE
    float *true_score;                 // [nq]: the true entity's sum until k_rank_finish
    int32_t *n_less, *n_equal;         // [nq], cleared by k_rank_true
    int32_t *bad;                      // counter of out-of-range indices
    // TransR: blockIdx.z walks the relations grp_first, grp_first + 1, ...; relation g owns the grouped queries
    // [grp_offsets[g], + grp_counts[g]) (h, t and the outputs are grouped arrays) and table number blockIdx.z.
    // With several relations per launch, those with more than grp_big queries are left to a launch of their own.
    const int32_t *grp_counts, *grp_offsets;
    int32_t grp_first, grp_big;
    int64_t table_stride;              // floats between the tables of consecutive blockIdx.z
};

// Narrows the arguments to the relation of this workgroup; false: nothing to do.
__device__ inline bool rank_group(RankArgs &a)
{
    if (!a.grp_counts) return true;
    const int32_t g = a.grp_first + (int32_t)blockIdx.z;
    const int32_t n = a.grp_counts[g];
    if (n == 0 || (gridDim.z > 1 && n > a.grp_big)) return false;
    const int64_t off = a.grp_offsets[g];
    a.X += (int64_t)blockIdx.z * a.table_stride;
    a.h += off; a.t += off;
    a.true_score += off; a.n_less += off; a.n_equal += off;
    a.nq = n;
    return true;
}

// The 8 x 8 block of a thread: query u is block row (u < 4 ? 0 : 64) + 4 ty + (u & 3) of the workgroup's 128,
// candidate v is (v < 4 ? 0 : 64) + 4 tx + (v & 3) of the tile's 128.
__device__ inline void rank_count(const float (&acc)[8][8], const float (&tr)[8], int32_t e0, int32_t e_end, int tx,
                                  int32_t (&less)[8], int32_t (&equal)[8])
{
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const bool valid = e0 + (v < 4 ? 0 : 64) + tx * 4 + (v & 3) < e_end;
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            less[u] += (valid && acc[u][v] < tr[u]) ? 1 : 0;
            equal[u] += (valid && acc[u][v] == tr[u]) ? 1 : 0;
        }
    }
}

// Adds a workgroup's counts to the queries' counters.  The 16 threads that share a query sit in consecutive lanes.
__device__ inline void rank_flush(const RankArgs &a, int64_t q0, int tx, int ty, int32_t (&less)[8], int32_t (&equal)[8])
{
#pragma unroll
    for (int u = 0; u < 8; ++u) {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) {
            less[u] += __shfl_xor(less[u], m, 16);
            equal[u] += __shfl_xor(equal[u], m, 16);
        }
        const int64_t q = q0 + (u < 4 ? 0 : 64) + ty * 4 + (u & 3);
        if (tx == 0 && q < a.nq) {
            if (less[u]) atomicAdd(&a.n_less[q], less[u]);
            if (equal[u]) atomicAdd(&a.n_equal[q], equal[u]);
        }
    }
}

// Clamped table rows of one query: q = h + r (tail side) or t - r (head side); the true entity is t or h.
struct RankRows {
    const float *pa, *pr, *ptrue;
    bool bad;
};
template <bool HEAD>
__device__ inline RankRows rank_rows(const RankArgs &a, int64_t qi)
{
    int32_t ih = a.h[qi], ir = a.r ? a.r[qi] : 0, it = a.t[qi];
    const bool bad = ih < 0 || ih >= a.n_ent || it < 0 || it >= a.n_ent || ir < 0 || ir >= a.n_rel;
    ih = min(max(ih, 0), a.n_ent - 1);
    it = min(max(it, 0), a.n_ent - 1);
    ir = min(max(ir, 0), a.n_rel - 1);
    return {a.X + (int64_t)(HEAD ? it : ih) * a.dim, a.X + ((int64_t)a.n_ent + ir) * a.dim,
            a.X + (int64_t)(HEAD ? ih : it) * a.dim, bad};
}

// One thread per query: the true entity's sum, formed step by step in index order exactly as the sweep forms
// every candidate's, so that the true entity ties with itself there.  Also clears the query's counters.
template <int DIST, bool HEAD>
__global__ __launch_bounds__(kThreads) void k_rank_true(RankArgs a)
{
    if (!rank_group(a)) return;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.nq) return;
    const RankRows rw = rank_rows<HEAD>(a, i);
    if (rw.bad) atomicAdd(a.bad, 1);
    float acc = 0.f;
    for (int j = 0; j < a.dim; j += 4) {
        const float4 va = ld4(rw.pa + j), vr = ld4(rw.pr + j), ve = ld4(rw.ptrue + j);
        const float av[4] = {va.x, va.y, va.z, va.w}, rv[4] = {vr.x, vr.y, vr.z, vr.w};
        const float ev[4] = {ve.x, ve.y, ve.z, ve.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float q = HEAD ? av[u] - rv[u] : av[u] + rv[u];
            acc = rank_step<DIST>(acc, HEAD ? ev[u] - q : q - ev[u]);
        }
    }
    a.true_score[i] = acc;        // the sum; k_rank_finish turns it into the distance after the sweep
    a.n_less[i] = 0;
    a.n_equal[i] = 0;
}

template <int DIST>
__global__ __launch_bounds__(kThreads) void k_rank_finish(float *true_score, int64_t nq)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < nq) true_score[i] = finish<DIST>(true_score[i]);
}

// (three waves per SIMD: the register budget that lets three workgroups share a compute unit)
template <int DIST, bool HEAD>
__global__ __launch_bounds__(kThreads, 3) void k_rank(RankArgs a)
{
    __shared__ __attribute__((aligned(16))) float s_q[kRankJ][kRankLd];
    __shared__ __attribute__((aligned(16))) float s_e[kRankJ][kRankLd];

    if (!rank_group(a)) return;                           // (uniform over the workgroup)
    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;               // candidate / query position of the 8 x 8 block
    const int64_t q0 = (int64_t)blockIdx.x * kRankQ;
    if (q0 >= a.nq) return;
    const int dim = a.dim;

    // The query this thread stages; past the end the last query is repeated and its counts are not stored.
    const int sc = tid & (kRankQ - 1);                    // staged query / candidate of this thread
    const int sj = (tid >> 7) * 4;                        // first float of its float4 inside a chunk (then + 8 i)
    const RankRows rw = rank_rows<HEAD>(a, min(q0 + sc, a.nq - 1));
    const float *pa = rw.pa, *pr = rw.pr;
    float tr[8];                                          // the true entities' sums (k_rank_true)
#pragma unroll
    for (int u = 0; u < 8; ++u) tr[u] = a.true_score[min(q0 + (u < 4 ? 0 : 64) + ty * 4 + (u & 3), a.nq - 1)];

    int32_t less[8], equal[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) less[u] = equal[u] = 0;

    const int32_t e_begin = (int32_t)blockIdx.y * a.slice;
    const int32_t e_end = min(e_begin + a.slice, a.n_ent);
    for (int32_t e0 = e_begin; e0 < e_end; e0 += kRankE) {
        float acc[8][8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int v = 0; v < 8; ++v) acc[u][v] = 0.f;
        const float *pe = a.X + (int64_t)min(e0 + sc, a.n_ent - 1) * dim;   // past the end: repeated, not counted
        for (int j0 = 0; j0 < dim; j0 += kRankJ) {
            // all twelve loads of the chunk go out together (addresses past the row's end are pulled back
            // inside it and their values replaced by zeros, which add nothing to a sum)
            float4 va[4], vr[4], ve[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = min(j0 + sj + 8 * i, dim - 4);
                va[i] = ld4(pa + j); vr[i] = ld4(pr + j); ve[i] = ld4(pe + j);
            }
            __syncthreads();                              // the previous chunk has been consumed
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jj = sj + 8 * i;
                float4 q4 = HEAD ? make_float4(va[i].x - vr[i].x, va[i].y - vr[i].y, va[i].z - vr[i].z, va[i].w - vr[i].w)
                                 : make_float4(va[i].x + vr[i].x, va[i].y + vr[i].y, va[i].z + vr[i].z, va[i].w + vr[i].w);
                float4 e4 = ve[i];
                if (j0 + jj >= dim) q4 = e4 = make_float4(0.f, 0.f, 0.f, 0.f);
                s_q[jj][sc] = q4.x; s_q[jj + 1][sc] = q4.y; s_q[jj + 2][sc] = q4.z; s_q[jj + 3][sc] = q4.w;
                s_e[jj][sc] = e4.x; s_e[jj + 1][sc] = e4.y; s_e[jj + 2][sc] = e4.z; s_e[jj + 3][sc] = e4.w;
            }
            __syncthreads();
            // the operands of step jj + 1 are requested before step jj is computed, so the LDS round trip hides
            // behind 128 vector operations
            float4 qa = *reinterpret_cast<const float4 *>(&s_q[0][ty * 4]);
            float4 qb = *reinterpret_cast<const float4 *>(&s_q[0][64 + ty * 4]);
            float4 ea = *reinterpret_cast<const float4 *>(&s_e[0][tx * 4]);
            float4 eb = *reinterpret_cast<const float4 *>(&s_e[0][64 + tx * 4]);
#pragma unroll 4
            for (int jj = 0; jj < kRankJ; ++jj) {
                const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
                const float ev[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
                const int jn = min(jj + 1, kRankJ - 1);
                qa = *reinterpret_cast<const float4 *>(&s_q[jn][ty * 4]);
                qb = *reinterpret_cast<const float4 *>(&s_q[jn][64 + ty * 4]);
                ea = *reinterpret_cast<const float4 *>(&s_e[jn][tx * 4]);
                eb = *reinterpret_cast<const float4 *>(&s_e[jn][64 + tx * 4]);
                __builtin_amdgcn_sched_barrier(0);        // keep the requests ahead of the arithmetic
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int v = 0; v < 8; ++v)
                        acc[u][v] = rank_step<DIST>(acc[u][v], HEAD ? ev[v] - qv[u] : qv[u] - ev[v]);
            }
        }
        rank_count(acc, tr, e0, e_end, tx, less, equal);
    }
    rank_flush(a, q0, tx, ty, less, equal);
}

// ---- TransH (Sec. 4.5) -----------------------------------------------------------------------------
// Candidate e as tail: x = h - e, y = x + d_r - (w_r.x) w_r; as head: x = e - t.  With b = h (tail side) or t
// (head side) and B = h + d_r or t - d_r, the projection coefficient splits into a part of the query and a
// part of the pair: s = w.b - w.e (tail) or w.e - w.b (head), and y_j = (B_j - e_j) - s w_j or
// (e_j - B_j) - s w_j.  The sweep therefore runs over the row twice: first the 8 x 8 dot products w_u.e_v,
// then the distances, three operations per element (difference, fused multiply-add, accumulate).
// Every sum runs in index order with fused multiply-adds, in the sweep and in k_rank_true_h alike.
struct RankRowsH {
    const float *pb, *pd, *pw, *ptrue;   // b = h or t, d_r, w_r, the true entity's row
    bool bad;
};
template <bool HEAD>
__device__ inline RankRowsH rank_rows_h(const RankArgs &a, int64_t qi)
{
    int32_t ih = a.h[qi], ir = a.r[qi], it = a.t[qi];
    const bool bad = ih < 0 || ih >= a.n_ent || it < 0 || it >= a.n_ent || ir < 0 || ir >= a.n_rel;
    ih = min(max(ih, 0), a.n_ent - 1);
    it = min(max(it, 0), a.n_ent - 1);
    ir = min(max(ir, 0), a.n_rel - 1);
    return {a.X + (int64_t)(HEAD ? it : ih) * a.dim, a.D + (int64_t)ir * a.dim, a.W + (int64_t)ir * a.dim,
            a.X + (int64_t)(HEAD ? ih : it) * a.dim, bad};
}

// w.v over a row, index order, fused multiply-adds (v = the query's own entity or a candidate).
__device__ inline float rank_dot_row(const float *__restrict__ pw, const float *__restrict__ pv, int dim)
{
    float s = 0.f;
    for (int j = 0; j < dim; j += 4) {
        const float4 w4 = ld4(pw + j), v4 = ld4(pv + j);
        s = __builtin_fmaf(w4.x, v4.x, s); s = __builtin_fmaf(w4.y, v4.y, s);
        s = __builtin_fmaf(w4.z, v4.z, s); s = __builtin_fmaf(w4.w, v4.w, s);
    }
    return s;
}

template <int DIST, bool HEAD>
__global__ __launch_bounds__(kThreads) void k_rank_true_h(RankArgs a)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= a.nq) return;
    const RankRowsH rw = rank_rows_h<HEAD>(a, i);
    if (rw.bad) atomicAdd(a.bad, 1);
    const float sb = rank_dot_row(rw.pw, rw.pb, a.dim), se = rank_dot_row(rw.pw, rw.ptrue, a.dim);
    const float ns = HEAD ? sb - se : se - sb;            // minus the projection coefficient
    float acc = 0.f;
    for (int j = 0; j < a.dim; j += 4) {
        const float4 b4 = ld4(rw.pb + j), d4 = ld4(rw.pd + j), w4 = ld4(rw.pw + j), e4 = ld4(rw.ptrue + j);
        const float bv[4] = {b4.x, b4.y, b4.z, b4.w}, dv[4] = {d4.x, d4.y, d4.z, d4.w};
        const float wv[4] = {w4.x, w4.y, w4.z, w4.w}, ev[4] = {e4.x, e4.y, e4.z, e4.w};
#pragma unroll
        for (int u = 0; u < 4; ++u) {
            const float B = HEAD ? bv[u] - dv[u] : bv[u] + dv[u];
            acc = rank_step<DIST>(acc, __builtin_fmaf(ns, wv[u], HEAD ? ev[u] - B : B - ev[u]));
        }
    }
    a.true_score[i] = acc;
    a.n_less[i] = 0;
    a.n_equal[i] = 0;
}

template <int DIST, bool HEAD>
__global__ __launch_bounds__(kThreads, 2) void k_rank_h(RankArgs a)
{
    __shared__ __attribute__((aligned(16))) float s_b[kRankJ][kRankLd];
    __shared__ __attribute__((aligned(16))) float s_w[kRankJ][kRankLd];
    __shared__ __attribute__((aligned(16))) float s_e[kRankJ][kRankLd];
    __shared__ float s_sb[kRankQ];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;
    const int64_t q0 = (int64_t)blockIdx.x * kRankQ;
    const int dim = a.dim;
    const int sc = tid & (kRankQ - 1);
    const int sj = (tid >> 7) * 4;
    const RankRowsH rw = rank_rows_h<HEAD>(a, min(q0 + sc, a.nq - 1));
    if (tid < kRankQ) s_sb[tid] = rank_dot_row(rw.pw, rw.pb, dim);   // w.b of the workgroup's queries
    float tr[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) tr[u] = a.true_score[min(q0 + (u < 4 ? 0 : 64) + ty * 4 + (u & 3), a.nq - 1)];
    __syncthreads();
    float sb[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) sb[u] = s_sb[(u < 4 ? 0 : 64) + ty * 4 + (u & 3)];

    int32_t less[8], equal[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) less[u] = equal[u] = 0;

    const int32_t e_begin = (int32_t)blockIdx.y * a.slice;
    const int32_t e_end = min(e_begin + a.slice, a.n_ent);
    for (int32_t e0 = e_begin; e0 < e_end; e0 += kRankE) {
        const float *pe = a.X + (int64_t)min(e0 + sc, a.n_ent - 1) * dim;
        // ---- first pass over the row: dot[u][v] = w_u . e_v --------------------------------------------
        float ns[8][8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int v = 0; v < 8; ++v) ns[u][v] = 0.f;
        for (int j0 = 0; j0 < dim; j0 += kRankJ) {
            float4 vw[4], ve[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int j = min(j0 + sj + 8 * i, dim - 4);
                vw[i] = ld4(rw.pw + j); ve[i] = ld4(pe + j);
            }
            __syncthreads();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jj = sj + 8 * i;
                float4 w4 = vw[i], e4 = ve[i];
                if (j0 + jj >= dim) w4 = e4 = make_float4(0.f, 0.f, 0.f, 0.f);
                s_w[jj][sc] = w4.x; s_w[jj + 1][sc] = w4.y; s_w[jj + 2][sc] = w4.z; s_w[jj + 3][sc] = w4.w;
                s_e[jj][sc] = e4.x; s_e[jj + 1][sc] = e4.y; s_e[jj + 2][sc] = e4.z; s_e[jj + 3][sc] = e4.w;
            }
            __syncthreads();
#pragma unroll 4
            for (int jj = 0; jj < kRankJ; ++jj) {
                const float4 wa = *reinterpret_cast<const float4 *>(&s_w[jj][ty * 4]);
                const float4 wb = *reinterpret_cast<const float4 *>(&s_w[jj][64 + ty * 4]);
                const float4 ea = *reinterpret_cast<const float4 *>(&s_e[jj][tx * 4]);
                const float4 eb = *reinterpret_cast<const float4 *>(&s_e[jj][64 + tx * 4]);
                const float wv[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
                const float ev[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int v = 0; v < 8; ++v) ns[u][v] = __builtin_fmaf(wv[u], ev[v], ns[u][v]);
            }
        }
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int v = 0; v < 8; ++v) ns[u][v] = HEAD ? sb[u] - ns[u][v] : ns[u][v] - sb[u];   // minus the coefficient
        // ---- second pass: the distances ------------------------------------------------------------------
        float acc[8][8];
#pragma unroll
        for (int u = 0; u < 8; ++u)
#pragma unroll
            for (int v = 0; v < 8; ++v) acc[u][v] = 0.f;
        for (int j0 = 0; j0 < dim; j0 += kRankJ) {
            __syncthreads();                              // the previous chunk has been consumed
#pragma unroll
            for (int half = 0; half < 2; ++half) {        // two batches of eight loads: fewer registers in flight
                float4 vb[2], vd[2], vw[2], ve[2];
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int j = min(j0 + sj + 8 * (2 * half + i), dim - 4);
                    vb[i] = ld4(rw.pb + j); vd[i] = ld4(rw.pd + j); vw[i] = ld4(rw.pw + j); ve[i] = ld4(pe + j);
                }
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const int jj = sj + 8 * (2 * half + i);
                    float4 B4 = HEAD ? make_float4(vb[i].x - vd[i].x, vb[i].y - vd[i].y, vb[i].z - vd[i].z, vb[i].w - vd[i].w)
                                     : make_float4(vb[i].x + vd[i].x, vb[i].y + vd[i].y, vb[i].z + vd[i].z, vb[i].w + vd[i].w);
                    float4 w4 = vw[i], e4 = ve[i];
                    if (j0 + jj >= dim) B4 = w4 = e4 = make_float4(0.f, 0.f, 0.f, 0.f);
                    s_b[jj][sc] = B4.x; s_b[jj + 1][sc] = B4.y; s_b[jj + 2][sc] = B4.z; s_b[jj + 3][sc] = B4.w;
                    s_w[jj][sc] = w4.x; s_w[jj + 1][sc] = w4.y; s_w[jj + 2][sc] = w4.z; s_w[jj + 3][sc] = w4.w;
                    s_e[jj][sc] = e4.x; s_e[jj + 1][sc] = e4.y; s_e[jj + 2][sc] = e4.z; s_e[jj + 3][sc] = e4.w;
                }
            }
            __syncthreads();
#pragma unroll 2
            for (int jj = 0; jj < kRankJ; ++jj) {
                const float4 ba = *reinterpret_cast<const float4 *>(&s_b[jj][ty * 4]);
                const float4 bb = *reinterpret_cast<const float4 *>(&s_b[jj][64 + ty * 4]);
                const float4 wa = *reinterpret_cast<const float4 *>(&s_w[jj][ty * 4]);
                const float4 wb = *reinterpret_cast<const float4 *>(&s_w[jj][64 + ty * 4]);
                const float4 ea = *reinterpret_cast<const float4 *>(&s_e[jj][tx * 4]);
                const float4 eb = *reinterpret_cast<const float4 *>(&s_e[jj][64 + tx * 4]);
                const float bv[8] = {ba.x, ba.y, ba.z, ba.w, bb.x, bb.y, bb.z, bb.w};
                const float wv[8] = {wa.x, wa.y, wa.z, wa.w, wb.x, wb.y, wb.z, wb.w};
                const float ev[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int v = 0; v < 8; ++v)
                        acc[u][v] = rank_step<DIST>(acc[u][v], __builtin_fmaf(ns[u][v], wv[u], HEAD ? ev[v] - bv[u] : bv[u] - ev[v]));
            }
        }
        rank_count(acc, tr, e0, e_end, tx, less, equal);
    }
    rank_flush(a, q0, tx, ty, less, equal);
}

// ---- TransR (Sec. 4.4) -----------------------------------------------------------------------------
// score = dist(M_r (h - t) + r).  M_r is linear, so for one relation the candidates can be projected once,
// p_e = M_r e, and the score of e as tail of (h, r, .) is dist((p_h + r) - p_e), as head of (., r, t)
// dist(p_e - (p_t - r)): the TransE sweep over the table [P_r; r] with a single relation.  Queries are
// grouped by relation (counting sort), and for every relation that occurs its projected table is built
// (k_rr_project, a plain fp32 product with sums in index order) and swept by k_rank_true / k_rank.  Relations
// with many queries get launches of their own; the many relations with few queries are taken several per
// launch (blockIdx.z), each with its own table, so that their small sweeps fill the chip together.
struct RankRWork {                      // partitions of the caller's work buffer
    int32_t *counts, *cursor, *offsets; // [n_rel], [n_rel], [n_rel + 1]
    int32_t *perm, *gh, *gt;            // [nq]: query at each grouped position, its clamped head and tail
    float *gts;                         // [nq] grouped outputs
    int32_t *gless, *gequal;
    float *table;                       // n_tables tables of (n_ent + 1) x rel_dim: P_r, then r
    int n_tables;
    size_t total;
};
constexpr int kRankBig = 1024;          // relations with more queries than this get a launch of their own
static RankRWork rank_r_work(const stx_config &cfg, int64_t nq, void *base)
{
    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = (off + bytes + 255) / 256 * 256; return (char *)base + o; };
    RankRWork w;
    w.counts = (int32_t *)take((size_t)cfg.n_rel * 4);
    w.cursor = (int32_t *)take((size_t)cfg.n_rel * 4);
    w.offsets = (int32_t *)take((size_t)(cfg.n_rel + 1) * 4);
    w.perm = (int32_t *)take((size_t)nq * 4);
    w.gh = (int32_t *)take((size_t)nq * 4);
    w.gt = (int32_t *)take((size_t)nq * 4);
    w.gts = (float *)take((size_t)nq * 4);
    w.gless = (int32_t *)take((size_t)nq * 4);
    w.gequal = (int32_t *)take((size_t)nq * 4);
    // relations with few queries are swept several per launch, each with a table of its own: up to 32, within 256 MiB
    const size_t table_bytes = (size_t)(cfg.n_ent + 1) * cfg.rel_dim * 4;
    const size_t fit = ((size_t)256 << 20) / table_bytes;
    w.n_tables = (int)(fit < 1 ? 1 : (fit > 32 ? 32 : fit));
    if (w.n_tables > cfg.n_rel) w.n_tables = (int)cfg.n_rel;
    w.table = (float *)take(table_bytes * w.n_tables);
    w.total = off;
    return w;
}
size_t rank_work_bytes(const stx_ctx *c, int64_t nq)
{
    return c->cfg.model == STX_TRANSR ? rank_r_work(c->cfg, nq, nullptr).total : 0;
}

__global__ __launch_bounds__(kThreads) void k_rr_clear(int32_t *counts, int32_t *cursor, int n_rel)
{
    const int i = (int)blockIdx.x * kThreads + threadIdx.x;
    if (i < n_rel) { counts[i] = 0; cursor[i] = 0; }
}

__global__ __launch_bounds__(kThreads) void k_rr_hist(const int32_t *h, const int32_t *r, const int32_t *t, int64_t nq,
                                                      int32_t n_ent, int32_t n_rel, int32_t *counts, int32_t *bad)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nq) return;
    const int32_t ih = h[i], ir = r[i], it = t[i];
    if (ih < 0 || ih >= n_ent || it < 0 || it >= n_ent || ir < 0 || ir >= n_rel) atomicAdd(bad, 1);
    atomicAdd(&counts[min(max(ir, 0), n_rel - 1)], 1);
}

// offsets[i] = counts[0] + ... + counts[i-1], offsets[n_rel] = nq.  One workgroup.
__global__ __launch_bounds__(kThreads) void k_rr_scan(const int32_t *counts, int32_t *offsets, int n_rel)
{
    __shared__ int32_t s_total;
    int32_t base = 0;
    for (int i0 = 0; i0 < n_rel; i0 += kThreads) {
        const int i = i0 + (int)threadIdx.x;
        const int32_t v = i < n_rel ? counts[i] : 0;
        const int32_t ex = block_exclusive_scan(v, &s_total);
        if (i < n_rel) offsets[i] = base + ex;
        __syncthreads();
        base += s_total;
    }
    if (threadIdx.x == 0) offsets[n_rel] = base;
}

// Grouped position of every query (any order inside a relation: a query's counts do not depend on it).
__global__ __launch_bounds__(kThreads) void k_rr_scatter(const int32_t *h, const int32_t *r, const int32_t *t, int64_t nq,
                                                         int32_t n_ent, int32_t n_rel, const int32_t *offsets,
                                                         int32_t *cursor, int32_t *perm, int32_t *gh, int32_t *gt)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nq) return;
    const int32_t ir = min(max(r[i], 0), n_rel - 1);
    const int32_t pos = offsets[ir] + atomicAdd(&cursor[ir], 1);
    perm[pos] = (int32_t)i;
    gh[pos] = min(max(h[i], 0), n_ent - 1);
    gt[pos] = min(max(t[i], 0), n_ent - 1);
}

__global__ __launch_bounds__(kThreads) void k_rr_unpermute(const int32_t *perm, const float *gts, const int32_t *gless,
                                                           const int32_t *gequal, int64_t nq, float *true_score,
                                                           int32_t *n_less, int32_t *n_equal)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= nq) return;
    const int32_t q = perm[i];
    true_score[q] = gts[i];
    n_less[q] = gless[i];
    n_equal[q] = gequal[i];
}

// T[e][a] = sum_j E[e][j] M[a][j] (index order, fused multiply-adds) for e < n_ent, a < k; T[n_ent][a] = rvec[a].
// Tiled like the sweep: 128 entities x 128 outputs per workgroup, 8 x 8 per thread.
// blockIdx.z walks the relations first, first + 1, ... as in the sweep (M, rvec: the whole tables).
__global__ __launch_bounds__(kThreads, 3) void k_rr_project(const float *__restrict__ E, const float *__restrict__ M,
                                                            const float *__restrict__ rvec, int32_t n_ent, int dim, int k,
                                                            float *__restrict__ T, const int32_t *__restrict__ counts,
                                                            int32_t first, int32_t big, int64_t table_stride)
{
    {
        const int32_t g = first + (int32_t)blockIdx.z, n = counts[g];
        if (n == 0 || (gridDim.z > 1 && n > big)) return;
        M += (int64_t)g * k * dim;
        rvec += (int64_t)g * k;
        T += (int64_t)blockIdx.z * table_stride;
    }
    __shared__ __attribute__((aligned(16))) float s_m[kRankJ][kRankLd];
    __shared__ __attribute__((aligned(16))) float s_e[kRankJ][kRankLd];
    const int tid = threadIdx.x, tx = tid & 15, ty = tid >> 4;
    const int32_t e0 = (int32_t)blockIdx.x * kRankE;
    const int a0 = (int)blockIdx.y * kRankQ;
    const int sc = tid & (kRankQ - 1), sj = (tid >> 7) * 4;
    const float *pm = M + (int64_t)min(a0 + sc, k - 1) * dim;
    const float *pe = E + (int64_t)min(e0 + sc, n_ent - 1) * dim;
    if (blockIdx.x == 0 && tid < kRankQ && a0 + tid < k) T[(int64_t)n_ent * k + a0 + tid] = rvec[a0 + tid];
    float acc[8][8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
#pragma unroll
        for (int v = 0; v < 8; ++v) acc[u][v] = 0.f;
    for (int j0 = 0; j0 < dim; j0 += kRankJ) {
        float4 vm[4], ve[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int j = min(j0 + sj + 8 * i, dim - 4);
            vm[i] = ld4(pm + j); ve[i] = ld4(pe + j);
        }
        __syncthreads();
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int jj = sj + 8 * i;
            float4 m4 = vm[i], e4 = ve[i];
            if (j0 + jj >= dim) m4 = e4 = make_float4(0.f, 0.f, 0.f, 0.f);
            s_m[jj][sc] = m4.x; s_m[jj + 1][sc] = m4.y; s_m[jj + 2][sc] = m4.z; s_m[jj + 3][sc] = m4.w;
            s_e[jj][sc] = e4.x; s_e[jj + 1][sc] = e4.y; s_e[jj + 2][sc] = e4.z; s_e[jj + 3][sc] = e4.w;
        }
        __syncthreads();
#pragma unroll 4
        for (int jj = 0; jj < kRankJ; ++jj) {
            const float4 ma = *reinterpret_cast<const float4 *>(&s_m[jj][ty * 4]);
            const float4 mb = *reinterpret_cast<const float4 *>(&s_m[jj][64 + ty * 4]);
            const float4 ea = *reinterpret_cast<const float4 *>(&s_e[jj][tx * 4]);
            const float4 eb = *reinterpret_cast<const float4 *>(&s_e[jj][64 + tx * 4]);
            const float mv[8] = {ma.x, ma.y, ma.z, ma.w, mb.x, mb.y, mb.z, mb.w};
            const float ev[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
#pragma unroll
            for (int u = 0; u < 8; ++u)
#pragma unroll
                for (int v = 0; v < 8; ++v) acc[u][v] = __builtin_fmaf(ev[v], mv[u], acc[u][v]);
        }
    }
#pragma unroll
    for (int v = 0; v < 8; ++v) {
        const int32_t e = e0 + (v < 4 ? 0 : 64) + tx * 4 + (v & 3);
        if (e >= n_ent) continue;
#pragma unroll
        for (int g = 0; g < 2; ++g) {                     // the thread's outputs: two runs of four consecutive a
            const int a = a0 + g * 64 + ty * 4;
            if (a < k) st4(T + (int64_t)e * k + a, make_float4(acc[4 * g][v], acc[4 * g + 1][v], acc[4 * g + 2][v], acc[4 * g + 3][v]));
        }
    }
}

// Launch shape of one sweep: query blocks, and candidate slices of whole tiles such that enough workgroups
// exist for the last, partly filled round of them to be a small share of the run (768 fit the chip at once).
struct RankShape {
    dim3 grid, qgrid;
    int32_t slice;
};
static RankShape rank_shape(int64_t nq, int32_t n_ent, int64_t min_tiles)
{
    const int64_t qblocks = (nq + kRankQ - 1) / kRankQ;
    const int64_t tiles = ((int64_t)n_ent + kRankE - 1) / kRankE;
    int64_t slices = (32768 + qblocks - 1) / qblocks;
    if (slices > (tiles + min_tiles - 1) / min_tiles) slices = (tiles + min_tiles - 1) / min_tiles;
    if (slices > 65535) slices = 65535;
    const int32_t slice = (int32_t)((tiles + slices - 1) / slices) * kRankE;
    slices = ((int64_t)n_ent + slice - 1) / slice;
    return {dim3((unsigned)qblocks, (unsigned)slices), dim3((unsigned)((nq + kThreads - 1) / kThreads)), slice};
}

// k_rank_true, the sweep and (L2 kinds) the square root for one table and one list of queries.
static void rank_sweep(stx_ctx *c, const RankArgs &a, const RankShape &sh, bool transh, int side, int nz = 1,
                       bool finish = true)
{
    const dim3 grid(sh.grid.x, sh.grid.y, (unsigned)nz), qgrid(sh.qgrid.x, 1, (unsigned)nz);
#define STX_RANK_GO(KT, KS, D, H)                                                                               \
    do {                                                                                                        \
        hipLaunchKernelGGL((KT<D, H>), qgrid, dim3(kThreads), 0, c->stream, a);                                 \
        ProfScope prof(c, #KS);                                                                                 \
        hipLaunchKernelGGL((KS<D, H>), grid, dim3(kThreads), 0, c->stream, a);                                  \
    } while (0)
#define STX_RANK(D)                                                                                             \
    do {                                                                                                        \
        if (transh) { if (side) STX_RANK_GO(k_rank_true_h, k_rank_h, D, true); else STX_RANK_GO(k_rank_true_h, k_rank_h, D, false); } \
        else        { if (side) STX_RANK_GO(k_rank_true, k_rank, D, true); else STX_RANK_GO(k_rank_true, k_rank, D, false); }         \
        if (finish && (D == STX_L2 || D == STX_TORUS_L2))                                                       \
            hipLaunchKernelGGL((k_rank_finish<D>), qgrid, dim3(kThreads), 0, c->stream, a.true_score, a.nq);    \
    } while (0)
    switch (c->cfg.dist) {
    case STX_L1: STX_RANK(STX_L1); break;
    case STX_L2: STX_RANK(STX_L2); break;
    case STX_TORUS_L1: STX_RANK(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_RANK(STX_L2_SQ); break;
    default: STX_RANK(STX_TORUS_L2); break;
    }
#undef STX_RANK
#undef STX_RANK_GO
}

stx_status launch_rank(stx_ctx *c, const stx_params *p, const int32_t *h, const int32_t *r, const int32_t *t,
                       int64_t nq, int side, float *true_score, int32_t *n_less, int32_t *n_equal, void *work)
{
    if (nq == 0) return STX_OK;
    const int32_t n_ent = (int32_t)c->cfg.n_ent, n_rel = (int32_t)c->cfg.n_rel;
    int32_t *bad = c->ctrl + CTRL_BAD_INDEX;
    if (c->cfg.model != STX_TRANSR) {
        const bool transh = c->cfg.model == STX_TRANSH;
        const RankShape sh = rank_shape(nq, n_ent, transh ? 4 : 2);   // TransH workgroups start with a dot product per query
        const RankArgs a{p->ent, transh ? p->rel : nullptr, transh ? p->w : nullptr, h, r, t, nq, n_ent, n_rel, c->cfg.dim,
                         sh.slice, true_score, n_less, n_equal, bad, nullptr, nullptr, 0, 0, 0};
        rank_sweep(c, a, sh, transh, side);
        return hip_ok(hipGetLastError());
    }
    // TransR: group the queries by relation, learn the group sizes (the one wait of this call), then one
    // projected table and one sweep per relation that occurs
    const RankRWork w = rank_r_work(c->cfg, nq, work);
    const int dim = c->cfg.dim, k = c->cfg.rel_dim;
    const dim3 rgrid((unsigned)((n_rel + kThreads - 1) / kThreads)), qgrid((unsigned)((nq + kThreads - 1) / kThreads));
    hipLaunchKernelGGL(k_rr_clear, rgrid, dim3(kThreads), 0, c->stream, w.counts, w.cursor, n_rel);
    hipLaunchKernelGGL(k_rr_hist, qgrid, dim3(kThreads), 0, c->stream, h, r, t, nq, n_ent, n_rel, w.counts, bad);
    hipLaunchKernelGGL(k_rr_scan, dim3(1), dim3(kThreads), 0, c->stream, w.counts, w.offsets, n_rel);
    hipLaunchKernelGGL(k_rr_scatter, qgrid, dim3(kThreads), 0, c->stream, h, r, t, nq, n_ent, n_rel, w.offsets, w.cursor,
                       w.perm, w.gh, w.gt);
    int32_t *counts = new (std::nothrow) int32_t[(size_t)n_rel];
    if (!counts) return STX_ERR_BAD_ARG;
    if (hipMemcpyAsync(counts, w.counts, (size_t)n_rel * 4, hipMemcpyDeviceToHost, c->stream) != hipSuccess ||
        hipStreamSynchronize(c->stream) != hipSuccess) {
        delete[] counts;
        return STX_ERR_HIP;
    }
    const int64_t stride = (int64_t)(n_ent + 1) * k;
    // relations first, first + 1, ... first + nz - 1 in one set of launches; max_n: the largest group among them
    auto sweep = [&](int32_t first, int nz, int64_t max_n, int32_t big) {
        const dim3 pgrid((unsigned)((n_ent + kRankE - 1) / kRankE), (unsigned)((k + kRankQ - 1) / kRankQ), (unsigned)nz);
        {
            ProfScope prof(c, "k_rr_project");
            hipLaunchKernelGGL(k_rr_project, pgrid, dim3(kThreads), 0, c->stream, p->ent, p->proj, p->rel, n_ent, dim, k,
                               w.table, w.counts, first, big, stride);
        }
        const RankShape sh = rank_shape(max_n, n_ent, 2);
        const RankArgs a{w.table, nullptr, nullptr, w.gh, nullptr, w.gt, max_n, n_ent, 1, k, sh.slice, w.gts, w.gless,
                         w.gequal, bad, w.counts, w.offsets, first, big, stride};
        rank_sweep(c, a, sh, false, side, nz, false);
    };
    for (int32_t rr = 0; rr < n_rel; ++rr)
        if (counts[rr] > kRankBig) sweep(rr, 1, counts[rr], 0x7fffffff);
    for (int32_t r0 = 0; r0 < n_rel; r0 += w.n_tables) {
        const int nz = n_rel - r0 < w.n_tables ? n_rel - r0 : w.n_tables;
        int64_t max_n = 0;
        for (int z = 0; z < nz; ++z)
            if (counts[r0 + z] <= kRankBig && counts[r0 + z] > max_n) max_n = counts[r0 + z];
        if (max_n > 0) sweep(r0, nz, max_n, nz > 1 ? kRankBig : 0x7fffffff);
    }
    if (c->cfg.dist == STX_L2) hipLaunchKernelGGL((k_rank_finish<STX_L2>), qgrid, dim3(kThreads), 0, c->stream, w.gts, nq);
    if (c->cfg.dist == STX_TORUS_L2)
        hipLaunchKernelGGL((k_rank_finish<STX_TORUS_L2>), qgrid, dim3(kThreads), 0, c->stream, w.gts, nq);
    delete[] counts;
    hipLaunchKernelGGL(k_rr_unpermute, qgrid, dim3(kThreads), 0, c->stream, w.perm, w.gts, w.gless, w.gequal, nq,
                       true_score, n_less, n_equal);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
