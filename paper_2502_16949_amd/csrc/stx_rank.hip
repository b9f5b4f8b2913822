// Link prediction by exhaustive scoring for TransE / TorusE: how many entities score below (and exactly
// like) the true entity of each test triplet.
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
    const float f = y - floorf(y);
    const float m = fminf(f, 1.0f - f);
    return DIST == STX_TORUS_L1 ? acc + m : __builtin_fmaf(m, m, acc);
}

struct RankArgs {
    const float *X;                    // [E;R], rows of dim floats
    const int32_t *h, *r, *t;          // [nq]
    int64_t nq;
    int32_t n_ent, n_rel;
    int dim;
    int32_t slice;                     // candidates per blockIdx.y, a multiple of kRankE
    float *true_score;                 // [nq]
    int32_t *n_less, *n_equal;         // [nq], zeroed before the launch
    int32_t *bad;                      // counter of out-of-range indices
};

__global__ __launch_bounds__(kThreads) void k_rank_clear(int32_t *a, int32_t *b, int64_t n)
{
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i < n) { a[i] = 0; b[i] = 0; }
}

template <int DIST, bool HEAD>
__global__ __launch_bounds__(kThreads) void k_rank(RankArgs a)
{
    __shared__ __attribute__((aligned(16))) float s_q[kRankJ][kRankLd];
    __shared__ __attribute__((aligned(16))) float s_e[kRankJ][kRankLd];
    __shared__ float s_true[kRankQ];

    const int tid = threadIdx.x;
    const int tx = tid & 15, ty = tid >> 4;               // candidate / query position of the 8 x 8 block
    const int64_t q0 = (int64_t)blockIdx.x * kRankQ;
    const int dim = a.dim;

    // The query this thread stages (and, in the first half of the workgroup, scores against its true entity).
    // Past the end the last query is repeated; its counts are not stored.
    const int sc = tid & (kRankQ - 1);                    // staged query / candidate of this thread
    const int sj = (tid >> 7) * 4;                        // first float of its float4 inside a chunk (then + 8 i)
    const int64_t qi = min(q0 + sc, a.nq - 1);
    int32_t ih = a.h[qi], ir = a.r[qi], it = a.t[qi];
    if (blockIdx.y == 0 && tid < kRankQ && q0 + sc < a.nq &&
        (ih < 0 || ih >= a.n_ent || it < 0 || it >= a.n_ent || ir < 0 || ir >= a.n_rel))
        atomicAdd(a.bad, 1);
    ih = min(max(ih, 0), a.n_ent - 1);
    it = min(max(it, 0), a.n_ent - 1);
    ir = min(max(ir, 0), a.n_rel - 1);
    // q = h + r (tail side) or t - r (head side); the true entity is t or h
    const float *pa = a.X + (int64_t)(HEAD ? it : ih) * dim;
    const float *pr = a.X + ((int64_t)a.n_ent + ir) * dim;
    const float *ptrue = a.X + (int64_t)(HEAD ? ih : it) * dim;

    if (tid < kRankQ) {
        float acc = 0.f;
        for (int j = 0; j < dim; j += 4) {
            const float4 va = ld4(pa + j), vr = ld4(pr + j), ve = ld4(ptrue + j);
            const float av[4] = {va.x, va.y, va.z, va.w}, rv[4] = {vr.x, vr.y, vr.z, vr.w};
            const float ev[4] = {ve.x, ve.y, ve.z, ve.w};
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const float q = HEAD ? av[u] - rv[u] : av[u] + rv[u];
                acc = rank_step<DIST>(acc, HEAD ? ev[u] - q : q - ev[u]);
            }
        }
        s_true[tid] = acc;
        if (blockIdx.y == 0 && q0 + tid < a.nq) a.true_score[q0 + tid] = finish<DIST>(acc);
    }
    __syncthreads();
    float tr[8];
#pragma unroll
    for (int u = 0; u < 8; ++u) tr[u] = s_true[(u < 4 ? 0 : 64) + ty * 4 + (u & 3)];

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
            __syncthreads();                              // the previous chunk has been consumed
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int jj = sj + 8 * i, j = j0 + jj;
                float4 q4 = make_float4(0.f, 0.f, 0.f, 0.f), e4 = q4;   // past the row's end: zeros add nothing
                if (j < dim) {
                    const float4 va = ld4(pa + j), vr = ld4(pr + j);
                    q4 = HEAD ? make_float4(va.x - vr.x, va.y - vr.y, va.z - vr.z, va.w - vr.w)
                              : make_float4(va.x + vr.x, va.y + vr.y, va.z + vr.z, va.w + vr.w);
                    e4 = ld4(pe + j);
                }
                s_q[jj][sc] = q4.x; s_q[jj + 1][sc] = q4.y; s_q[jj + 2][sc] = q4.z; s_q[jj + 3][sc] = q4.w;
                s_e[jj][sc] = e4.x; s_e[jj + 1][sc] = e4.y; s_e[jj + 2][sc] = e4.z; s_e[jj + 3][sc] = e4.w;
            }
            __syncthreads();
#pragma unroll 4
            for (int jj = 0; jj < kRankJ; ++jj) {
                const float4 qa = *reinterpret_cast<const float4 *>(&s_q[jj][ty * 4]);
                const float4 qb = *reinterpret_cast<const float4 *>(&s_q[jj][64 + ty * 4]);
                const float4 ea = *reinterpret_cast<const float4 *>(&s_e[jj][tx * 4]);
                const float4 eb = *reinterpret_cast<const float4 *>(&s_e[jj][64 + tx * 4]);
                const float qv[8] = {qa.x, qa.y, qa.z, qa.w, qb.x, qb.y, qb.z, qb.w};
                const float ev[8] = {ea.x, ea.y, ea.z, ea.w, eb.x, eb.y, eb.z, eb.w};
#pragma unroll
                for (int u = 0; u < 8; ++u)
#pragma unroll
                    for (int v = 0; v < 8; ++v)
                        acc[u][v] = rank_step<DIST>(acc[u][v], HEAD ? ev[v] - qv[u] : qv[u] - ev[v]);
            }
        }
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
    // the 16 threads that share a query block sit in consecutive lanes
#pragma unroll
    for (int u = 0; u < 8; ++u) {
#pragma unroll
        for (int m = 8; m >= 1; m >>= 1) {
            less[u] += __shfl_xor(less[u], m, 16);
            equal[u] += __shfl_xor(equal[u], m, 16);
        }
        const int64_t q = q0 + (u < 4 ? 0 : 64) + ty * 4 + (u & 3);
        if (tx == 0 && q < a.nq) {
            atomicAdd(&a.n_less[q], less[u]);
            atomicAdd(&a.n_equal[q], equal[u]);
        }
    }
}

stx_status launch_rank(stx_ctx *c, const stx_params *p, const int32_t *h, const int32_t *r, const int32_t *t,
                       int64_t nq, int side, float *true_score, int32_t *n_less, int32_t *n_equal)
{
    if (nq == 0) return STX_OK;
    const int32_t n_ent = (int32_t)c->cfg.n_ent;
    const int64_t qblocks = (nq + kRankQ - 1) / kRankQ;
    // Candidate slices: enough workgroups to fill the chip several times over, but whole tiles per slice.
    const int64_t tiles = ((int64_t)n_ent + kRankE - 1) / kRankE;
    int64_t slices = (4096 + qblocks - 1) / qblocks;
    if (slices > tiles) slices = tiles;
    if (slices > 65535) slices = 65535;
    const int32_t slice = (int32_t)((tiles + slices - 1) / slices) * kRankE;
    slices = ((int64_t)n_ent + slice - 1) / slice;
    hipLaunchKernelGGL(k_rank_clear, dim3((unsigned)((nq + kThreads - 1) / kThreads)), dim3(kThreads), 0, c->stream,
                       n_less, n_equal, nq);
    const RankArgs a{p->ent, h, r, t, nq, n_ent, (int32_t)c->cfg.n_rel, c->cfg.dim, slice, true_score, n_less, n_equal,
                     c->ctrl + CTRL_BAD_INDEX};
    const dim3 grid((unsigned)qblocks, (unsigned)slices);
#define STX_RANK(D)                                                                                             \
    do {                                                                                                        \
        ProfScope prof(c, "k_rank");                                                                            \
        if (side) hipLaunchKernelGGL((k_rank<D, true>), grid, dim3(kThreads), 0, c->stream, a);                 \
        else hipLaunchKernelGGL((k_rank<D, false>), grid, dim3(kThreads), 0, c->stream, a);                     \
    } while (0)
    switch (c->cfg.dist) {
    case STX_L1: STX_RANK(STX_L1); break;
    case STX_L2: STX_RANK(STX_L2); break;
    case STX_TORUS_L1: STX_RANK(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_RANK(STX_L2_SQ); break;
    default: STX_RANK(STX_TORUS_L2); break;
    }
#undef STX_RANK
    return hip_ok(hipGetLastError());
}

}  // namespace stx
