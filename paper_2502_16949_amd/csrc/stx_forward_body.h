// Device-side bodies of the fused TransE / TorusE forward step and of the final loss sum, shared by the
// kernels that run them alone (stx_forward.hip) and by the launches that run them beside another,
// independent piece of work (stx_step.hip).
#pragma once

#include "stx_rowops.h"

namespace stx {

// Packed dL/dy row of an L1-kind distance: record `row` of gs = coefficient (fp32), then the sign bytes.
template <int LPR, int ITERS, int DIST>
__device__ inline void write_grad_row_packed(uint8_t *__restrict__ gs, int gstride, float *__restrict__ coefs,
                                             int64_t row, int d4, int lig, const RowVec<ITERS> &x, float coef)
{
    uint8_t *rec = gs + row * gstride;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) rec[j] = (uint8_t)sign_bits<DIST>(x.v[it]);
    }
    if (lig == 0) coefs[row] = coef;
}

template <int LPR, int ITERS, int DIST>
__device__ inline void write_grad_row(float *__restrict__ g, int d4, int lig, const RowVec<ITERS> &x, float coef,
                                      float dist)
{
    const float cs = coef_scale<DIST>(coef, dist);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4)
            st4(g + 4 * j, make_float4(dterm<DIST>(x.v[it].x, cs), dterm<DIST>(x.v[it].y, cs),
                                       dterm<DIST>(x.v[it].z, cs), dterm<DIST>(x.v[it].w, cs)));
    }
}

// Sum of the per-workgroup loss partials in a fixed order (one workgroup, after the forward kernel).
// ARENA: the body's LDS array lives in the kFinishLds bytes at `lds` (8-byte aligned) instead of its own.
template <bool ARENA = false>
__device__ inline void finish_loss_body(const float *__restrict__ partials, int n, float scale,
                                        float *__restrict__ loss, unsigned char *lds = nullptr)
{
    double *s_acc;
    if constexpr (ARENA) {
        s_acc = reinterpret_cast<double *>(lds);
    } else {
        __shared__ double o_acc[kThreads];
        s_acc = o_acc;
    }
    const int tid = threadIdx.x;
    double a = 0.0;
    int i = tid;
    for (; i + 7 * kThreads < n; i += 8 * kThreads) {   // eight loads in flight, added in index order
        float v[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) v[u] = partials[i + u * kThreads];
#pragma unroll
        for (int u = 0; u < 8; ++u) a += (double)v[u];
    }
    for (; i < n; i += kThreads) a += (double)partials[i];
    s_acc[tid] = a;
    __syncthreads();
    for (int off = kThreads / 2; off >= 1; off >>= 1) {
        if (tid < off) s_acc[tid] += s_acc[tid + off];
        __syncthreads();
    }
    if (tid == 0) loss[0] = (float)(s_acc[0] * (double)scale);
}

// The forward step for batches whose negatives come from the sampler (Sec. 5.3: every negative keeps the relation
// and one entity of its positive), at most NB negatives per positive.  One group per positive: its lanes fetch the
// 3 + 3k column ids in ONE load (lane s < 3: id s of the positive; lane 3 + 3q + s: id s of negative q) and share
// them by shuffles; then the positive's three rows and the ONE row in which each negative differs are requested
// together (3 + k table rows instead of 3 + 3k), so a wavefront pays two dependent memory round trips in all.
// x is formed by the same two roundings in the same order as a full gather would: the bits are those of
// forward_stacked_body.  A group that finds another kind of negative (a caller's own) does nothing and stores
// `serial` in *general_flag: the caller then runs the general kernel over those groups.
template <int LPR, int ITERS, int DIST, bool PACKED, int NB>
__device__ inline void forward_fast_body(const int block, const ForwardArgs &a, int32_t *general_flag, int32_t serial)
{
    static_assert(LPR >= 3 + 3 * NB, "one lane per column id");
    const int32_t *__restrict__ colidx = a.colidx;
    const float *__restrict__ X = a.X;
    const int32_t b = a.b, k = a.k;
    const int dim = a.dim, d4 = dim / 4, gstride = a.gstride;
    float *__restrict__ scores = a.scores;
    constexpr int GROUPS = kThreads / LPR;
    __shared__ float s_loss[GROUPS];
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int32_t i = block * GROUPS + grp;
    float hinge_sum = 0.f;
    if (i < b) {
        const int32_t row0 = b + i * k;
        int32_t mine = 0;
        if (lig < 3 + 3 * k) mine = colidx[lig < 3 ? 3 * (int64_t)i + lig : 3 * (int64_t)row0 + (lig - 3)];
        const int32_t c0 = __shfl(mine, 0, LPR), c1 = __shfl(mine, 1, LPR), c2 = __shfl(mine, 2, LPR);
        int32_t ce[NB];
        unsigned tail_mask = 0;
        bool shared = true;
#pragma unroll
        for (int q = 0; q < NB; ++q) {
            const int32_t nh = __shfl(mine, 3 + 3 * q, LPR), nr = __shfl(mine, 4 + 3 * q, LPR), nt = __shfl(mine, 5 + 3 * q, LPR);
            const bool ts = nh == c0;
            ce[q] = ts ? nt : nh;
            tail_mask |= ts ? 1u << q : 0u;
            if (q < k) shared = shared && nr == c1 && (ts || nt == c2);
        }
        if (shared) {
            const float wr = a.rel_weight ? a.rel_weight[c1 - a.n_ent] : 1.0f;
            // (lanes past the row's width hold zeros and take part in the reductions only)
            RowVec<ITERS> hr, pr, pt, e[NB];
            load_vec<LPR, ITERS>(X + (int64_t)c0 * dim, d4, lig, hr);
            load_vec<LPR, ITERS>(X + (int64_t)c1 * dim, d4, lig, pr);
            load_vec<LPR, ITERS>(X + (int64_t)c2 * dim, d4, lig, pt);
#pragma unroll
            for (int q = 0; q < NB; ++q)
                if (q < k) {
                    // a row used once does not displace the others when the table is far larger than the caches
                    if (a.stream_rows) load_vec_stream<LPR, ITERS>(X + (int64_t)ce[q] * dim, d4, lig, e[q]);
                    else load_vec<LPR, ITERS>(X + (int64_t)ce[q] * dim, d4, lig, e[q]);
                }
            RowVec<ITERS> x;
#pragma unroll
            for (int it = 0; it < ITERS; ++it) {
                hr.v[it] = add4(hr.v[it], pr.v[it]);
                x.v[it] = sub4(hr.v[it], pt.v[it]);
            }
            const float npos = row_distance<LPR, ITERS, DIST>(x);
            const float dpos = wr * npos;
            if (lig == 0) scores[i] = dpos;
            uint8_t *recs = reinterpret_cast<uint8_t *>(a.G);
            float *gcoef = PACKED ? reinterpret_cast<float *>(recs + packed_coef_offset((int64_t)b * (1 + k), gstride)) : nullptr;
            int n_active = 0;
            const RowVec<ITERS> xp = x;
#pragma unroll
            for (int q = 0; q < NB; ++q)
                if (q < k) {
#pragma unroll
                    for (int it = 0; it < ITERS; ++it)
                        x.v[it] = (tail_mask >> q & 1u) ? sub4(hr.v[it], e[q].v[it]) : sub4(add4(e[q].v[it], pr.v[it]), pt.v[it]);
                    const float nneg = row_distance<LPR, ITERS, DIST>(x);
                    const float dneg = wr * nneg;
                    const float arg = (a.margin + dpos) - dneg;
                    const bool active = arg > 0.f;
                    const int32_t row = row0 + q;
                    if (lig == 0) scores[row] = dneg;
                    if (active) { hinge_sum += arg; ++n_active; }
                    if (PACKED)
                        write_grad_row_packed<LPR, ITERS, DIST>(recs, gstride, gcoef, row, d4, lig, x, active ? -a.scale * wr : 0.f);
                    else
                        write_grad_row<LPR, ITERS, DIST>(a.G + (int64_t)row * dim, d4, lig, x, active ? -a.scale * wr : 0.f, nneg);
                }
            if (PACKED)
                write_grad_row_packed<LPR, ITERS, DIST>(recs, gstride, gcoef, i, d4, lig, xp, (float)n_active * a.scale * wr);
            else
                write_grad_row<LPR, ITERS, DIST>(a.G + (int64_t)i * dim, d4, lig, xp, (float)n_active * a.scale * wr, npos);
        } else if (lig == 0 && general_flag) {
            *general_flag = serial;
        }
    }
    if (lig == 0) s_loss[grp] = hinge_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float sum = 0.f;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) sum += s_loss[g];
        a.loss_partials[block] = sum;
    }
}

// One group per positive i: rows i and b + i*k + kk (kk < k).
// FROM_Y = false: the translated vector of a row is gathered from the stacked table X (TransE/TorusE).
// FROM_Y = true : it is row `row` of the dense buffer G (TransR: y = M_r (h - t) + r was put there by
//                 the projection kernel), and dL/dy overwrites it in place; every row is read and then
//                 written by one group only.
// PACKED (L1 kinds, gathered rows only): dL/dx is written as records of gstride bytes at G (sign bytes), the
// rows' coefficients behind the records of the batch.
// `block` is the index of the workgroup among those of the forward pass (the launch may hold others).
// K1: at most one negative per positive (the benchmarks' shape): no registers are kept for a batch of them, and
// more wavefronts fit (same arithmetic in the same order, so the same bits).
template <int LPR, int ITERS, int DIST, bool FROM_Y, bool PACKED, bool K1 = false>
__device__ inline void forward_stacked_body(const int block, const ForwardArgs &a)
{
    const int32_t *__restrict__ colidx = a.colidx;
    const float *__restrict__ X = a.X;
    const int32_t b = a.b, k = a.k;
    const int dim = a.dim, gstride = a.gstride;
    const float margin = a.margin, scale = a.scale;
    float *__restrict__ scores = a.scores;
    float *G = a.G;
    float *gcoef = PACKED ? reinterpret_cast<float *>(reinterpret_cast<uint8_t *>(a.G) +
                                                      packed_coef_offset((int64_t)b * (1 + k), gstride))
                          : nullptr;
    float *__restrict__ loss_partials = a.loss_partials;
    static_assert(!PACKED || (is_sign_kind(DIST) && !FROM_Y), "packed rows need an L1-kind distance");
    constexpr int GROUPS = kThreads / LPR;
    __shared__ float s_loss[GROUPS];
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int64_t i = (int64_t)block * GROUPS + grp;
    const int d4 = dim / 4;
    float hinge_sum = 0.f;
    if (i < b) {   // uniform within the group; shuffles below stay inside the group
        // Negatives are taken NB at a time so that the kernel pays two memory round trips per batch (all
        // column ids, then all table rows) instead of two per row; the positive rides with the first batch.
        constexpr int NB = K1 ? 1 : (ITERS <= 2 ? 4 : 2);
        RowVec<ITERS> xp;
        float dpos = 0.f, npos = 0.f;   // the positive's score and its norm (they differ by the relation's weight)
        int n_active = 0;
        int32_t cp[3] = {0, 0, 0};
        if (!FROM_Y) { cp[0] = colidx[3 * i]; cp[1] = colidx[3 * i + 1]; cp[2] = colidx[3 * i + 2]; }
        // Table 2, TransM row: a fixed weight per relation multiplies the norm (1 when there is none; the
        // negatives of a positive keep its relation).  Multiplying by 1 changes no bit.
        const float wr = (!FROM_Y && a.rel_weight) ? a.rel_weight[cp[1] - a.n_ent] : 1.0f;
        for (int kk0 = 0; kk0 < k || kk0 == 0; kk0 += NB) {
            const int nb = min(NB, k - kk0);
            const int64_t row0 = (int64_t)b + i * k + kk0;
            int32_t cn[NB][3];
            RowVec<ITERS> xn[NB];
            if (!FROM_Y) {
#pragma unroll
                for (int q = 0; q < NB; ++q) {
                    const int64_t rr = q < nb ? row0 + q : i;   // past the end: re-read the positive's ids
                    cn[q][0] = colidx[3 * rr]; cn[q][1] = colidx[3 * rr + 1]; cn[q][2] = colidx[3 * rr + 2];
                }
            }
            if (kk0 == 0) {
                if (FROM_Y) load_vec<LPR, ITERS>(G + i * dim, d4, lig, xp);
                else gather_row<LPR, ITERS, true>(X, dim, d4, lig, cp[0], cp[1], cp[2], xp);
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                if (q < nb) {
                    if (FROM_Y) load_vec<LPR, ITERS>(G + (row0 + q) * dim, d4, lig, xn[q]);
                    else gather_row<LPR, ITERS, true>(X, dim, d4, lig, cn[q][0], cn[q][1], cn[q][2], xn[q]);
                }
            }
            if (kk0 == 0) {
                npos = row_distance<LPR, ITERS, DIST>(xp);
                dpos = wr * npos;
                if (lig == 0) scores[i] = dpos;
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                if (q < nb) {
                    const int64_t row = row0 + q;
                    const float nneg = row_distance<LPR, ITERS, DIST>(xn[q]);
                    const float dneg = wr * nneg;
                    const float arg = (margin + dpos) - dneg;
                    const bool active = arg > 0.f;
                    if (lig == 0) scores[row] = dneg;
                    if (active) { hinge_sum += arg; ++n_active; }
                    if (PACKED)
                        write_grad_row_packed<LPR, ITERS, DIST>(reinterpret_cast<uint8_t *>(G), gstride, gcoef, row, d4,
                                                                lig, xn[q], active ? -scale * wr : 0.f);
                    else
                        write_grad_row<LPR, ITERS, DIST>(G + row * dim, d4, lig, xn[q], active ? -scale * wr : 0.f,
                                                         nneg);
                }
            }
        }
        if (PACKED)
            write_grad_row_packed<LPR, ITERS, DIST>(reinterpret_cast<uint8_t *>(G), gstride, gcoef, i, d4, lig, xp,
                                                    (float)n_active * scale * wr);
        else
            write_grad_row<LPR, ITERS, DIST>(G + i * dim, d4, lig, xp, (float)n_active * scale * wr, npos);
    }
    if (lig == 0) s_loss[grp] = hinge_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float sum = 0.f;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) sum += s_loss[g];
        loss_partials[block] = sum;
    }
}

}  // namespace stx

namespace stx {

// Most negatives per positive that forward_fast_body takes with groups of LPR lanes (one lane per column id) and
// ITERS float4 per lane (wide rows: one, or the rows in flight would not fit the registers).
template <int LPR, int ITERS = 1>
constexpr int fast_negatives() { return (LPR >= 16 && ITERS == 1) ? 4 : 1; }

// The forward step inside the launches of stx_train_step, whose negatives are the sampler's: the fast body where the
// row width and the number of negatives allow it.  K1: the launch was chosen for at most one negative per positive.
template <int LPR, int ITERS, int DIST, bool PACKED, bool K1>
__device__ inline void forward_step_body(const int block, const ForwardArgs &fa)
{
    if constexpr (ITERS == 1 && K1) {
        forward_fast_body<LPR, 1, DIST, PACKED, 1>(block, fa, nullptr, 0);
    } else if constexpr (ITERS == 1 && LPR >= 16) {
        if (fa.k <= 4) forward_fast_body<LPR, 1, DIST, PACKED, 4>(block, fa, nullptr, 0);
        else forward_stacked_body<LPR, ITERS, DIST, false, PACKED, K1>(block, fa);
    } else {
        forward_stacked_body<LPR, ITERS, DIST, false, PACKED, K1>(block, fa);
    }
}

}  // namespace stx
