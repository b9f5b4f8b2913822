// Device-side body of the TransH forward step (see stx_transh.hip), shared by the kernel that runs it alone
// and by the launch that runs it beside the first pass of the sort (stx_step.hip).
#pragma once

#include "stx_rowops.h"

namespace stx {

struct TranshArgs {
    const int32_t *colidx;
    const float *E, *D, *W;
    int32_t n_ent, b, k;
    int dim;
    float margin, scale;
    float *scores, *GX, *GY, *GW;
    float *loss_partials;
};

// One row of the batch in registers: x = h - t, y, the dot product s = w . x and the distance.
template <int LPR, int ITERS, int DIST>
struct HRow {
    RowVec<ITERS> x, y;
    float s, dist;

    // h, t: the two entity rows as loaded; w, dr: the relation's normal and translation
    __device__ inline void project(const RowVec<ITERS> &h, const RowVec<ITERS> &t, const RowVec<ITERS> &w,
                                   const RowVec<ITERS> &dr)
    {
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
            x.v[it] = make_float4(h.v[it].x - t.v[it].x, h.v[it].y - t.v[it].y, h.v[it].z - t.v[it].z,
                                  h.v[it].w - t.v[it].w);
        s = group_dot<LPR, ITERS>(w, x);
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            y.v[it].x = (x.v[it].x + dr.v[it].x) - s * w.v[it].x;
            y.v[it].y = (x.v[it].y + dr.v[it].y) - s * w.v[it].y;
            y.v[it].z = (x.v[it].z + dr.v[it].z) - s * w.v[it].z;
            y.v[it].w = (x.v[it].w + dr.v[it].w) - s * w.v[it].w;
        }
        dist = row_distance<LPR, ITERS, DIST>(y);
    }

    __device__ inline void write_grads(const RowVec<ITERS> &w, int d4, int lig, float coef, float *__restrict__ gx_row,
                                       float *__restrict__ gy_row, float *__restrict__ gw_row) const
    {
        const float cs = coef_scale<DIST>(coef, dist);
        RowVec<ITERS> gy, gx, gw;
#pragma unroll
        for (int it = 0; it < ITERS; ++it)
            gy.v[it] = make_float4(dterm<DIST>(y.v[it].x, cs), dterm<DIST>(y.v[it].y, cs),
                                   dterm<DIST>(y.v[it].z, cs), dterm<DIST>(y.v[it].w, cs));
        const float a = group_dot<LPR, ITERS>(gy, w);
#pragma unroll
        for (int it = 0; it < ITERS; ++it) {
            gx.v[it] = make_float4(gy.v[it].x - a * w.v[it].x, gy.v[it].y - a * w.v[it].y,
                                   gy.v[it].z - a * w.v[it].z, gy.v[it].w - a * w.v[it].w);
            gw.v[it] = make_float4(-(a * x.v[it].x + s * gy.v[it].x), -(a * x.v[it].y + s * gy.v[it].y),
                                   -(a * x.v[it].z + s * gy.v[it].z), -(a * x.v[it].w + s * gy.v[it].w));
        }
        store_vec<LPR, ITERS>(gx_row, d4, lig, gx);
        store_vec<LPR, ITERS>(gy_row, d4, lig, gy);
        store_vec<LPR, ITERS>(gw_row, d4, lig, gw);
    }
};

// One lane group per positive i and its k negatives (rows b + i*k + kk).  A corrupted triplet keeps the
// relation of its positive (the build writes the batch that way), so w_r and d_r are fetched once per
// group; the negatives are taken NB at a time so that their column ids, then their entity rows, are
// in flight together.  `block` is the index of the workgroup among those of the forward pass.
// K1: at most one negative per positive (the benchmarks' shape): no registers are kept for a batch of them.
template <int LPR, int ITERS, int DIST, bool K1 = false>
__device__ inline void forward_transh_body(const int block, const TranshArgs &a)
{
    constexpr int GROUPS = kThreads / LPR;
    constexpr int NB = K1 ? 1 : (ITERS <= 2 ? 4 : 2);
    __shared__ float s_loss[GROUPS];
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int64_t i = (int64_t)block * GROUPS + grp;
    const int dim = a.dim, d4 = dim / 4;
    const int32_t b = a.b, k = a.k;
    float hinge_sum = 0.f;
    if (i < b) {
        const int32_t *__restrict__ colidx = a.colidx;
        const int32_t ch = colidx[3 * i], cr = colidx[3 * i + 1] - a.n_ent, ct = colidx[3 * i + 2];
        RowVec<ITERS> w, dr;
        HRow<LPR, ITERS, DIST> pos;
        int n_active = 0;
        for (int kk0 = 0; kk0 < k || kk0 == 0; kk0 += NB) {
            const int nb = min(NB, k - kk0);
            const int64_t row0 = (int64_t)b + i * k + kk0;
            int32_t cn[NB][2];
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                const int64_t rr = q < nb ? row0 + q : i;   // past the end: the positive's ids again
                cn[q][0] = colidx[3 * rr]; cn[q][1] = colidx[3 * rr + 2];
            }
            RowVec<ITERS> ph, pt, nh[NB], nt[NB];
            if (kk0 == 0) {
                load_vec<LPR, ITERS>(a.E + (int64_t)ch * dim, d4, lig, ph);
                load_vec<LPR, ITERS>(a.E + (int64_t)ct * dim, d4, lig, pt);
                load_vec<LPR, ITERS>(a.W + (int64_t)cr * dim, d4, lig, w);
                load_vec<LPR, ITERS>(a.D + (int64_t)cr * dim, d4, lig, dr);
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                if (q < nb) {
                    load_vec<LPR, ITERS>(a.E + (int64_t)cn[q][0] * dim, d4, lig, nh[q]);
                    load_vec<LPR, ITERS>(a.E + (int64_t)cn[q][1] * dim, d4, lig, nt[q]);
                }
            }
            if (kk0 == 0) {
                pos.project(ph, pt, w, dr);
                if (lig == 0) a.scores[i] = pos.dist;
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                if (q < nb) {
                    const int64_t row = row0 + q;
                    HRow<LPR, ITERS, DIST> neg;
                    neg.project(nh[q], nt[q], w, dr);
                    const float arg = (a.margin + pos.dist) - neg.dist;
                    const bool active = arg > 0.f;
                    if (lig == 0) a.scores[row] = neg.dist;
                    if (active) { hinge_sum += arg; ++n_active; }
                    neg.write_grads(w, d4, lig, active ? -a.scale : 0.f, a.GX + row * dim, a.GY + row * dim,
                                    a.GW + row * dim);
                }
            }
        }
        pos.write_grads(w, d4, lig, (float)n_active * a.scale, a.GX + i * dim, a.GY + i * dim, a.GW + i * dim);
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

}  // namespace stx
