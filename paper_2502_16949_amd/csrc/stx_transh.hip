// TransH forward, fused with the hinge and the backward pass through the hyperplane projection.
//
// SparseTransX Sec. 4.5: with x = h - t from the `ht` incidence product (Sec. 4.2.1), the translated
// vector is y = (x + d_r) - (w_r . x) w_r.  One lane group owns a positive row and its k negatives:
// it computes the distances, the margin-ranking hinge (Sec. 5.3), and then for every row writes the
// three vectors the transposed products need:
//   gy = dL/dy                                   -> summed per relation column into dL/d(d_r)
//   gx = gy - (gy . w) w                         -> summed with signs per entity column into dL/dE
//   gw = -((gy . w) x + (w . x) gy)              -> summed per relation column into dL/dw_r
#include "stx_rowops.h"

namespace stx {

template <int LPR, int ITERS, int DIST>
struct HRow {
    RowVec<ITERS> x, y;
    float s, dist;
    int32_t r;

    __device__ inline void compute(const float *__restrict__ E, const float *__restrict__ D,
                                   const float *__restrict__ W, int dim, int d4, int lig, int32_t n_ent,
                                   const int32_t *__restrict__ cols)
    {
        r = cols[1] - n_ent;
        gather_row<LPR, ITERS, false>(E, dim, d4, lig, cols[0], 0, cols[2], x);
        RowVec<ITERS> w, dr;
        load_vec<LPR, ITERS>(W + (int64_t)r * dim, d4, lig, w);
        load_vec<LPR, ITERS>(D + (int64_t)r * dim, d4, lig, dr);
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

    __device__ inline void write_grads(const float *__restrict__ W, int dim, int d4, int lig, float coef,
                                       float *__restrict__ gx_row, float *__restrict__ gy_row,
                                       float *__restrict__ gw_row) const
    {
        const float cs = coef_scale<DIST>(coef, dist);
        RowVec<ITERS> w, gy, gx, gw;
        load_vec<LPR, ITERS>(W + (int64_t)r * dim, d4, lig, w);
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

template <int LPR, int ITERS, int DIST>
__global__ __launch_bounds__(kThreads) void k_forward_transh(const int32_t *__restrict__ colidx,
                                                             const float *__restrict__ E,
                                                             const float *__restrict__ D,
                                                             const float *__restrict__ W, int32_t n_ent, int32_t b,
                                                             int32_t k, int dim, float margin, float scale,
                                                             float *__restrict__ scores, float *__restrict__ GX,
                                                             float *__restrict__ GY, float *__restrict__ GW,
                                                             float *__restrict__ loss_partials)
{
    constexpr int GROUPS = kThreads / LPR;
    __shared__ float s_loss[GROUPS];
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int64_t i = (int64_t)blockIdx.x * GROUPS + grp;
    const int d4 = dim / 4;
    float hinge_sum = 0.f;
    if (i < b) {
        HRow<LPR, ITERS, DIST> pos;
        pos.compute(E, D, W, dim, d4, lig, n_ent, colidx + 3 * i);
        if (lig == 0) scores[i] = pos.dist;
        int n_active = 0;
        for (int kk = 0; kk < k; ++kk) {
            const int64_t row = (int64_t)b + i * k + kk;
            HRow<LPR, ITERS, DIST> neg;
            neg.compute(E, D, W, dim, d4, lig, n_ent, colidx + 3 * row);
            const float arg = (margin + pos.dist) - neg.dist;
            const bool active = arg > 0.f;
            if (lig == 0) scores[row] = neg.dist;
            if (active) { hinge_sum += arg; ++n_active; }
            neg.write_grads(W, dim, d4, lig, active ? -scale : 0.f, GX + row * dim, GY + row * dim, GW + row * dim);
        }
        pos.write_grads(W, dim, d4, lig, (float)n_active * scale, GX + i * dim, GY + i * dim, GW + i * dim);
    }
    if (lig == 0) s_loss[grp] = hinge_sum;
    __syncthreads();
    if (threadIdx.x == 0) {
        float a = 0.f;
#pragma unroll
        for (int g = 0; g < GROUPS; ++g) a += s_loss[g];
        loss_partials[blockIdx.x] = a;
    }
}

template <int LPR, int ITERS>
static void transh_go(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores, float *loss,
                      float scale)
{
    constexpr int GROUPS = kThreads / LPR;
    dim3 grid((unsigned)((inc->b + GROUPS - 1) / GROUPS));
#define STX_FWD(DD)                                                                                              \
    hipLaunchKernelGGL((k_forward_transh<LPR, ITERS, DD>), grid, dim3(kThreads), 0, c->stream, inc->a_colidx,    \
                       p->ent, p->rel, p->w, (int32_t)c->cfg.n_ent, inc->b, inc->k, c->cfg.dim, c->cfg.margin,   \
                       scale, scores, c->gbuf[0], c->gbuf[1], c->gbuf[2], c->loss_partials)
    {
    ProfScope prof(c, "k_forward_transh");
    switch (c->cfg.dist) {
    case STX_L1: STX_FWD(STX_L1); break;
    case STX_L2: STX_FWD(STX_L2); break;
    case STX_TORUS_L1: STX_FWD(STX_TORUS_L1); break;
    default: STX_FWD(STX_TORUS_L2); break;
    }
    }
#undef STX_FWD
    launch_finish_loss(c, (int)grid.x, scale, loss);
}

stx_status launch_forward_transh(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores,
                                 float *loss)
{
    if (inc->n_rows == 0) return launch_finish_loss(c, 0, 1.0f, loss);
    float scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    Launch L = row_launch(c->cfg.dim);
    STX_DISPATCH_ROW(L, transh_go, c, inc, p, scores, loss, scale);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
