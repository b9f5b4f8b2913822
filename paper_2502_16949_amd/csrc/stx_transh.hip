// TransH forward, fused with the hinge and the backward pass through the hyperplane projection.
//
// SparseTransX Sec. 4.5: with x = h - t from the `ht` incidence product (Sec. 4.2.1), the translated
// vector is y = (x + d_r) - (w_r . x) w_r.  One lane group owns a positive row and its k negatives:
// it computes the distances, the margin-ranking hinge (Sec. 5.3), and then for every row writes the
// three vectors the transposed products need:
//   gy = dL/dy                                   -> summed per relation column into dL/d(d_r)
//   gx = gy - (gy . w) w                         -> summed with signs per entity column into dL/dE
//   gw = -((gy . w) x + (w . x) gy)              -> summed per relation column into dL/dw_r
#include "stx_transh_body.h"

namespace stx {

template <int LPR, int ITERS, int DIST>
__global__ __launch_bounds__(kThreads) void k_forward_transh(TranshArgs a)
{
    forward_transh_body<LPR, ITERS, DIST>((int)blockIdx.x, a);
}

template <int LPR, int ITERS>
static void transh_go(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores, float *loss,
                      float scale)
{
    constexpr int GROUPS = kThreads / LPR;
    dim3 grid((unsigned)((inc->b + GROUPS - 1) / GROUPS));
    const TranshArgs ta{inc->a_colidx, p->ent, p->rel, p->w, (int32_t)c->cfg.n_ent, inc->b, inc->k, c->cfg.dim,
                        c->cfg.margin, scale, scores, c->gbuf[0], c->gbuf[1], c->gbuf[2], c->loss_partials};
#define STX_FWD(DD)                                                                                              \
    hipLaunchKernelGGL((k_forward_transh<LPR, ITERS, DD>), grid, dim3(kThreads), 0, c->stream, ta)
    {
    ProfScope prof(c, "k_forward_transh");
    switch (c->cfg.dist) {
    case STX_L1: STX_FWD(STX_L1); break;
    case STX_L2: STX_FWD(STX_L2); break;
    case STX_TORUS_L1: STX_FWD(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_FWD(STX_L2_SQ); break;
    default: STX_FWD(STX_TORUS_L2); break;
    }
    }
#undef STX_FWD
    if (c->defer_finish) { c->fin_n = (int)grid.x; c->fin_scale = scale; c->fin_loss = loss; }
    else launch_finish_loss(c, (int)grid.x, scale, loss);
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
