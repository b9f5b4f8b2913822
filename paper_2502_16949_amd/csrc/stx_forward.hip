// Forward product C = A.X and the fused TransE / TorusE forward step.
//
// Every row of the incidence matrix A has exactly three entries (SparseTransX Sec. 4.2.2, Appendix B),
// so the sparse-dense product is a three-row gather: x_i = (X[h] + X[n_ent + r]) - X[t], with the `ht`
// form (Sec. 4.2.1) dropping the middle term.  A sub-wavefront group of LPR lanes owns one row and
// moves it as float4 per lane, so a 128-wide fp32 row is one 512-byte coalesced access by 32 lanes.
//
// The fused forward kernel gives one group a positive row and its k negatives: it computes the
// distances (Sec. 4.3, 4.6), the margin-ranking hinge (Sec. 5.3) and writes dL/dx of each of those
// rows straight away, so x itself never goes to memory.
#include "stx_emit_body.h"
#include "stx_forward_body.h"

namespace stx {

template <int LPR, int ITERS, bool HRT>
__global__ __launch_bounds__(kThreads) void k_spmm(const int32_t *__restrict__ colidx, const float *__restrict__ X,
                                                   int64_t n_rows, int dim, int32_t rel_off, float *__restrict__ C)
{
    const int lig = threadIdx.x % LPR;
    const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    if (row >= n_rows) return;
    const int d4 = dim / 4;
    int32_t c0 = colidx[3 * row], c1 = colidx[3 * row + 1] - rel_off, c2 = colidx[3 * row + 2];
    RowVec<ITERS> x;
    gather_row<LPR, ITERS, HRT>(X, dim, d4, lig, c0, c1, c2, x);
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) st4(C + row * dim + 4 * j, x.v[it]);
    }
}

__global__ __launch_bounds__(kThreads) void k_finish_loss(const float *__restrict__ partials, int n, float scale,
                                                          float *__restrict__ loss)
{
    finish_loss_body(partials, n, scale, loss);
}

template <int LPR, int ITERS, int DIST, bool FROM_Y, bool PACKED>
__global__ __launch_bounds__(kThreads, ITERS == 1 ? 8 : 1) void k_forward_stacked(ForwardArgs a)
{
    forward_stacked_body<LPR, ITERS, DIST, FROM_Y, PACKED>((int)blockIdx.x, a);
}

// TransR in stx_train_step: the first kernel of the next batch's build (which also counts the rows per relation)
// rides with the distances over the rows of y; nothing after this launch reads the A arrays it overwrites.
template <int LPR, int ITERS, int DIST>
__global__ __launch_bounds__(kThreads) void k_forward_y_emit(ForwardArgs a, EmitAhead ea)
{
    if ((int)blockIdx.x < ea.ntiles) emit_body<kSortItems, true, true, true>((int)blockIdx.x, ea.ntiles, ea.args);
    else forward_stacked_body<LPR, ITERS, DIST, true, false>((int)blockIdx.x - ea.ntiles, a);
}

__global__ void k_zero_loss(float *loss) { loss[0] = 0.f; }

__global__ __launch_bounds__(kThreads) void k_copy_f32(float *__restrict__ dst, const float *__restrict__ src, int64_t n4)
{
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n4; i += (int64_t)gridDim.x * kThreads)
        st4(dst + 4 * i, ld4(src + 4 * i));
}

stx_status launch_copy_f32(stx_ctx *c, float *dst, const float *src, int64_t n)
{
    if (n == 0) return STX_OK;
    int64_t n4 = n / 4, blocks = (n4 + kThreads - 1) / kThreads;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_copy_f32, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, dst, src, n4);
    return hip_ok(hipGetLastError());
}

stx_status launch_finish_loss(stx_ctx *c, int n_partials, float scale, float *loss)
{
    if (n_partials <= 0) hipLaunchKernelGGL(k_zero_loss, dim3(1), dim3(1), 0, c->stream, loss);
    else {
        ProfScope prof(c, "k_finish_loss");
        hipLaunchKernelGGL(k_finish_loss, dim3(1), dim3(kThreads), 0, c->stream, c->loss_partials, n_partials, scale,
                           loss);
    }
    return hip_ok(hipGetLastError());
}

// ---- dispatch --------------------------------------------------------------------------------------
template <int LPR, int ITERS>
static void spmm_go(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *out, bool hrt)
{
    int64_t threads = inc->n_rows * LPR;
    dim3 grid((unsigned)((threads + kThreads - 1) / kThreads));
    if (hrt)
        hipLaunchKernelGGL((k_spmm<LPR, ITERS, true>), grid, dim3(kThreads), 0, c->stream, inc->a_colidx, p->ent,
                           inc->n_rows, c->cfg.dim, 0, out);
    else
        hipLaunchKernelGGL((k_spmm<LPR, ITERS, false>), grid, dim3(kThreads), 0, c->stream, inc->a_colidx, p->ent,
                           inc->n_rows, c->cfg.dim, 0, out);
}

stx_status launch_spmm(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *out)
{
    if (inc->n_rows == 0) return STX_OK;
    Launch L = row_launch(c->cfg.dim);
    bool hrt = c->cfg.model == STX_TRANSE || c->cfg.model == STX_TORUSE;
    STX_DISPATCH_ROW(L, spmm_go, c, inc, p, out, hrt);
    return hip_ok(hipGetLastError());
}

template <int LPR, int ITERS>
static void forward_go(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores, float *loss,
                       float scale, bool from_y, int width)
{
    constexpr int GROUPS = kThreads / LPR;
    dim3 grid((unsigned)((inc->b + GROUPS - 1) / GROUPS));
    const ForwardArgs fa{inc->a_colidx, p->ent, inc->b, inc->k, width, c->cfg.margin, scale, scores, c->gbuf[0],
                         packed_stride(c->cfg.dim), c->loss_partials, from_y ? nullptr : p->rel_weight,
                         (int32_t)c->cfg.n_ent};
    // (the next batch's first build kernel, if one is due and counts rows per relation as TransR's do)
    EmitAhead ea{};
    if (from_y && c->ahead.armed && !c->ahead.emit_done && c->ahead.args.rc.cur) ea = take_emit_ahead(c);
    const dim3 grid_e(grid.x + (unsigned)ea.ntiles);
#define STX_FWD(D, Y, P)                                                                                        \
    hipLaunchKernelGGL((k_forward_stacked<LPR, ITERS, D, Y, P>), grid, dim3(kThreads), 0, c->stream, fa)
#define STX_FWD2(D)                                                                                             \
    do {                                                                                                        \
        if (from_y && ea.ntiles)                                                                                \
            hipLaunchKernelGGL((k_forward_y_emit<LPR, ITERS, D>), grid_e, dim3(kThreads), 0, c->stream, fa, ea); \
        else if (from_y) STX_FWD(D, true, false);                                                               \
        else if (is_sign_kind(D)) STX_FWD(D, false, is_sign_kind(D));                                           \
        else STX_FWD(D, false, false);                                                                          \
    } while (0)
    {
    ProfScope prof(c, "k_forward_stacked");
    switch (c->cfg.dist) {
    case STX_L1: STX_FWD2(STX_L1); break;
    case STX_L2: STX_FWD2(STX_L2); break;
    case STX_TORUS_L1: STX_FWD2(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_FWD2(STX_L2_SQ); break;
    default: STX_FWD2(STX_TORUS_L2); break;
    }
    }
#undef STX_FWD2
#undef STX_FWD
    if (c->defer_finish) { c->fin_n = (int)grid.x; c->fin_scale = scale; c->fin_loss = loss; }
    else launch_finish_loss(c, (int)grid.x, scale, loss);
}

stx_status launch_forward_stacked(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores,
                                  float *loss)
{
    if (inc->n_rows == 0) return launch_finish_loss(c, 0, 1.0f, loss);
    float scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    Launch L = row_launch(c->cfg.dim);
    STX_DISPATCH_ROW(L, forward_go, c, inc, p, scores, loss, scale, false, c->cfg.dim);
    return hip_ok(hipGetLastError());
}

// Distances, hinge and dL/dy over rows of y already stored in gbuf[0] (row width = out_dim).
stx_status launch_forward_from_y(stx_ctx *c, const stx_incidence *inc, const stx_params *p, float *scores,
                                 float *loss)
{
    float scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    Launch L = row_launch(c->out_dim);
    STX_DISPATCH_ROW(L, forward_go, c, inc, p, scores, loss, scale, true, c->out_dim);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
