// Launches in which two independent pieces of one training step share the GPU.
//
// At the batch sizes of the paper's benchmarks (Sec. 5.3: 32,768 positives) every kernel of a step is
// short and the step is a chain of dependent launches, so its duration is the sum of their latencies.
// Two links of that chain do not depend on each other: the forward pass (SparseTransX Sec. 4.3) needs
// only A, which the first kernel of the build writes, while the sort that produces A^T for the
// backward pass (Appendix G) goes on for several more launches; and the final sum of the loss needs
// only the forward pass.  stx_train_step therefore runs the forward pass in the launch of a scatter pass
// of the sort (the first one; or, when the first stages of this batch's build already ran inside the
// previous step's launches, the histogram pass or the last scatter pass), and the loss sum in the launch
// of a later pass or of the transposed product.  In those later launches the first kernel of the next
// batch's build comes along as well.  The sort's workgroups take the low block indices so that they start
// first: they are few and long, the forward workgroups many and short.
#include "stx_emit_body.h"
#include "stx_forward_body.h"
#include "stx_sort_body.h"
#include "stx_transh_body.h"

namespace stx {

// LDS of the launches below that run bodies of the sort beside a forward pass: the larger of the two bodies' needs
constexpr int kRideLds = kScatterLds > emit_lds(true, false) ? kScatterLds : emit_lds(true, false);

// (a later pass, FIRST false, can also take the first kernel of the next batch's build along: ea.ntiles > 0)
template <int LPR, int ITERS, int DIST, bool PACKED, bool FIRST, bool K1>
__global__ __launch_bounds__(kThreads) void k_fwd_scatter(ForwardArgs fa, ScatterArgs sa, EmitAhead ea)
{
    __shared__ __align__(16) unsigned char s_arena[kRideLds];   // one block of LDS for the sort's bodies
    int block = (int)blockIdx.x;
    if (block < sa.ntiles) { scatter_body<FIRST, false, kSortItems, true>(block, sa, s_arena); return; }
    block -= sa.ntiles;
    if constexpr (!FIRST) {
        if (block < ea.ntiles) { emit_body<kSortItems, true, true, false, true>(block, ea.ntiles, ea.args, s_arena); return; }
        block -= ea.ntiles;
    }
    forward_step_body<LPR, ITERS, DIST, PACKED, K1>(block, fa);
}

template <int LPR, int ITERS, int DIST, bool FIRST, bool K1>
__global__ __launch_bounds__(kThreads, 4) void k_fwdh_scatter(TranshArgs ta, ScatterArgs sa, EmitAhead ea)
{
    __shared__ __align__(16) unsigned char s_arena[kRideLds];
    int block = (int)blockIdx.x;
    if (block < sa.ntiles) { scatter_body<FIRST, false, kSortItems, true>(block, sa, s_arena); return; }
    block -= sa.ntiles;
    if constexpr (!FIRST) {
        if (block < ea.ntiles) { emit_body<kSortItems, true, true, false, true>(block, ea.ntiles, ea.args, s_arena); return; }
        block -= ea.ntiles;
    }
    forward_transh_body<LPR, ITERS, DIST, K1>(block, ta);
}

__global__ __launch_bounds__(kThreads) void k_hist_finish(const int32_t *__restrict__ keys, int32_t nnz, int shift,
                                                          int radix, int32_t *__restrict__ table,
                                                          const float *__restrict__ partials, int n_partials,
                                                          float scale, float *__restrict__ loss)
{
    if (blockIdx.x == 0) finish_loss_body(partials, n_partials, scale, loss);
    else hist_body<kSortItems>((int)blockIdx.x - 1, keys, nnz, shift, radix, table);
}

// When the first scatter pass of a build ran ahead of time (in a launch of the previous step), the forward
// pass shares the launch of the next histogram pass instead, and the sum of the loss that of the scatter
// pass after it.  The first kernel of the next batch's build can come along (ea.ntiles > 0).
template <int LPR, int ITERS, int DIST, bool PACKED>
__global__ __launch_bounds__(kThreads) void k_fwd_hist(ForwardArgs fa, const int32_t *__restrict__ keys, int32_t nnz,
                                                       int shift, int radix, int32_t *__restrict__ table, int ntiles,
                                                       EmitAhead ea)
{
    __shared__ __align__(16) unsigned char s_arena[emit_lds(true, false)];
    int block = (int)blockIdx.x;
    if (block < ntiles) { hist_body<kSortItems>(block, keys, nnz, shift, radix, table); return; }
    block -= ntiles;
    if (block < ea.ntiles) { emit_body<kSortItems, true, true, false, true>(block, ea.ntiles, ea.args, s_arena); return; }
    forward_step_body<LPR, ITERS, DIST, PACKED, false>(block - ea.ntiles, fa);
}

template <int LPR, int ITERS, int DIST>
__global__ __launch_bounds__(kThreads) void k_fwdh_hist(TranshArgs ta, const int32_t *__restrict__ keys, int32_t nnz,
                                                        int shift, int radix, int32_t *__restrict__ table, int ntiles,
                                                        EmitAhead ea)
{
    __shared__ __align__(16) unsigned char s_arena[emit_lds(true, false)];
    int block = (int)blockIdx.x;
    if (block < ntiles) { hist_body<kSortItems>(block, keys, nnz, shift, radix, table); return; }
    block -= ntiles;
    if (block < ea.ntiles) { emit_body<kSortItems, true, true, false, true>(block, ea.ntiles, ea.args, s_arena); return; }
    forward_transh_body<LPR, ITERS, DIST>(block - ea.ntiles, ta);
}

__global__ __launch_bounds__(kThreads) void k_scatter_finish(ScatterArgs sa, const float *__restrict__ partials,
                                                             int n_partials, float scale, float *__restrict__ loss)
{
    if (blockIdx.x == 0) finish_loss_body(partials, n_partials, scale, loss);
    else scatter_body<false, false, kSortItems>((int)blockIdx.x - 1, sa);
}

template <int LPR, int ITERS>
static void fwd_scatter_go(stx_ctx *c, const ForwardArgs &fa, const ScatterArgs &sa, unsigned blocks, bool first,
                           const EmitAhead &ea)
{
#define STX_FS(D, P)                                                                                            \
    do {                                                                                                        \
        if (first && fa.k <= 1)                                                                                 \
            hipLaunchKernelGGL((k_fwd_scatter<LPR, ITERS, D, P, true, true>), dim3(blocks), dim3(kThreads), 0,  \
                               c->stream, fa, sa, ea);                                                          \
        else if (first)                                                                                         \
            hipLaunchKernelGGL((k_fwd_scatter<LPR, ITERS, D, P, true, false>), dim3(blocks), dim3(kThreads), 0, \
                               c->stream, fa, sa, ea);                                                          \
        else if (fa.k <= 1)                                                                                     \
            hipLaunchKernelGGL((k_fwd_scatter<LPR, ITERS, D, P, false, true>), dim3(blocks), dim3(kThreads), 0, \
                               c->stream, fa, sa, ea);                                                          \
        else                                                                                                    \
            hipLaunchKernelGGL((k_fwd_scatter<LPR, ITERS, D, P, false, false>), dim3(blocks), dim3(kThreads),   \
                               0, c->stream, fa, sa, ea);                                                       \
    } while (0)
    switch (c->cfg.dist) {
    case STX_L1: STX_FS(STX_L1, true); break;
    case STX_L2: STX_FS(STX_L2, false); break;
    case STX_TORUS_L1: STX_FS(STX_TORUS_L1, true); break;
    case STX_L2_SQ: STX_FS(STX_L2_SQ, false); break;
    default: STX_FS(STX_TORUS_L2, false); break;
    }
#undef STX_FS
}

template <int LPR, int ITERS>
static void fwdh_scatter_go(stx_ctx *c, const TranshArgs &ta, const ScatterArgs &sa, unsigned blocks, bool first,
                            const EmitAhead &ea)
{
#define STX_FS(D)                                                                                               \
    do {                                                                                                        \
        if (first && ta.k <= 1)                                                                                 \
            hipLaunchKernelGGL((k_fwdh_scatter<LPR, ITERS, D, true, true>), dim3(blocks), dim3(kThreads), 0,    \
                               c->stream, ta, sa, ea);                                                          \
        else if (first)                                                                                         \
            hipLaunchKernelGGL((k_fwdh_scatter<LPR, ITERS, D, true, false>), dim3(blocks), dim3(kThreads), 0,   \
                               c->stream, ta, sa, ea);                                                          \
        else if (ta.k <= 1)                                                                                     \
            hipLaunchKernelGGL((k_fwdh_scatter<LPR, ITERS, D, false, true>), dim3(blocks), dim3(kThreads), 0,   \
                               c->stream, ta, sa, ea);                                                          \
        else                                                                                                    \
            hipLaunchKernelGGL((k_fwdh_scatter<LPR, ITERS, D, false, false>), dim3(blocks), dim3(kThreads), 0,  \
                               c->stream, ta, sa, ea);                                                          \
    } while (0)
    switch (c->cfg.dist) {
    case STX_L1: STX_FS(STX_L1); break;
    case STX_L2: STX_FS(STX_L2); break;
    case STX_TORUS_L1: STX_FS(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_FS(STX_L2_SQ); break;
    default: STX_FS(STX_TORUS_L2); break;
    }
#undef STX_FS
}

template <int LPR>
static void fwd_hist_go(stx_ctx *c, const ForwardArgs &fa, const int32_t *keys, int32_t nnz, int shift, int radix,
                        int ntiles, unsigned blocks, const EmitAhead &ea)
{
#define STX_FH(D, P)                                                                                            \
    hipLaunchKernelGGL((k_fwd_hist<LPR, 1, D, P>), dim3(blocks), dim3(kThreads), 0, c->stream, fa, keys, nnz, shift, \
                       radix, c->table1, ntiles, ea)
    switch (c->cfg.dist) {
    case STX_L1: STX_FH(STX_L1, true); break;
    case STX_L2: STX_FH(STX_L2, false); break;
    case STX_TORUS_L1: STX_FH(STX_TORUS_L1, true); break;
    case STX_L2_SQ: STX_FH(STX_L2_SQ, false); break;
    default: STX_FH(STX_TORUS_L2, false); break;
    }
#undef STX_FH
}

template <int LPR>
static void fwdh_hist_go(stx_ctx *c, const TranshArgs &ta, const int32_t *keys, int32_t nnz, int shift, int radix,
                         int ntiles, unsigned blocks, const EmitAhead &ea)
{
#define STX_FH(D)                                                                                               \
    hipLaunchKernelGGL((k_fwdh_hist<LPR, 1, D>), dim3(blocks), dim3(kThreads), 0, c->stream, ta, keys, nnz, shift,  \
                       radix, c->table1, ntiles, ea)
    switch (c->cfg.dist) {
    case STX_L1: STX_FH(STX_L1); break;
    case STX_L2: STX_FH(STX_L2); break;
    case STX_TORUS_L1: STX_FH(STX_TORUS_L1); break;
    case STX_L2_SQ: STX_FH(STX_L2_SQ); break;
    default: STX_FH(STX_TORUS_L2); break;
    }
#undef STX_FH
}

bool launch_fwd_hist(stx_ctx *c, const stx_incidence *inc, StepFusion *f, const int32_t *keys, int32_t nnz, int shift,
                     int radix, int ntiles)
{
    const bool stacked = c->cfg.model == STX_TRANSE || c->cfg.model == STX_TORUSE;
    const bool transh = c->cfg.model == STX_TRANSH;
    const Launch L = row_launch(c->cfg.dim);
    if (!(stacked || transh) || L.iters != 1 || inc->n_rows == 0) return false;
    f->scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) f->scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    const int groups = kThreads / L.lpr;
    f->n_partials = (inc->b + groups - 1) / groups;
    const int32_t *colidx = f->colidx ? f->colidx : inc->a_colidx;
    const EmitAhead ea = take_emit_ahead(c);
    const unsigned blocks = (unsigned)(ntiles + ea.ntiles + f->n_partials);
    if (transh) {
        const TranshArgs ta{colidx, f->p->ent, f->p->rel, f->p->w, (int32_t)c->cfg.n_ent, inc->b, inc->k,
                            c->cfg.dim, c->cfg.margin, f->scale, f->scores, c->gbuf[0], c->gbuf[1], c->gbuf[2],
                            c->loss_partials};
        ProfScope prof(c, "k_fwdh_hist");
        if (L.lpr == 8) fwdh_hist_go<8>(c, ta, keys, nnz, shift, radix, ntiles, blocks, ea);
        else if (L.lpr == 16) fwdh_hist_go<16>(c, ta, keys, nnz, shift, radix, ntiles, blocks, ea);
        else if (L.lpr == 32) fwdh_hist_go<32>(c, ta, keys, nnz, shift, radix, ntiles, blocks, ea);
        else fwdh_hist_go<64>(c, ta, keys, nnz, shift, radix, ntiles, blocks, ea);
        f->forward_done = true;
        return true;
    }
    const ForwardArgs fa{colidx, f->p->ent, inc->b, inc->k, c->cfg.dim, c->cfg.margin, f->scale, f->scores,
                         c->gbuf[0], packed_stride(c->cfg.dim), c->loss_partials, f->p->rel_weight,
                         (int32_t)c->cfg.n_ent};
    ProfScope prof(c, "k_fwd_hist");
    if (L.lpr == 8) fwd_hist_go<8>(c, fa, keys, nnz, shift, radix, ntiles, blocks, ea);
    else if (L.lpr == 16) fwd_hist_go<16>(c, fa, keys, nnz, shift, radix, ntiles, blocks, ea);
    else if (L.lpr == 32) fwd_hist_go<32>(c, fa, keys, nnz, shift, radix, ntiles, blocks, ea);
    else fwd_hist_go<64>(c, fa, keys, nnz, shift, radix, ntiles, blocks, ea);
    f->forward_done = true;
    return true;
}

void launch_scatter_finish(stx_ctx *c, StepFusion *f, const ScatterArgs &sa)
{
    ProfScope prof(c, "k_scatter_finish");
    hipLaunchKernelGGL(k_scatter_finish, dim3((unsigned)sa.ntiles + 1), dim3(kThreads), 0, c->stream, sa, c->loss_partials,
                       f->n_partials, f->scale, f->loss);
    f->finish_done = true;
}

bool launch_fwd_scatter(stx_ctx *c, const stx_incidence *inc, StepFusion *f, const ScatterArgs &sa, bool first)
{
    const bool stacked = c->cfg.model == STX_TRANSE || c->cfg.model == STX_TORUSE;
    const bool transh = c->cfg.model == STX_TRANSH;
    const Launch L = row_launch(c->cfg.dim);
    if (!(stacked || transh) || L.iters != 1 || inc->n_rows == 0) return false;
    f->scale = 1.0f;
    if (c->cfg.reduce == STX_MEAN && inc->k > 0) f->scale = 1.0f / (float)((int64_t)inc->b * inc->k);
    const int groups = kThreads / L.lpr;
    f->n_partials = (inc->b + groups - 1) / groups;
    const int32_t *colidx = f->colidx ? f->colidx : inc->a_colidx;
    const EmitAhead ea = first ? EmitAhead{} : take_emit_ahead(c);
    if (transh) {
        const TranshArgs ta{colidx, f->p->ent, f->p->rel, f->p->w, (int32_t)c->cfg.n_ent, inc->b, inc->k,
                            c->cfg.dim, c->cfg.margin, f->scale, f->scores, c->gbuf[0], c->gbuf[1], c->gbuf[2],
                            c->loss_partials};
        const unsigned blocks = (unsigned)(sa.ntiles + ea.ntiles + f->n_partials);
        ProfScope prof(c, "k_fwdh_scatter");
        if (L.lpr == 8) fwdh_scatter_go<8, 1>(c, ta, sa, blocks, first, ea);
        else if (L.lpr == 16) fwdh_scatter_go<16, 1>(c, ta, sa, blocks, first, ea);
        else if (L.lpr == 32) fwdh_scatter_go<32, 1>(c, ta, sa, blocks, first, ea);
        else fwdh_scatter_go<64, 1>(c, ta, sa, blocks, first, ea);
        f->forward_done = true;
        return true;
    }
    const ForwardArgs fa{colidx, f->p->ent, inc->b, inc->k, c->cfg.dim, c->cfg.margin, f->scale, f->scores,
                         c->gbuf[0], packed_stride(c->cfg.dim), c->loss_partials, f->p->rel_weight,
                         (int32_t)c->cfg.n_ent};
    const unsigned blocks = (unsigned)(sa.ntiles + ea.ntiles + f->n_partials);
    ProfScope prof(c, "k_fwd_scatter");
    if (L.lpr == 8) fwd_scatter_go<8, 1>(c, fa, sa, blocks, first, ea);
    else if (L.lpr == 16) fwd_scatter_go<16, 1>(c, fa, sa, blocks, first, ea);
    else if (L.lpr == 32) fwd_scatter_go<32, 1>(c, fa, sa, blocks, first, ea);
    else fwd_scatter_go<64, 1>(c, fa, sa, blocks, first, ea);
    f->forward_done = true;
    return true;
}

void launch_hist_finish(stx_ctx *c, StepFusion *f, const int32_t *keys, int32_t nnz, int shift, int radix, int ntiles)
{
    ProfScope prof(c, "k_hist_finish");
    hipLaunchKernelGGL(k_hist_finish, dim3((unsigned)ntiles + 1), dim3(kThreads), 0, c->stream, keys, nnz, shift, radix,
                       c->table1, c->loss_partials, f->n_partials, f->scale, f->loss);
    f->finish_done = true;
}

}  // namespace stx
