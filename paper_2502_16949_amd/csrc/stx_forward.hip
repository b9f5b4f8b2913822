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

// general_flag (may be null): the kernel runs only if *general_flag == serial, i.e. if the fast kernel before it met
// a positive whose negatives it does not cover; it then redoes the whole batch (the same bits where both apply).
template <int LPR, int ITERS, int DIST, bool FROM_Y, bool PACKED>
__global__ __launch_bounds__(kThreads, ITERS == 1 ? 8 : 1) void k_forward_stacked(ForwardArgs a, const int32_t *general_flag,
                                                                                 int32_t serial)
{
    if (general_flag && *general_flag != serial) return;
    forward_stacked_body<LPR, ITERS, DIST, FROM_Y, PACKED>((int)blockIdx.x, a);
}

// (rows of one float4 per lane: 64 registers, every workgroup of a large batch resident at once; wider rows hold
// four rows of ITERS float4 per lane)
template <int LPR, int ITERS, int DIST, bool PACKED, int NB>
__global__ __launch_bounds__(kThreads, ITERS == 1 ? 8 : (ITERS == 2 ? 4 : 2)) void k_forward_fast(ForwardArgs a, int32_t *general_flag,
                                                                                                 int32_t serial)
{
    forward_fast_body<LPR, ITERS, DIST, PACKED, NB>((int)blockIdx.x, a, general_flag, serial);
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

// Scattered reads of known volume: thread i reads the 32 bytes at the start of slot (i * 40503) mod n_slots (an
// odd multiplier, so a power-of-two number of slots is visited once each when n_reads == n_slots), `slot_bytes`
// apart: like the sign records the transposed product fetches, one memory sector per lane with no two lanes of a
// wavefront in one line when slot_bytes >= 128.  The sums go to `sink` so that the loads are kept.
__global__ __launch_bounds__(kThreads) void k_read_sectors(const char *__restrict__ src, int64_t n_slots, int slot_bytes,
                                                           int64_t n_reads, float *__restrict__ sink)
{
    float acc = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < n_reads; i += (int64_t)gridDim.x * kThreads) {
        const int64_t slot = (i * 40503) % n_slots;
        const float *q = reinterpret_cast<const float *>(src + slot * slot_bytes);
        const float4 a = ld4(q), b = ld4(q + 4);
        acc += (a.x + a.y + a.z + a.w) + (b.x + b.y + b.z + b.w);
    }
    if (acc == 12345.678f) sink[blockIdx.x] = acc;   // practically never: the loads must only be kept
}

stx_status launch_read_sectors(stx_ctx *c, const void *src, int64_t n_slots, int slot_bytes, int64_t n_reads, float *sink)
{
    if (n_reads == 0) return STX_OK;
    int64_t blocks = (n_reads + kThreads - 1) / kThreads;
    if (blocks > 16384) blocks = 16384;
    hipLaunchKernelGGL(k_read_sectors, dim3((unsigned)blocks), dim3(kThreads), 0, c->stream, static_cast<const char *>(src),
                       n_slots, slot_bytes, n_reads, sink);
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
                         (int32_t)c->cfg.n_ent, from_y ? 0 : big_tables(c)};
    // (the next batch's first build kernel, if one is due and counts rows per relation as TransR's do)
    EmitAhead ea{};
    if (from_y && c->ahead.armed && !c->ahead.emit_done && c->ahead.args.rc.cur) ea = take_emit_ahead(c);
    const dim3 grid_e(grid.x + (unsigned)ea.ntiles);
    // Few negatives per positive (four with rows of one float4 per lane, one with wider rows): the kernel that
    // fetches the positive's rows once (forward_fast_body).  It covers negatives that keep the relation and one entity of their positive; when the
    // batch was not drawn by the library's sampler in this build, the general kernel is enqueued behind it and runs
    // only if the fast one met another kind of negative.
    const bool fast = !from_y && inc->k <= fast_negatives<LPR, ITERS>();
    const bool sampled = c->sampled_inc == inc;
    int32_t *flag = c->ctrl + CTRL_GENERAL;
    const int32_t serial = fast ? ++c->fwd_serial : 0;
#define STX_FWD(D, Y, P)                                                                                        \
    hipLaunchKernelGGL((k_forward_stacked<LPR, ITERS, D, Y, P>), grid, dim3(kThreads), 0, c->stream, fa,        \
                       fast ? flag : nullptr, serial)
#define STX_FAST(D, P)                                                                                          \
    do {                                                                                                        \
        if (inc->k <= 1)                                                                                        \
            hipLaunchKernelGGL((k_forward_fast<LPR, ITERS, D, P, 1>), grid, dim3(kThreads), 0, c->stream, fa, flag, serial); \
        else                                                                                                    \
            hipLaunchKernelGGL((k_forward_fast<LPR, ITERS, D, P, fast_negatives<LPR, ITERS>()>), grid, dim3(kThreads), 0, \
                               c->stream, fa, flag, serial);                                                    \
    } while (0)
#define STX_FWD2(D)                                                                                             \
    do {                                                                                                        \
        if (from_y && ea.ntiles)                                                                                \
            hipLaunchKernelGGL((k_forward_y_emit<LPR, ITERS, D>), grid_e, dim3(kThreads), 0, c->stream, fa, ea); \
        else if (from_y) STX_FWD(D, true, false);                                                               \
        else {                                                                                                  \
            if (fast) {                                                                                         \
                ProfScope prof(c, "k_forward_stacked");                                                         \
                STX_FAST(D, is_sign_kind(D));                                                                   \
            }                                                                                                   \
            if (!fast || !sampled) {                                                                            \
                ProfScope prof(c, fast ? "k_forward_general" : "k_forward_stacked");                            \
                STX_FWD(D, false, is_sign_kind(D));                                                             \
            }                                                                                                   \
        }                                                                                                       \
    } while (0)
    if (from_y) {
        ProfScope prof(c, "k_forward_stacked");
        switch (c->cfg.dist) {
        case STX_L1: STX_FWD2(STX_L1); break;
        case STX_L2: STX_FWD2(STX_L2); break;
        case STX_TORUS_L1: STX_FWD2(STX_TORUS_L1); break;
        case STX_L2_SQ: STX_FWD2(STX_L2_SQ); break;
        default: STX_FWD2(STX_TORUS_L2); break;
        }
    } else {
        switch (c->cfg.dist) {
        case STX_L1: STX_FWD2(STX_L1); break;
        case STX_L2: STX_FWD2(STX_L2); break;
        case STX_TORUS_L1: STX_FWD2(STX_TORUS_L1); break;
        case STX_L2_SQ: STX_FWD2(STX_L2_SQ); break;
        default: STX_FWD2(STX_TORUS_L2); break;
        }
    }
#undef STX_FAST
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
