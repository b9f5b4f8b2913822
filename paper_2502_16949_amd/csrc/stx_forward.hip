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
#include "stx_rowops.h"

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

// Packed dL/dy row of an L1-kind distance: record `row` of gs = coefficient (fp32), then the sign bytes.
template <int LPR, int ITERS, int DIST>
__device__ inline void write_grad_row_packed(uint8_t *__restrict__ gs, int gstride, int64_t row, int d4, int lig,
                                             const RowVec<ITERS> &x, float coef)
{
    uint8_t *rec = gs + row * gstride;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) rec[4 + j] = (uint8_t)sign_bits<DIST>(x.v[it]);
    }
    if (lig == 0) *reinterpret_cast<float *>(rec) = coef;
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

// Sum of the per-workgroup loss partials in a fixed order (one workgroup, launched after the forward).
__global__ __launch_bounds__(kThreads) void k_finish_loss(const float *__restrict__ partials, int n, float scale,
                                                          float *__restrict__ loss)
{
    __shared__ double s_acc[kThreads];
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

// One group per positive i: rows i and b + i*k + kk (kk < k).
// FROM_Y = false: the translated vector of a row is gathered from the stacked table X (TransE/TorusE).
// FROM_Y = true : it is row `row` of the dense buffer G (TransR: y = M_r (h - t) + r was put there by
//                 the projection kernel), and dL/dy overwrites it in place; every row is read and then
//                 written by one group only.
// PACKED (L1 kinds, gathered rows only): dL/dx is written as records of gstride bytes at G (coefficient + sign bytes).
template <int LPR, int ITERS, int DIST, bool FROM_Y, bool PACKED>
__global__ __launch_bounds__(kThreads) void k_forward_stacked(const int32_t *__restrict__ colidx,
                                                              const float *__restrict__ X, int32_t b, int32_t k,
                                                              int dim, float margin, float scale,
                                                              float *__restrict__ scores, float *G,
                                                              int gstride,
                                                              float *__restrict__ loss_partials)
{
    static_assert(!PACKED || (is_sign_kind(DIST) && !FROM_Y), "packed rows need an L1-kind distance");
    constexpr int GROUPS = kThreads / LPR;
    __shared__ float s_loss[GROUPS];
    const int lig = threadIdx.x % LPR, grp = threadIdx.x / LPR;
    const int64_t i = (int64_t)blockIdx.x * GROUPS + grp;
    const int d4 = dim / 4;
    float hinge_sum = 0.f;
    if (i < b) {   // uniform within the group; shuffles below stay inside the group
        // Negatives are taken NB at a time so that the kernel pays two memory round trips per batch (all
        // column ids, then all table rows) instead of two per row; the positive rides with the first batch.
        constexpr int NB = ITERS <= 2 ? 4 : 2;
        RowVec<ITERS> xp;
        float dpos = 0.f;
        int n_active = 0;
        int32_t cp[3] = {0, 0, 0};
        if (!FROM_Y) { cp[0] = colidx[3 * i]; cp[1] = colidx[3 * i + 1]; cp[2] = colidx[3 * i + 2]; }
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
                dpos = row_distance<LPR, ITERS, DIST>(xp);
                if (lig == 0) scores[i] = dpos;
            }
#pragma unroll
            for (int q = 0; q < NB; ++q) {
                if (q < nb) {
                    const int64_t row = row0 + q;
                    const float dneg = row_distance<LPR, ITERS, DIST>(xn[q]);
                    const float arg = (margin + dpos) - dneg;
                    const bool active = arg > 0.f;
                    if (lig == 0) scores[row] = dneg;
                    if (active) { hinge_sum += arg; ++n_active; }
                    if (PACKED)
                        write_grad_row_packed<LPR, ITERS, DIST>(reinterpret_cast<uint8_t *>(G), gstride, row, d4, lig,
                                                                xn[q], active ? -scale : 0.f);
                    else
                        write_grad_row<LPR, ITERS, DIST>(G + row * dim, d4, lig, xn[q], active ? -scale : 0.f, dneg);
                }
            }
        }
        if (PACKED)
            write_grad_row_packed<LPR, ITERS, DIST>(reinterpret_cast<uint8_t *>(G), gstride, i, d4, lig, xp,
                                                    (float)n_active * scale);
        else
            write_grad_row<LPR, ITERS, DIST>(G + i * dim, d4, lig, xp, (float)n_active * scale, dpos);
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
#define STX_FWD(D, Y, P)                                                                                        \
    hipLaunchKernelGGL((k_forward_stacked<LPR, ITERS, D, Y, P>), grid, dim3(kThreads), 0, c->stream,            \
                       inc->a_colidx, p->ent, inc->b, inc->k, width, c->cfg.margin, scale, scores, c->gbuf[0],  \
                       packed_stride(c->cfg.dim), c->loss_partials)
#define STX_FWD2(D)                                                                                             \
    do {                                                                                                        \
        if (from_y) STX_FWD(D, true, false);                                                                    \
        else if (is_sign_kind(D)) STX_FWD(D, false, is_sign_kind(D));                                           \
        else STX_FWD(D, false, false);                                                                          \
    } while (0)
    {
    ProfScope prof(c, "k_forward_stacked");
    switch (c->cfg.dist) {
    case STX_L1: STX_FWD2(STX_L1); break;
    case STX_L2: STX_FWD2(STX_L2); break;
    case STX_TORUS_L1: STX_FWD2(STX_TORUS_L1); break;
    default: STX_FWD2(STX_TORUS_L2); break;
    }
    }
#undef STX_FWD2
#undef STX_FWD
    launch_finish_loss(c, (int)grid.x, scale, loss);
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
