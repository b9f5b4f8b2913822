// The three-entry product under the semirings of SparseTransX Appendix D, and its backward.
//
// Appendix D keeps the incidence matrix (a head, a relation and a tail column per row) and swaps the
// operators of the sparse-dense product: the row's entries are multiplied instead of added, with real
// products for DistMult (h r t), complex ones for ComplEx (h r conj(t)) and RotatE (h r - t).  A table
// row of a complex kind holds dim/2 numbers as (re, im) pairs, so a lane's float4 is two of them.
// Every real product and sum is rounded once, in the order written in cmul() and below.
//
// Backward for a real loss, given G = dL/dZ: every entry of a row receives G times the (conjugated)
// product of the row's other two factors.  k_semiring_terms writes these three rows per matrix row (the
// tail's negated), and the transposed product of the translational models sums them per column: head and
// relation entries add their row, tail entries subtract theirs.
#include <mutex>

#include "stx_rowops.h"

namespace stx {

enum { SR_DISTMULT = 0, SR_COMPLEX = 1, SR_ROTATE = 2 };

// (a.x + i a.y)(b.x + i b.y)
__device__ inline float2 cmul(float2 a, float2 b)
{
    const float ac = a.x * b.x, bd = a.y * b.y, ad = a.x * b.y, bc = a.y * b.x;
    return make_float2(ac - bd, ad + bc);
}
__device__ inline float2 conj2(float2 a) { return make_float2(a.x, -a.y); }
__device__ inline float2 lo2(float4 v) { return make_float2(v.x, v.y); }
__device__ inline float2 hi2(float4 v) { return make_float2(v.z, v.w); }
__device__ inline float4 join(float2 a, float2 b) { return make_float4(a.x, a.y, b.x, b.y); }
__device__ inline float4 mul4(float4 a, float4 b) { return make_float4(a.x * b.x, a.y * b.y, a.z * b.z, a.w * b.w); }
__device__ inline float4 neg4(float4 a) { return make_float4(-a.x, -a.y, -a.z, -a.w); }

template <int KIND>
__device__ inline float4 product(float4 h, float4 r, float4 t)
{
    if (KIND == SR_DISTMULT) return mul4(mul4(h, r), t);
    const float2 p0 = cmul(lo2(h), lo2(r)), p1 = cmul(hi2(h), hi2(r));
    if (KIND == SR_COMPLEX) return join(cmul(p0, conj2(lo2(t))), cmul(p1, conj2(hi2(t))));
    return make_float4(p0.x - t.x, p0.y - t.y, p1.x - t.z, p1.y - t.w);
}

template <int LPR, int ITERS, int KIND>
__global__ __launch_bounds__(kThreads) void k_semiring(const int32_t *__restrict__ colidx, const float *__restrict__ X,
                                                       int64_t n_rows, int dim, float *__restrict__ Z)
{
    const int lig = threadIdx.x % LPR;
    const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    if (row >= n_rows) return;
    const int d4 = dim / 4;
    const float *ph = X + (int64_t)colidx[3 * row] * dim, *pr = X + (int64_t)colidx[3 * row + 1] * dim;
    const float *pt = X + (int64_t)colidx[3 * row + 2] * dim;
    float4 h[ITERS], r[ITERS], t[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {   // all loads first
        const int j = min(lig + it * LPR, d4 - 1);
        h[it] = ld4(ph + 4 * j); r[it] = ld4(pr + 4 * j); t[it] = ld4(pt + 4 * j);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int j = lig + it * LPR;
        if (j < d4) st4_stream(Z + row * dim + 4 * j, product<KIND>(h[it], r[it], t[it]));
    }
}

// terms[row][0] = dL/dh, [1] = dL/dr, [2] = -dL/dt of this row, each `dim` floats.
template <int LPR, int ITERS, int KIND>
__global__ __launch_bounds__(kThreads) void k_semiring_terms(const int32_t *__restrict__ colidx,
                                                             const float *__restrict__ X, const float *__restrict__ G,
                                                             int64_t n_rows, int dim, float *__restrict__ terms)
{
    const int lig = threadIdx.x % LPR;
    const int64_t row = ((int64_t)blockIdx.x * kThreads + threadIdx.x) / LPR;
    if (row >= n_rows) return;
    const int d4 = dim / 4;
    const float *ph = X + (int64_t)colidx[3 * row] * dim, *pr = X + (int64_t)colidx[3 * row + 1] * dim;
    const float *pt = X + (int64_t)colidx[3 * row + 2] * dim, *pg = G + row * dim;
    float *out = terms + row * 3 * dim;
    float4 h[ITERS], r[ITERS], t[ITERS], g[ITERS];
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int j = min(lig + it * LPR, d4 - 1);
        h[it] = ld4(ph + 4 * j); r[it] = ld4(pr + 4 * j);
        t[it] = KIND == SR_ROTATE ? make_float4(0.f, 0.f, 0.f, 0.f) : ld4(pt + 4 * j);
        g[it] = ld4_stream(pg + 4 * j);
    }
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        const int j = lig + it * LPR;
        if (j >= d4) continue;
        float4 dh, dr, ndt;
        if (KIND == SR_DISTMULT) {
            const float4 gr = mul4(g[it], r[it]), gh = mul4(g[it], h[it]);
            dh = mul4(gr, t[it]);
            dr = mul4(gh, t[it]);
            ndt = neg4(mul4(gh, r[it]));
        } else {
            const float2 g0 = lo2(g[it]), g1 = hi2(g[it]);
            const float2 gr0 = cmul(g0, conj2(lo2(r[it]))), gr1 = cmul(g1, conj2(hi2(r[it])));
            const float2 gh0 = cmul(g0, conj2(lo2(h[it]))), gh1 = cmul(g1, conj2(hi2(h[it])));
            if (KIND == SR_COMPLEX) {
                dh = join(cmul(gr0, lo2(t[it])), cmul(gr1, hi2(t[it])));
                dr = join(cmul(gh0, lo2(t[it])), cmul(gh1, hi2(t[it])));
                const float2 c0 = cmul(cmul(conj2(g0), lo2(h[it])), lo2(r[it]));
                const float2 c1 = cmul(cmul(conj2(g1), hi2(h[it])), hi2(r[it]));
                ndt = neg4(join(c0, c1));
            } else {
                dh = join(gr0, gr1);
                dr = join(gh0, gh1);
                ndt = g[it];   // dL/dt = -g
            }
        }
        st4(out + 4 * j, dh);
        st4(out + dim + 4 * j, dr);
        st4(out + 2 * dim + 4 * j, ndt);
    }
}

template <int LPR, int ITERS>
static void semiring_go(stx_ctx *c, const stx_incidence *inc, const stx_params *p, int kind, const float *gz,
                        float *out)
{
    const int64_t threads = inc->n_rows * LPR;
    const dim3 grid((unsigned)((threads + kThreads - 1) / kThreads)), block(kThreads);
    const int dim = c->cfg.dim;
#define STX_SR(K)                                                                                               \
    do {                                                                                                        \
        if (gz) {                                                                                               \
            ProfScope prof(c, "k_semiring_terms");                                                              \
            hipLaunchKernelGGL((k_semiring_terms<LPR, ITERS, K>), grid, block, 0, c->stream, inc->a_colidx,     \
                               p->ent, gz, inc->n_rows, dim, out);                                              \
        } else {                                                                                                \
            ProfScope prof(c, "k_semiring");                                                                    \
            hipLaunchKernelGGL((k_semiring<LPR, ITERS, K>), grid, block, 0, c->stream, inc->a_colidx, p->ent,   \
                               inc->n_rows, dim, out);                                                          \
        }                                                                                                       \
    } while (0)
    if (kind == SR_DISTMULT) STX_SR(SR_DISTMULT);
    else if (kind == SR_COMPLEX) STX_SR(SR_COMPLEX);
    else STX_SR(SR_ROTATE);
#undef STX_SR
}

stx_status launch_semiring(stx_ctx *c, const stx_incidence *inc, const stx_params *p, int kind, float *z_out)
{
    if (inc->n_rows == 0) return STX_OK;
    Launch L = row_launch(c->cfg.dim);
    STX_DISPATCH_ROW(L, semiring_go, c, inc, p, kind, nullptr, z_out);
    return hip_ok(hipGetLastError());
}

// Scratch of stx_spmm_semiring_t_static: the per-row terms of the backward product, for callers that can bring
// no work buffer.  Every GPU the library runs on holds its own copy of the array, at its own address, until the
// process ends.  In host code the array's name is only a handle for the symbol look-up below, never an address.
static __device__ __align__(256) unsigned char scratch[STX_STATIC_WORK_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];   // device address of `scratch` on each GPU, null until first asked for
}  // namespace

stx_status static_work(float **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return STX_ERR_HIP;
    if (dev < 0 || dev >= kMaxDevices) return STX_ERR_UNSUPPORTED;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return STX_ERR_HIP;
        g_scratch_ptr[dev] = ptr;
    }
    *out = static_cast<float *>(g_scratch_ptr[dev]);
    return STX_OK;
}

stx_status launch_semiring_t(stx_ctx *c, const stx_incidence *inc, const stx_params *p, int kind, const float *gz,
                             float *work, float *out_rows)
{
    if (inc->n_rows == 0) return STX_OK;
    const int dim = c->cfg.dim;
    Launch L = row_launch(dim);
    STX_DISPATCH_ROW(L, semiring_go, c, inc, p, kind, gz, work);
    stx_status s = hip_ok(hipGetLastError());
    if (s != STX_OK) return s;
    // sorted entries: entity columns first (heads add their row of `work`, tails subtract the row 2*dim
    // floats further on), then the relation columns (the row dim floats further on)
    return launch_seg_reduce(c, inc, 0, inc->nnz, work, work + dim, 2 * inc->n_rows, 3 * dim, dim, out_rows, c->ld,
                             false, nullptr, nullptr, 2 * dim);
}

}  // namespace stx
