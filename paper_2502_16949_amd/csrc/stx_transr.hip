// TransR: the per-relation projection products on the matrix cores.
//
// SparseTransX Sec. 4.4 rearranges M_r h + r - M_r t into M_r (h - t) + r, so the `ht` incidence
// product (Sec. 4.2.1) feeds one projection per row.  Rows with the same relation share M_r, and the
// relation columns of the sorted A^T (stx_build.hip) already list every relation's rows contiguously,
// so the projections are dense products over runs of that list:
//
//   forward   Y_g  = X_g . M_r^T + r        (n_g x d)(d x k)      k_transr_project
//   backward  GX_g = GY_g . M_r             (n_g x k)(k x d)      k_transr_gx
//             dM_r = GY_g^T . X_g           (k x n_g)(n_g x d)    k_transr_dm (+ k_transr_dm_fixup)
//
// Operands are rounded to bfloat16 (round to nearest even) as they are loaded, products accumulate in
// fp32 in v_mfma_f32_32x32x16_bf16; x = h - t is formed in fp32 first.  Work is cut by entries of the
// sorted list, not by relation (group sizes are power-law distributed): a workgroup owns a fixed chunk
// of entries and walks the runs of equal relation inside it, masking rows of other relations, so a
// chunk inside a big relation is one dense tile and a chunk in the tail costs one tile per relation.
//
// MFMA 32x32x16 operand layout (64 lanes): lane l holds, for the A operand, row (l % 32) and the eight
// consecutive K elements 8*(l / 32) ..; for the B operand, column (l % 32) and the same eight K
// elements; accumulator register v holds row 8*(v / 4) + 4*(l / 32) + v % 4 of column l % 32.
#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

__device__ inline bf16x8 cvt8(float4 a, float4 b)
{
    bf16x8 r;
    r[0] = (__bf16)a.x; r[1] = (__bf16)a.y; r[2] = (__bf16)a.z; r[3] = (__bf16)a.w;
    r[4] = (__bf16)b.x; r[5] = (__bf16)b.y; r[6] = (__bf16)b.z; r[7] = (__bf16)b.w;
    return r;
}
__device__ inline bf16x8 zero8()
{
    bf16x8 r;
#pragma unroll
    for (int i = 0; i < 8; ++i) r[i] = (__bf16)0.0f;
    return r;
}
__device__ inline float4 sub4(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }
__device__ inline floatx16 zero16()
{
    floatx16 r;
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = 0.f;
    return r;
}

constexpr int kMaxNT = kMaxProjDim / 32 / 2;   // 32-column tiles per wavefront (two wavefronts share the columns)

struct ProjArgs {
    const int32_t *colidx, *packed, *seg_id, *seg_ptr, *touched_cols;
    const float *E, *M, *Rv;
    int32_t n_ent, e_begin, e_end;
    int d, k;
};

// One workgroup per kProjRows sorted relation entries.  Wavefront w: rows 32*(w/2).., column tiles w%2, w%2+2, ..
// GX = false: Y[row] = bf16(E[h]-E[t]) . bf16(M_r)^T + r_vec       (out width k, reduction over d)
// GX = true : GX[row] = bf16(GY[row]) . bf16(M_r)                   (out width d, reduction over k)
template <bool GX>
__global__ __launch_bounds__(kThreads) void k_transr_rows(ProjArgs p, const float *__restrict__ gy,
                                                          float *__restrict__ out)
{
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6, wr = w >> 1, wc = w & 1;
    const int l31 = l & 31, kg = l >> 5;
    const int n_out = GX ? p.d : p.k, n_red = GX ? p.k : p.d;
    const int32_t e_first = p.e_begin + (int32_t)blockIdx.x * kProjRows + 32 * wr;
    if (e_first >= p.e_end) return;                       // no barrier is used below: wavefronts are independent
    const int32_t e_last = min(e_first + 31, p.e_end - 1);
    const int32_t e = e_first + l31;
    const bool valid = e <= e_last;
    const int32_t row = valid ? (p.packed[e] >> 2) : 0;
    const int32_t seg = valid ? p.seg_id[e] : -1;
    const float *pa0, *pa1 = nullptr;
    if (GX) {
        pa0 = gy + (int64_t)row * p.k;
    } else {
        pa0 = p.E + (int64_t)(valid ? p.colidx[3 * row] : 0) * p.d;
        pa1 = p.E + (int64_t)(valid ? p.colidx[3 * row + 2] : 0) * p.d;
    }
    const int32_t s_first = p.seg_id[e_first], s_last = p.seg_id[e_last];
    const int ntiles = n_out / 32, ntw = (ntiles - wc + 1) / 2;

    for (int32_t s = s_first; s <= s_last; ++s) {
        const int32_t r = p.touched_cols[s] - p.n_ent;
        const float *Mr = p.M + (int64_t)r * p.k * p.d;
        const bool mine = valid && seg == s;
        floatx16 acc[kMaxNT];
#pragma unroll
        for (int q = 0; q < kMaxNT; ++q) acc[q] = zero16();
        for (int ks = 0; ks < n_red / 16; ++ks) {
            const int j0 = 16 * ks + 8 * kg;
            bf16x8 a = zero8();
            if (mine) {
                if (GX) a = cvt8(ld4(pa0 + j0), ld4(pa0 + j0 + 4));
                else a = cvt8(sub4(ld4(pa0 + j0), ld4(pa1 + j0)), sub4(ld4(pa0 + j0 + 4), ld4(pa1 + j0 + 4)));
            }
#pragma unroll
            for (int q = 0; q < kMaxNT; ++q) {
                if (q < ntw) {
                    const int n = (wc + 2 * q) * 32 + l31;
                    bf16x8 bfrag;
                    if (GX) {   // B[K = a][N = j] = M_r[a][j]: eight rows of M_r at column n
                        const float *pm = Mr + (int64_t)j0 * p.d + n;
#pragma unroll
                        for (int i = 0; i < 8; ++i) bfrag[i] = (__bf16)pm[(int64_t)i * p.d];
                    } else {    // B[K = j][N = a] = M_r[a][j]: eight consecutive elements of row n of M_r
                        const float *pm = Mr + (int64_t)n * p.d + j0;
                        bfrag = cvt8(ld4(pm), ld4(pm + 4));
                    }
                    acc[q] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, bfrag, acc[q], 0, 0, 0);
                }
            }
        }
#pragma unroll
        for (int q = 0; q < kMaxNT; ++q) {
            if (q < ntw) {
                const int n = (wc + 2 * q) * 32 + l31;
                const float add = GX ? 0.f : p.Rv[(int64_t)r * p.k + n];
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int m = 8 * (v >> 2) + 4 * kg + (v & 3);
                    const int32_t row_m = __shfl(row, m), seg_m = __shfl(seg, m);
                    if (seg_m == s) out[(int64_t)row_m * n_out + n] = acc[q][v] + add;
                }
            }
        }
    }
}

// dL/dM_r = sum over the rows i of relation r of bf16(gy_i) bf16(x_i)^T, x_i = E[h_i] - E[t_i].
// One workgroup per kProjRowsDm sorted relation entries; the reduction runs over rows, 16 per MFMA.
// Wavefront w owns output column tiles w, w+4, ..; for each it walks the row tiles four at a time.
// A run of a relation that lies inside the chunk is stored to dM_r directly; a run that crosses the
// chunk's border is stored as a partial matrix (slot 0: it began before the chunk, slot 1: it goes on
// after it) for k_transr_dm_fixup.
__global__ __launch_bounds__(kThreads) void k_transr_dm(ProjArgs p, const float *__restrict__ gy,
                                                        float *__restrict__ g_proj, float *__restrict__ partials)
{
    __shared__ int32_t s_row[kProjRowsDm], s_h[kProjRowsDm], s_t[kProjRowsDm];
    const int tid = threadIdx.x, l = tid & 63, w = tid >> 6, l31 = l & 31, kg = l >> 5;
    const int32_t c0 = p.e_begin + (int32_t)blockIdx.x * kProjRowsDm;
    const int32_t c1 = min(c0 + kProjRowsDm, p.e_end);
    {
        const int32_t e = c0 + tid;
        int32_t row = 0, hh = 0, tt = 0;
        if (e < c1) {
            row = p.packed[e] >> 2;
            hh = p.colidx[3 * row];
            tt = p.colidx[3 * row + 2];
        }
        s_row[tid] = row; s_h[tid] = hh; s_t[tid] = tt;
    }
    __syncthreads();
    const int32_t s_first = p.seg_id[c0], s_last = p.seg_id[c1 - 1];
    const int mtiles = p.k / 32, ntiles = p.d / 32;
    const int64_t kd = (int64_t)p.k * p.d;

    for (int32_t s = s_first; s <= s_last; ++s) {
        const int32_t sb = p.seg_ptr[s], se = p.seg_ptr[s + 1];
        const int32_t q0 = max(sb, c0) - c0, q1 = min(se, c1) - c0;   // positions in the chunk
        const int32_t r = p.touched_cols[s] - p.n_ent;
        float *dst = (sb >= c0 && se <= c1) ? g_proj + (int64_t)r * kd
                                            : partials + ((int64_t)blockIdx.x * 2 + (sb < c0 ? 0 : 1)) * kd;
        for (int nt = w; nt < ntiles; nt += 4) {
            const int j = nt * 32 + l31;
            for (int mt0 = 0; mt0 < mtiles; mt0 += 4) {
                floatx16 acc[4];
#pragma unroll
                for (int q = 0; q < 4; ++q) acc[q] = zero16();
                for (int i0 = q0; i0 < q1; i0 += 16) {
                    bf16x8 bx;                                   // B[K = i][N = j] = x_i[j]
                    bf16x8 ax[4];                                // A[M = a][K = i] = gy_i[a]
#pragma unroll
                    for (int i = 0; i < 8; ++i) {
                        const int q = i0 + 8 * kg + i;
                        const bool ok = q < q1;
                        const int qq = ok ? q : q0;
                        const float xv = p.E[(int64_t)s_h[qq] * p.d + j] - p.E[(int64_t)s_t[qq] * p.d + j];
                        bx[i] = (__bf16)(ok ? xv : 0.f);
                        const float *pg = gy + (int64_t)s_row[qq] * p.k + l31;
#pragma unroll
                        for (int m = 0; m < 4; ++m)
                            ax[m][i] = (__bf16)((ok && mt0 + m < mtiles) ? pg[(mt0 + m) * 32] : 0.f);
                    }
#pragma unroll
                    for (int m = 0; m < 4; ++m)
                        if (mt0 + m < mtiles) acc[m] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(ax[m], bx, acc[m], 0, 0, 0);
                }
#pragma unroll
                for (int m = 0; m < 4; ++m) {
                    if (mt0 + m < mtiles) {
#pragma unroll
                        for (int v = 0; v < 16; ++v) {
                            const int a = (mt0 + m) * 32 + 8 * (v >> 2) + 4 * kg + (v & 3);
                            dst[(int64_t)a * p.d + j] = acc[m][v];
                        }
                    }
                }
            }
        }
    }
}

// The chunk in which a border-crossing run of a relation ends adds up the run's partial matrices in
// chunk order: (first chunk, slot 1), then slot 0 of every later chunk up to this one.
__global__ __launch_bounds__(kThreads) void k_transr_dm_fixup(ProjArgs p, float *__restrict__ g_proj,
                                                              const float *__restrict__ partials)
{
    const int32_t j = (int32_t)blockIdx.x + 1;
    const int32_t c0 = p.e_begin + j * kProjRowsDm;
    if (c0 >= p.e_end) return;
    const int32_t c1 = min(c0 + kProjRowsDm, p.e_end);
    const int32_t s = p.seg_id[c0];
    const int32_t sb = p.seg_ptr[s], se = p.seg_ptr[s + 1];
    if (sb >= c0 || se > c1) return;                      // starts here, or goes on: not the closing chunk
    const int32_t j0 = (sb - p.e_begin) / kProjRowsDm;
    const int64_t kd = (int64_t)p.k * p.d;
    float *dst = g_proj + (int64_t)(p.touched_cols[s] - p.n_ent) * kd;
    // blockIdx.y slices the matrix: 4 consecutive elements per thread, 1024 per workgroup
    const int64_t idx = ((int64_t)blockIdx.y * kThreads + threadIdx.x) * 4;
    if (idx >= kd) return;
    float4 a = ld4(partials + ((int64_t)j0 * 2 + 1) * kd + idx);
    int32_t jj = j0 + 1;
    for (; jj + 3 <= j; jj += 4) {    // four partial matrices in flight, added in chunk order
        float4 v[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) v[u] = ld4(partials + ((int64_t)(jj + u) * 2) * kd + idx);
#pragma unroll
        for (int u = 0; u < 4; ++u) { a.x += v[u].x; a.y += v[u].y; a.z += v[u].z; a.w += v[u].w; }
    }
    for (; jj <= j; ++jj) {
        float4 v = ld4(partials + ((int64_t)jj * 2) * kd + idx);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    st4(dst + idx, a);
}

// M_r <- M_r - lr * dL/dM_r for every relation present in the batch (one workgroup per relation;
// it looks its column up in the sorted touched list and leaves if absent).
__global__ __launch_bounds__(kThreads) void k_sgd_proj(const int32_t *__restrict__ touched_cols,
                                                       const int32_t *__restrict__ n_touched, int32_t n_ent,
                                                       int64_t kd, float *__restrict__ M,
                                                       const float *__restrict__ g_proj, float lr)
{
    const int32_t target = n_ent + (int32_t)blockIdx.x;
    int32_t lo = 0, hi = n_touched[0];
    while (lo < hi) {                                     // first position with touched_cols[pos] >= target
        const int32_t mid = (lo + hi) >> 1;
        if (touched_cols[mid] < target) lo = mid + 1; else hi = mid;
    }
    if (lo >= n_touched[0] || touched_cols[lo] != target) return;
    float *m = M + (int64_t)blockIdx.x * kd;
    const float *g = g_proj + (int64_t)blockIdx.x * kd;
    for (int64_t idx = (int64_t)threadIdx.x * 4; idx < kd; idx += kThreads * 4) {
        float4 x = ld4(m + idx), gg = ld4(g + idx);
        const float s0 = lr * gg.x, s1 = lr * gg.y, s2 = lr * gg.z, s3 = lr * gg.w;
        st4(m + idx, make_float4(x.x - s0, x.y - s1, x.z - s2, x.w - s3));
    }
}

// ---------------------------------------------------------------------------------------------------
static ProjArgs proj_args(stx_ctx *c, const stx_incidence *inc, const stx_params *p)
{
    ProjArgs a;
    a.colidx = inc->a_colidx; a.packed = inc->at_packed; a.seg_id = inc->at_seg_id; a.seg_ptr = inc->at_seg_ptr;
    a.touched_cols = inc->at_touched_cols;
    a.E = p->ent; a.M = p->proj; a.Rv = p->rel;
    a.n_ent = (int32_t)c->cfg.n_ent;
    a.e_begin = (int32_t)(2 * inc->n_rows);               // relation columns follow the entity columns
    a.e_end = (int32_t)inc->nnz;
    a.d = c->cfg.dim; a.k = c->cfg.rel_dim;
    return a;
}

stx_status launch_transr_project(stx_ctx *c, const stx_incidence *inc, const stx_params *p)
{
    if (inc->n_rows == 0) return STX_OK;
    ProjArgs a = proj_args(c, inc, p);
    const int chunks = (int)((inc->n_rows + kProjRows - 1) / kProjRows);
    ProfScope prof(c, "k_transr_project");
    hipLaunchKernelGGL(k_transr_rows<false>, dim3(chunks), dim3(kThreads), 0, c->stream, a, (const float *)nullptr,
                       c->gbuf[0]);
    return hip_ok(hipGetLastError());
}

stx_status launch_transr_backward(stx_ctx *c, const stx_incidence *inc, const stx_params *p, stx_grads *g)
{
    if (inc->n_rows == 0) return STX_OK;
    ProjArgs a = proj_args(c, inc, p);
    const int chunks = (int)((inc->n_rows + kProjRows - 1) / kProjRows);
    const int chunks_dm = (int)((inc->n_rows + kProjRowsDm - 1) / kProjRowsDm);
    {
        ProfScope prof(c, "k_transr_gx");
        hipLaunchKernelGGL(k_transr_rows<true>, dim3(chunks), dim3(kThreads), 0, c->stream, a, c->gbuf[0], c->gbuf[1]);
    }
    {
        ProfScope prof(c, "k_transr_dm");
        hipLaunchKernelGGL(k_transr_dm, dim3(chunks_dm), dim3(kThreads), 0, c->stream, a, c->gbuf[0], g->proj,
                           c->gbuf[2]);
    }
    if (chunks_dm > 1) {
        ProfScope prof(c, "k_transr_dm_fixup");
        hipLaunchKernelGGL(k_transr_dm_fixup,
                           dim3(chunks_dm - 1, (unsigned)(((int64_t)a.k * a.d + 4 * kThreads - 1) / (4 * kThreads))),
                           dim3(kThreads), 0, c->stream, a, g->proj, c->gbuf[2]);
    }
    return hip_ok(hipGetLastError());
}

stx_status launch_transr_sgd_proj(stx_ctx *c, const stx_incidence *inc, stx_params *p, const stx_grads *g, float lr)
{
    if (inc->n_rows == 0) return STX_OK;
    ProfScope prof(c, "k_sgd_proj");
    hipLaunchKernelGGL(k_sgd_proj, dim3((unsigned)c->cfg.n_rel), dim3(kThreads), 0, c->stream, inc->at_touched_cols,
                       inc->n_touched, (int32_t)c->cfg.n_ent, (int64_t)c->cfg.rel_dim * c->cfg.dim, p->proj, g->proj,
                       lr);
    return hip_ok(hipGetLastError());
}

}  // namespace stx
