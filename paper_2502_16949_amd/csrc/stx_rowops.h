// Row-level pieces shared by the forward kernels: a table row held as float4 slices by the LPR lanes of
// a group, the `hrt` / `ht` gathers of SparseTransX Sec. 4.2, and the distance terms of Sec. 4.3 / 4.6.
#pragma once

#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

template <int ITERS>
struct RowVec {
    float4 v[ITERS];
};

__device__ inline float4 add4(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ inline float4 sub4(float4 a, float4 b) { return make_float4(a.x - b.x, a.y - b.y, a.z - b.z, a.w - b.w); }

template <int LPR, int ITERS>
__device__ inline void load_vec(const float *__restrict__ p, int d4, int lig, RowVec<ITERS> &x)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        x.v[it] = j < d4 ? ld4(p + 4 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
// the same with non-temporal loads: for rows that are used once and should not displace others in the caches
template <int LPR, int ITERS>
__device__ inline void load_vec_stream(const float *__restrict__ p, int d4, int lig, RowVec<ITERS> &x)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        x.v[it] = j < d4 ? ld4_stream(p + 4 * j) : make_float4(0.f, 0.f, 0.f, 0.f);
    }
}
template <int LPR, int ITERS>
__device__ inline void store_vec(float *__restrict__ p, int d4, int lig, const RowVec<ITERS> &x)
{
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) st4(p + 4 * j, x.v[it]);
    }
}

// x = (X[c0] + X[c1]) - X[c2] (hrt) or X[c0] - X[c2] (ht): each operation rounded once, in this order.
template <int LPR, int ITERS, bool HRT>
__device__ inline void gather_row(const float *__restrict__ X, int dim, int d4, int lig, int32_t c0, int32_t c1,
                                  int32_t c2, RowVec<ITERS> &x)
{
    const float *p0 = X + (int64_t)c0 * dim, *p2 = X + (int64_t)c2 * dim;
    const float *p1 = HRT ? X + (int64_t)c1 * dim : p0;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        int j = lig + it * LPR;
        if (j < d4) {
            float4 a = ld4(p0 + 4 * j), c = ld4(p2 + 4 * j);
            if (HRT) {
                float4 b = ld4(p1 + 4 * j);
                a.x += b.x; a.y += b.y; a.z += b.z; a.w += b.w;
            }
            x.v[it] = make_float4(a.x - c.x, a.y - c.y, a.z - c.z, a.w - c.w);
        } else {
            x.v[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        }
    }
}

// ---- distance pieces -------------------------------------------------------------------------------
template <int DIST>
__device__ inline float term(float y)
{
    if (DIST == STX_L1) return fabsf(y);
    if (DIST == STX_L2 || DIST == STX_L2_SQ) return y * y;
    float f = y - floorf(y);
    float m = fminf(f, 1.0f - f);
    return DIST == STX_TORUS_L1 ? m : m * m;
}
template <int DIST>
__device__ inline float finish(float acc)
{
    return (DIST == STX_L2 || DIST == STX_TORUS_L2) ? sqrtf(acc) : acc;
}
// d(dist)/dy times coef.  cs = coef for the L1 kinds, coef / dist (0 if dist == 0) for the L2 kinds,
// 2 coef for the squared L2 norm.
template <int DIST>
__device__ inline float dterm(float y, float cs)
{
    if (DIST == STX_L1) return y > 0.f ? cs : (y < 0.f ? -cs : 0.f);
    if (DIST == STX_L2 || DIST == STX_L2_SQ) return y * cs;
    float f = y - floorf(y);
    float sg = (f > 0.f && f < 0.5f) ? 1.f : (f > 0.5f ? -1.f : 0.f);
    if (DIST == STX_TORUS_L1) return sg * cs;
    return sg * fminf(f, 1.0f - f) * cs;
}
// For the L1 kinds d(dist)/dy is -1, 0 or +1, so a row of dL/dy is one coefficient times a sign pattern.
// Such rows are stored packed: one byte per four elements, two bits each holding the element's sign as a
// two's-complement number (01: +1, 11: -1, 00: 0), plus the coefficient: 36 bytes instead of 512 at dim 128.
// The reader sign-extends the two bits, converts to float and does one fused multiply-add with the
// coefficient, which is exact: c * (+-1 or 0) has no rounding, so the sum equals adding +c, -c or 0.
template <int DIST>
__device__ inline unsigned sign_bits(float4 y)
{
    const float v[4] = {y.x, y.y, y.z, y.w};
    unsigned b = 0;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const float s = dterm<DIST>(v[q], 1.0f);
        b |= (s > 0.f ? 1u : (s < 0.f ? 3u : 0u)) << (2 * q);
    }
    return b;
}
constexpr bool is_sign_kind(int dist) { return dist == STX_L1 || dist == STX_TORUS_L1; }

template <int DIST>
__device__ inline float coef_scale(float coef, float dist)
{
    if (DIST == STX_L2 || DIST == STX_TORUS_L2) return dist > 0.f ? coef / dist : 0.f;
    if (DIST == STX_L2_SQ) return 2.0f * coef;
    return coef;
}

template <int LPR, int ITERS, int DIST>
__device__ inline float row_distance(const RowVec<ITERS> &x)
{
    float acc = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        acc += term<DIST>(x.v[it].x);
        acc += term<DIST>(x.v[it].y);
        acc += term<DIST>(x.v[it].z);
        acc += term<DIST>(x.v[it].w);
    }
    return finish<DIST>(group_sum<LPR>(acc));
}

template <int LPR, int ITERS>
__device__ inline float group_dot(const RowVec<ITERS> &a, const RowVec<ITERS> &b)
{
    float acc = 0.f;
#pragma unroll
    for (int it = 0; it < ITERS; ++it) {
        acc += a.v[it].x * b.v[it].x;
        acc += a.v[it].y * b.v[it].y;
        acc += a.v[it].z * b.v[it].z;
        acc += a.v[it].w * b.v[it].w;
    }
    return group_sum<LPR>(acc);
}

#define STX_DISPATCH_ROW(L, FN, ...)                                                      \
    do {                                                                                  \
        if (L.lpr == 8 && L.iters == 1) FN<8, 1>(__VA_ARGS__);                            \
        else if (L.lpr == 16 && L.iters == 1) FN<16, 1>(__VA_ARGS__);                     \
        else if (L.lpr == 32 && L.iters == 1) FN<32, 1>(__VA_ARGS__);                     \
        else if (L.lpr == 64 && L.iters == 1) FN<64, 1>(__VA_ARGS__);                     \
        else if (L.lpr == 64 && L.iters == 2) FN<64, 2>(__VA_ARGS__);                     \
        else if (L.lpr == 64 && L.iters == 3) FN<64, 3>(__VA_ARGS__);                     \
        else FN<64, 4>(__VA_ARGS__);                                                      \
    } while (0)

}  // namespace stx
