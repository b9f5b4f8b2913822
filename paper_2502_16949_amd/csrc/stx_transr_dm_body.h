// TransR: the product that forms dL/dM_r (SparseTransX Sec. 4.4, backward of the projection) and the sum of
// its partial matrices, as device functions: stx_transr.hip wraps them in kernels of their own, and the
// launches of the transposed incidence product (stx_backward.hip) can take them along, since both read
// only what the forward pass left behind and write different arrays.
#pragma once

#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float floatx16;

__device__ inline uint32_t bf16_bits(float v) { return (uint32_t)__builtin_bit_cast(uint16_t, (__bf16)v); }
__device__ inline uint32_t pack2(float lo, float hi) { return bf16_bits(lo) | (bf16_bits(hi) << 16); }
__device__ inline uint4 pack8(float4 a, float4 b)
{
    return make_uint4(pack2(a.x, a.y), pack2(a.z, a.w), pack2(b.x, b.y), pack2(b.z, b.w));
}
__device__ inline bf16x8 as_frag(uint4 v) { return __builtin_bit_cast(bf16x8, v); }
__device__ inline uint4 ld16(const uint16_t *p) { return *reinterpret_cast<const uint4 *>(p); }
__device__ inline floatx16 zero16()
{
    floatx16 r;
#pragma unroll
    for (int i = 0; i < 16; ++i) r[i] = 0.f;
    return r;
}

// dL/dM_r = sum over the rows i of relation r of bf16(gy_i) bf16(x_i)^T, x_i = E[h_i] - E[t_i].
// One workgroup per dM item (up to four 64-entry tiles of one relation) and per 128 x 128 block of the
// matrix (yblock); the reduction runs over entries, 16 per MFMA, both operands read in operand order
// from the transposed tiles.  Wavefront w owns the 64 x 64 quarter (w/2, w%2).  A relation with one
// item gets its matrix written directly; otherwise every item writes a partial matrix into its slot
// and transr_dm_fixup_body adds the slots in order.  No barrier and no LDS in here; the fragments of
// a reduction step are requested right before its products, and the compiler moves those requests
// ahead as far as 128 registers allow, which keeps four workgroups on a CU.
__device__ inline void transr_dm_body(const int item, const int yblock, const DmArgs &p)
{
    const int4 it = p.dm_items[item];                     // readable for every item of the launch bound
    if (item >= p.counts[1]) return;
    const int rel = it.x, tile0 = it.y, entries = it.z, slot = it.w;
    const int l = threadIdx.x & 63, w = threadIdx.x >> 6, l31 = l & 31, kg = l >> 5;
    const int mtl = p.k >> 5, ntl = p.d >> 5, dblocks = (p.d + 127) >> 7;
    const int kb = yblock / dblocks, db = yblock - kb * dblocks;
    const int mt0 = 4 * kb + 2 * (w >> 1), nt0 = 4 * db + 2 * (w & 1);
    if (mt0 >= mtl || nt0 >= ntl) return;
    const bool m1 = mt0 + 1 < mtl, n1 = nt0 + 1 < ntl;
    floatx16 acc[2][2];
#pragma unroll
    for (int i = 0; i < 4; ++i) acc[i >> 1][i & 1] = zero16();
    const int ntile = (entries + 63) >> 6;
    for (int t = 0; t < ntile; ++t) {
        const int nks = (min(64, entries - 64 * t) + 15) >> 4;
        const uint16_t *ga = p.gyt + ((int64_t)(tile0 + t) * 64 * p.k) + (int64_t)l * 8;
        const uint16_t *xb = p.xt + ((int64_t)(tile0 + t) * 64 * p.d) + (int64_t)l * 8;
#pragma unroll
        for (int ks = 0; ks < 4; ++ks) {
            if (ks < nks) {
                const uint4 z = make_uint4(0, 0, 0, 0);
                const uint4 a0 = ld16(ga + (int64_t)(ks * mtl + mt0) * 512);
                const uint4 a1 = m1 ? ld16(ga + (int64_t)(ks * mtl + mt0 + 1) * 512) : z;
                const uint4 b0 = ld16(xb + (int64_t)(ks * ntl + nt0) * 512);
                const uint4 b1 = n1 ? ld16(xb + (int64_t)(ks * ntl + nt0 + 1) * 512) : z;
                acc[0][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a0), as_frag(b0), acc[0][0], 0, 0, 0);
                if (n1) acc[0][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a0), as_frag(b1), acc[0][1], 0, 0, 0);
                if (m1) acc[1][0] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a1), as_frag(b0), acc[1][0], 0, 0, 0);
                if (m1 && n1) acc[1][1] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(as_frag(a1), as_frag(b1), acc[1][1], 0, 0, 0);
            }
        }
    }
    const int64_t kd = (int64_t)p.k * p.d;
    const bool update = slot < 0 && p.fused;             // the relation's only item: apply the step right here
    float *dst = slot >= 0 ? p.partials + slot * kd : (update ? p.M + rel * kd : p.g_proj + rel * kd);
#pragma unroll
    for (int mi = 0; mi < 2; ++mi) {
#pragma unroll
        for (int ni = 0; ni < 2; ++ni) {
            if ((mi == 0 || m1) && (ni == 0 || n1)) {
                const int j = 32 * (nt0 + ni) + l31;
                float old[16];
                if (update) {
#pragma unroll
                    for (int v = 0; v < 16; ++v)
                        old[v] = dst[(int64_t)(32 * (mt0 + mi) + 8 * (v >> 2) + 4 * kg + (v & 3)) * p.d + j];
                }
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int a = 32 * (mt0 + mi) + 8 * (v >> 2) + 4 * kg + (v & 3);
                    float val = acc[mi][ni][v];
                    if (update) { const float step = p.lr * val; val = old[v] - step; }
                    dst[(int64_t)a * p.d + j] = val;
                }
            }
        }
    }
}

// Elements of the matrix per workgroup of the sum below: four consecutive ones per thread.
constexpr int kDmFixupSlice = 4 * kThreads;

// Fix-up item `item` (a relation with several dM items): adds up the relation's partial matrices in item
// order (slice `yslice` of the matrix) and stores the sum, or applies the update with it.
__device__ inline void transr_dm_fixup_body(const int item, const int yslice, const DmArgs &p)
{
    if (item >= p.counts[2]) return;
    const int4 tail = p.fix_items[item];                  // {relation, first slot, slots, 0}
    const int parts = tail.z;
    const int64_t kd = (int64_t)p.k * p.d;
    const int64_t idx = ((int64_t)yslice * kThreads + threadIdx.x) * 4;
    if (idx >= kd) return;
    const float *src = p.partials + (int64_t)tail.y * kd + idx;
    float4 a = ld4(src);
    int u = 1;
    // (a relation with a quarter of a large batch's rows has more than a hundred partial matrices: sixteen in
    // flight, then four, added in item order)
    for (; u + 15 < parts; u += 16) {
        float4 v[16];
#pragma unroll
        for (int q = 0; q < 16; ++q) v[q] = ld4(src + (int64_t)(u + q) * kd);
#pragma unroll
        for (int q = 0; q < 16; ++q) { a.x += v[q].x; a.y += v[q].y; a.z += v[q].z; a.w += v[q].w; }
    }
    for (; u + 3 < parts; u += 4) {
        float4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) v[q] = ld4(src + (int64_t)(u + q) * kd);
#pragma unroll
        for (int q = 0; q < 4; ++q) { a.x += v[q].x; a.y += v[q].y; a.z += v[q].z; a.w += v[q].w; }
    }
    for (; u < parts; ++u) {
        float4 v = ld4(src + (int64_t)u * kd);
        a.x += v.x; a.y += v.y; a.z += v.z; a.w += v.w;
    }
    const int64_t off = (int64_t)tail.x * kd + idx;
    if (p.fused) {
        const float4 m = ld4(p.M + off);
        const float s0 = p.lr * a.x, s1 = p.lr * a.y, s2 = p.lr * a.z, s3 = p.lr * a.w;
        st4(p.M + off, make_float4(m.x - s0, m.y - s1, m.z - s2, m.w - s3));
    } else {
        st4(p.g_proj + off, a);
    }
}

}  // namespace stx
