// Device-side bodies of the radix-sort passes over the column ids of A (see stx_build.hip), shared by the
// kernels that run them alone and by the launches that run them beside another, independent piece of
// work (stx_step.hip).
#pragma once

#include "stx_device.h"
#include "stx_internal.h"

namespace stx {

// Tile histograms of the digit at `shift` for the later passes.
template <int ITEMS>
__device__ inline void hist_body(const int block, const int32_t *__restrict__ keys, int32_t nnz, int shift,
                                 int radix, int32_t *__restrict__ table)
{
    __shared__ int32_t s_hist[256];
    const int tid = threadIdx.x;
    s_hist[tid] = 0;
    __syncthreads();
    const int32_t base = block * (kThreads * ITEMS);
    int32_t kv[ITEMS];                                   // all loads first, so that they are in flight together
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int32_t e = base + it * kThreads + tid;
        kv[it] = e < nnz ? keys[e] : 0;
    }
    // The lanes of a wavefront that hold the same digit are found by a ballot per bit, and one of them adds their
    // number: power-law keys put many lanes on one counter, and LDS serialises atomics on one address.
    const int bits = 31 - __clz(radix), lane = tid & 63;
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        const int32_t e = base + it * kThreads + tid;
        const bool valid = e < nnz;
        const int dgt = (kv[it] >> shift) & (radix - 1);
        const uint64_t m = digit_class_mask(dgt, valid, bits);
        if (valid && ((m >> lane) >> 1) == 0) atomicAdd(&s_hist[dgt], (int32_t)__popcll(m));   // highest lane of its class
    }
    __syncthreads();
    if (tid < radix) table[block * radix + tid] = s_hist[tid];
}

// Stable scatter of one tile by the digit at `shift`.  Element order inside a tile is
// (wavefront, iteration, lane): wavefront w owns the contiguous span [w*512, (w+1)*512) of the tile.
// The rank of a key among equal digits is
//   (count in earlier wavefronts) + (count in earlier iterations of this wavefront) + (equal lanes below),
// the last term from a ballot match over the digit's bits.  The base offset of a (digit, tile) is the
// number of keys with a smaller digit anywhere plus those with the same digit in earlier tiles: read
// derived here from the raw tile counts: directly when there are few tiles (TWO_LEVEL false), through
// the group sums of k_super_sums otherwise.
// `block` is the tile (the index of the workgroup among those of the scatter; the launch may hold others).
// ARENA: the body's LDS arrays live in the kScatterLds bytes at `lds` instead of arrays of its own.
template <bool FIRST, bool TWO_LEVEL, int ITEMS, bool ARENA = false>
__device__ inline void scatter_body(const int block, const ScatterArgs &a, unsigned char *lds = nullptr)
{
    const int32_t *__restrict__ keys_in = a.keys_in;
    const int32_t *__restrict__ pay_in = a.pay_in;
    int32_t *__restrict__ keys_out = a.keys_out;
    int32_t *__restrict__ pay_out = a.pay_out;
    const int32_t nnz = a.nnz;
    const int shift = a.shift, bits = a.bits, ntiles = a.ntiles;
    const int32_t *__restrict__ table = a.table;
    const int32_t *__restrict__ super = a.super;
    int32_t *s_goff, (*s_hist)[256], *s_tot, *s_bel;
    if constexpr (ARENA) {
        int32_t *p = reinterpret_cast<int32_t *>(lds);
        s_goff = p; s_hist = reinterpret_cast<int32_t (*)[256]>(p + 256); s_tot = p + 1280; s_bel = p + 2304;
    } else {
        __shared__ int32_t o_goff[256];
        __shared__ int32_t o_hist[4][256];
        __shared__ int32_t o_tot[TWO_LEVEL ? 1 : 1024], o_bel[TWO_LEVEL ? 1 : 1024];
        s_goff = o_goff; s_hist = o_hist; s_tot = o_tot; s_bel = o_bel;
    }
    const int tid = threadIdx.x, lane = tid & 63, w = tid >> 6;
    const int radix = 1 << bits;
    for (int i = tid; i < 4 * 256; i += kThreads) (&s_hist[0][0])[i] = 0;
    int32_t key[ITEMS], pay[ITEMS], rank[ITEMS];
    const int32_t wave_base = block * (kThreads * ITEMS) + w * (64 * ITEMS);
    const uint64_t lanes_below = (1ull << lane) - 1ull;
    auto load_items = [&]() {
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {             // all loads at once, so that they are in flight together
            const int32_t e = wave_base + it * 64 + lane;
            const bool valid = e < nnz;
            key[it] = valid ? keys_in[e] : 0;
            pay[it] = FIRST ? e : (valid ? pay_in[e] : 0);
        }
    };
    // Large sorts: the tile's keys are requested before the offsets are derived from the histogram tables (a dozen
    // dependent round trips with the two-level table), so that the two waits overlap.  The small sorts share
    // launches with kernels that are capped at 64 registers and keep the order that needs fewer of them.
    constexpr bool EARLY = ITEMS > kSortItems && !ARENA;
    if constexpr (EARLY) load_items();
    if (TWO_LEVEL) {
        int32_t below = 0, total = 0;
        if (tid < radix) {
            const int me = block, g_me = me / kSuperTile, ngroups = (ntiles + kSuperTile - 1) / kSuperTile;
            // (integer sums: any order gives the same offsets; eight loads are in flight per step)
            constexpr int U = 8;
            for (int g0 = 0; g0 < ngroups; g0 += U) {
                int32_t v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = g0 + u < ngroups ? super[(g0 + u) * radix + tid] : 0;
#pragma unroll
                for (int u = 0; u < U; ++u) {
                    total += v[u];
                    below += g0 + u < g_me ? v[u] : 0;
                }
            }
            for (int t0 = g_me * kSuperTile; t0 < me; t0 += U) {
                int32_t v[U];
#pragma unroll
                for (int u = 0; u < U; ++u) v[u] = t0 + u < me ? table[(t0 + u) * radix + tid] : 0;
#pragma unroll
                for (int u = 0; u < U; ++u) below += v[u];
            }
        }
        int32_t base = block_exclusive_scan(total, nullptr);
        s_goff[tid] = base + below;
    } else {
        // All 256 threads share the table: a thread owns four neighbouring digits (one 16-byte load per
        // tile row) and every `parts`-th tile; up to SCAN loads are in flight per thread (few enough registers
        // that this body does not lower the occupancy of the kernels it shares launches with).
        const int me = block;
        int32_t below = 0, total = 0;
        if (radix >= 4) {
            const int r4 = radix >> 2, parts = kThreads / r4, d4 = tid % r4, q = tid / r4;
            int4 tot = make_int4(0, 0, 0, 0), bel = make_int4(0, 0, 0, 0);
            constexpr int SCAN = 8;
            for (int t0 = q; t0 < ntiles; t0 += SCAN * parts) {
                int4 v[SCAN];
#pragma unroll
                for (int u = 0; u < SCAN; ++u) {
                    const int t = t0 + u * parts;
                    v[u] = t < ntiles ? *reinterpret_cast<const int4 *>(table + t * radix + 4 * d4)
                                      : make_int4(0, 0, 0, 0);
                }
#pragma unroll
                for (int u = 0; u < SCAN; ++u) {
                    const int t = t0 + u * parts;
                    tot.x += v[u].x; tot.y += v[u].y; tot.z += v[u].z; tot.w += v[u].w;
                    if (t < me) { bel.x += v[u].x; bel.y += v[u].y; bel.z += v[u].z; bel.w += v[u].w; }
                }
            }
            *reinterpret_cast<int4 *>(&s_tot[q * radix + 4 * d4]) = tot;
            *reinterpret_cast<int4 *>(&s_bel[q * radix + 4 * d4]) = bel;
            __syncthreads();
            if (tid < radix)
                for (int qq = 0; qq < parts; ++qq) {
                    total += s_tot[qq * radix + tid];
                    below += s_bel[qq * radix + tid];
                }
        } else if (tid < radix) {   // two bins only
            for (int t = 0; t < ntiles; ++t) {
                const int32_t v = table[t * radix + tid];
                total += v;
                below += t < me ? v : 0;
            }
        }
        int32_t base = block_exclusive_scan(total, nullptr);
        s_goff[tid] = base + below;
    }
    __syncthreads();

    if constexpr (!EARLY) load_items();
#pragma unroll
    for (int it = 0; it < ITEMS; ++it) {
        int32_t e = wave_base + it * 64 + lane;
        bool valid = e < nnz;
        int dgt = (key[it] >> shift) & (radix - 1);
        const uint64_t m = digit_class_mask(dgt, valid, bits);
        int32_t prior = s_hist[w][dgt];
        rank[it] = prior + __popcll(m & lanes_below);
        bool leader = valid && ((m >> lane) >> 1) == 0;   // highest lane of its digit class
        if (leader) s_hist[w][dgt] = prior + __popcll(m);
    }
    __syncthreads();
    int32_t tile_count = 0;                              // keys of the tile with digit `tid`
    if (tid < radix) {
#pragma unroll
        for (int w2 = 0; w2 < 4; ++w2) {
            int32_t c = s_hist[w2][tid];
            s_hist[w2][tid] = tile_count;
            tile_count += c;
        }
    }
    // Large sorts (tiles of kBigSortItems keys per thread): the tile is put in order in LDS first and written from
    // there, so that neighbouring lanes write neighbouring addresses and a digit's keys of one tile (16 on
    // average with 256 digits: 64 bytes) fill whole sectors; written straight from the registers every key is a
    // partial write of its own, and the pass moves 2.5 times the bytes it has to.
    constexpr bool LOCAL = ITEMS > kSortItems && !ARENA;
    if constexpr (LOCAL) {
        __shared__ int32_t s_dstart[256];
        __shared__ int32_t s_k[kThreads * ITEMS], s_p[kThreads * ITEMS];
        s_dstart[tid] = block_exclusive_scan(tile_count, nullptr);   // (its barriers also publish s_hist)
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            const int32_t e = wave_base + it * 64 + lane;
            if (e < nnz) {
                const int dgt = (key[it] >> shift) & (radix - 1);
                const int32_t lp = s_dstart[dgt] + s_hist[w][dgt] + rank[it];
                s_k[lp] = key[it];
                s_p[lp] = pay[it];
            }
        }
        __syncthreads();
        const int32_t tile_n = min(kThreads * ITEMS, nnz - block * (kThreads * ITEMS));
        for (int32_t i = tid; i < tile_n; i += kThreads) {
            const int32_t kv = s_k[i];
            const int dgt = (kv >> shift) & (radix - 1);
            const int32_t pos = s_goff[dgt] + (i - s_dstart[dgt]);
            keys_out[pos] = kv;
            pay_out[pos] = s_p[i];
        }
    } else {
        __syncthreads();
#pragma unroll
        for (int it = 0; it < ITEMS; ++it) {
            int32_t e = wave_base + it * 64 + lane;
            if (e < nnz) {
                int dgt = (key[it] >> shift) & (radix - 1);
                int32_t pos = s_goff[dgt] + s_hist[w][dgt] + rank[it];
                keys_out[pos] = key[it];
                pay_out[pos] = pay[it];
            }
        }
    }
}

}  // namespace stx
