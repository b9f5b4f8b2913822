// C-ABI entry points of libstx: argument checks, workspace layout, call-order state, and dispatch to
// the kernel launchers.  No arithmetic of the method happens here.
#include <cstdio>
#include <new>

#include "stx_internal.h"

using namespace stx;

namespace {

inline size_t align_up(size_t v, size_t a = 256) { return (v + a - 1) / a * a; }

struct Layout {
    size_t ctrl, keys[3], pay[2], cix[2], table, table1, super, tile_heads, loss_partials, partials, gbuf[4], total;
    size_t tr_items, tr_dm_items, tr_fix_items, tr_counts, tr_m16, tr_m16t, tr_xt, tr_gyt;
    size_t colmap, rel_cnt;
    int map_words;
    int64_t rows_max, nnz_max, cols_max;
    int ld, out_dim, ntiles_max, fwd_blocks_max, n_gbuf;
    int sort_bits, sort_passes, digit_bits;
};

stx_status check_config(const stx_config *c)
{
    if (!c) return STX_ERR_NULL;
    if (c->model < STX_TRANSE || c->model > STX_TORUSE) return STX_ERR_BAD_ARG;
    if (c->dist < STX_L1 || c->dist > STX_L2_SQ) return STX_ERR_BAD_ARG;
    if (c->reduce != STX_SUM && c->reduce != STX_MEAN) return STX_ERR_BAD_ARG;
    if (c->dim <= 0 || c->dim % 4 != 0 || c->dim > kMaxDim) return STX_ERR_BAD_ARG;
    if (c->model == STX_TRANSR && (c->rel_dim <= 0 || c->rel_dim % 4 != 0 || c->rel_dim > kMaxDim))
        return STX_ERR_BAD_ARG;
    // the matrix-core path of TransR works on 32-wide tiles and bfloat16 operands
    if (c->model == STX_TRANSR && (c->dim % 32 != 0 || c->rel_dim % 32 != 0 || c->dim > kMaxProjDim ||
                                   c->rel_dim > kMaxProjDim || !(c->flags & STX_FLAG_BF16_PROJ)))
        return STX_ERR_UNSUPPORTED;
    if (c->n_ent <= 0 || c->n_rel <= 0 || c->n_ent + c->n_rel >= (int64_t)1 << 31) return STX_ERR_BAD_ARG;
    if (c->max_batch <= 0 || c->max_neg < 0) return STX_ERR_BAD_ARG;
    if (3 * (int64_t)c->max_batch * (1 + (int64_t)c->max_neg) >= ((int64_t)1 << 29)) return STX_ERR_BAD_ARG;
    if (!(c->margin >= 0.0f)) return STX_ERR_BAD_ARG;
    if (c->flags & ~(STX_FLAG_RENORM_W | STX_FLAG_BF16_PROJ)) return STX_ERR_BAD_ARG;
    return STX_OK;
}

Layout make_layout(const stx_config *c)
{
    Layout L{};
    L.rows_max = (int64_t)c->max_batch * (1 + c->max_neg);
    L.nnz_max = 3 * L.rows_max;
    L.cols_max = L.nnz_max < c->n_ent + c->n_rel ? L.nnz_max : c->n_ent + c->n_rel;
    int rel_dim = c->model == STX_TRANSR ? c->rel_dim : c->dim;
    L.ld = c->dim > rel_dim ? c->dim : rel_dim;
    L.out_dim = rel_dim;
    L.ntiles_max = (int)((L.nnz_max + kSortTile - 1) / kSortTile);
    Launch rl = row_launch(c->dim);
    L.fwd_blocks_max = (int)((c->max_batch + (kThreads / rl.lpr) - 1) / (kThreads / rl.lpr));
    if (c->model == STX_TRANSR) {   // one loss partial per row item of the fused forward kernel
        const int64_t items = L.rows_max / kProjRows + (L.rows_max < c->n_rel ? L.rows_max : c->n_rel) + 1;
        if (items > L.fwd_blocks_max) L.fwd_blocks_max = (int)items;
    }
    int64_t ncol = c->n_ent + c->n_rel;
    L.sort_bits = 1;
    while (((int64_t)1 << L.sort_bits) < ncol) ++L.sort_bits;
    L.sort_passes = (L.sort_bits + 7) / 8;
    L.digit_bits = (L.sort_bits + L.sort_passes - 1) / L.sort_passes;
    L.n_gbuf = (c->model == STX_TRANSH || c->model == STX_TRANSR) ? 3 : 1;

    size_t off = 0;
    auto take = [&](size_t bytes) { size_t o = off; off = align_up(off + bytes); return o; };
    L.ctrl = take(CTRL_WORDS * sizeof(int32_t));
    for (int i = 0; i < 3; ++i) L.keys[i] = take((size_t)L.nnz_max * 4);
    for (int i = 0; i < 2; ++i) L.pay[i] = take((size_t)L.nnz_max * 4);
    for (int i = 0; i < 2; ++i) L.cix[i] = take((size_t)L.nnz_max * 4);
    L.table = take((size_t)256 * L.ntiles_max * 4);
    L.table1 = take((size_t)256 * L.ntiles_max * 4);
    L.super = take((size_t)256 * (L.ntiles_max / kSuperTile + 1) * 4);
    L.tile_heads = take((size_t)(L.ntiles_max + 1) * 4);
    L.loss_partials = take((size_t)(L.fwd_blocks_max + 1) * 4);
    // two partial rows per tile of the transposed product; TransH runs a second product over the relation
    // entries in the same launch
    L.partials = take((size_t)(L.nnz_max / kSegTileMin + L.rows_max / kSegTileMin + 4) * 2 * L.ld * 4);
    for (int i = 0; i < 4; ++i) {
        size_t bytes = (size_t)L.rows_max * L.ld * 4;
        const size_t pk_bytes = (size_t)packed_coef_offset(L.rows_max, packed_stride(c->dim)) + (size_t)L.rows_max * 4;
        if (i == 0 && bytes < pk_bytes) bytes = pk_bytes;   // packed dL/dx records and coefficients (tiny dims only)
        if (c->model == STX_TRANSR && i == 2)   // partial dL/dM_r matrices: two per chunk of the dM product
            bytes = (size_t)(L.rows_max / kProjRowsDm + 2) * 2 * (size_t)c->rel_dim * c->dim * 4;
        L.gbuf[i] = i < L.n_gbuf ? take(bytes) : 0;
    }
    {
        const int64_t words = (c->n_ent + c->n_rel + 31) / 32;
        L.map_words = words <= kMapMaxWords ? (int)words : 0;
        L.colmap = take((size_t)3 * L.map_words * 4 + 4);
    }
    if (c->model == STX_TRANSR) {
        // every relation segment adds at most one item that is not full
        const size_t segs = (size_t)(L.rows_max < c->n_rel ? L.rows_max : c->n_rel);
        const size_t items = (size_t)L.rows_max / kProjRows + segs, dm_items = (size_t)L.rows_max / kProjRowsDm + segs;
        const size_t kd = (size_t)c->rel_dim * c->dim;
        L.tr_items = take((items + 1) * 16);
        L.tr_dm_items = take((dm_items + 1) * 16);
        L.tr_fix_items = take(((size_t)L.rows_max / (kProjRowsDm + 1) + 1) * 16);
        L.tr_counts = take(64 * sizeof(int32_t));
        L.tr_m16 = take((size_t)c->n_rel * kd * 2);
        L.tr_m16t = take((size_t)c->n_rel * kd * 2);
        L.tr_xt = take((items + 1) * kProjRows * c->dim * 2);
        L.tr_gyt = take((items + 1) * kProjRows * c->rel_dim * 2);
        L.rel_cnt = take((size_t)2 * c->n_rel * 4);
    }
    L.total = off;
    return L;
}

stx_status check_incidence_arrays(const stx_incidence *inc)
{
    if (!inc) return STX_ERR_NULL;
    if (!inc->a_rowptr || !inc->a_colidx || !inc->a_vals || !inc->at_touched_cols || !inc->at_seg_ptr ||
        !inc->at_row_idx || !inc->at_sign || !inc->at_seg_id || !inc->at_packed || !inc->n_touched)
        return STX_ERR_NULL;
    return STX_OK;
}

stx_status check_built(const stx_ctx *ctx, const stx_incidence *inc)
{
    stx_status s = check_incidence_arrays(inc);
    if (s != STX_OK) return s;
    if (inc->b < 0 || inc->b > ctx->cfg.max_batch || inc->k < 0 || inc->k > ctx->cfg.max_neg) return STX_ERR_BAD_ARG;
    if (inc->n_rows != (int64_t)inc->b * (1 + inc->k) || inc->nnz != 3 * inc->n_rows) return STX_ERR_BAD_ARG;
    return STX_OK;
}

stx_status check_params(const stx_ctx *ctx, const stx_params *p)
{
    if (!p || !p->ent) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSH && (!p->rel || !p->w)) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSR && (!p->rel || !p->proj)) return STX_ERR_NULL;
    if (p->rel_weight && ctx->cfg.model != STX_TRANSE && ctx->cfg.model != STX_TORUSE) return STX_ERR_UNSUPPORTED;
    return STX_OK;
}

bool stacked(const stx_ctx *c) { return c->cfg.model == STX_TRANSE || c->cfg.model == STX_TORUSE; }

// After a stx_train_step that named its next batch, the A arrays of inc already hold that next batch while
// inc->b, k, n_rows and the A^T arrays describe the batch just trained: a call that reads A must not pair them.
stx_status check_a_current(const stx_ctx *ctx, const stx_incidence *inc)
{
    return (ctx->ahead.armed && ctx->ahead.emit_done && ctx->ahead.inc == inc) ? STX_ERR_STATE : STX_OK;
}

}  // namespace

extern "C" {

stx_status stx_workspace_bytes(const stx_config *cfg, size_t *bytes)
{
    if (!bytes) return STX_ERR_NULL;
    stx_status s = check_config(cfg);
    if (s != STX_OK) return s;
    *bytes = make_layout(cfg).total;
    return STX_OK;
}

stx_status stx_create(const stx_config *cfg, void *workspace, size_t workspace_bytes, void *stream, stx_ctx **out)
{
    if (!out) return STX_ERR_NULL;
    *out = nullptr;
    stx_status s = check_config(cfg);
    if (s != STX_OK) return s;
    if (!workspace) return STX_ERR_NULL;
    Layout L = make_layout(cfg);
    if (workspace_bytes < L.total || ((uintptr_t)workspace & 255u)) return STX_ERR_WORKSPACE;
    stx_ctx *c = new (std::nothrow) stx_ctx();
    if (!c) return STX_ERR_BAD_ARG;
    c->cfg = *cfg;
    if (cfg->model != STX_TRANSR) c->cfg.rel_dim = cfg->dim;
    c->stream = (hipStream_t)stream;
    c->ld = L.ld;
    c->out_dim = L.out_dim;
    c->rows_max = L.rows_max;
    c->nnz_max = L.nnz_max;
    c->cols_max = L.cols_max;
    c->sort_bits = L.sort_bits;
    c->sort_passes = L.sort_passes;
    c->digit_bits = L.digit_bits;
    c->ntiles_max = L.ntiles_max;
    c->fwd_blocks_max = L.fwd_blocks_max;
    char *base = (char *)workspace;
    c->ctrl = (int32_t *)(base + L.ctrl);
    for (int i = 0; i < 3; ++i) c->keys[i] = (int32_t *)(base + L.keys[i]);
    for (int i = 0; i < 2; ++i) c->pay[i] = (int32_t *)(base + L.pay[i]);
    c->table = (int32_t *)(base + L.table);
    c->table1 = (int32_t *)(base + L.table1);
    for (int i = 0; i < 2; ++i) c->cix[i] = (int32_t *)(base + L.cix[i]);
    c->cix_cur = 0;
    c->super = (int32_t *)(base + L.super);
    c->tile_heads = (int32_t *)(base + L.tile_heads);
    c->loss_partials = (float *)(base + L.loss_partials);
    c->partials = (float *)(base + L.partials);
    for (int i = 0; i < 4; ++i) c->gbuf[i] = i < L.n_gbuf ? (float *)(base + L.gbuf[i]) : nullptr;
    const bool tr = cfg->model == STX_TRANSR;
    c->tr_items = tr ? (int32_t *)(base + L.tr_items) : nullptr;
    c->tr_dm_items = tr ? (int32_t *)(base + L.tr_dm_items) : nullptr;
    c->tr_fix_items = tr ? (int32_t *)(base + L.tr_fix_items) : nullptr;
    c->tr_counts = tr ? (int32_t *)(base + L.tr_counts) : nullptr;
    c->tr_m16 = tr ? (uint16_t *)(base + L.tr_m16) : nullptr;
    c->tr_m16t = tr ? (uint16_t *)(base + L.tr_m16t) : nullptr;
    c->tr_xt = tr ? (uint16_t *)(base + L.tr_xt) : nullptr;
    c->tr_gyt = tr ? (uint16_t *)(base + L.tr_gyt) : nullptr;
    const bool rc = tr && cfg->n_rel <= kRelCntMax;
    c->rel_cnt[0] = rc ? (int32_t *)(base + L.rel_cnt) : nullptr;
    c->rel_cnt[1] = rc ? c->rel_cnt[0] + cfg->n_rel : nullptr;
    c->cnt_cur = 0;
    c->cnt_ptr = nullptr;
    c->cnt_inc = nullptr;
    c->prep_inc = nullptr;
    c->prep_whole = 0;
    c->tr_fused_inc = nullptr;
    c->dm_ride = DmRideState{};
    c->step_colidx = nullptr;
    c->step_colidx_inc = nullptr;
    c->defer_finish = false;
    c->fin_n = 0;
    c->fin_scale = 1.0f;
    c->fin_loss = nullptr;
    c->fwd_inc = nullptr;
    c->fwd_rows = 0;
    c->ahead.armed = false;
    c->ahead.emit_done = c->ahead.scatter_done = c->ahead.hist_done = false;
    c->ahead.scatter_ok = c->ahead.hist_ok = false;
    c->ahead.late_only = false;
    c->ahead.inc = nullptr;
    c->sorted_inc = nullptr;
    c->sampled_inc = nullptr;
    c->fwd_serial = 0;
    c->sorted_keys = nullptr;
    c->prof_ev = nullptr;
    c->prof_tag = nullptr;
    c->prof_cap = c->prof_n = 0;
    c->prof_every = 1;
    c->prof_seen = 0;
    c->prof_name[0] = 0;
    c->map_words = L.map_words;
    c->map_cur = 0;
    c->colmap[0] = L.map_words ? (uint32_t *)(base + L.colmap) : nullptr;
    c->colmap[1] = L.map_words ? c->colmap[0] + L.map_words : nullptr;
    c->colmap[2] = L.map_words ? c->colmap[1] + L.map_words : nullptr;
    c->segw.allowed = c->segw.armed = false;
    s = launch_clear_ctrl(c);
    if (s == STX_OK) s = launch_clear_maps(c);
    if (s == STX_OK) s = launch_clear_rel_counts(c);
    if (s != STX_OK) { delete c; return s; }
    *out = c;
    return STX_OK;
}

static void prof_release(stx_ctx *ctx)
{
    if (ctx->prof_ev) {
        for (int i = 0; i < 2 * ctx->prof_cap; ++i) (void)hipEventDestroy(ctx->prof_ev[i]);
        delete[] ctx->prof_ev;
        delete[] ctx->prof_tag;
    }
    ctx->prof_ev = nullptr;
    ctx->prof_tag = nullptr;
    ctx->prof_cap = ctx->prof_n = 0;
    ctx->prof_name[0] = 0;
    ctx->prof_every = 1;
    ctx->prof_seen = 0;
}

stx_status stx_destroy(stx_ctx *ctx)
{
    if (!ctx) return STX_ERR_NULL;
    prof_release(ctx);
    delete ctx;
    return STX_OK;
}

stx_status stx_profile_kernel(stx_ctx *ctx, const char *kernel_name, int32_t max_records)
{
    if (!ctx) return STX_ERR_NULL;
    if (max_records < 0 || max_records > (1 << 20)) return STX_ERR_BAD_ARG;
    prof_release(ctx);
    if (!kernel_name || max_records == 0) return STX_OK;
    size_t len = __builtin_strlen(kernel_name);
    if (len == 0 || len >= sizeof(ctx->prof_name)) return STX_ERR_BAD_ARG;
    ctx->prof_ev = new (std::nothrow) hipEvent_t[2 * (size_t)max_records];
    ctx->prof_tag = new (std::nothrow) const char *[(size_t)max_records];
    if (!ctx->prof_ev || !ctx->prof_tag) {
        delete[] ctx->prof_ev;
        delete[] ctx->prof_tag;
        ctx->prof_ev = nullptr;
        ctx->prof_tag = nullptr;
        return STX_ERR_BAD_ARG;
    }
    for (int i = 0; i < 2 * max_records; ++i)
        if (hipEventCreate(&ctx->prof_ev[i]) != hipSuccess) {
            for (int j = 0; j < i; ++j) (void)hipEventDestroy(ctx->prof_ev[j]);
            delete[] ctx->prof_ev;
            delete[] ctx->prof_tag;
            ctx->prof_ev = nullptr;
            ctx->prof_tag = nullptr;
            return STX_ERR_HIP;
        }
    ctx->prof_cap = max_records;
    __builtin_memcpy(ctx->prof_name, kernel_name, len + 1);
    return STX_OK;
}

stx_status stx_profile_every(stx_ctx *ctx, int32_t every)
{
    if (!ctx) return STX_ERR_NULL;
    if (every < 1) return STX_ERR_BAD_ARG;
    ctx->prof_every = every;
    ctx->prof_seen = 0;
    return STX_OK;
}

stx_status stx_profile_dump(stx_ctx *ctx, char *text, size_t text_bytes)
{
    if (!ctx || !text) return STX_ERR_NULL;
    if (text_bytes == 0) return STX_ERR_BAD_ARG;
    text[0] = 0;
    if (!ctx->prof_ev) return STX_ERR_STATE;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return STX_ERR_HIP;
    const int kMaxNames = 64;
    const char *names[kMaxNames];
    double total_ms[kMaxNames];
    int count[kMaxNames], n_names = 0;
    for (int i = 0; i < ctx->prof_n; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]) != hipSuccess) return STX_ERR_HIP;
        int j = 0;
        while (j < n_names && __builtin_strcmp(names[j], ctx->prof_tag[i]) != 0) ++j;
        if (j == n_names) {
            if (n_names == kMaxNames) continue;
            names[n_names] = ctx->prof_tag[i];
            total_ms[n_names] = 0.0;
            count[n_names] = 0;
            ++n_names;
        }
        total_ms[j] += ms;
        ++count[j];
    }
    size_t used = 0;
    for (int j = 0; j < n_names; ++j) {
        int w = snprintf(text + used, text_bytes - used, "%s %.3f %d\n", names[j], total_ms[j] * 1e3 / count[j], count[j]);
        if (w < 0 || (size_t)w >= text_bytes - used) break;
        used += (size_t)w;
    }
    ctx->prof_n = 0;
    return STX_OK;
}

stx_status stx_profile_read(stx_ctx *ctx, double *avg_us, int32_t *n)
{
    if (!ctx || !avg_us || !n) return STX_ERR_NULL;
    *avg_us = 0.0;
    *n = 0;
    if (!ctx->prof_ev) return STX_ERR_STATE;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return STX_ERR_HIP;
    double total_ms = 0.0;
    for (int i = 0; i < ctx->prof_n; ++i) {
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, ctx->prof_ev[2 * i], ctx->prof_ev[2 * i + 1]) != hipSuccess) return STX_ERR_HIP;
        total_ms += ms;
    }
    *n = ctx->prof_n;
    if (ctx->prof_n) *avg_us = total_ms * 1e3 / ctx->prof_n;
    ctx->prof_n = 0;
    return STX_OK;
}

stx_status stx_sample_negatives(stx_ctx *ctx, const int32_t *h, const int32_t *r, const int32_t *t, int64_t m,
                                int32_t k, uint64_t seed, uint64_t epoch, int64_t m_total, int64_t global_offset,
                                int32_t *neg_h, int32_t *neg_t)
{
    (void)r;
    if (!ctx) return STX_ERR_NULL;
    if (m < 0 || k < 0 || m_total < 0 || global_offset < 0) return STX_ERR_BAD_ARG;
    if (m == 0 || k == 0) return STX_OK;
    if (!h || !t || !neg_h || !neg_t) return STX_ERR_NULL;
    if (m * (int64_t)k > ((int64_t)1 << 40)) return STX_ERR_BAD_ARG;
    uint64_t base = (epoch * (uint64_t)m_total + (uint64_t)global_offset) * (uint64_t)k;
    return launch_sample(ctx, h, t, m, k, seed, base, neg_h, neg_t);
}

stx_status stx_build_incidence(stx_ctx *ctx, const int32_t *h, const int32_t *r, const int32_t *t,
                               const int32_t *neg_h, const int32_t *neg_t, int32_t b, int32_t k, stx_incidence *inc)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_incidence_arrays(inc);
    if (s != STX_OK) return s;
    if (b < 0 || k < 0 || b > ctx->cfg.max_batch || k > ctx->cfg.max_neg) return STX_ERR_BAD_ARG;
    if (b > 0 && (!h || !r || !t)) return STX_ERR_NULL;
    if (b > 0 && k > 0 && (!neg_h || !neg_t)) return STX_ERR_NULL;
    inc->b = b;
    inc->k = k;
    inc->n_rows = (int64_t)b * (1 + k);
    inc->nnz = 3 * inc->n_rows;
    if (ctx->fwd_inc == inc) ctx->fwd_inc = nullptr;   // rebuilt: a stored forward no longer matches
    return launch_build(ctx, h, r, t, neg_h, neg_t, b, k, inc);
}

stx_status stx_check_indices(stx_ctx *ctx, int64_t *n_bad)
{
    if (!ctx) return STX_ERR_NULL;
    int32_t bad = 0;
    if (hipMemcpyAsync(&bad, ctx->ctrl + CTRL_BAD_INDEX, sizeof(bad), hipMemcpyDeviceToHost, ctx->stream) !=
        hipSuccess)
        return STX_ERR_HIP;
    if (hipStreamSynchronize(ctx->stream) != hipSuccess) return STX_ERR_HIP;
    if (n_bad) *n_bad = bad;
    if (bad) {
        stx_status s = launch_clear_ctrl(ctx);   // the block holds nothing but this counter
        if (s != STX_OK) return s;
        return STX_ERR_INDEX_RANGE;
    }
    return STX_OK;
}

stx_status stx_spmm(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, float *c_out)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    if (!p || !p->ent || !c_out) return STX_ERR_NULL;
    if ((s = check_a_current(ctx, inc)) != STX_OK) return s;
    return launch_spmm(ctx, inc, p, c_out);
}

stx_status stx_spmm_semiring(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind, float *z_out)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    if (!p || !p->ent || !z_out) return STX_ERR_NULL;
    if (kind < STX_DISTMULT || kind > STX_ROTATE) return STX_ERR_BAD_ARG;
    if (!stacked(ctx)) return STX_ERR_UNSUPPORTED;
    if ((s = check_a_current(ctx, inc)) != STX_OK) return s;
    return launch_semiring(ctx, inc, p, kind, z_out);
}

stx_status stx_spmm_semiring_t(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind,
                               const float *gz, float *work, stx_grads *g)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    if (!p || !p->ent || !gz || !work || !g || !g->rows) return STX_ERR_NULL;
    if (kind < STX_DISTMULT || kind > STX_ROTATE) return STX_ERR_BAD_ARG;
    if (((uintptr_t)gz & 15u) || ((uintptr_t)work & 15u)) return STX_ERR_BAD_ARG;
    if (!stacked(ctx)) return STX_ERR_UNSUPPORTED;
    if ((s = check_a_current(ctx, inc)) != STX_OK) return s;
    return launch_semiring_t(ctx, inc, p, kind, gz, work, g->rows);
}

stx_status stx_spmm_semiring_t_static(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind,
                                      const float *gz, stx_grads *g)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    if (!p || !p->ent || !gz || !g || !g->rows) return STX_ERR_NULL;
    if (kind < STX_DISTMULT || kind > STX_ROTATE) return STX_ERR_BAD_ARG;
    if ((uintptr_t)gz & 15u) return STX_ERR_BAD_ARG;
    if (!stacked(ctx)) return STX_ERR_UNSUPPORTED;
    if ((uint64_t)inc->n_rows * 3u * (uint64_t)ctx->cfg.dim * sizeof(float) > (uint64_t)STX_STATIC_WORK_BYTES)
        return STX_ERR_STATIC_LIMIT;
    if ((s = check_a_current(ctx, inc)) != STX_OK) return s;
    float *work = nullptr;
    s = static_work(&work);
    if (s != STX_OK) return s;
    return launch_semiring_t(ctx, inc, p, kind, gz, work, g->rows);
}

stx_status stx_rank_work_bytes(const stx_ctx *ctx, int64_t nq, size_t *bytes)
{
    if (!ctx || !bytes) return STX_ERR_NULL;
    if (nq < 0 || nq > ((int64_t)1 << 31) - 256) return STX_ERR_BAD_ARG;
    *bytes = rank_work_bytes(ctx, nq);
    return STX_OK;
}

stx_status stx_rank(stx_ctx *ctx, const stx_params *p, const int32_t *h, const int32_t *r, const int32_t *t,
                    int64_t nq, int32_t side, float *true_score, int32_t *n_less, int32_t *n_equal, void *work,
                    size_t work_bytes)
{
    if (!ctx) return STX_ERR_NULL;
    if (!p || !p->ent) return STX_ERR_NULL;
    if (nq < 0 || nq > ((int64_t)1 << 31) - 256 || (side != STX_TAIL && side != STX_HEAD)) return STX_ERR_BAD_ARG;
    if (ctx->cfg.model == STX_TRANSH && (!p->rel || !p->w)) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSR && (!p->rel || !p->proj)) return STX_ERR_NULL;
    if (nq == 0) return STX_OK;
    if (!h || !r || !t || !true_score || !n_less || !n_equal) return STX_ERR_NULL;
    const size_t need = rank_work_bytes(ctx, nq);
    if (need > 0 && !work) return STX_ERR_NULL;
    if (need > 0 && (work_bytes < need || ((uintptr_t)work & 255u))) return STX_ERR_WORKSPACE;
    return launch_rank(ctx, p, h, r, t, nq, side, true_score, n_less, n_equal, work);
}

// The forward pass; from_step: called by stx_train_step, whose own launches keep A and A^T paired.
static stx_status run_forward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, float *scores, float *loss,
                              bool from_step)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    s = check_params(ctx, p);
    if (s != STX_OK) return s;
    if (!scores || !loss) return STX_ERR_NULL;
    if (!from_step && (s = check_a_current(ctx, inc)) != STX_OK) return s;
    if (stacked(ctx)) s = launch_forward_stacked(ctx, inc, p, scores, loss);
    else if (ctx->cfg.model == STX_TRANSH) s = launch_forward_transh(ctx, inc, p, scores, loss);
    else {   // TransR: y = M_r (h - t) + r on the matrix cores, then distances / hinge / dL/dy over the rows of y
        if (inc->n_rows == 0) s = launch_finish_loss(ctx, 0, 1.0f, loss);
        else if (transr_fused_ok(ctx, inc)) {
            s = launch_transr_fused(ctx, inc, p, scores, loss);
        } else {
            s = launch_transr_project(ctx, inc, p);
            if (s == STX_OK) s = launch_forward_from_y(ctx, inc, p, scores, loss);
        }
    }
    if (s == STX_OK) {
        ctx->fwd_inc = inc;
        ctx->fwd_rows = inc->n_rows;
    }
    return s;
}

stx_status stx_forward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, float *scores, float *loss)
{
    return run_forward(ctx, inc, p, scores, loss, false);
}

// The backward pass.  lr == nullptr: gradients go to g.  Otherwise the update is applied where a
// gradient would be stored and g is not touched (it may be null).
static stx_status run_backward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, stx_grads *g,
                               const float *lr)
{
    const int dim = ctx->cfg.dim;
    const int64_t ent_end = 2 * inc->n_rows;   // sorted entries of entity columns come first, then relation columns
    float *rows = lr ? nullptr : g->rows;
    if (stacked(ctx)) {   // dL/dX = A^T G over all columns of X = [E;R] (Appendix G)
        const bool pk = packed_grad(ctx);
        const SegFusedHost fh{p->ent, nullptr, 0x7fffffff, lr ? *lr : 0.f, ctx->cfg.model == STX_TORUSE ? 1 : 0};
        const float *coefs = pk ? reinterpret_cast<const float *>(reinterpret_cast<const char *>(ctx->gbuf[0]) +
                                                                  packed_coef_offset(inc->n_rows, packed_stride(dim)))
                                : ctx->gbuf[0];
        return launch_seg_reduce(ctx, inc, 0, inc->nnz, ctx->gbuf[0], coefs, inc->nnz, pk ? packed_stride(dim) : dim, dim,
                                 rows, ctx->ld, pk, lr ? &fh : nullptr);
    }
    const SegFusedHost fh{p->ent, p->rel, (int32_t)ctx->cfg.n_ent, lr ? *lr : 0.f, 0};
    if (ctx->cfg.model == STX_TRANSH) {
        // entity columns: signed sums of gx; relation columns: sums of gy (-> d_r) and of gw (-> w_r)
        // (both products in the same pair of launches)
        const SegSecondHost second{(int32_t)ent_end, (int32_t)inc->nnz, ctx->gbuf[2], lr ? nullptr : g->w_rows, p->w,
                                   (ctx->cfg.flags & STX_FLAG_RENORM_W) ? 2 : 0};
        return launch_seg_reduce(ctx, inc, 0, inc->nnz, ctx->gbuf[0], ctx->gbuf[1], ent_end, dim, dim, rows, ctx->ld,
                                 false, lr ? &fh : nullptr, &second);
    }
    // TransR: gx = M_r^T gy and dL/dM_r on the matrix cores, then entity columns sum gx (signed, width dim)
    // and relation columns sum gy (width rel_dim)
    stx_status s = launch_transr_backward(ctx, inc, p, g, lr);
    if (s != STX_OK) return s;
    // (the first of these launches takes the dL/dM_r product along or launches it)
    if (dim == ctx->cfg.rel_dim) {   // rows of equal width: one product over all columns, as for TransH
        s = launch_seg_reduce(ctx, inc, 0, inc->nnz, ctx->gbuf[1], ctx->gbuf[0], ent_end, dim, dim, rows, ctx->ld,
                              false, lr ? &fh : nullptr);
    } else {
        s = launch_seg_reduce(ctx, inc, 0, ent_end, ctx->gbuf[1], ctx->gbuf[1], ent_end, dim, dim, rows, ctx->ld, false,
                              lr ? &fh : nullptr);
        if (s != STX_OK) return s;
        s = launch_seg_reduce(ctx, inc, ent_end, inc->nnz, ctx->gbuf[0], ctx->gbuf[0], inc->nnz, ctx->cfg.rel_dim,
                              ctx->cfg.rel_dim, rows, ctx->ld, false, lr ? &fh : nullptr);
    }
    if (s != STX_OK) return s;
    return launch_transr_dm_late(ctx);   // (nothing left to do unless no launch above ran)
}

stx_status stx_backward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, stx_grads *g)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    s = check_params(ctx, p);
    if (s != STX_OK) return s;
    if (!g || !g->rows) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSH && !g->w_rows) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSR && !g->proj) return STX_ERR_NULL;
    if (ctx->fwd_inc != inc || ctx->fwd_rows != inc->n_rows) return STX_ERR_STATE;
    return run_backward(ctx, inc, p, g, nullptr);
}

stx_status stx_sgd_step(stx_ctx *ctx, stx_params *p, const stx_incidence *inc, const stx_grads *g, float lr)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    s = check_params(ctx, p);
    if (s != STX_OK) return s;
    if (!g || !g->rows) return STX_ERR_NULL;
    if (!(lr == lr)) return STX_ERR_BAD_ARG;
    if (ctx->cfg.model == STX_TRANSH && !g->w_rows) return STX_ERR_NULL;
    if (ctx->cfg.model == STX_TRANSR && !g->proj) return STX_ERR_NULL;
    ctx->fwd_inc = nullptr;   // the tables change: a stored forward no longer matches them
    const int dim = ctx->cfg.dim;
    if (stacked(ctx)) {
        SgdTables T{p->ent, dim, ctx->cfg.model == STX_TORUSE ? 1 : 0, ctx->cfg.n_ent + ctx->cfg.n_rel, nullptr, dim,
                    nullptr, 0};
        return launch_sgd_rows(ctx, inc, T, g->rows, nullptr, lr);
    }
    if (ctx->cfg.model == STX_TRANSH) {
        SgdTables T{p->ent, dim, 0, ctx->cfg.n_ent, p->rel, dim, p->w, (ctx->cfg.flags & STX_FLAG_RENORM_W) ? 2 : 0};
        return launch_sgd_rows(ctx, inc, T, g->rows, g->w_rows, lr);
    }
    SgdTables T{p->ent, dim, 0, ctx->cfg.n_ent, p->rel, ctx->cfg.rel_dim, nullptr, 0};
    s = launch_sgd_rows(ctx, inc, T, g->rows, nullptr, lr);
    if (s != STX_OK) return s;
    return launch_transr_sgd_proj(ctx, inc, p, g, lr);
}

stx_status stx_backward_sgd(stx_ctx *ctx, const stx_incidence *inc, stx_params *p, stx_grads *g, float lr)
{
    if (!ctx) return STX_ERR_NULL;
    stx_status s = check_built(ctx, inc);
    if (s != STX_OK) return s;
    s = check_params(ctx, p);
    if (s != STX_OK) return s;
    if (!(lr == lr)) return STX_ERR_BAD_ARG;
    if (ctx->fwd_inc != inc || ctx->fwd_rows != inc->n_rows) return STX_ERR_STATE;
    ctx->fwd_inc = nullptr;   // the tables change: a stored forward no longer matches them
    return run_backward(ctx, inc, p, g, &lr);
}

stx_status stx_train_step(stx_ctx *ctx, const stx_batch *bt, stx_incidence *inc, stx_params *p, stx_grads *g, float lr,
                          float *scores, float *loss)
{
    if (!ctx || !bt) return STX_ERR_NULL;
    stx_status s = check_incidence_arrays(inc);
    if (s != STX_OK) return s;
    const int32_t b = bt->b, k = bt->k;
    if (b < 0 || k < 0 || b > ctx->cfg.max_batch || k > ctx->cfg.max_neg) return STX_ERR_BAD_ARG;
    if (bt->m_total < 0 || bt->global_offset < 0) return STX_ERR_BAD_ARG;
    if (b > 0 && (!bt->h || !bt->r || !bt->t)) return STX_ERR_NULL;
    if (b > 0 && k > 0 && (!bt->neg_h || !bt->neg_t)) return STX_ERR_NULL;
    s = check_params(ctx, p);
    if (s != STX_OK) return s;
    if (!scores || !loss) return STX_ERR_NULL;
    if (!(lr == lr)) return STX_ERR_BAD_ARG;
    inc->b = b;
    inc->k = k;
    inc->n_rows = (int64_t)b * (1 + k);
    inc->nnz = 3 * inc->n_rows;
    ctx->fwd_inc = nullptr;
    SampleArgs sa{bt->neg_h, bt->neg_t, bt->seed,
                  (bt->epoch * (uint64_t)bt->m_total + (uint64_t)bt->global_offset) * (uint64_t)k};
    // (the next batch's first build kernels may ride in this step's launches: the build prepares them)
    StepFusion fusion{p, scores, loss, false, false, 0, 1.0f, b > 0 ? bt->next : nullptr, nullptr};
    // the fused transposed product of one float4 per lane can run the build's last kernel in its own launch
    // (TransR: when its work items come from the rows-per-relation counts, not from the segment lists)
    ctx->segw.allowed = (ctx->cfg.model != STX_TRANSR || ctx->rel_cnt[0] != nullptr) && row_launch(ctx->cfg.dim).iters == 1;
    s = launch_build(ctx, bt->h, bt->r, bt->t, nullptr, nullptr, b, k, inc, &sa, &fusion);
    ctx->segw.allowed = false;
    // a stage of the next build that no launch took along: the buffers go back to their roles
    auto unwind_ahead = [&]() {
        if (ctx->ahead.armed && !ctx->ahead.emit_done) {
            ctx->ahead.armed = false;
            if (!ctx->ahead.late_only) {   // (a large sort's first kernel takes no rotating buffer)
                ctx->map_cur = (ctx->map_cur + 2) % 3;
                ctx->cix_cur ^= 1;
                if (ctx->ahead.args.rc.cur) ctx->cnt_cur ^= 1;
            }
        }
    };
    if (s != STX_OK) { launch_seg_write_late(ctx); unwind_ahead(); return s; }
    if (!fusion.forward_done) {
        // the sum of the loss rides in the backward pass's first launch: TransR's row products take it along, and
        // so does a transposed product that takes the build's last kernel along
        ctx->defer_finish = ctx->cfg.model == STX_TRANSR || ctx->segw.armed;
        s = run_forward(ctx, inc, p, scores, loss, true);
        ctx->defer_finish = false;
    } else {   // the forward pass shared a launch with the sort; the sum of the loss may still be missing
        if (!fusion.finish_done) {
            if (ctx->segw.armed) {   // the launch that takes the build's last kernel along takes this sum as well
                ctx->fin_n = fusion.n_partials;
                ctx->fin_scale = fusion.scale;
                ctx->fin_loss = loss;
            } else {
                s = launch_finish_loss(ctx, fusion.n_partials, fusion.scale, loss);
            }
        }
        ctx->fwd_inc = inc;
        ctx->fwd_rows = inc->n_rows;
    }
    if (s != STX_OK) { launch_seg_write_late(ctx); unwind_ahead(); return s; }
    s = stx_backward_sgd(ctx, inc, p, g, lr);
    unwind_ahead();
    if (ctx->segw.armed) {   // no launch took the build's last kernel along
        const stx_status s2 = launch_seg_write_late(ctx);
        if (s == STX_OK) s = s2;
    }
    if (ctx->fin_n > 0) {   // nothing took the deferred loss sum along (or the backward pass failed)
        const stx_status s2 = launch_finish_loss(ctx, ctx->fin_n, ctx->fin_scale, ctx->fin_loss);
        ctx->fin_n = 0;
        if (s == STX_OK) s = s2;
    }
    return s;
}

stx_status stx_copy_f32(stx_ctx *ctx, float *dst, const float *src, int64_t n)
{
    if (!ctx || !dst || !src) return STX_ERR_NULL;
    if (n < 0 || n % 4 != 0 || ((uintptr_t)dst & 15u) || ((uintptr_t)src & 15u)) return STX_ERR_BAD_ARG;
    return launch_copy_f32(ctx, dst, src, n);
}

stx_status stx_read_sectors(stx_ctx *ctx, const void *src, int64_t n_slots, int32_t slot_bytes, int64_t n_reads,
                            float *sink)
{
    if (!ctx || !src || !sink) return STX_ERR_NULL;
    if (n_slots <= 0 || n_reads < 0 || slot_bytes < 32 || slot_bytes % 16 != 0 || ((uintptr_t)src & 15u))
        return STX_ERR_BAD_ARG;
    return launch_read_sectors(ctx, src, n_slots, slot_bytes, n_reads, sink);
}

const char *stx_status_string(stx_status s)
{
    switch (s) {
    case STX_OK: return "ok";
    case STX_ERR_NULL: return "null pointer";
    case STX_ERR_BAD_ARG: return "bad argument";
    case STX_ERR_INDEX_RANGE: return "triplet index out of range";
    case STX_ERR_WORKSPACE: return "workspace too small or misaligned";
    case STX_ERR_STATE: return "call order violated";
    case STX_ERR_UNSUPPORTED: return "not supported";
    case STX_ERR_HIP: return "HIP runtime error";
    case STX_ERR_STATIC_LIMIT: return "request larger than the library's fixed scratch (STX_STATIC_WORK_BYTES)";
    }
    return "unknown status";
}

}  // extern "C"
