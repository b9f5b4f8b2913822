// Internal declarations shared by the HIP translation units of libstx.  Not part of the C ABI.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "stx.h"
#include "stx_measure.h"

namespace stx {

constexpr int kThreads = 256;          // every kernel here runs 256-thread workgroups (4 wavefronts)
constexpr int kSortItems = 4;          // keys per thread in the radix-sort kernels
constexpr int kSortTile = kThreads * kSortItems;
constexpr int kBigSortItems = 16;      // ... in large sorts: a digit's keys of one tile then fill whole memory lines
constexpr int kSegWItems = 8;          // sorted entries per thread in the kernels that derive the segments
constexpr int kSegWTile = kThreads * kSegWItems;
constexpr int kSegTileMin = 64;        // fewest sorted entries a workgroup of the transposed product may own
constexpr int kSuperTile = 32;         // sort tiles per group when the histogram table is scanned in two levels
constexpr int kSelfScanTiles = 512;   // up to this many sort tiles, scatter workgroups scan the histograms themselves
constexpr int kMapMaxWords = 2048;     // presence bitmap of the columns: kept when n_ent + n_rel <= 32 * this
constexpr int kRelCntMax = 4096;       // TransR: rows per relation are counted while A is written when n_rel <= this
constexpr int kMaxDim = 1024;
constexpr int kMaxProjDim = 256;        // TransR: dim and rel_dim are multiples of 32 up to this
constexpr int kProjRows = 64;           // TransR: entries of one relation per work item of the two row products
constexpr int kProjRowsDm = 256;        // ... and per work item of the product that forms dL/dM_r

// Slots of the control block at the start of the workspace (int32 each).
enum { CTRL_BAD_INDEX = 0, CTRL_GENERAL = 1 /* see k_forward_fast */, CTRL_WORDS = 64 };

struct Launch {            // how a row of `width` floats maps onto lanes
    int lpr;               // lanes per row: power of two in 8..64
    int iters;             // float4 per lane: ceil(width/4 / lpr), 1..4
};
inline Launch row_launch(int width)
{
    int q = width / 4, lpr = 8;
    while (lpr < 64 && lpr < q) lpr <<= 1;
    return {lpr, (q + lpr - 1) / lpr};
}


// LDS bytes of the kernel bodies that can run as part of another kernel's launch.  Such a kernel hands every
// body the same block of LDS (the bodies' own arrays would add up and cost it wavefronts per CU).
constexpr int kScatterLds = (256 + 4 * 256 + 2 * 1024) * 4;
constexpr int kSegWriteLds = (kThreads + 4) * 4;
constexpr int kFinishLds = kThreads * 8;
constexpr int emit_lds(bool map, bool rc) { return (256 + (map ? kMapMaxWords : 4) + (rc ? kRelCntMax : 4)) * 4; }

// What the first kernel of a build (k_emit, stx_emit_body.h) takes; plain data, shared with the host code
// that prepares a build ahead of time.
struct BatchPtrs {
    const int32_t *h, *r, *t, *nh, *nt;
    int32_t b, k;
    // SAMPLE: the negatives are drawn here (as k_sample draws them) and also written to nh_out / nt_out
    int32_t *nh_out, *nt_out;
    uint64_t seed, base_ctr;
};

// Presence bitmap of the batch's columns (one bit per column of [E;R]), kept when the table has few
// enough columns for a workgroup to scan the whole map: the segment of a column is then its rank among
// the set bits, and k_seg_write needs no count of segment heads per tile from a kernel before it.
// Three maps rotate: a build sets bits in one and clears the next one, which the build two before it used; the
// map of the build just before it stays intact, because that build's last kernel may run late (SegWriteLate).
struct ColMap {
    uint32_t *cur, *other;
    int words;
};

// TransR: rows per relation of the batch, for the work-item lists of the projection products.  Two
// buffers alternate like the bitmaps: a build adds into one and clears the other.
struct RelCnt {
    int32_t *cur, *other;
    int n_rel;
};

// One thread per entry e = 3*row + slot of A.  Writes the CSR arrays and the sort keys (= column ids),
// and the histogram of the first digit for this tile.
// Everything k_emit needs, by value, so that the same body can run in a launch shared with another kernel.
struct EmitArgs {
    BatchPtrs bp;
    int32_t n_ent, n_rel, nnz;
    int32_t *rowptr, *colidx;
    float *vals;
    int32_t *keys;
    int radix, ntiles;
    int32_t *table, *ctrl;
    ColMap map;
    RelCnt rc;
    int32_t *colidx2;              // a second copy of colidx, kept by the context (see stx_ctx::cix), or null
};

// Arguments of a scatter pass of the sort (by value into its kernel).
struct ScatterArgs {
    const int32_t *keys_in, *pay_in;
    int32_t *keys_out, *pay_out;
    int32_t nnz;
    int shift, bits, ntiles;
    const int32_t *table, *super;
};

// Arguments of a histogram pass of the sort (a later digit).
struct HistArgs {
    const int32_t *keys;
    int32_t nnz;
    int shift, radix;
    int32_t *table;
    int ntiles;
};

// Arguments of the last kernel of a build (k_seg_write, stx_segw_body.h), by value.
struct SegWriteArgs {
    const int32_t *keys, *pay;     // sorted
    int32_t nnz;
    const int32_t *tile_heads;
    int32_t *n_touched, *touched_cols, *seg_ptr, *row_idx;
    int8_t *sign;
    int32_t *seg_id, *packed;
    ColMap map;
};

// stx_train_step: the fused transposed product of one float4 per lane reads the sorted keys and payloads
// itself, so the last kernel of the build need not run before it: it waits here (`armed`) and runs as extra
// workgroups of that product's launch (the fix-up launch after it is the first reader of its arrays).
struct SegWriteLate {
    bool allowed, armed;
    bool use_map;
    SegWriteArgs args;
    int ntiles;
};

// stx_train_step with a next batch: the first kernels of the next build (k_emit, then the first scatter pass
// of the sort, then the histogram pass of the second digit) depend on nothing this step computes and run as
// extra workgroups of this step's launches, one stage per launch, because each stage needs all of the one
// before it: in the forward pass's launch, the transposed product's and its fix-up's when the forward pass
// runs in a launch that can take a stage along, else in the last two.  `armed`: prepared for the batch that
// `args` describes; `*_done`: that stage ran, and the next build may skip it if it is given this very batch;
// `*_ok`: the stage may run ahead at all (shape of the sort).
struct EmitAheadState {
    bool armed;
    bool emit_done, scatter_done, hist_done;
    bool scatter_ok, hist_ok;
    // a large sort: the first kernel alone runs ahead, and only in the fix-up launch that ends the step (it
    // overwrites the caller's A arrays, of which no copy is kept for the launches before that one)
    bool late_only;
    EmitArgs args;
    ScatterArgs sargs;
    HistArgs hargs;
    int ntiles;
    const stx_incidence *inc;
};

}  // namespace stx

// TransR: arguments of the product that forms dL/dM_r and of the sum of its partial matrices (stx_transr.hip).
struct DmArgs {
    const int4 *dm_items, *fix_items;
    const int32_t *counts;       // [1] = number of dM items, [2] = number of fix-up items
    int n_fix;                   // most fix-up items the batch can have (launch bound of the sums)
    const uint16_t *gyt, *xt;    // operand-order transposed tiles written by the row kernels
    float *g_proj, *partials;
    int d, k;
    float *M;                    // fused update: M_r <- M_r - lr * dL/dM_r replaces the store of dL/dM_r
    float lr;
    int fused;
    int n_items;                 // workgroups (blockIdx.x) that are dM items; one more may follow:
    const float *fin_partials;   // a deferred final sum of the loss that the launch takes along (fin_n == 0: none)
    int fin_n;
    float fin_scale;
    float *fin_loss;
};
// Those two, left by the backward pass of stx_train_step for the launches of the transposed incidence product to
// take along (both widths at most 128: one workgroup per dM item).  fixup: a relation can have several items.
struct DmRideState {
    bool armed, fixup;
    DmArgs args;
    int items;
};

struct stx_ctx {
    stx_config cfg;
    hipStream_t stream;
    int ld;                        // floats per gradient row: max(dim, rel_dim)
    int out_dim;                   // width of y: rel_dim for TransR, dim otherwise
    int64_t rows_max, nnz_max, cols_max;
    int sort_bits, sort_passes, digit_bits;
    int ntiles_max;                // radix-sort tiles at nnz_max
    int fwd_blocks_max;
    // workspace partitions (device)
    int32_t *ctrl;
    int32_t *keys[3];              // [0], [1]: ping-pong of the sort; [2]: the unsorted keys of the batch being built
    int32_t *pay[2];
    int32_t *table;                // [256 * ntiles_max] tile histograms of the first digit (written by k_emit)
    int32_t *table1;               // ... and of the later digits: a next batch's first kernel may run beside them
    int32_t *cix[2];               // copies of A's column ids that the forward pass of stx_train_step reads: the
    int cix_cur;                   // next batch's first kernel may overwrite the caller's arrays meanwhile
    int32_t *super;                // [256 * (ntiles_max / kSuperTile + 1)] group sums of the tile histograms
    int32_t *tile_heads;           // [ntiles_max + 1]
    float *loss_partials;          // [fwd_blocks_max]
    float *partials;               // [(nnz_max/kSegTileMin + 2) * 2 * ld]
    float *gbuf[4];                // per-row buffers, rows_max x ld each (how many depends on the model)
    uint32_t *colmap[3];           // presence bitmaps of the columns (adjacent), or null when the table is too wide
    int map_words, map_cur;        // words per map (0: not kept); which map the next build fills (they rotate)
    // TransR only: work items, bfloat16 operand copies of the projection matrices, transposed operand tiles
    int32_t *tr_items, *tr_dm_items, *tr_fix_items, *tr_counts;
    uint16_t *tr_m16, *tr_m16t, *tr_xt, *tr_gyt;
    int32_t *rel_cnt[2];           // rows per relation of a batch (two buffers alternate, like the bitmaps), or null
    int cnt_cur;
    const int32_t *cnt_ptr;        // counts of the last build ...
    const stx_incidence *cnt_inc;  // ... which was of this incidence
    const stx_incidence *prep_inc; // incidence whose TransR preparation already ran beside its sort
    int prep_whole;                // ... with row items that name whole lists (k_transr_fused) or 64-entry pieces
    const stx_incidence *tr_fused_inc;   // incidence whose forward pass was k_transr_fused (dL/dx and the tiles exist)
    DmRideState dm_ride;
    const int32_t *step_colidx;    // stx_train_step: the context's own copy of this batch's column ids, or null ...
    const stx_incidence *step_colidx_inc;   // ... of this incidence
    // stx_train_step: the final sum of the loss is not launched by the forward pass but rides in the first
    // launch of the backward pass (nothing in between needs it), when that launch can take it along
    bool defer_finish;
    int fin_n;                     // loss partials waiting to be summed (0: none)
    float fin_scale;
    float *fin_loss;
    // optional live timing of one kernel (stx_profile_kernel): event pairs around its launches
    char prof_name[48];
    hipEvent_t *prof_ev;           // 2 * prof_cap events, null when profiling is off
    const char **prof_tag;         // kernel name of each recorded pair (string literals of the launch sites)
    int prof_cap, prof_n;
    int prof_every, prof_seen;     // bracket every prof_every-th selected launch
    // host-side call-order state
    const stx_incidence *sorted_inc;   // incidence of the last build, whose sorted keys are still in keys[]
    const int32_t *sorted_keys;
    const stx_incidence *sampled_inc;  // incidence whose negatives the library's sampler drew inside its build, or null
    int32_t fwd_serial;            // number of the last forward pass that used the fast kernel (never 0 once used)
    const stx_incidence *fwd_inc;  // incidence of the last stx_forward, null if none
    int64_t fwd_rows;
    stx::EmitAheadState ahead;
    stx::SegWriteLate segw;
};

namespace stx {

// Arguments of the forward-step body and of a scatter pass of the sort (by value into their kernels).
struct ForwardArgs {
    const int32_t *colidx;
    const float *X;
    int32_t b, k;
    int dim;
    float margin, scale;
    float *scores, *G;
    int gstride;
    float *loss_partials;
    const float *rel_weight;   // fixed weight of every relation's distance, or null (gathered rows only)
    int32_t n_ent;
    int32_t stream_rows;       // the table is far larger than the caches: rows used once are fetched past them
};


// stx_train_step: forward-pass work that may share launches with the sort of A^T.  launch_build fills
// in what it has done; the caller launches the rest.
struct StepFusion {
    const stx_params *p;
    float *scores, *loss;
    bool forward_done, finish_done;
    int n_partials;            // loss partials the forward pass wrote
    float scale;               // of the loss (1, or 1 / pairs for the mean)
    const stx_batch *next;     // the batch of the next call, or null
    const int32_t *colidx;     // A's column ids for the forward pass (the context's copy; filled in by the build)
};

// stx_build.hip
stx_status launch_sample(stx_ctx *, const int32_t *h, const int32_t *t, int64_t m, int32_t k, uint64_t seed,
                         uint64_t base_ctr, int32_t *nh, int32_t *nt);
struct SampleArgs {            // negatives drawn inside the build (same numbers as launch_sample) and stored here
    int32_t *neg_h, *neg_t;
    uint64_t seed, base_ctr;
};
stx_status launch_build(stx_ctx *, const int32_t *h, const int32_t *r, const int32_t *t, const int32_t *nh,
                        const int32_t *nt, int32_t b, int32_t k, stx_incidence *inc,
                        const SampleArgs *sample = nullptr, StepFusion *fusion = nullptr);
// Prepares the first kernel of the build of `next` (as stx_train_step would launch it) to run inside the next
// fused transposed product of this context; false: this configuration or batch does not allow it.
bool prepare_emit_ahead(stx_ctx *, const stx_batch *next, stx_incidence *inc);
// A launch that can take a stage of the next build along asks for it here (null args / zero tiles: none).
struct EmitAhead {
    EmitArgs args;
    int ntiles;
};
struct ScatterAhead {
    ScatterArgs args;
    int ntiles;
};
struct HistAhead {
    HistArgs args;
    int ntiles;
};
struct DmRide {
    DmArgs args;
    int blocks;                    // workgroups of the launch that play this part (0: none)
};
// (fixup_launch: the caller is the fix-up launch of the transposed product, the last launch of a step)
EmitAhead take_emit_ahead(stx_ctx *, bool fixup_launch = false);
ScatterAhead take_scatter_ahead(stx_ctx *);
HistAhead take_hist_ahead(stx_ctx *);
stx_status launch_seg_write_late(stx_ctx *);
// stx_transr.hip: item lists and bf16 copies of M_r in the launch of the first scatter pass; false: not possible
bool launch_prep_scatter(stx_ctx *, const stx_incidence *, const stx_params *, const ScatterArgs &, bool first);
// stx_step.hip
// (first: the sort's first pass, whose payloads are the positions; false: shape not covered)
bool launch_fwd_scatter(stx_ctx *, const stx_incidence *, StepFusion *, const ScatterArgs &, bool first);
// the forward pass beside a histogram pass; a scatter pass beside the sum of the loss (when the first scatter
// pass already ran ahead of time)
bool launch_fwd_hist(stx_ctx *, const stx_incidence *, StepFusion *, const int32_t *keys, int32_t nnz, int shift,
                     int radix, int ntiles);
void launch_scatter_finish(stx_ctx *, StepFusion *, const ScatterArgs &);
void launch_hist_finish(stx_ctx *, StepFusion *, const int32_t *keys, int32_t nnz, int shift, int radix, int ntiles);
stx_status launch_clear_ctrl(stx_ctx *);
stx_status launch_clear_maps(stx_ctx *);
stx_status launch_clear_rel_counts(stx_ctx *);
// stx_forward.hip
stx_status launch_spmm(stx_ctx *, const stx_incidence *, const stx_params *, float *c_out);
stx_status launch_forward_stacked(stx_ctx *, const stx_incidence *, const stx_params *, float *scores, float *loss);
stx_status launch_copy_f32(stx_ctx *, float *dst, const float *src, int64_t n);
stx_status launch_read_sectors(stx_ctx *, const void *src, int64_t n_slots, int slot_bytes, int64_t n_reads, float *sink);
// stx_backward.hip
// out_rows[segment] = signed sum of source rows over the sorted entries [e_begin, e_end); entries
// before `split` read src_a, the others src_b (both with ld_src floats per row, `width` of them used).
// packed_src: src_a holds packed L1-kind sign records (see packed_stride), ld_src is the record size in bytes,
// and src_b the rows' coefficients.
// second: another product of the same row width over the entries [e_begin, e_end), all reading `src`, that
// runs in the same two launches (its workgroups follow the first product's).
// tail_off (dense source rows only): entries with value -1 read their row tail_off floats further on.
// fused: no gradient row is written; the table row of the column (rows of `width` floats; `table` for
// columns below n_split, row column - n_split of `table_b` for the others) becomes row - lr * gradient
// instead (mode 1: then its fractional part; mode 2: then rescaled to unit length).  The second
// product's columns all lie at or above n_split and update its own table in its own mode.
struct SegSecondHost {
    int32_t e_begin, e_end;
    const float *src;
    float *out_rows;
    float *fused_table;
    int fused_mode;
};
struct SegFusedHost {
    float *table, *table_b;
    int32_t n_split;
    float lr;
    int mode;
};
stx_status launch_seg_reduce(stx_ctx *, const stx_incidence *, int64_t e_begin, int64_t e_end, const float *src_a,
                             const float *src_b, int64_t split, int ld_src, int width, float *out_rows, int ld_out,
                             bool packed_src = false, const SegFusedHost *fused = nullptr,
                             const SegSecondHost *second = nullptr, int tail_off = 0);
struct SgdTables {
    float *table_a; int width_a; int mode_a;   // columns [0, n_split)
    int64_t n_split;
    float *table_b; int width_b;               // columns >= n_split, gradient in the same rows array (may be null)
    float *table_w; int mode_w;                // columns >= n_split, gradient in w_rows, width_a (may be null)
};
stx_status launch_sgd_rows(stx_ctx *, const stx_incidence *, const SgdTables &, const float *grad_rows,
                           const float *w_rows, float lr);
stx_status launch_forward_from_y(stx_ctx *, const stx_incidence *, const stx_params *, float *scores, float *loss);
// stx_rank.hip
stx_status launch_rank(stx_ctx *, const stx_params *, const int32_t *h, const int32_t *r, const int32_t *t, int64_t nq,
                       int side, float *true_score, int32_t *n_less, int32_t *n_equal, void *work);
size_t rank_work_bytes(const stx_ctx *, int64_t nq);   // scratch launch_rank needs for nq queries (0 unless TransR)
// stx_semiring.hip
stx_status launch_semiring(stx_ctx *, const stx_incidence *, const stx_params *, int kind, float *z_out);
stx_status launch_semiring_t(stx_ctx *, const stx_incidence *, const stx_params *, int kind, const float *gz,
                             float *work, float *out_rows);
// device address, on the current GPU, of the library's fixed scratch array of STX_STATIC_WORK_BYTES bytes
stx_status static_work(float **out);
// stx_transr.hip
stx_status launch_transr_project(stx_ctx *, const stx_incidence *, const stx_params *);
// the forward pass, dL/dy, dL/dx and the tiles of the dM product in one kernel, for the shapes transr_fused_ok names
bool transr_fused_ok(const stx_ctx *, const stx_incidence *);
stx_status launch_transr_fused(stx_ctx *, const stx_incidence *, const stx_params *, float *scores, float *loss);
// fused_lr: if not null, M_r <- M_r - lr * dL/dM_r is applied in place of the store of dL/dM_r (g may be null)
stx_status launch_transr_backward(stx_ctx *, const stx_incidence *, const stx_params *, stx_grads *,
                                  const float *fused_lr = nullptr);
// launches what dm_ride holds as kernels of its own (a launch that could not take it along calls this first)
stx_status launch_transr_dm_late(stx_ctx *);
// the sum of the partial matrices alone, after a launch that took the product of dm_ride along but not the sum
stx_status launch_transr_dm_fixup_late(stx_ctx *);
stx_status launch_transr_sgd_proj(stx_ctx *, const stx_incidence *, stx_params *, const stx_grads *, float lr);
// stx_transh.hip
stx_status launch_forward_transh(stx_ctx *, const stx_incidence *, const stx_params *, float *scores, float *loss);
stx_status launch_finish_loss(stx_ctx *, int n_partials, float scale, float *loss);

// TransE / TorusE with an L1-kind distance keep dL/dx packed inside gbuf[0]: per row a record of dim/4 sign
// bytes, padded to a multiple of 32 bytes (one 32-byte memory sector at dim 128, which is what a random
// read of it costs), and, in an array of their own behind the records of the batch, the rows' fp32
// coefficients (4 bytes a row: 5 MB at 1.3 M rows, read out of the caches).
inline bool packed_grad(const stx_ctx *c)
{
    return (c->cfg.model == STX_TRANSE || c->cfg.model == STX_TORUSE) &&
           (c->cfg.dist == STX_L1 || c->cfg.dist == STX_TORUS_L1);
}
// (bytes per sign record: a power of two, so that a record's address is a shift of its row)
inline int packed_stride(int dim)
{
    int s = 32;
    while (s < dim / 4) s <<= 1;
    return s;
}
// byte offset of the coefficient array from the start of the records of a batch of `rows` rows
__host__ __device__ inline int64_t packed_coef_offset(int64_t rows, int stride) { return (rows * stride + 255) / 256 * 256; }

// Tables beyond the reach of the last-level cache: their updated rows are stored past the caches, and rows the
// forward pass uses once are fetched past them.  Rows of a small table are read again by the next step's forward
// pass, which runs measurably faster when the update leaves them cached (TransH at 15,000 entities: 30 against 37
// microseconds).
inline int big_tables(const stx_ctx *c)
{
    return (c->cfg.n_ent + c->cfg.n_rel) * (int64_t)c->cfg.dim * 4 > ((int64_t)128 << 20) ? 1 : 0;
}

inline stx_status hip_ok(hipError_t e) { return e == hipSuccess ? STX_OK : STX_ERR_HIP; }

// Brackets the launches of the kernel selected with stx_profile_kernel by a pair of events on the
// context's stream.  Costs one string compare per launch when profiling is off.
struct ProfScope {
    stx_ctx *c;
    bool on;
    ProfScope(stx_ctx *ctx, const char *kernel) : c(ctx), on(false)
    {
        if (c->prof_ev && c->prof_n < c->prof_cap &&
            (c->prof_name[0] == '*' || __builtin_strcmp(kernel, c->prof_name) == 0) &&
            (c->prof_every <= 1 || c->prof_seen++ % c->prof_every == 0)) {
            on = true;
            c->prof_tag[c->prof_n] = kernel;
            (void)hipEventRecord(c->prof_ev[2 * c->prof_n], c->stream);
        }
    }
    ~ProfScope()
    {
        if (on) {
            (void)hipEventRecord(c->prof_ev[2 * c->prof_n + 1], c->stream);
            ++c->prof_n;
        }
    }
};

}  // namespace stx
