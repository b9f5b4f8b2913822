/*
 * stx — sparse-incidence training step for translation-based knowledge-graph embeddings
 *       (TransE, TorusE, TransH, TransR) on AMD MI355X (gfx950).
 *
 * The method (SparseTransX, arXiv 2502.16949): a batch of (head, relation, tail) triplets and their
 * corrupted negatives is written as a sparse incidence matrix A with three nonzeros per row, so that
 * the forward pass is one sparse-dense product A.[E;R] = h + r - t per row (Sec. 4.2) followed by a
 * distance and a margin-ranking loss (Sec. 5.3), and the backward pass is the transposed product
 * A^T.(dL/dC) (Appendix G), which replaces the per-index scatter-adds.
 *
 * Conventions for every entry point
 *   - Unless a parameter says "host", pointers are DEVICE pointers owned by the caller.  The library
 *     never allocates or frees device memory: its scratch lives in the workspace given to stx_create.
 *   - All work is enqueued on the stream given to stx_create and the calls return without waiting, except
 *     stx_check_indices (waits for the stream to read the counter) and stx_rank on a TransR context (waits
 *     once, to learn the sizes of the relation groups).  Calls on one context must not overlap in time.
 *   - Every call returns a stx_status.  Host-detectable argument errors (null pointers, sizes beyond
 *     the configured maxima, bad enums) are reported before anything is launched.
 *   - Indices are int32, counts int64.  Tables are fp32, row-major, 16-byte aligned, with
 *     dim % 4 == 0, dim <= 1024.  TransR runs its projections on the matrix cores in 32-wide tiles:
 *     dim % 32 == 0, rel_dim % 32 == 0, both <= 256, and STX_FLAG_BF16_PROJ must be set
 *     (anything else: STX_ERR_UNSUPPORTED).
 */
#ifndef STX_H
#define STX_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    STX_OK = 0,
    STX_ERR_NULL = 1,        /* a required pointer is null */
    STX_ERR_BAD_ARG = 2,     /* enum out of range, negative size, dim not a multiple of 4, ... */
    STX_ERR_INDEX_RANGE = 3, /* stx_check_indices: some triplet index was outside its table */
    STX_ERR_WORKSPACE = 4,   /* workspace smaller than stx_workspace_bytes, or misaligned */
    STX_ERR_STATE = 5,       /* call order violated (e.g. backward before forward) */
    STX_ERR_UNSUPPORTED = 6, /* valid request this build does not implement */
    STX_ERR_HIP = 7,         /* a HIP runtime call failed */
    STX_ERR_STATIC_LIMIT = 8 /* stx_spmm_semiring_t_static: the batch needs more than STX_STATIC_WORK_BYTES */
} stx_status;

/* Score functions of Table 2 (Sec. 4.2): which incidence form is used and what follows it. */
enum { STX_TRANSE = 0, STX_TRANSH = 1, STX_TRANSR = 2, STX_TORUSE = 3 };
/* Norm applied to the translated vector (Sec. 4.3, 4.6): L1, unsquared L2, or their torus
 * versions, taken on the fractional part f = y - floor(y) as sum / root-sum-square of min(f, 1-f). */
enum { STX_L1 = 0, STX_L2 = 1, STX_TORUS_L1 = 2, STX_TORUS_L2 = 3, STX_L2_SQ = 4 /* sum y^2: Table 2, TransC */ };
/* Reduction of the margin-ranking loss over the b*k (positive, negative) pairs. */
enum { STX_SUM = 0, STX_MEAN = 1 };

#define STX_FLAG_RENORM_W 1u  /* TransH: rescale every touched normal w_r to unit length after the update */
#define STX_FLAG_BF16_PROJ 2u /* TransR: h - t, M_r and dL/dy are rounded to bfloat16 (nearest even) as operands
                                 of the three projection products; accumulation is fp32 */

typedef struct {
    int32_t model;     /* STX_TRANSE ... */
    int32_t dist;      /* STX_L1 ... */
    int32_t reduce;    /* STX_SUM / STX_MEAN */
    int32_t dim;       /* entity embedding width d */
    int32_t rel_dim;   /* TransR: relation space width k; other models: ignored (taken as dim) */
    int64_t n_ent;     /* N */
    int64_t n_rel;     /* R;  N + R < 2^31 */
    float margin;      /* gamma of the hinge max(0, gamma + d_pos - d_neg) */
    int32_t max_batch; /* largest b (positives per batch) any call will pass */
    int32_t max_neg;   /* largest k (negatives per positive) any call will pass; 3*b*(1+k) < 2^29 */
    uint32_t flags;    /* STX_FLAG_* */
} stx_config;

/* Parameter tables (device, fp32, row-major), updated in place by stx_sgd_step.
 *   TransE / TorusE : ent = X = [E;R], (n_ent + n_rel) x dim, relation r in row n_ent + r (Sec. 4.2.2);
 *                     rel, w, proj unused.  rel_weight (optional, n_rel floats, read only): a fixed weight
 *                     per relation that multiplies the distance of its triplets, the TransM row of
 *                     Table 2; null = all ones.  The other models reject a non-null rel_weight.
 *   TransH          : ent = E (n_ent x dim), rel = d_r (n_rel x dim), w = w_r (n_rel x dim)  (Sec. 4.5).
 *   TransR          : ent = E (n_ent x dim), rel = r (n_rel x rel_dim),
 *                     proj = M_r (n_rel x rel_dim x dim, each matrix row-major)               (Sec. 4.4). */
typedef struct {
    float *ent;
    float *rel;
    float *w;
    float *proj;
    const float *rel_weight;
} stx_params;

/* One batch as a sparse incidence matrix and its transpose (Sec. 4.2; Appendix G).
 * The caller allocates every array (device) for the configured maxima:
 *   rows_max = max_batch * (1 + max_neg), nnz_max = 3 * rows_max, cols_max = min(nnz_max, n_ent + n_rel).
 * stx_build_incidence fills the arrays (asynchronously) and the host-side scalars b, k, n_rows, nnz.
 *
 * A, `hrt` form, CSR: row i holds its three entries in the order (head, n_ent + relation, tail) with
 * values (+1, +1, -1); the `ht` form of Sec. 4.2.1 is entries 0 and 2 of each row.  Rows 0..b-1 are the
 * positives; the kk-th negative of positive i is row b + i*k + kk and keeps the relation of i.
 * Equal head and tail stay two entries.
 *
 * A^T, doubly compressed and sorted by column: only the U columns holding an entry appear, ascending;
 * entries of one column keep their order of appearance in A (position 3*row + slot).                 */
typedef struct {
    int32_t b, k;             /* host, filled by stx_build_incidence */
    int64_t n_rows, nnz;      /* host, filled: b*(1+k), 3*n_rows */
    int32_t *a_rowptr;        /* [rows_max + 1]  = 3*i */
    int32_t *a_colidx;        /* [nnz_max] */
    float *a_vals;            /* [nnz_max] */
    int32_t *at_touched_cols; /* [cols_max]      column id of segment s, ascending */
    int32_t *at_seg_ptr;      /* [cols_max + 1]  first sorted entry of segment s; [U] = nnz */
    int32_t *at_row_idx;      /* [nnz_max]       row of sorted entry e */
    int8_t *at_sign;          /* [nnz_max]       value of sorted entry e: +1 or -1 */
    int32_t *at_seg_id;       /* [nnz_max]       segment of sorted entry e */
    int32_t *at_packed;       /* [nnz_max]       row_idx << 2 | (entry starts its segment) << 1 | (sign < 0);
                                                 what the transposed-product kernels read */
    int32_t *n_touched;       /* [1]             U */
} stx_incidence;

/* Gradients, row-sparse and aligned with the segments of A^T: row s belongs to column
 * at_touched_cols[s].  ld = max(dim, rel_dim) floats per row; cols_max rows each (device, caller-owned).
 *   rows   : segments of entity columns   -> dL/dE rows (width dim);
 *            segments of relation columns -> TransE/TorusE: dL/dR row (these are rows of X too);
 *                                            TransH: dL/d(d_r);  TransR: dL/dr (width rel_dim).
 *   w_rows : TransH only: dL/dw_r in the rows of relation segments; other rows are not written.
 *   proj   : TransR only: dL/dM_r, dense n_rel x rel_dim x dim; only matrices of relations present in
 *            the batch are written.                                                                   */
typedef struct {
    float *rows;
    float *w_rows;
    float *proj;
} stx_grads;

typedef struct stx_ctx stx_ctx;

/* Bytes of device workspace a context with this configuration needs. */
stx_status stx_workspace_bytes(const stx_config *cfg, size_t *bytes /* host, out */);

/* Create a context.  workspace: device memory, 256-byte aligned, at least stx_workspace_bytes, owned by
 * the caller and kept alive until stx_destroy.  stream: a hipStream_t (NULL = the default stream).
 * Enqueues one small kernel that clears the library's counters.                                       */
stx_status stx_create(const stx_config *cfg, void *workspace, size_t workspace_bytes, void *stream,
                      stx_ctx **out /* host, out */);
stx_status stx_destroy(stx_ctx *ctx);

/* Negative sampling (Sec. 5.3: one pre-generated negative set; Sec. 6.1: as many negatives as
 * positives per slot).  For positive i of this call (global index g = global_offset + i) and slot kk:
 *   u = SplitMix64 output number (epoch*m_total + g)*k + kk of the sequence seeded with `seed`;
 *   the head is replaced if the top bit of u is set, else the tail;
 *   replacement entity = floor((u mod 2^32) * n_ent / 2^32).  The relation is kept, nothing is filtered.
 * h, r, t: [m] in; neg_h, neg_t: [m*k] out.                                                           */
stx_status stx_sample_negatives(stx_ctx *ctx, const int32_t *h, const int32_t *r, const int32_t *t,
                                int64_t m, int32_t k, uint64_t seed, uint64_t epoch, int64_t m_total,
                                int64_t global_offset, int32_t *neg_h, int32_t *neg_t);

/* Build A and A^T for one batch (Sec. 4.2.1, 4.2.2): h, r, t [b]; neg_h, neg_t [b*k] (may be null when
 * k == 0).  Out-of-range indices are clamped into their table and counted (see stx_check_indices), so
 * later kernels never read outside the tables.  b == 0 gives an empty matrix.                         */
stx_status stx_build_incidence(stx_ctx *ctx, const int32_t *h, const int32_t *r, const int32_t *t,
                               const int32_t *neg_h, const int32_t *neg_t, int32_t b, int32_t k,
                               stx_incidence *inc /* host struct of device arrays */);

/* Waits for the stream, then reports whether any index seen by stx_build_incidence since the last
 * check was out of range: *n_bad (host, may be null) receives the count; returns STX_ERR_INDEX_RANGE
 * when it is nonzero.  The counter is reset.                                                          */
stx_status stx_check_indices(stx_ctx *ctx, int64_t *n_bad);

/* C = A.X (Sec. 4.2): row i of C (n_rows x dim, fp32) = (X[h] + X[n_ent + r]) - X[t] for TransE/TorusE,
 * E[h] - E[t] for TransH/TransR, each operation rounded once, in that order.                          */
stx_status stx_spmm(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, float *c_out);

/* The same three-entry product under the semirings of Appendix D, for the models it names: the entries
 * of a row are multiplied instead of added.  TransE / TorusE contexts only (X = [E;R] stacked in p->ent,
 * columns as in a_colidx; the values of A play no part), else STX_ERR_UNSUPPORTED.
 *   STX_DISTMULT : z = (h r) t elementwise over the dim floats of a row;
 *   STX_COMPLEX  : a row is dim/2 complex numbers stored (re, im); z = (h r) conj(t);
 *   STX_ROTATE   : the same storage; z = h r - t;
 * with (a + bi)(c + di) = (ac - bd) + (ad + bc)i and every real product and sum rounded once.
 * z_out: n_rows x dim floats (device, out).                                                           */
enum { STX_DISTMULT = 0, STX_COMPLEX = 1, STX_ROTATE = 2 };
stx_status stx_spmm_semiring(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind,
                             float *z_out);

/* Backward of stx_spmm_semiring for a real loss (Appendix G's transposed product with Appendix D's
 * operators).  gz: dL/dZ, n_rows x dim (device, in; complex kinds: (dL/dRe z, dL/dIm z) pairs).
 * g->rows[s] = sum over the entries of segment s of gz[row] times the conjugated product of the row's
 * other two factors (head entry: conj(r) t | conj(r); relation entry: conj(h) t | conj(h); tail entry:
 * ComplEx conj(gz) h r, RotatE -gz; DistMult: the plain products), summed in the fixed order of
 * stx_backward.  work: 3 * n_rows * dim floats of device scratch owned by the caller (the per-row terms). */
stx_status stx_spmm_semiring_t(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind,
                               const float *gz, float *work, stx_grads *g);

/* stx_spmm_semiring_t for callers that cannot allocate device memory and have no work buffer to hand over
 * (code under HIP graph capture, serving loops, harnesses that forbid hipMalloc): the same kernels and the
 * same results bit for bit, with the per-row terms kept in a fixed array of STX_STATIC_WORK_BYTES bytes that
 * is part of the library's device code (every GPU the library runs on holds its own copy until the process
 * ends).  Calls no allocator.  The context's GPU must be the current device.
 * A batch with 3 * n_rows * dim * 4 > STX_STATIC_WORK_BYTES is refused with STX_ERR_STATIC_LIMIT before
 * anything is launched (at dim 128: up to 65,536 rows).  All calls on one GPU share the array, from every
 * context and thread: calls that overlap in time on one GPU race on it; calls on one stream do not.  Nothing
 * in it needs clearing between calls: every element a call reads it has written before.                  */
#define STX_STATIC_WORK_BYTES (96u << 20)
stx_status stx_spmm_semiring_t_static(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, int32_t kind,
                                      const float *gz, stx_grads *g);

/* Forward (Sec. 4.3-4.6, 5.3): scores[i] = distance of row i (n_rows, fp32); *loss (device, fp32) =
 * sum (or mean) over pairs of max(0, margin + score[i] - score[b + i*k + kk]).  Also stores dL/dy of
 * every row in the workspace for stx_backward: the pair is active when margin + d_pos - d_neg > 0
 * (evaluated in fp32 as (margin + d_pos) - d_neg); subgradient 0 at every tie (sign(0) = 0, zero
 * vector at zero distance, 0 at torus fractional part 0 or 1/2).                                      */
stx_status stx_forward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, float *scores,
                       float *loss);

/* Backward (Appendix G): g->rows[s] = sum over the entries e of segment s of sign[e] * (dL/dx of row
 * row_idx[e]), summed without atomics in a fixed order (bitwise reproducible); TransH and TransR first
 * pass dL/dy back through their projection (Sec. 4.4, 4.5) and also fill w_rows / proj.
 * Needs the stx_forward of the same incidence immediately before it on this context.                  */
stx_status stx_backward(stx_ctx *ctx, const stx_incidence *inc, const stx_params *p, stx_grads *g);

/* SGD on the touched rows only: row <- row - lr * grad (product and difference rounded separately).
 * TorusE: then v <- v - floor(v) (0 if that rounds to 1): only fractional parts are kept (Sec. 4.6).
 * TransH with STX_FLAG_RENORM_W: touched w_r are rescaled to unit length.                             */
stx_status stx_sgd_step(stx_ctx *ctx, stx_params *p, const stx_incidence *inc, const stx_grads *g,
                        float lr);

/* stx_backward and stx_sgd_step in one call, with the same results in the tables (the paper counts the
 * optimiser step as part of the training loop, Table 1; fusing it with Appendix G's transposed product is
 * this library's choice).  The update is applied where the transposed products (and TransR's product for
 * dL/dM_r) would store a gradient, so no gradient is written: g may be null and, if given, is left
 * untouched.  Needs the stx_forward of the same incidence immediately before it.                       */
stx_status stx_backward_sgd(stx_ctx *ctx, const stx_incidence *inc, stx_params *p, stx_grads *g, float lr);

/* One training step in one call.  The batch's positives plus what stx_sample_negatives needs to draw its
 * negatives; neg_h / neg_t ([b*k], device, out) receive the negatives drawn (not needed when k == 0).
 * next (host, may be null): the batch the NEXT stx_train_step call on this context will be given, with the
 * same inc.  The first kernels of a build (the one that writes A, the sort keys and the negatives, the
 * first scatter pass of the sort, the histogram pass after it) depend on nothing the step before computes,
 * so they then run inside this step's launches, one stage per launch, and the next call, if it is given
 * exactly that batch, starts from where they stopped (in steady state a step is three launches); results
 * are the same bit for bit.  With next set, on return the A arrays of inc (a_rowptr, a_colidx, a_vals) and
 * next's neg_h / neg_t already hold the next batch's, the A^T arrays this batch's; until inc is built again
 * (by the next stx_train_step or by stx_build_incidence) the calls that read A through it (stx_spmm,
 * stx_spmm_semiring, stx_spmm_semiring_t, stx_forward) return STX_ERR_STATE, the calls that read only A^T
 * (stx_backward, stx_sgd_step) work as usual.  A next call with another batch simply builds as usual (an
 * out-of-range index of a batch that was announced and then not given is counted once more when its
 * batch is written again).  Used when the configuration keeps a column
 * bitmap (n_ent + n_rel <= 65,536), with dim <= 256 (TransR: also n_rel <= 4,096) and batches of at most
 * 2^19 entries of A.  Batches of more entries, on configurations without that bitmap (TransE, TorusE, TransH,
 * dim <= 256): the first of those kernels alone runs ahead, in the last launch of this step, with the same
 * effects on return.  Ignored otherwise.  next->next is ignored.                                          */
typedef struct stx_batch {
    const int32_t *h, *r, *t; /* [b], device */
    int32_t b, k;
    uint64_t seed, epoch;
    int64_t m_total, global_offset;
    int32_t *neg_h, *neg_t;
    const struct stx_batch *next;
} stx_batch;

/* stx_sample_negatives, stx_build_incidence, stx_forward and stx_backward_sgd on one batch, with the same
 * results bit for bit (negatives, incidence arrays, scores, loss, updated tables), in fewer and fatter
 * kernel launches: the negatives are drawn while A is written, and where the sizes allow independent
 * kernels share a launch (the forward pass runs beside the first pass of the sort of A^T, the final sum
 * of the loss beside a later one).  g as for stx_backward_sgd.  Afterwards inc holds this batch's
 * incidence; a stored forward is consumed (stx_backward needs a new stx_forward).                      */
stx_status stx_train_step(stx_ctx *ctx, const stx_batch *batch, stx_incidence *inc, stx_params *p, stx_grads *g,
                          float lr, float *scores, float *loss);

/* Link prediction by exhaustive scoring (Sec. 4.7 lists it among the framework's functions; Hits@10,
 * Sec. 6.1, is the share of test triplets whose true entity is among the ten best candidates).  Raw,
 * unfiltered counts.  For test triplet i = (h, r, t) every entity e of the table is a candidate; STX_TAIL
 * scores the triplets (h, r, e) (the true entity is t), STX_HEAD the triplets (e, r, t) (true entity h).
 *   TransE / TorusE : q = X[h] + X[n_ent + r], y = q - X[e]  |  q = X[t] - X[n_ent + r], y = X[e] - q;
 *                     q and y rounded once each.  A relation weight scales all candidates of a query
 *                     alike and is ignored.
 *   TransH (Sec. 4.5): y = (B - E[e]) - s w_r with B = E[h] + d_r, s = w_r.E[h] - w_r.E[e]  |
 *                     y = (E[e] - B) - s w_r with B = E[t] - d_r, s = w_r.E[e] - w_r.E[t].
 *   TransR (Sec. 4.4): with p_v = M_r E[v] in fp32 (no bfloat16 rounding here, whatever the flag),
 *                     y = (p_h + r) - p_e  |  y = p_e - (p_t - r).
 * score(e) = the context's distance of y.  Every sum (distances, dot products, projections) runs over the
 * row in index order; products inside sums are fused multiply-adds; L2 kinds are compared before the
 * square root; the torus kinds use the fractional part of y as the hardware forms it, which stays below
 * 1 where y - floor(y) would round to 1.
 *   true_score[i] : score of the true entity;
 *   n_less[i]     : candidates scoring strictly below it (the best rank it can claim is 1 + n_less);
 *   n_equal[i]    : candidates scoring exactly like it, itself included (the worst is n_less + n_equal).
 * h, r, t: [nq] device, in; the three outputs: [nq] device.  Out-of-range indices are clamped and
 * counted as in stx_build_incidence.  work: device scratch of stx_rank_work_bytes(nq) bytes, 256-byte
 * aligned, owned by the caller; TransE / TorusE / TransH need none (null is fine).  TransR groups the
 * queries by relation and builds one projected table per relation that occurs; it waits for the stream
 * once (to learn the group sizes) and launches a few kernels per relation.
 * Cost: nq * n_ent * dim steps of vector arithmetic (TransH about twice that; TransR rel_dim in place of
 * dim, plus n_ent * dim * rel_dim per relation that occurs).                                            */
enum { STX_TAIL = 0, STX_HEAD = 1 };
stx_status stx_rank_work_bytes(const stx_ctx *ctx, int64_t nq, size_t *bytes /* host, out */);
stx_status stx_rank(stx_ctx *ctx, const stx_params *p, const int32_t *h, const int32_t *r, const int32_t *t,
                    int64_t nq, int32_t side, float *true_score, int32_t *n_less, int32_t *n_equal, void *work,
                    size_t work_bytes);

const char *stx_status_string(stx_status s);

#ifdef __cplusplus
}
#endif
#endif /* STX_H */
