/*
 * stxo — CPU oracle for the sparse translation-based KGE training step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the GPU
 * library is checked against.  Only tests, the smoke check and the benchmark's
 * cpu_baseline leg may call it; the product path never does.  It shares no code,
 * header or table with the HIP sources.
 *
 * What it follows (section / equation of the SparseTransX paper, arXiv 2502.16949):
 *   - incidence matrix, `ht` form .......... Sec. 4.2.1 (two nonzeros per row: +1 head, -1 tail)
 *   - incidence matrix, `hrt` form ......... Sec. 4.2.2 (+1 head, +1 at column N+r, -1 tail;
 *                                            table X=[E;R], entities first, relations last)
 *   - TransE score ......................... Sec. 4.3, Eq. 1, Table 2
 *   - TransR score M_r(h-t)+r .............. Sec. 4.4, Eq. 2, Table 2
 *   - TransH score (h-t)+d_r-(w.(h-t))w .... Sec. 4.5, Eq. 3 and the derivation after it
 *   - TorusE score ......................... Sec. 4.6, Eq. 4 (torus distance on fractional parts)
 *   - loss: margin ranking, one pre-generated negative set ... Sec. 5.3
 *   - backward of C=AX is A^T dL/dC ........ Appendix G
 *   - three nonzeros per row, cost O(3 m n) . Appendices B, C
 *   - semiring products and their backward . Appendix D
 *   - link prediction by exhaustive scoring . Sec. 4.7, Sec. 6.1 (Hits@10)
 *
 * The method reaches exactly the result of the gather/scatter definition (Sec. 6, "Model
 * Accuracies": the sparse form does not change the computational steps), so every model function
 * below is that definition written out: per-triplet gathers, per-triplet scatters, double
 * accumulators.  The generic CSR products further down exist only so tests can check that
 * A.X equals the per-row h+r-t and that A^T.G equals the scatter.
 *
 * Readings where the paper is silent (hinge form, tie handling, sampler, SGD, wrap) are listed
 * beside each function.
 *
 * Parity pins: every function here is pinned by tests that run without a GPU
 * (tests/test_oracle_*.py); none is "parity unpinned".
 *
 * Build: gcc -O2 -std=c99 -ffp-contract=off -fno-fast-math -shared -fPIC stxo.c -o libstxo.so -lm
 */
#include <complex.h>
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { STXO_TRANSE = 0, STXO_TRANSH = 1, STXO_TRANSR = 2, STXO_TORUSE = 3 };
enum { STXO_L1 = 0, STXO_L2 = 1, STXO_TORUS_L1 = 2, STXO_TORUS_L2 = 3, STXO_L2_SQ = 4 };
enum { STXO_SUM = 0, STXO_MEAN = 1 };

typedef struct {
    int32_t model, dist, reduce;
    int32_t dim, rel_dim;
    int64_t n_ent, n_rel;
    float margin;
    int32_t bf16_proj; /* TransR only: round x, M_r (and gy in backward) to bfloat16 before the products */
} stxo_cfg;

/* Tables.  TransE/TorusE: ent = X = [E;R], (n_ent+n_rel) x dim, relation r in row n_ent+r.
 * TransH: ent = E (n_ent x dim), rel = d_r (n_rel x dim), w = w_r (n_rel x dim).
 * TransR: ent = E (n_ent x dim), rel = r (n_rel x rel_dim), proj = M_r (n_rel x rel_dim x dim, row-major). */
typedef struct {
    const float *ent, *rel, *w, *proj;
    /* Optional (NULL: every weight is 1): a fixed positive weight per relation that multiplies the
     * distance of every triplet of that relation, as in the TransM row of Table 2, w_r ||h + r - t||.
     * It is a constant of the model, not a trained parameter: no gradient is formed for it. */
    const float *rel_weight;
} stxo_tables;

static double rel_w(const stxo_tables *tb, int32_t rr) { return tb->rel_weight ? (double)tb->rel_weight[rr] : 1.0; }

/* One batch: b positives (h,r,t) and b*k negatives (nh,nt); the negative (i,kk) keeps r[i].
 * Row order of the incidence matrix: positives 0..b-1, then negative (i,kk) at b + i*k + kk. */
typedef struct {
    const int32_t *h, *r, *t, *nh, *nt;
    int32_t b, k;
} stxo_batch;

/* ------------------------------------------------------------------------------------------ */
/* Counter-based random numbers: output number `counter` (from 0) of the SplitMix64 sequence
 * (Steele, Lea, Flood, "Fast splittable pseudorandom number generators", OOPSLA 2014; the
 * 64-bit finaliser and the golden-gamma increment of that paper) started at `seed`.          */
uint64_t stxo_rng_u64(uint64_t seed, uint64_t counter)
{
    uint64_t z = seed + (counter + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* Negative sampling (Sec. 5.3: generated once per positive, outside the loop; Sec. 6.1: equal
 * numbers of positives and negatives).  The paper names no algorithm; the reading used:
 * for positive with global index g = global_offset + i and slot kk, draw
 * u = rng(seed, (epoch*m_total + g)*k + kk); corrupt the head if the top bit of u is set, else
 * the tail; replacement entity = floor(low32(u) * n_ent / 2^32).  No rejection or filtering; the
 * relation is never corrupted.                                                               */
void stxo_sample_negatives(const int32_t *h, const int32_t *r, const int32_t *t, int64_t m, int32_t k,
                           int64_t n_ent, uint64_t seed, uint64_t epoch, int64_t m_total,
                           int64_t global_offset, int32_t *neg_h, int32_t *neg_t)
{
    (void)r;
    for (int64_t i = 0; i < m; ++i) {
        for (int32_t kk = 0; kk < k; ++kk) {
            uint64_t g = (uint64_t)(global_offset + i);
            uint64_t ctr = (epoch * (uint64_t)m_total + g) * (uint64_t)k + (uint64_t)kk;
            uint64_t u = stxo_rng_u64(seed, ctr);
            uint64_t lo = u & 0xFFFFFFFFull;
            int32_t e = (int32_t)((lo * (uint64_t)n_ent) >> 32);
            int head = (int)(u >> 63);
            neg_h[i * k + kk] = head ? e : h[i];
            neg_t[i * k + kk] = head ? t[i] : e;
        }
    }
}

/* ------------------------------------------------------------------------------------------ */
static void batch_row(const stxo_batch *bt, int64_t row, int32_t *hh, int32_t *rr, int32_t *tt)
{
    if (row < bt->b) {
        *hh = bt->h[row]; *rr = bt->r[row]; *tt = bt->t[row];
    } else {
        int64_t j = row - bt->b;
        *hh = bt->nh[j]; *rr = bt->r[j / bt->k]; *tt = bt->nt[j];
    }
}

/* Incidence matrix of a batch in the `hrt` form (Sec. 4.2.2) as CSR, plus its transpose.
 *   A: rowptr[i] = 3i; slots of row i in the order (head, N+relation, tail), values (+1,+1,-1).
 *      The `ht` form (Sec. 4.2.1) is slots 0 and 2 of every row.
 *      A self-loop (h == t) keeps both entries; nothing is merged.
 *   A^T, doubly compressed: only columns with at least one entry appear.
 *      touched_cols[0..U)  ascending column ids
 *      seg_ptr[0..U]       start of each column's run in the sorted entry list, seg_ptr[U] = nnz
 *      row_idx[e], sign[e] row and value of sorted entry e
 *      seg_id[e]           index into touched_cols of sorted entry e
 *      Entries of one column are ordered by their position 3*row+slot in A (stable counting sort).
 * Returns 0, or 1 if an index is out of range (nothing is written then).                      */
int stxo_build_incidence(const stxo_batch *bt, int64_t n_ent, int64_t n_rel,
                         int32_t *rowptr, int32_t *colidx, float *vals,
                         int32_t *touched_cols, int32_t *seg_ptr, int32_t *row_idx, int8_t *sign,
                         int32_t *seg_id, int32_t *n_touched)
{
    int64_t rows = (int64_t)bt->b * (1 + bt->k);
    int64_t nnz = 3 * rows;
    int64_t ncol = n_ent + n_rel;
    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        batch_row(bt, i, &hh, &rr, &tt);
        if (hh < 0 || hh >= n_ent || tt < 0 || tt >= n_ent || rr < 0 || rr >= n_rel) return 1;
    }
    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        batch_row(bt, i, &hh, &rr, &tt);
        rowptr[i] = (int32_t)(3 * i);
        colidx[3 * i + 0] = hh;               vals[3 * i + 0] = 1.0f;
        colidx[3 * i + 1] = (int32_t)(n_ent + rr); vals[3 * i + 1] = 1.0f;
        colidx[3 * i + 2] = tt;               vals[3 * i + 2] = -1.0f;
    }
    rowptr[rows] = (int32_t)nnz;

    int64_t *count = (int64_t *)calloc((size_t)ncol + 1, sizeof(int64_t));
    if (!count) return 2;
    for (int64_t e = 0; e < nnz; ++e) count[colidx[e] + 1]++;
    for (int64_t c = 0; c < ncol; ++c) count[c + 1] += count[c]; /* count[c] = first sorted position of column c */
    int32_t u = 0;
    int32_t *col_seg = (int32_t *)malloc((size_t)ncol * sizeof(int32_t));
    if (!col_seg) { free(count); return 2; }
    for (int64_t c = 0; c < ncol; ++c) {
        if (count[c + 1] > count[c]) {
            touched_cols[u] = (int32_t)c;
            seg_ptr[u] = (int32_t)count[c];
            col_seg[c] = u;
            ++u;
        } else col_seg[c] = -1;
    }
    seg_ptr[u] = (int32_t)nnz;
    *n_touched = u;
    for (int64_t e = 0; e < nnz; ++e) { /* ascending e within each column: stable */
        int32_t c = colidx[e];
        int64_t p = count[c]++;
        row_idx[p] = (int32_t)(e / 3);
        sign[p] = (int8_t)((e % 3) == 2 ? -1 : 1);
        seg_id[p] = col_seg[c];
    }
    free(col_seg);
    free(count);
    return 0;
}

/* ------------------------------------------------------------------------------------------ */
/* Generic CSR products (test helpers for the invariants of Sec. 4.2 and Appendix G).           */

/* C = A X in fp32, each row accumulated left to right over its stored entries, starting from the
 * first product (not from zero), one rounding per operation, no fused multiply-add.           */
void stxo_spmm_csr(int64_t nrows, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                   const float *X, int32_t d, float *C)
{
    for (int64_t i = 0; i < nrows; ++i) {
        for (int32_t j = 0; j < d; ++j) {
            int32_t p0 = rowptr[i], p1 = rowptr[i + 1];
            float acc = 0.0f;
            for (int32_t p = p0; p < p1; ++p) {
                volatile float prod = vals[p] * X[(int64_t)colidx[p] * d + j];
                acc = (p == p0) ? prod : (float)(acc + prod);
            }
            C[i * d + j] = acc;
        }
    }
}

/* The semiring products of Appendix D over rows with three stored entries (head, relation, tail
 * columns, in that order, as in the hrt incidence matrix): the model's multiplication takes the
 * place of the sum over the row's entries.  fp32, every real product and sum rounded once.
 *   kind 0, DistMult: z_j = (h_j r_j) t_j
 *   kind 1, ComplEx : rows are d/2 complex numbers stored (re, im); z = (h r) conj(t)
 *   kind 2, RotatE  : the same storage; z = h r - t
 * with the complex product (a+bi)(c+di) = (ac - bd) + (ad + bc)i.                              */
static void cmul(float a, float b, float c, float d, float *re, float *im)
{
    volatile float ac = a * c, bd = b * d, ad = a * d, bc = b * c;
    *re = ac - bd;
    *im = ad + bc;
}

int stxo_spmm_semiring(int64_t nrows, const int32_t *colidx, const float *X, int32_t d, int32_t kind, float *Z)
{
    if (kind < 0 || kind > 2 || (kind != 0 && d % 2 != 0)) return 1;
    for (int64_t i = 0; i < nrows; ++i) {
        const float *h = X + (int64_t)colidx[3 * i] * d, *r = X + (int64_t)colidx[3 * i + 1] * d;
        const float *t = X + (int64_t)colidx[3 * i + 2] * d;
        float *z = Z + i * d;
        if (kind == 0) {
            for (int32_t j = 0; j < d; ++j) {
                volatile float hr = h[j] * r[j];
                z[j] = hr * t[j];
            }
        } else {
            for (int32_t j = 0; j < d; j += 2) {
                float re, im;
                cmul(h[j], h[j + 1], r[j], r[j + 1], &re, &im);
                if (kind == 1) cmul(re, im, t[j], -t[j + 1], &z[j], &z[j + 1]);
                else { z[j] = re - t[j]; z[j + 1] = im - t[j + 1]; }
            }
        }
    }
    return 0;
}

/* Backward of the semiring products for a real-valued loss L (Appendix D names the products only;
 * Appendix G's rule "the gradient flows back along the entries of the row" carries over, with the
 * model's product in place of the sign).  G = dL/dZ, rows of d floats; for the complex kinds a pair
 * holds (dL/dRe z, dL/dIm z).  With g the complex number made of such a pair, the chain rule gives
 * dL/dv = g conj(dz/dv) for a factor v the product is holomorphic in, and dL/dv = conj(g) (dz/dconj(v))
 * for ComplEx's tail, which enters conjugated:
 *   DistMult  dL/dh = g r t         dL/dr = g h t         dL/dt = g h r       (real numbers)
 *   ComplEx   dL/dh = g conj(r) t   dL/dr = g conj(h) t   dL/dt = conj(g) h r
 *   RotatE    dL/dh = g conj(r)     dL/dr = g conj(h)     dL/dt = -g
 * out (ncols x d, double, caller-zeroed) += these rows at the row's head, relation and tail columns,
 * looping over the rows in ascending order; scale (same shape) += a bound on the magnitudes of the real
 * products behind each element (the products of the factors' |re| + |im|), the error scale that a
 * comparison in single precision needs.                                                              */
static double l1mod(double complex v) { return fabs(creal(v)) + fabs(cimag(v)); }

int stxo_spmm_semiring_t(int64_t nrows, const int32_t *colidx, const float *X, int32_t d, int32_t kind,
                         const float *G, double *out, double *scale)
{
    if (kind < 0 || kind > 2 || (kind != 0 && d % 2 != 0)) return 1;
    for (int64_t i = 0; i < nrows; ++i) {
        const int64_t ch = colidx[3 * i], cr = colidx[3 * i + 1], ct = colidx[3 * i + 2];
        const float *h = X + ch * d, *r = X + cr * d, *t = X + ct * d, *g = G + i * d;
        if (kind == 0) {
            for (int32_t j = 0; j < d; ++j) {
                const double gj = g[j], hj = h[j], rj = r[j], tj = t[j];
                out[ch * d + j] += gj * rj * tj;
                out[cr * d + j] += gj * hj * tj;
                out[ct * d + j] += gj * hj * rj;
                scale[ch * d + j] += fabs(gj * rj * tj);
                scale[cr * d + j] += fabs(gj * hj * tj);
                scale[ct * d + j] += fabs(gj * hj * rj);
            }
            continue;
        }
        for (int32_t j = 0; j < d; j += 2) {
            const double complex gz = g[j] + I * (double)g[j + 1], hz = h[j] + I * (double)h[j + 1];
            const double complex rz = r[j] + I * (double)r[j + 1], tz = t[j] + I * (double)t[j + 1];
            double complex dh, dr, dt;
            double sh, sr, st;
            if (kind == 1) {
                dh = gz * conj(rz) * tz;  sh = l1mod(gz) * l1mod(rz) * l1mod(tz);
                dr = gz * conj(hz) * tz;  sr = l1mod(gz) * l1mod(hz) * l1mod(tz);
                dt = conj(gz) * hz * rz;  st = l1mod(gz) * l1mod(hz) * l1mod(rz);
            } else {
                dh = gz * conj(rz);       sh = l1mod(gz) * l1mod(rz);
                dr = gz * conj(hz);       sr = l1mod(gz) * l1mod(hz);
                dt = -gz;                 st = l1mod(gz);
            }
            out[ch * d + j] += creal(dh); out[ch * d + j + 1] += cimag(dh);
            out[cr * d + j] += creal(dr); out[cr * d + j + 1] += cimag(dr);
            out[ct * d + j] += creal(dt); out[ct * d + j + 1] += cimag(dt);
            scale[ch * d + j] += sh; scale[ch * d + j + 1] += sh;
            scale[cr * d + j] += sr; scale[cr * d + j + 1] += sr;
            scale[ct * d + j] += st; scale[ct * d + j + 1] += st;
        }
    }
    return 0;
}

/* out (ncols x d, double, caller-zeroed) += A^T G, looping over the rows of A.                 */
void stxo_spmm_csr_t(int64_t nrows, const int32_t *rowptr, const int32_t *colidx, const float *vals,
                     const float *G, int32_t d, double *out)
{
    for (int64_t i = 0; i < nrows; ++i)
        for (int32_t p = rowptr[i]; p < rowptr[i + 1]; ++p)
            for (int32_t j = 0; j < d; ++j)
                out[(int64_t)colidx[p] * d + j] += (double)vals[p] * (double)G[i * d + j];
}

/* ------------------------------------------------------------------------------------------ */
static float bf16_round(float v)
{ /* round-to-nearest-even to 8 significand bits (bfloat16), result held in a float */
    uint32_t u;
    memcpy(&u, &v, 4);
    if ((u & 0x7F800000u) == 0x7F800000u) return v; /* inf / nan unchanged */
    uint32_t lsb = (u >> 16) & 1u;
    u += 0x7FFFu + lsb;
    u &= 0xFFFF0000u;
    memcpy(&v, &u, 4);
    return v;
}
float stxo_bf16_round(float v) { return bf16_round(v); }

static int is_stacked(const stxo_cfg *c) { return c->model == STXO_TRANSE || c->model == STXO_TORUSE; }
static int out_dim(const stxo_cfg *c) { return c->model == STXO_TRANSR ? c->rel_dim : c->dim; }

/* x of one row: fp32, (h + r) - t for the hrt models, h - t for the ht models (Sec. 4.2). */
static void row_x(const stxo_cfg *c, const stxo_tables *tb, int32_t hh, int32_t rr, int32_t tt, float *x)
{
    int32_t d = c->dim;
    const float *eh = tb->ent + (int64_t)hh * d, *et = tb->ent + (int64_t)tt * d;
    if (is_stacked(c)) {
        const float *er = tb->ent + (c->n_ent + rr) * (int64_t)d;
        for (int32_t j = 0; j < d; ++j) {
            volatile float s = eh[j] + er[j];
            x[j] = s - et[j];
        }
    } else {
        for (int32_t j = 0; j < d; ++j) x[j] = eh[j] - et[j];
    }
}

/* y of one row in double (length out_dim), and s = w.x for TransH.  yabs (optional): for every
 * element of y the sum of the absolute values of the terms it is made of, i.e. the scale against
 * which an fp32 evaluation of y can be off. */
static void row_y(const stxo_cfg *c, const stxo_tables *tb, int32_t rr, const float *x, double *y, double *s_out,
                  double *yabs)
{
    int32_t d = c->dim;
    if (is_stacked(c)) {
        for (int32_t j = 0; j < d; ++j) { y[j] = (double)x[j]; if (yabs) yabs[j] = fabs((double)x[j]); }
    } else if (c->model == STXO_TRANSH) {
        const float *w = tb->w + (int64_t)rr * d, *dr = tb->rel + (int64_t)rr * d;
        double s = 0.0;
        for (int32_t j = 0; j < d; ++j) s += (double)w[j] * (double)x[j];
        for (int32_t j = 0; j < d; ++j) {
            y[j] = ((double)x[j] + (double)dr[j]) - s * (double)w[j];
            if (yabs) yabs[j] = fabs((double)x[j]) + fabs((double)dr[j]) + fabs(s * (double)w[j]);
        }
        if (s_out) *s_out = s;
    } else { /* TransR */
        int32_t kd = c->rel_dim;
        const float *M = tb->proj + (int64_t)rr * kd * d, *rv = tb->rel + (int64_t)rr * kd;
        for (int32_t a = 0; a < kd; ++a) {
            double acc = 0.0, aacc = 0.0;
            for (int32_t j = 0; j < d; ++j) {
                float m = M[(int64_t)a * d + j], xv = x[j];
                if (c->bf16_proj) { m = bf16_round(m); xv = bf16_round(xv); }
                acc += (double)m * (double)xv;
                aacc += fabs((double)m * (double)xv);
            }
            y[a] = acc + (double)rv[a];
            if (yabs) yabs[a] = aacc + fabs((double)rv[a]);
        }
    }
}

/* Distance of Table 2's norm: L1, L2 (unsquared), the squared L2 norm of the TransC row of that
 * table, or the torus versions on f = y - floor(y): torus-L1 = sum min(f,1-f); torus-L2 =
 * sqrt(sum min(f,1-f)^2).  For the torus the fractional part is taken in fp32 (y is the fp32 x
 * there), the sum in double.                                                                  */
static double row_dist(const stxo_cfg *c, const double *y, int32_t n)
{
    double acc = 0.0;
    switch (c->dist) {
    case STXO_L1: for (int32_t j = 0; j < n; ++j) acc += fabs(y[j]); return acc;
    case STXO_L2: for (int32_t j = 0; j < n; ++j) acc += y[j] * y[j]; return sqrt(acc);
    case STXO_L2_SQ: for (int32_t j = 0; j < n; ++j) acc += y[j] * y[j]; return acc;
    default:
        for (int32_t j = 0; j < n; ++j) {
            float yf = (float)y[j];
            float f = yf - floorf(yf);
            float g = 1.0f - f;
            float m = f < g ? f : g;
            acc += (c->dist == STXO_TORUS_L1) ? (double)m : (double)m * (double)m;
        }
        return c->dist == STXO_TORUS_L1 ? acc : sqrt(acc);
    }
}

/* d(dist)/dy.  Subgradient 0 at every tie: sign(0)=0, zero vector at ||y||=0, 0 at f in {0, 1/2}. */
static void row_ddist(const stxo_cfg *c, const double *y, int32_t n, double dist, double *g)
{
    for (int32_t j = 0; j < n; ++j) {
        switch (c->dist) {
        case STXO_L1: g[j] = (y[j] > 0) - (y[j] < 0); break;
        case STXO_L2: g[j] = dist > 0 ? y[j] / dist : 0.0; break;
        case STXO_L2_SQ: g[j] = 2.0 * y[j]; break;
        default: {
            float yf = (float)y[j];
            float f = yf - floorf(yf);
            double sg = (f > 0.0f && f < 0.5f) ? 1.0 : (f > 0.5f ? -1.0 : 0.0);
            if (c->dist == STXO_TORUS_L1) g[j] = sg;
            else {
                float gg = 1.0f - f;
                double m = f < gg ? f : gg;
                g[j] = dist > 0 ? sg * m / dist : 0.0;
            }
        }
        }
    }
}

/* Forward: x (optional, rows x dim fp32), scores (rows, double), the hinge argument
 * margin + d_pos - d_neg of every (positive, negative) pair (b*k, double, optional) and the loss
 * sum (or mean over the b*k pairs) of max(0, that argument).                                  */
int stxo_forward(const stxo_cfg *c, const stxo_tables *tb, const stxo_batch *bt,
                 float *x_out, double *scores, double *hinge_arg, double *loss)
{
    int32_t d = c->dim, n = out_dim(c);
    int64_t rows = (int64_t)bt->b * (1 + bt->k);
    float *x = (float *)malloc(sizeof(float) * (size_t)d);
    double *y = (double *)malloc(sizeof(double) * (size_t)n);
    if (!x || !y) return 2;
    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        batch_row(bt, i, &hh, &rr, &tt);
        row_x(c, tb, hh, rr, tt, x);
        if (x_out) memcpy(x_out + i * d, x, sizeof(float) * (size_t)d);
        row_y(c, tb, rr, x, y, NULL, NULL);
        scores[i] = rel_w(tb, rr) * row_dist(c, y, n);
    }
    double total = 0.0;
    for (int64_t i = 0; i < bt->b; ++i)
        for (int32_t kk = 0; kk < bt->k; ++kk) {
            int64_t p = i * bt->k + kk;
            double a = (double)c->margin + scores[i] - scores[bt->b + p];
            if (hinge_arg) hinge_arg[p] = a;
            if (a > 0) total += a;
        }
    if (c->reduce == STXO_MEAN) total /= (double)((int64_t)bt->b * bt->k);
    *loss = total;
    free(x); free(y);
    return 0;
}

/* Link prediction by exhaustive scoring (the "predicting links" facility of Sec. 4.7; Hits@10, the
 * accuracy measure of Sec. 6.1, is the share of test triplets whose true entity ranks among the ten
 * best).  The paper fixes no protocol; the reading taken here is the usual
 * raw (unfiltered) one: for a test triplet (h, r, t) every entity e of the table is a candidate,
 * side 0 (tail prediction) scores the triplets (h, r, e), true entity t; side 1 (head prediction)
 * scores (e, r, t), true entity h; smaller is better.
 *   TransE / TorusE: query point q = h + r (tail side) or t - r (head side), score of e =
 *     distance(q - e) or distance(e - q); q and the difference are each rounded once to fp32 (for the
 *     tail side that is the x of the training score, bit for bit).  A relation weight (Table 2, TransM)
 *     would scale all candidates of a query alike and plays no part.
 *   TransH: the training score of the triplet with e in place of the true entity (Sec. 4.5):
 *     x = h - e or e - t in fp32, y = x + d_r - (w_r.x) w_r, distance(y), by row_x / row_y above.
 *   TransR: likewise (Sec. 4.4): y = M_r x + r on the fp32 operands as they are (rounding the operands to
 *     bfloat16 is an option of the training configuration; a configuration that sets it is refused here).
 * The distance is the model's (row_dist, summed in double).  Outputs per query:
 *   true_score : the true entity's score;
 *   n_less     : candidates scoring strictly below the true entity and outside the band below;
 *   n_band     : candidates with |score - true| <= tol * (scale + scale of the true entity), the true
 *                entity among them, where scale is the distance taken over the sums of magnitudes of
 *                the terms behind each element of y (the score itself for TransE / TorusE; twice that
 *                for the squared L2 norm of a computed y): the size against which a single-precision
 *                evaluation of the score can be off.
 * abs_tol (optional, one value per query) widens the band by an absolute amount: a caller that knows an
 * error term of the evaluation it checks which the scales above do not cover passes it here.
 * With tol = 0 the band holds the exact ties, the best rank the true entity can claim is 1 + n_less
 * and the worst n_less + n_band.  With tol > 0 the band holds every candidate whose order against
 * the true entity a single-precision evaluation may decide either way.                          */
int stxo_rank(const stxo_cfg *c, const stxo_tables *tb, const int32_t *h, const int32_t *r, const int32_t *t,
              int64_t nq, int32_t side, double tol, const double *abs_tol, double *true_score, int64_t *n_less,
              int64_t *n_band)
{
    if ((c->model == STXO_TRANSR && c->bf16_proj) || side < 0 || side > 1) return 1;
    const int32_t d = c->dim, n = out_dim(c);
    const float *X = tb->ent;
    float *q = (float *)malloc(sizeof(float) * (size_t)d);
    float *x = (float *)malloc(sizeof(float) * (size_t)d);
    double *y = (double *)malloc(sizeof(double) * (size_t)(d > n ? d : n));
    double *ya = (double *)malloc(sizeof(double) * (size_t)(d > n ? d : n));
    double *score = (double *)malloc(sizeof(double) * (size_t)c->n_ent);
    double *scale = (double *)malloc(sizeof(double) * (size_t)c->n_ent);
    if (!q || !x || !y || !ya || !score || !scale) return 2;
    for (int64_t i = 0; i < nq; ++i) {
        if (is_stacked(c)) {
            const float *eh = X + (int64_t)h[i] * d, *et = X + (int64_t)t[i] * d;
            const float *er = X + (c->n_ent + r[i]) * (int64_t)d;
            for (int32_t j = 0; j < d; ++j) q[j] = side == 0 ? eh[j] + er[j] : et[j] - er[j];
        }
        for (int64_t e = 0; e < c->n_ent; ++e) {
            if (is_stacked(c)) {
                const float *ee = X + e * d;
                for (int32_t j = 0; j < d; ++j) {
                    const float diff = side == 0 ? q[j] - ee[j] : ee[j] - q[j];
                    y[j] = (double)diff;
                }
                score[e] = scale[e] = row_dist(c, y, d);
            } else {
                row_x(c, tb, side == 0 ? h[i] : (int32_t)e, r[i], side == 0 ? (int32_t)e : t[i], x);
                row_y(c, tb, r[i], x, y, NULL, ya);
                score[e] = row_dist(c, y, n);
                scale[e] = (c->dist == STXO_L2_SQ ? 2.0 : 1.0) * row_dist(c, ya, n);
            }
        }
        const int64_t te = side == 0 ? t[i] : h[i];
        const double st = score[te];
        int64_t less = 0, band = 0;
        for (int64_t e = 0; e < c->n_ent; ++e) {
            if (fabs(score[e] - st) <= tol * (scale[e] + scale[te]) + (abs_tol ? abs_tol[i] : 0.0)) ++band;
            else if (score[e] < st) ++less;
        }
        true_score[i] = st;
        n_less[i] = less;
        n_band[i] = band;
    }
    free(q); free(x); free(y); free(ya); free(score); free(scale);
    return 0;
}

/* Backward by explicit scatter, rows in ascending order, double accumulators.
 * active_override (b*k bytes, may be NULL): use these hinge flags instead of the oracle's own
 * (margin + d_pos - d_neg > 0, strict).
 * Outputs are dense, caller-zeroed, double; each has a twin `a_*` receiving the sum of the
 * absolute values of the separately rounded terms that make up the same element (the comparison
 * scale; e.g. for TransH's gx = gy - a w both |gy| and |a w| count, for TransR's gx = M^T gy every
 * |gy_a M_aj|):
 *   g_ent : stacked models (n_ent+n_rel) x dim; otherwise n_ent x dim
 *   g_rel : TransH n_rel x dim (d_r); TransR n_rel x rel_dim (r); unused for stacked models
 *   g_w   : TransH n_rel x dim
 *   g_proj: TransR n_rel x rel_dim x dim
 * For TransH and TransR, y itself is a computed quantity, so the scale of dL/dy_j used in those sums
 * is max(|dL/dy_j|, |coef|/dist * sum|terms of y_j|) for the L2 kinds (2 |coef| * sum|terms of y_j|
 * for the squared L2 norm).
 * gy_out (optional, rows x out_dim doubles): dL/dy of every row.
 * ambiguous (optional, rows bytes): set to 1 for rows of TransH/TransR with an L1-kind distance in
 * which some y_j lies within 1e-5 * sum|terms of y_j| of a point where the subgradient jumps (0, or
 * fractional part 0 / one half on the torus): there an fp32 evaluation may pick the other branch.
 * An element whose terms are all zero is zero in any precision and never sets the flag. */
#define STXO_TIE_WIDTH 1e-5
int stxo_backward(const stxo_cfg *c, const stxo_tables *tb, const stxo_batch *bt,
                  const uint8_t *active_override,
                  double *g_ent, double *a_ent, double *g_rel, double *a_rel,
                  double *g_w, double *a_w, double *g_proj, double *a_proj, double *gy_out,
                  uint8_t *ambiguous)
{
    int32_t d = c->dim, n = out_dim(c), b = bt->b, k = bt->k;
    int64_t rows = (int64_t)b * (1 + k);
    double scale = c->reduce == STXO_MEAN ? 1.0 / (double)((int64_t)b * k) : 1.0;
    float *x = (float *)malloc(sizeof(float) * (size_t)d);
    double *y = (double *)malloc(sizeof(double) * (size_t)n);
    double *gd = (double *)malloc(sizeof(double) * (size_t)n);
    double *gx = (double *)malloc(sizeof(double) * (size_t)d);
    double *ax = (double *)malloc(sizeof(double) * (size_t)d); /* sum of |products| that make up gx */
    double *yabs = (double *)malloc(sizeof(double) * (size_t)n);
    double *ug = (double *)malloc(sizeof(double) * (size_t)n);  /* scale of each dL/dy_j */
    double *dist = (double *)malloc(sizeof(double) * (size_t)rows);   /* the norm itself ... */
    double *wrow = (double *)malloc(sizeof(double) * (size_t)rows);   /* ... and the row's relation weight */
    double *coef = (double *)calloc((size_t)rows, sizeof(double));
    if (!x || !y || !gd || !gx || !ax || !yabs || !ug || !dist || !wrow || !coef) return 2;

    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        batch_row(bt, i, &hh, &rr, &tt);
        row_x(c, tb, hh, rr, tt, x);
        row_y(c, tb, rr, x, y, NULL, NULL);
        dist[i] = row_dist(c, y, n);
        wrow[i] = rel_w(tb, rr);
    }
    for (int64_t i = 0; i < b; ++i)
        for (int32_t kk = 0; kk < k; ++kk) {
            int64_t p = i * k + kk;
            int act = active_override ? (active_override[p] != 0)
                                      : ((double)c->margin + wrow[i] * dist[i] - wrow[b + p] * dist[b + p] > 0);
            if (act) { coef[i] += scale; coef[b + p] -= scale; }
        }
    for (int64_t i = 0; i < rows; ++i) coef[i] *= wrow[i];   /* score = weight * norm */
    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        double s = 0.0;
        batch_row(bt, i, &hh, &rr, &tt);
        row_x(c, tb, hh, rr, tt, x);
        row_y(c, tb, rr, x, y, &s, yabs);
        row_ddist(c, y, n, dist[i], gd);
        for (int32_t j = 0; j < n; ++j) gd[j] *= coef[i]; /* gd is now dL/dy */
        if (gy_out) memcpy(gy_out + i * n, gd, sizeof(double) * (size_t)n);
        {
            int l2kind = c->dist == STXO_L2 || c->dist == STXO_TORUS_L2, amb = 0;
            for (int32_t j = 0; j < n; ++j) {
                ug[j] = fabs(gd[j]);
                if (is_stacked(c)) continue;            /* there y is the exact fp32 x */
                if (l2kind) {
                    double alt = dist[i] > 0 ? fabs(coef[i]) / dist[i] * yabs[j] : 0.0;
                    if (alt > ug[j]) ug[j] = alt;
                } else if (c->dist == STXO_L2_SQ) {
                    double alt = 2.0 * fabs(coef[i]) * yabs[j];
                    if (alt > ug[j]) ug[j] = alt;
                } else if (yabs[j] == 0.0) {
                    continue;                           /* every term is 0: y_j is 0 in any precision */
                } else if (c->dist == STXO_L1) {
                    if (fabs(y[j]) <= STXO_TIE_WIDTH * yabs[j]) amb = 1;
                } else {
                    double f = y[j] - floor(y[j]);
                    double dd = fmin(fmin(f, 1.0 - f), fabs(f - 0.5));
                    if (dd <= STXO_TIE_WIDTH * yabs[j]) amb = 1;
                }
            }
            if (ambiguous) ambiguous[i] = (uint8_t)amb;
        }

        if (is_stacked(c)) {
            for (int32_t j = 0; j < d; ++j) { gx[j] = gd[j]; ax[j] = fabs(gd[j]); }
            double *gr = g_ent + (c->n_ent + rr) * (int64_t)d, *ar = a_ent + (c->n_ent + rr) * (int64_t)d;
            for (int32_t j = 0; j < d; ++j) { gr[j] += gx[j]; ar[j] += fabs(gx[j]); }
        } else if (c->model == STXO_TRANSH) {
            const float *w = tb->w + (int64_t)rr * d;
            double a = 0.0;
            for (int32_t j = 0; j < d; ++j) a += gd[j] * (double)w[j];
            for (int32_t j = 0; j < d; ++j) {
                gx[j] = gd[j] - a * (double)w[j];
                ax[j] = ug[j] + fabs(a * (double)w[j]);
            }
            double *gr = g_rel + (int64_t)rr * d, *ar = a_rel + (int64_t)rr * d;
            double *gw = g_w + (int64_t)rr * d, *aw = a_w + (int64_t)rr * d;
            for (int32_t j = 0; j < d; ++j) {
                gr[j] += gd[j]; ar[j] += ug[j];
                double term = -(a * (double)x[j] + s * gd[j]);
                gw[j] += term; aw[j] += fabs(a * (double)x[j]) + fabs(s) * ug[j];
            }
        } else { /* TransR: y = M x + r */
            int32_t kd = c->rel_dim;
            const float *M = tb->proj + (int64_t)rr * kd * d;
            double *gM = g_proj + (int64_t)rr * kd * d, *aM = a_proj + (int64_t)rr * kd * d;
            double *gr = g_rel + (int64_t)rr * kd, *ar = a_rel + (int64_t)rr * kd;
            for (int32_t j = 0; j < d; ++j) { gx[j] = 0.0; ax[j] = 0.0; }
            for (int32_t a = 0; a < kd; ++a) {
                double gya = gd[a];
                gr[a] += gya; ar[a] += ug[a];
                double gq = c->bf16_proj ? (double)bf16_round((float)gya) : gya;
                for (int32_t j = 0; j < d; ++j) {
                    float m = M[(int64_t)a * d + j], xv = x[j];
                    if (c->bf16_proj) { m = bf16_round(m); xv = bf16_round(xv); }
                    gx[j] += gq * (double)m;
                    ax[j] += ug[a] * fabs((double)m);
                    double term = gq * (double)xv;
                    gM[(int64_t)a * d + j] += term; aM[(int64_t)a * d + j] += ug[a] * fabs((double)xv);
                }
            }
        }
        double *gh = g_ent + (int64_t)hh * d, *ah = a_ent + (int64_t)hh * d;
        double *gt = g_ent + (int64_t)tt * d, *at = a_ent + (int64_t)tt * d;
        for (int32_t j = 0; j < d; ++j) { gh[j] += gx[j]; ah[j] += ax[j]; }
        for (int32_t j = 0; j < d; ++j) { gt[j] -= gx[j]; at[j] += ax[j]; }
    }
    free(x); free(y); free(gd); free(gx); free(ax); free(yabs); free(ug); free(dist); free(wrow); free(coef);
    return 0;
}

/* SGD on the rows marked in `touched` (n_rows bytes): v <- v - lr*g with the gradient first rounded
 * to fp32, product and difference each rounded once (no fused multiply-add).
 * mode 1 (torus, Sec. 4.6: only fractional parts are kept): then v <- v - floor(v), and 0 if that
 *         rounds up to 1.
 * mode 2 (TransH normals): then the row is divided by its Euclidean norm (sum in double), unless
 *         the norm is 0.                                                                      */
void stxo_sgd(float *table, int64_t n_rows, int32_t dim, const double *grad, const uint8_t *touched,
              float lr, int32_t mode)
{
    for (int64_t i = 0; i < n_rows; ++i) {
        if (!touched[i]) continue;
        float *v = table + i * dim;
        for (int32_t j = 0; j < dim; ++j) {
            float g = (float)grad[i * dim + j];
            volatile float step = lr * g;
            float nv = v[j] - step;
            if (mode == 1) {
                nv = nv - floorf(nv);
                if (nv >= 1.0f) nv = 0.0f;
            }
            v[j] = nv;
        }
        if (mode == 2) {
            double ss = 0.0;
            for (int32_t j = 0; j < dim; ++j) ss += (double)v[j] * (double)v[j];
            if (ss > 0) {
                double inv = 1.0 / sqrt(ss);
                for (int32_t j = 0; j < dim; ++j) v[j] = (float)((double)v[j] * inv);
            }
        }
    }
}

/* Torus wrap of a whole table (used once on the initial TorusE table). */
void stxo_wrap(float *table, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        float v = table[i] - floorf(table[i]);
        table[i] = v >= 1.0f ? 0.0f : v;
    }
}

/* Gradient of one column of the stacked / entity table for a stacked model, computed directly from
 * the definition by scanning every row of the batch: for spot checks at sizes where the dense
 * tables of stxo_backward are too large.  out and aout have `dim` doubles.                    */
int stxo_grad_column_stacked(const stxo_cfg *c, const stxo_tables *tb, const stxo_batch *bt,
                             const uint8_t *active, int64_t col, double *out, double *aout)
{
    if (!is_stacked(c)) return 1;
    int32_t d = c->dim, b = bt->b, k = bt->k;
    int64_t rows = (int64_t)b * (1 + k);
    double scale = c->reduce == STXO_MEAN ? 1.0 / (double)((int64_t)b * k) : 1.0;
    float *x = (float *)malloc(sizeof(float) * (size_t)d);
    double *y = (double *)malloc(sizeof(double) * (size_t)d);
    double *gd = (double *)malloc(sizeof(double) * (size_t)d);
    if (!x || !y || !gd) return 2;
    for (int32_t j = 0; j < d; ++j) { out[j] = 0; aout[j] = 0; }
    for (int64_t i = 0; i < rows; ++i) {
        int32_t hh, rr, tt;
        batch_row(bt, i, &hh, &rr, &tt);
        int hit_h = hh == col, hit_r = (c->n_ent + rr) == col, hit_t = tt == col;
        if (!hit_h && !hit_r && !hit_t) continue;
        double coef = 0.0;
        if (i < b) { for (int32_t kk = 0; kk < k; ++kk) if (active[i * k + kk]) coef += scale; }
        else if (active[i - b]) coef = -scale;
        coef *= rel_w(tb, rr);
        row_x(c, tb, hh, rr, tt, x);
        row_y(c, tb, rr, x, y, NULL, NULL);
        double dist = row_dist(c, y, d);
        row_ddist(c, y, d, dist, gd);
        for (int32_t j = 0; j < d; ++j) {
            double g = gd[j] * coef;
            if (hit_h) { out[j] += g; aout[j] += fabs(g); }
            if (hit_r) { out[j] += g; aout[j] += fabs(g); }
            if (hit_t) { out[j] -= g; aout[j] += fabs(g); }
        }
    }
    free(x); free(y); free(gd);
    return 0;
}
