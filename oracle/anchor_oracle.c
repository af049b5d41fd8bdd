/*
 * anchor_oracle.c -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, fp64 CPU statement of what AnchorAttention's sparse causal
 * prefill computes for ONE query head of ONE sequence (arXiv 2505.23520,
 * Section 3 and Algorithms 1-3).  It exists so that the GPU library can be
 * checked against something that can be read next to the paper.  Nothing in
 * the product path may include, link or call this file; it shares no code
 * with the HIP kernels.
 *
 * Notation (0-indexed tokens): r query row, j key column, b_q query block
 * size, i = r / b_q query block, g = i / step group, G_g = g*step*b_q the
 * group's first row, n_init the number of initial tokens, w the reach of the
 * local window before the group start, W_g = max(n_init, G_g - w) the first
 * key of the group's window, S(r,j) = sigma * <q_r, k_j>.
 *
 *   anchor set     A(r) = { j < n_init, j <= r }  u  { W_g <= j <= r }
 *   candidates     C_g  = [ n_init, W_g )
 *   selected set   I_g  = { j in C_g : exists block i in g with
 *                           xbar_i - sigma*<qbar_i, k_j> <= theta }
 *   attended set   P(r) = A(r) u I_g
 *
 * All inputs are float arrays whose values are exactly the values the GPU
 * sees (bf16 inputs are widened to float without change); every sum, max,
 * exp and mean below is carried in double.  There is no tiling, no online
 * softmax and no reuse between steps: each function is the definition
 * written out.  OpenMP only distributes independent rows / columns.
 *
 * Parity status: every function here is pinned by tests/test_oracle_pins.py
 * (dense causal attention through a library routine at theta=+inf, a band
 * mask at theta=-inf, closed forms for constant keys, a hand-worked golden
 * example, and an independent mask-based brute force; the block-granularity
 * variant by its reduction to the stripe test at b_kv = 1 and on keys that are
 * constant inside each block, by linearity of the pooled score, and by its own
 * brute force).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    int64_t N;       /* tokens in this sequence                               */
    int32_t d;       /* head dimension                                         */
    int32_t b_q;     /* query block size                                       */
    int32_t n_init;  /* initial ("sink") tokens always attended               */
    int32_t w;       /* window reach, in tokens, before the group's first row */
    int32_t step;    /* query blocks that share one selected-column list      */
    double  sigma;   /* score scale, 1/sqrt(d) in the paper (Eq. 1)           */
    double  theta;   /* difference threshold in natural-log units (Sec. 3.2)  */
} ao_cfg;

/* First key of the local window of group g (Alg. 1, window range, in tokens). */
int64_t ao_window_start(const ao_cfg *c, int64_t g)
{
    int64_t G = g * (int64_t)c->step * c->b_q;
    int64_t W = G - c->w;
    return W > c->n_init ? W : c->n_init;
}

/* S(r,j) = sigma * <q_r, k_j>  (Eq. 1 scaling). */
static double score(const ao_cfg *c, const float *qr, const float *kj)
{
    double s = 0.0;
    for (int t = 0; t < c->d; ++t) s += (double)qr[t] * (double)kj[t];
    return c->sigma * s;
}

/* 1 iff key j belongs to the anchor set A(r)  (Eq. 1; Alg. 1). */
static int in_anchor(const ao_cfg *c, int64_t r, int64_t j)
{
    if (j > r) return 0;                       /* causal prefill */
    if (j < c->n_init) return 1;               /* initial tokens */
    int64_t g = (r / c->b_q) / c->step;
    return j >= ao_window_start(c, g);         /* local window   */
}

/*
 * Anchor state of rows [r0, r1)  (Alg. 1's cached results):
 *   M[r-r0]   = max_{j in A(r)} S(r,j)                 -- the anchor, Eq. 1
 *   L[r-r0]   = sum_{j in A(r)} exp(S(r,j) - M)
 *   Acc[r-r0] = sum_{j in A(r)} exp(S(r,j) - M) * v_j  (may be NULL)
 */
void ao_anchor_rows(const ao_cfg *c, const float *q, const float *k, const float *v,
                    int64_t r0, int64_t r1, double *M, double *L, double *Acc)
{
    const int d = c->d;
#pragma omp parallel for schedule(dynamic, 8)
    for (int64_t r = r0; r < r1; ++r) {
        const float *qr = q + r * d;
        double m = -INFINITY;
        for (int64_t j = 0; j <= r; ++j)
            if (in_anchor(c, r, j)) {
                double s = score(c, qr, k + j * d);
                if (s > m) m = s;
            }
        double l = 0.0;
        double *acc = Acc ? Acc + (r - r0) * d : NULL;
        if (acc) for (int t = 0; t < d; ++t) acc[t] = 0.0;
        for (int64_t j = 0; j <= r; ++j)
            if (in_anchor(c, r, j)) {
                double p = exp(score(c, qr, k + j * d) - m);
                l += p;
                if (acc) for (int t = 0; t < d; ++t) acc[t] += p * (double)v[j * d + t];
            }
        M[r - r0] = m;
        L[r - r0] = l;
    }
}

/*
 * Block-average pooling of query block i  (Sec. 3.2; Alg. 2's two avgpool
 * lines): qbar = mean of the block's query rows, xbar = mean of the block's
 * anchors.  M_blk holds the anchors of the block's rows, first row first.
 * A ragged last block averages over the rows that exist.
 */
void ao_pool_block(const ao_cfg *c, const float *q, const double *M_blk, int64_t i,
                   double *xbar, double *qbar)
{
    int64_t r0 = i * c->b_q, r1 = r0 + c->b_q;
    if (r1 > c->N) r1 = c->N;
    double n = (double)(r1 - r0);
    double sx = 0.0;
    for (int t = 0; t < c->d; ++t) qbar[t] = 0.0;
    for (int64_t r = r0; r < r1; ++r) {
        sx += M_blk[r - r0];
        for (int t = 0; t < c->d; ++t) qbar[t] += (double)q[r * c->d + t];
    }
    *xbar = sx / n;
    for (int t = 0; t < c->d; ++t) qbar[t] /= n;
}

/*
 * Difference-aware selection for group g  (Sec. 3.2 mask; Alg. 2; the
 * step-sharing rule of Sec. 3.4).  nb = number of blocks of the group that
 * exist; xbar[nb], qbar[nb][d] are their pooled anchors / queries.
 * For every j in [0, N):
 *   margin[j] = min_i ( xbar_i - sigma*<qbar_i,k_j> ) - theta   for j in C_g,
 *               +inf elsewhere
 *   sel[j]    = 1 iff margin[j] <= 0
 * Returns |I_g|.
 */
int64_t ao_select_group(const ao_cfg *c, const float *k, int64_t g, int nb,
                        const double *xbar, const double *qbar,
                        uint8_t *sel, double *margin)
{
    const int d = c->d;
    const int64_t W = ao_window_start(c, g);
    int64_t count = 0;
#pragma omp parallel for schedule(static) reduction(+ : count)
    for (int64_t j = 0; j < c->N; ++j) {
        double mg = INFINITY;
        if (j >= c->n_init && j < W) {
            for (int b = 0; b < nb; ++b) {
                double s = 0.0;
                for (int t = 0; t < d; ++t) s += qbar[b * d + t] * (double)k[j * d + t];
                double diff = xbar[b] - c->sigma * s;
                if (diff < mg) mg = diff;
            }
            mg -= c->theta;
        }
        if (margin) margin[j] = mg;
        sel[j] = (mg <= 0.0) ? 1 : 0;
        count += sel[j];
    }
    return count;
}

/*
 * Block-granularity identification for group g: the variant that Sec. 2.1.2 and
 * Table 1 set against stripe granularity.  Granularity (b_q, b_kv) takes one
 * decision per key block, granularity (b_q, 1) (ao_select_group above) one per
 * key column.  The paper does not spell the block test out; here it is the
 * difference test of Sec. 3.2 with the key replaced by the block's average key:
 *   key block J = [J*b_kv, (J+1)*b_kv), a candidate iff it lies inside C_g
 *   kbar_J      = mean of the block's keys
 *   margin_J    = min_i ( xbar_i - sigma*<qbar_i, kbar_J> ) - theta
 *   sel[j] = 1 and margin[j] = margin_J for every j in J iff margin_J <= 0
 * n_init and W_g must be multiples of b_kv, so that C_g is a union of whole
 * key blocks; returns -1 (nothing written) otherwise.  Returns |I_g|.
 */
int64_t ao_select_group_blocks(const ao_cfg *c, const float *k, int64_t g, int nb,
                               const double *xbar, const double *qbar, int32_t b_kv,
                               uint8_t *sel, double *margin)
{
    const int d = c->d;
    const int64_t W = ao_window_start(c, g);
    if (b_kv <= 0 || c->n_init % b_kv != 0 || W % b_kv != 0) return -1;
    for (int64_t j = 0; j < c->N; ++j) {
        sel[j] = 0;
        if (margin) margin[j] = INFINITY;
    }
    int64_t count = 0;
    double *kbar = (double *)malloc((size_t)d * sizeof(double));
    for (int64_t J = c->n_init / b_kv; J < W / b_kv; ++J) {
        for (int t = 0; t < d; ++t) kbar[t] = 0.0;
        for (int64_t j = J * b_kv; j < (J + 1) * b_kv; ++j)
            for (int t = 0; t < d; ++t) kbar[t] += (double)k[j * d + t];
        for (int t = 0; t < d; ++t) kbar[t] /= (double)b_kv;
        double mg = INFINITY;
        for (int b = 0; b < nb; ++b) {
            double s = 0.0;
            for (int t = 0; t < d; ++t) s += qbar[b * d + t] * kbar[t];
            double diff = xbar[b] - c->sigma * s;
            if (diff < mg) mg = diff;
        }
        mg -= c->theta;
        for (int64_t j = J * b_kv; j < (J + 1) * b_kv; ++j) {
            if (margin) margin[j] = mg;
            sel[j] = (mg <= 0.0) ? 1 : 0;
            count += sel[j];
        }
    }
    free(kbar);
    return count;
}

/*
 * Attention of rows [r0, r1) (all inside group g) over P(r) = A(r) u I_g
 * (Sec. 3.3, Eq. 3-5; the result Alg. 3 reaches), as a plain two-pass
 * softmax:  O_r = sum_P softmax(S(r,.))_j v_j,  lse_r = log sum_P exp S(r,j).
 * sel is the group's N-byte selection map.  Returns the number of (r,j)
 * pairs attended.
 */
int64_t ao_attend_rows(const ao_cfg *c, const float *q, const float *k, const float *v,
                       int64_t r0, int64_t r1, const uint8_t *sel,
                       double *O, double *lse)
{
    const int d = c->d;
    int64_t pairs = 0;
#pragma omp parallel for schedule(dynamic, 4) reduction(+ : pairs)
    for (int64_t r = r0; r < r1; ++r) {
        const float *qr = q + r * d;
        double *s = (double *)malloc((size_t)(r + 1) * sizeof(double));
        double m = -INFINITY;
        for (int64_t j = 0; j <= r; ++j) {
            if (in_anchor(c, r, j) || sel[j]) {
                s[j] = score(c, qr, k + j * d);
                if (s[j] > m) m = s[j];
                pairs += 1;
            } else {
                s[j] = -INFINITY;
            }
        }
        double l = 0.0;
        double *o = O + (r - r0) * d;
        for (int t = 0; t < d; ++t) o[t] = 0.0;
        for (int64_t j = 0; j <= r; ++j)
            if (s[j] != -INFINITY) {
                double p = exp(s[j] - m);
                l += p;
                for (int t = 0; t < d; ++t) o[t] += p * (double)v[j * d + t];
            }
        for (int t = 0; t < d; ++t) o[t] /= l;
        lse[r - r0] = m + log(l);
        free(s);
    }
    return pairs;
}
