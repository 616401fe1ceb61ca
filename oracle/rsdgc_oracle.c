/*
 * RS-DGC local gradient compressor -- CPU ORACLE.
 *
 * THIS FILE IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step
 * implementation of what the paper's per-iteration sparsifier computes, used
 * only by the tests, by the smoke check and by the benchmark's CPU-baseline
 * leg.  The GPU library shares no code with it and never calls it.
 *
 * Every step follows the paper's own definition, in the paper's order:
 *
 *   step 1  v = r + g                      Eq. 12, second line (with u = g)
 *   step 2  NSI at every centre            Eqs. 6-10 (Section III-C)
 *   step 3  k = ceil(G / (p*p) * rho_l)    Eq. 11
 *   step 4  rank the NSI values, take k    Algorithm 1 ("conduct a ranking")
 *   step 5  keep whole neighbourhoods      Section III-C, sentence after Eq. 11
 *   step 6  emit (index, value) pairs      same sentence ("transmit ... index")
 *   step 7  residual = what was not sent   Eq. 12 (v accumulates the unsent part)
 *   step 8  decompress (scatter)           Eq. 12, third line (sum of sparse(v))
 *
 * With momentum correction (Eq. 12 in full) step 1 becomes
 *   step 1m u = m*u + g,  v = r + u        Eq. 12, first and second line
 * and step 7 also restarts u from zero where v was sent (the masking of the
 * method Eq. 12 is taken from).
 *
 * The receiving side of one iteration (Eq. 12, third line):
 *   step 9  S = sum over the nodes' messages of sparse(v_k), accumulated in
 *           message order with binary32 adds; w = w - eta * S (one binary32
 *           multiply, one binary32 subtract).
 *
 * The other reading of Section III-C ("a convolution kernel as a whole", Eq. 11's
 * G / p^2): the matrix is cut into ceil(R/p) x ceil(C/p) non-overlapping p x p
 * blocks, each block is one neighbourhood:
 *   step B2  NSI of every block (Eqs. 8-10 over the block's p*p slots, zero
 *            outside the matrix, divisor p*p)
 *   step B3  k = min(ceil(G / (p*p) * rho_l), number of blocks)      Eq. 11
 *   step B4  rank the blocks, take k (ties: lower block index)
 *   step B6  emit per kept block its index and its p*p values (row-major,
 *            zero for slots outside the matrix), blocks in ascending order
 *   step B7  residual = v outside the kept blocks, +0 inside
 *
 * Once per epoch (Section III-B, Algorithm 1's outer loop) the per-layer keep
 * ratios come from the weights:
 *   step D  mu = |w| (Eq. 3); rank all weights of the network together; the
 *           K = ceil(rho * G) top-ranked survive (Eq. 4); rho_l = survivors of
 *           layer l / G_l (Eq. 5).  Equal |w| rank by layer, then by index.
 *
 * Readings taken where the paper is silent (each is also a parameter or a
 * documented convention of the GPU library):
 *   - every element is the centre of one neighbourhood (stride-1 window);
 *   - p is odd, half width h = (p-1)/2, window |dx| <= h, |dy| <= h (Eq. 7);
 *   - a window slot outside the matrix holds the value 0 and the divisor is
 *     always p*p (Eqs. 9-10 sum p^2 terms with 1/p^2 in front);
 *   - mean uses |g|, std uses the signed values with the signed mean and the
 *     1/p^2 (population) normalisation, exactly as printed in Eqs. 9-10;
 *   - statistics are evaluated in IEEE double from the float32 values and the
 *     score is rounded once to float32; the ranking key is that float32;
 *   - ties in the ranking go to the lower flat index (stable descending sort);
 *   - kept positions get residual +0.0f.
 *
 * Floating point: no fast-math, no contraction (compile with
 * -ffp-contract=off); float adds are single IEEE binary32 operations.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ---------------------------------------------------------------- step 1 */
/* Eq. 12, line 2 with u = g (no momentum): one binary32 add per element.   */
void rsdgc_oracle_accumulate(const float *r, const float *g, float *v, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float s = r[i] + g[i];
        v[i] = s;
    }
}

/* --------------------------------------------------------------- step 1m */
/* Eq. 12, lines 1 and 2: u_new = m*u + g (one binary32 multiply, one
 * binary32 add), v = r + u_new (one binary32 add).                         */
void rsdgc_oracle_momentum(const float *u, const float *g, const float *r, float m,
                           float *u_new, float *v, int64_t n)
{
    for (int64_t i = 0; i < n; ++i) {
        volatile float mu = m * u[i];
        volatile float un = mu + g[i];
        volatile float s = r[i] + un;
        u_new[i] = un;
        v[i] = s;
    }
}

/* ---------------------------------------------------------------- step 2 */
/* Value of window slot (x, y); slots outside the R x C matrix are zero.    */
static double slot(const float *v, int64_t R, int64_t C, int64_t x, int64_t y)
{
    if (x < 0 || x >= R || y < 0 || y >= C)
        return 0.0;
    return (double)v[x * C + y];
}

/* Eqs. 8-10 at one centre (x0, y0), in double. x = row, y = column.        */
double rsdgc_oracle_nsi_at(const float *v, int64_t R, int64_t C, int p,
                           double alpha, int64_t x0, int64_t y0)
{
    const int h = (p - 1) / 2;
    const double n = (double)p * (double)p;

    double sum_abs = 0.0, sum = 0.0;
    for (int dx = -h; dx <= h; ++dx)
        for (int dy = -h; dy <= h; ++dy) {
            double w = slot(v, R, C, x0 + dx, y0 + dy);
            sum_abs += fabs(w);
            sum += w;
        }
    const double mean_abs = sum_abs / n;   /* Eq. 9  */
    const double mean = sum / n;           /* inner mean of Eq. 10 */

    double sq = 0.0;
    for (int dx = -h; dx <= h; ++dx)
        for (int dy = -h; dy <= h; ++dy) {
            double d = slot(v, R, C, x0 + dx, y0 + dy) - mean;
            sq += d * d;
        }
    const double std = sqrt(sq / n);       /* Eq. 10 */

    return alpha * mean_abs + (1.0 - alpha) * std;   /* Eq. 8 */
}

/* NSI map of one layer: one score per element, rounded once to float32.    */
void rsdgc_oracle_nsi(const float *v, int64_t R, int64_t C, int p, double alpha,
                      float *nsi)
{
    for (int64_t x = 0; x < R; ++x)
        for (int64_t y = 0; y < C; ++y)
            nsi[x * C + y] = (float)rsdgc_oracle_nsi_at(v, R, C, p, alpha, x, y);
}

/* ---------------------------------------------------------------- step 3 */
/* Eq. 11: k = ceil( (G / p^2) * rho ), evaluated in double in that order,
 * clamped to [0, G].                                                       */
int64_t rsdgc_oracle_k(int64_t G, int p, double rho)
{
    double q = (double)G / (double)((int64_t)p * (int64_t)p);
    double kf = ceil(q * rho);
    if (!(kf > 0.0))
        return 0;
    if (kf > (double)G)
        return G;
    return (int64_t)kf;
}

/* ---------------------------------------------------------------- step 4 */
typedef struct {
    float score;
    uint32_t index;
} ranked_t;

/* Descending score, ascending index among equal scores. */
static int rank_cmp(const void *a, const void *b)
{
    const ranked_t *p = (const ranked_t *)a, *q = (const ranked_t *)b;
    if (p->score > q->score) return -1;
    if (p->score < q->score) return 1;
    if (p->index < q->index) return -1;
    if (p->index > q->index) return 1;
    return 0;
}

static int u32_cmp(const void *a, const void *b)
{
    uint32_t p = *(const uint32_t *)a, q = *(const uint32_t *)b;
    return (p > q) - (p < q);
}

/* Full ranking of all G centres; the first k are selected.
 * centres[k] receives their flat indices in ASCENDING index order;
 * *tau receives the k-th largest score (untouched if k == 0).
 * Returns 0, or -1 if memory ran out.                                      */
int rsdgc_oracle_select(const float *nsi, int64_t G, int64_t k,
                        uint32_t *centres, float *tau)
{
    if (k <= 0)
        return 0;
    ranked_t *all = (ranked_t *)malloc((size_t)G * sizeof(ranked_t));
    if (!all)
        return -1;
    for (int64_t i = 0; i < G; ++i) {
        all[i].score = nsi[i];
        all[i].index = (uint32_t)i;
    }
    qsort(all, (size_t)G, sizeof(ranked_t), rank_cmp);
    for (int64_t j = 0; j < k; ++j)
        centres[j] = all[j].index;
    *tau = all[k - 1].score;
    free(all);
    qsort(centres, (size_t)k, sizeof(uint32_t), u32_cmp);
    return 0;
}

/* ---------------------------------------------------------------- step 5 */
/* mask[i] = 1 iff element i lies in the p x p window (Eq. 7) of a selected
 * centre.                                                                   */
void rsdgc_oracle_dilate(const uint32_t *centres, int64_t k, int64_t R, int64_t C,
                         int p, uint8_t *mask)
{
    const int h = (p - 1) / 2;
    memset(mask, 0, (size_t)(R * C));
    for (int64_t j = 0; j < k; ++j) {
        int64_t x0 = (int64_t)centres[j] / C, y0 = (int64_t)centres[j] % C;
        for (int dx = -h; dx <= h; ++dx)
            for (int dy = -h; dy <= h; ++dy) {
                int64_t x = x0 + dx, y = y0 + dy;
                if (x < 0 || x >= R || y < 0 || y >= C)
                    continue;
                mask[x * C + y] = 1;
            }
    }
}

/* ---------------------------------------------------------------- step 6 */
/* Kept (index, value) pairs in ascending flat index; returns their number. */
int64_t rsdgc_oracle_emit(const float *v, const uint8_t *mask, int64_t G,
                          uint32_t *idx, float *val)
{
    int64_t n = 0;
    for (int64_t i = 0; i < G; ++i)
        if (mask[i]) {
            idx[n] = (uint32_t)i;
            val[n] = v[i];
            ++n;
        }
    return n;
}

/* ---------------------------------------------------------------- step 7 */
/* What was sent leaves the accumulator; what was not sent stays.           */
void rsdgc_oracle_residual(const float *v, const uint8_t *mask, int64_t G,
                           float *r_new)
{
    for (int64_t i = 0; i < G; ++i)
        r_new[i] = mask[i] ? 0.0f : v[i];
}

/* Momentum masking: where v was sent the momentum restarts from +0.         */
void rsdgc_oracle_mask_momentum(const float *u_new, const uint8_t *mask, int64_t G,
                                float *u_out)
{
    for (int64_t i = 0; i < G; ++i)
        u_out[i] = mask[i] ? 0.0f : u_new[i];
}

/* ---------------------------------------------------------------- step 8 */
/* accumulate == 0: dense = 0 then dense[idx] = val;
 * accumulate != 0: dense[idx] += val (one binary32 add).                   */
void rsdgc_oracle_decompress(const uint32_t *idx, const float *val, int64_t n,
                             float *dense, int64_t G, int accumulate)
{
    if (!accumulate)
        for (int64_t i = 0; i < G; ++i)
            dense[i] = 0.0f;
    for (int64_t j = 0; j < n; ++j) {
        if (accumulate) {
            volatile float s = dense[idx[j]] + val[j];
            dense[idx[j]] = s;
        } else {
            dense[idx[j]] = val[j];
        }
    }
}

/* ------------------------------------------------------- one whole layer */
/* Steps 1-7 for one layer, in order.  r is updated in place.
 * Outputs (caller-allocated): idx/val capacity min(k*p*p, G); centres
 * capacity k; nsi_out (nullable) G floats; v_out (nullable) G floats.
 * Returns the number of emitted pairs, or -1 on allocation failure.        */
int64_t rsdgc_oracle_compress_layer(const float *g, float *r, int64_t R, int64_t C,
                                    int p, double alpha, double rho,
                                    uint32_t *idx, float *val, uint32_t *centres,
                                    int64_t *k_out, float *tau_out,
                                    float *nsi_out, float *v_out)
{
    const int64_t G = R * C;
    float *v = (float *)malloc((size_t)G * sizeof(float));
    float *nsi = (float *)malloc((size_t)G * sizeof(float));
    uint8_t *mask = (uint8_t *)malloc((size_t)G);
    if (!v || !nsi || !mask) {
        free(v); free(nsi); free(mask);
        return -1;
    }
    rsdgc_oracle_accumulate(r, g, v, G);                      /* step 1 */
    rsdgc_oracle_nsi(v, R, C, p, alpha, nsi);                 /* step 2 */
    const int64_t k = rsdgc_oracle_k(G, p, rho);              /* step 3 */
    float tau = 0.0f;
    if (rsdgc_oracle_select(nsi, G, k, centres, &tau) != 0) { /* step 4 */
        free(v); free(nsi); free(mask);
        return -1;
    }
    rsdgc_oracle_dilate(centres, k, R, C, p, mask);           /* step 5 */
    const int64_t n = rsdgc_oracle_emit(v, mask, G, idx, val);/* step 6 */
    rsdgc_oracle_residual(v, mask, G, r);                     /* step 7 */
    if (k_out) *k_out = k;
    if (tau_out) *tau_out = tau;
    if (nsi_out) memcpy(nsi_out, nsi, (size_t)G * sizeof(float));
    if (v_out) memcpy(v_out, v, (size_t)G * sizeof(float));
    free(v); free(nsi); free(mask);
    return n;
}

/* The same with momentum correction: steps 1m, 2-7; u and r are updated in
 * place (u: m*u + g, then +0 where sent; r: as above).                      */
int64_t rsdgc_oracle_compress_layer_momentum(const float *g, float *u, float *r, float m,
                                             int64_t R, int64_t C, int p, double alpha,
                                             double rho, uint32_t *idx, float *val,
                                             uint32_t *centres, int64_t *k_out,
                                             float *tau_out, float *nsi_out, float *v_out)
{
    const int64_t G = R * C;
    float *v = (float *)malloc((size_t)G * sizeof(float));
    float *un = (float *)malloc((size_t)G * sizeof(float));
    float *nsi = (float *)malloc((size_t)G * sizeof(float));
    uint8_t *mask = (uint8_t *)malloc((size_t)G);
    if (!v || !un || !nsi || !mask) {
        free(v); free(un); free(nsi); free(mask);
        return -1;
    }
    rsdgc_oracle_momentum(u, g, r, m, un, v, G);              /* step 1m */
    rsdgc_oracle_nsi(v, R, C, p, alpha, nsi);                 /* step 2 */
    const int64_t k = rsdgc_oracle_k(G, p, rho);              /* step 3 */
    float tau = 0.0f;
    if (rsdgc_oracle_select(nsi, G, k, centres, &tau) != 0) { /* step 4 */
        free(v); free(un); free(nsi); free(mask);
        return -1;
    }
    rsdgc_oracle_dilate(centres, k, R, C, p, mask);           /* step 5 */
    const int64_t n = rsdgc_oracle_emit(v, mask, G, idx, val);/* step 6 */
    rsdgc_oracle_residual(v, mask, G, r);                     /* step 7 */
    rsdgc_oracle_mask_momentum(un, mask, G, u);               /* step 7, momentum */
    if (k_out) *k_out = k;
    if (tau_out) *tau_out = tau;
    if (nsi_out) memcpy(nsi_out, nsi, (size_t)G * sizeof(float));
    if (v_out) memcpy(v_out, v, (size_t)G * sizeof(float));
    free(v); free(un); free(nsi); free(mask);
    return n;
}

/* ---------------------------------------------------------------- step D */
/* Eqs. 3-5: per-layer keep ratios from a cross-layer ranking of |w|.
 * w_all holds the layers back to back; layer l is w_all[off[l] .. off[l+1]).
 * rho is the global keep fraction.  Returns 0, or -1 on allocation failure. */
typedef struct {
    float mu;
    int32_t layer;
    int64_t index;
} weight_item;

static int weight_cmp(const void *a, const void *b)
{
    const weight_item *p = (const weight_item *)a, *q = (const weight_item *)b;
    if (p->mu > q->mu) return -1;
    if (p->mu < q->mu) return 1;
    if (p->layer < q->layer) return -1;
    if (p->layer > q->layer) return 1;
    if (p->index < q->index) return -1;
    if (p->index > q->index) return 1;
    return 0;
}

int rsdgc_oracle_dynamic_ratios(const float *w_all, const int64_t *off, int32_t L, double rho,
                                double *ratio_out)
{
    const int64_t N = off[L];
    weight_item *it = (weight_item *)malloc((size_t)(N > 0 ? N : 1) * sizeof(weight_item));
    int64_t *kept = (int64_t *)calloc((size_t)L, sizeof(int64_t));
    if (!it || !kept) {
        free(it); free(kept);
        return -1;
    }
    for (int32_t l = 0; l < L; ++l)
        for (int64_t i = off[l]; i < off[l + 1]; ++i) {
            it[i].mu = fabsf(w_all[i]);                       /* Eq. 3 */
            it[i].layer = l;
            it[i].index = i - off[l];
        }
    qsort(it, (size_t)N, sizeof(weight_item), weight_cmp);    /* cross-layer ranking */
    double kf = ceil(rho * (double)N);                        /* survivors (Eq. 4) */
    if (kf < 0.0) kf = 0.0;
    if (kf > (double)N) kf = (double)N;
    const int64_t K = (int64_t)kf;
    for (int64_t j = 0; j < K; ++j)
        ++kept[it[j].layer];
    for (int32_t l = 0; l < L; ++l) {                         /* Eq. 5 */
        const int64_t Gl = off[l + 1] - off[l];
        ratio_out[l] = Gl > 0 ? (double)kept[l] / (double)Gl : 0.0;
    }
    free(it); free(kept);
    return 0;
}

/* ---------------------------------------------------------------- step 9 */
/* Eq. 12, third line, for one layer: the messages of n_msgs nodes are summed
 * into a dense sum (message 0 first), then w <- w - eta * sum.              */
int rsdgc_oracle_apply(float *w, int64_t G, int32_t n_msgs, const uint32_t *const *idx,
                       const float *const *val, const int64_t *n, float eta)
{
    float *sum = (float *)malloc((size_t)(G > 0 ? G : 1) * sizeof(float));
    if (!sum)
        return -1;
    for (int64_t i = 0; i < G; ++i)
        sum[i] = 0.0f;
    for (int32_t k = 0; k < n_msgs; ++k)
        rsdgc_oracle_decompress(idx[k], val[k], n[k], sum, G, 1);
    for (int64_t i = 0; i < G; ++i) {
        volatile float step = eta * sum[i];
        volatile float wn = w[i] - step;
        w[i] = wn;
    }
    free(sum);
    return 0;
}

/* ------------------------------------------------------- block reading -- */
/* Eqs. 8-10 over block (bx, by): rows bx*p .. bx*p+p-1, columns by*p .. by*p+p-1. */
double rsdgc_oracle_block_nsi_at(const float *v, int64_t R, int64_t C, int p, double alpha,
                                 int64_t bx, int64_t by)
{
    const double n = (double)p * (double)p;
    double sum_abs = 0.0, sum = 0.0;
    for (int dx = 0; dx < p; ++dx)
        for (int dy = 0; dy < p; ++dy) {
            double w = slot(v, R, C, bx * p + dx, by * p + dy);
            sum_abs += fabs(w);
            sum += w;
        }
    const double mean_abs = sum_abs / n;   /* Eq. 9  */
    const double mean = sum / n;
    double sq = 0.0;
    for (int dx = 0; dx < p; ++dx)
        for (int dy = 0; dy < p; ++dy) {
            double d = slot(v, R, C, bx * p + dx, by * p + dy) - mean;
            sq += d * d;
        }
    const double std = sqrt(sq / n);       /* Eq. 10 */
    return alpha * mean_abs + (1.0 - alpha) * std;   /* Eq. 8 */
}

/* Block NSI map: ceil(R/p) x ceil(C/p) scores, each rounded once to float32. */
void rsdgc_oracle_block_nsi(const float *v, int64_t R, int64_t C, int p, double alpha, float *nsi)
{
    const int64_t BR = (R + p - 1) / p, BC = (C + p - 1) / p;
    for (int64_t bx = 0; bx < BR; ++bx)
        for (int64_t by = 0; by < BC; ++by)
            nsi[bx * BC + by] = (float)rsdgc_oracle_block_nsi_at(v, R, C, p, alpha, bx, by);
}

/* Steps 1, B2-B7 for one layer.  r is updated in place.  blocks: capacity k block
 * indices; val: capacity k*p*p values (p*p per kept block, in block order).
 * Returns the number of kept blocks, or -1 on allocation failure.           */
int64_t rsdgc_oracle_compress_layer_blocks(const float *g, float *r, int64_t R, int64_t C, int p,
                                           double alpha, double rho, uint32_t *blocks, float *val,
                                           float *tau_out, float *nsi_out, float *v_out)
{
    const int64_t G = R * C;
    const int64_t BR = (R + p - 1) / p, BC = (C + p - 1) / p, NB = BR * BC;
    float *v = (float *)malloc((size_t)G * sizeof(float));
    float *nsi = (float *)malloc((size_t)NB * sizeof(float));
    if (!v || !nsi) {
        free(v); free(nsi);
        return -1;
    }
    rsdgc_oracle_accumulate(r, g, v, G);                       /* step 1 */
    rsdgc_oracle_block_nsi(v, R, C, p, alpha, nsi);            /* step B2 */
    int64_t k = rsdgc_oracle_k(G, p, rho);                     /* step B3 */
    if (k > NB) k = NB;
    float tau = 0.0f;
    if (rsdgc_oracle_select(nsi, NB, k, blocks, &tau) != 0) {  /* step B4 */
        free(v); free(nsi);
        return -1;
    }
    for (int64_t i = 0; i < G; ++i)                            /* step B7, first half */
        r[i] = v[i];
    for (int64_t j = 0; j < k; ++j) {                          /* steps B6, B7 */
        const int64_t bx = blocks[j] / BC, by = blocks[j] % BC;
        for (int dx = 0; dx < p; ++dx)
            for (int dy = 0; dy < p; ++dy) {
                const int64_t x = bx * p + dx, y = by * p + dy;
                const int inside = x < R && y < C;
                val[j * p * p + dx * p + dy] = inside ? v[x * C + y] : 0.0f;
                if (inside) r[x * C + y] = 0.0f;
            }
    }
    if (tau_out) *tau_out = tau;
    if (nsi_out) memcpy(nsi_out, nsi, (size_t)NB * sizeof(float));
    if (v_out) memcpy(v_out, v, (size_t)G * sizeof(float));
    free(v); free(nsi);
    return k;
}

/* The block reading with momentum correction: Eq. 12's first two lines (step 1m), then steps
 * B2-B7 on v = r + u_new; u and r are updated in place and both restart from +0 on every slot
 * of a kept block (what Eq. 12's line 1 accumulates for a sent position must not be sent again).
 * Arguments and return value as above.                                                         */
int64_t rsdgc_oracle_compress_layer_blocks_momentum(const float *g, float *u, float *r, float m,
                                                    int64_t R, int64_t C, int p, double alpha,
                                                    double rho, uint32_t *blocks, float *val,
                                                    float *tau_out, float *nsi_out, float *v_out)
{
    const int64_t G = R * C;
    const int64_t BR = (R + p - 1) / p, BC = (C + p - 1) / p, NB = BR * BC;
    float *v = (float *)malloc((size_t)G * sizeof(float));
    float *un = (float *)malloc((size_t)G * sizeof(float));
    float *nsi = (float *)malloc((size_t)NB * sizeof(float));
    if (!v || !un || !nsi) {
        free(v); free(un); free(nsi);
        return -1;
    }
    rsdgc_oracle_momentum(u, g, r, m, un, v, G);               /* step 1m */
    rsdgc_oracle_block_nsi(v, R, C, p, alpha, nsi);            /* step B2 */
    int64_t k = rsdgc_oracle_k(G, p, rho);                     /* step B3 */
    if (k > NB) k = NB;
    float tau = 0.0f;
    if (rsdgc_oracle_select(nsi, NB, k, blocks, &tau) != 0) {  /* step B4 */
        free(v); free(un); free(nsi);
        return -1;
    }
    for (int64_t i = 0; i < G; ++i) {                          /* step B7, first half */
        r[i] = v[i];
        u[i] = un[i];
    }
    for (int64_t j = 0; j < k; ++j) {                          /* steps B6, B7 */
        const int64_t kx = blocks[j] / BC, ky = blocks[j] % BC;
        for (int dx = 0; dx < p; ++dx)
            for (int dy = 0; dy < p; ++dy) {
                const int64_t x = kx * p + dx, y = ky * p + dy;
                const int within = x < R && y < C;
                val[j * p * p + dx * p + dy] = within ? v[x * C + y] : 0.0f;
                if (within) {
                    r[x * C + y] = 0.0f;
                    u[x * C + y] = 0.0f;
                }
            }
    }
    if (tau_out) *tau_out = tau;
    if (nsi_out) memcpy(nsi_out, nsi, (size_t)NB * sizeof(float));
    if (v_out) memcpy(v_out, v, (size_t)G * sizeof(float));
    free(v); free(un); free(nsi);
    return k;
}

/* Inverse of step B6: dense = 0 (accumulate == 0) or kept; dense[block slot] = or += value. */
void rsdgc_oracle_decompress_blocks(const uint32_t *blocks, const float *val, int64_t k,
                                    int64_t R, int64_t C, int p, float *dense, int accumulate)
{
    const int64_t BC = (C + p - 1) / p;
    if (!accumulate)
        for (int64_t i = 0; i < R * C; ++i)
            dense[i] = 0.0f;
    for (int64_t j = 0; j < k; ++j) {
        const int64_t bx = blocks[j] / BC, by = blocks[j] % BC;
        for (int dx = 0; dx < p; ++dx)
            for (int dy = 0; dy < p; ++dy) {
                const int64_t x = bx * p + dx, y = by * p + dy;
                if (x >= R || y >= C) continue;
                if (accumulate) {
                    volatile float s = dense[x * C + y] + val[j * p * p + dx * p + dy];
                    dense[x * C + y] = s;
                } else {
                    dense[x * C + y] = val[j * p * p + dx * p + dy];
                }
            }
    }
}

/* Eq. 12, third line, with block messages (the block reading of Section III-C): the messages
 * are summed in the order given (float32 adds, each block slot inside the matrix once per
 * message), then w <- w - eta * sum with one float32 multiply and one float32 subtract.     */
int rsdgc_oracle_apply_blocks(float *w, int64_t R, int64_t C, int p, int32_t n_msgs,
                              const uint32_t *const *blocks, const float *const *val,
                              const int64_t *n, float eta)
{
    const int64_t G = R * C;
    float *sum = (float *)malloc((size_t)(G > 0 ? G : 1) * sizeof(float));
    if (!sum)
        return -1;
    for (int64_t i = 0; i < G; ++i)
        sum[i] = 0.0f;
    for (int32_t k = 0; k < n_msgs; ++k)
        rsdgc_oracle_decompress_blocks(blocks[k], val[k], n[k], R, C, p, sum, 1);
    for (int64_t i = 0; i < G; ++i) {
        volatile float step = eta * sum[i];
        volatile float wn = w[i] - step;
        w[i] = wn;
    }
    free(sum);
    return 0;
}
