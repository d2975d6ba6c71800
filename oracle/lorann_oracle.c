/*
 * CPU oracle for the query phase of LoRANN (clustering-based ANN search with reduced-rank-regression
 * score computation and 8-bit quantization).
 *
 * THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, step-by-step statement of what the search computes,
 * used only by the tests, the smoke check and the benchmark's CPU-baseline leg.  It shares no code with the
 * HIP library and must never serve as a fallback for it.
 *
 * The search is an approximation whose result depends on every rounding step, so the oracle follows the
 * algorithm in the paper's order (Sec. 2.2 template; Sec. 3.2 scores; Sec. 3.3 quantization; Sec. 4.1
 * dimensionality reduction).  Floating-point contractions accumulate in double and round once to float;
 * the integer stages are exact.  Notation: q query, q' = P^T q its d'-dimensional projection, mu_l
 * centroids, A_c [d' x r] and B_c [r x m_c] the int8 factors of cluster c with step sizes DeltaA_c and
 * DeltaB_c (real value ~= Delta * code), w clusters probed, m candidates kept (the paper's t), k returned.
 *
 * Readings of points the paper leaves open (all stated again in the tests):
 *   - rounding of the query quantization: round-half-to-even (rintf), codes clamped to [-127, 127];
 *   - the intermediate vector x'^T A is re-quantized per (query, cluster) pair; with one scalar DeltaA per
 *     cluster the de-quantize / re-quantize pair of Sec. 3.3 cancels to an integer expression:
 *     z_j = round_half_away(127 R_j / max|R|);
 *   - a zero vector (max = 0) gets all-zero codes and scale 0;
 *   - ties in each of the three selections go to the lower index;
 *   - returned dissimilarities: squared Euclidean, negative inner product, 1 - <q, c> / |q| (cosine
 *     corpora are unit-norm by construction, Sec. 3.1).
 */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

enum { ORACLE_IP = 0, ORACLE_L2 = 1, ORACLE_COS = 2 };

typedef struct {
    int32_t metric;
    int64_t n;
    int32_t d, dp, r, L;
    const float *centroids;        /* [L][dp] */
    const float *P;                /* [d][dp] or NULL (identity, dp == d) */
    const int8_t *A;               /* [L][r][dp] */
    const int8_t *B;               /* [n][r] */
    const float *scale_A;          /* [L] */
    const float *scale_B;          /* [L] */
    const int64_t *offsets;        /* [L+1] */
    const float *corpus;           /* [n][d] rows in cluster order */
    const int64_t *ids;            /* [n] or NULL */
    const float *sqnorms;          /* [n] squared row norms from oracle_corpus_sqnorms (Euclidean), or NULL */
    /* Sec. 3.3 as printed: absmax quantization of EACH COLUMN of A_c and B_c.  Both NULL: one step size per
     * cluster (scale_A, scale_B above).  Both set: scale_A / scale_B are ignored. */
    const float *col_scale_A;      /* [L][r]  step size of column j of A_c */
    const float *pt_scale_B;       /* [n]     step size of the column of B_c that belongs to a corpus row */
    /* Sec. 4.2 mixed-precision decomposition: the first component of the projected query and the first row of
     * every A_c and B_c are not quantized.  Both NULL: everything is quantized.  Both set (needs the column-wise
     * step sizes above): the codes' first components (A[c][j][0], B[t][0]) are not read. */
    const float *first_row_A;      /* [L][r]  A_c[0][j] in float */
    const float *first_row_B;      /* [n]     B_c[0][t] in float, for the column that belongs to a corpus row */
} oracle_index;

/* Optional per-stage outputs of oracle_search; any pointer may be NULL. */
typedef struct {
    float *qproj;        /* [nq][dp]      projected queries                     */
    int8_t *q8;          /* [nq][dp]      quantized projected queries           */
    float *dx;           /* [nq]          query step size                       */
    int32_t *sel;        /* [nq][w]       selected clusters, best first         */
    float *sel_g;        /* [nq][w]       their centroid dissimilarities        */
    int32_t *R;          /* [nq][w][r]    int32 accumulators of q'_i8^T A_c     */
    int8_t *z;           /* [nq][w][r]    re-quantized intermediate vectors     */
    float *sigma;        /* [nq][w]       combined scale of each pair           */
    int64_t *cand_rows;  /* [nq][m]       candidate rows (score desc, row asc), -1 padded */
    float *cand_scores;  /* [nq][m]       their estimated scores (0 where padded) */
    float *rho0;         /* [nq][w]       mixed precision: unquantized first component of each pair's r */
    float *pair_best;    /* [nq][w]       highest estimated score among the points of each pair's cluster */
                         /*               (-inf for an empty cluster)                                     */
} oracle_dump;

/* ---- Step 1 (Sec. 4.1): q' = P^T q, double accumulation over i ascending, one rounding to float. ---- */
void oracle_project(const float *q, int32_t d, int32_t dp, const float *P, float *qp)
{
    if (!P) { memcpy(qp, q, sizeof(float) * (size_t)dp); return; }
    for (int32_t j = 0; j < dp; ++j) {
        double acc = 0.0;
        for (int32_t i = 0; i < d; ++i) acc += (double)q[i] * (double)P[(size_t)i * dp + j];
        qp[j] = (float)acc;
    }
}

/* ---- Step 2 (Sec. 2.2 routing, Sec. 3.1 reduction to inner products, Sec. 4.1 routing in d' dims). ---- */
/* Dissimilarity of q' to every centroid: inner product / cosine -> -<q', mu>; Euclidean -> |mu|^2 - 2<q', mu>
 * (the |q'|^2 term is common to all centroids). */
void oracle_centroid_dissim(const float *qp, int32_t dp, const float *centroids, int32_t L, int32_t metric, float *g)
{
    for (int32_t l = 0; l < L; ++l) {
        const float *mu = centroids + (size_t)l * dp;
        double dot = 0.0, nrm = 0.0;
        for (int32_t i = 0; i < dp; ++i) { dot += (double)qp[i] * (double)mu[i]; nrm += (double)mu[i] * (double)mu[i]; }
        g[l] = (metric == ORACLE_L2) ? (float)(nrm - 2.0 * dot) : (float)(-dot);
    }
}

typedef struct { float key; int64_t idx; } keyidx;
static int cmp_key_asc(const void *a, const void *b)
{
    const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
    if (x->key < y->key) return -1;
    if (x->key > y->key) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}
static int cmp_key_desc(const void *a, const void *b)
{
    const keyidx *x = (const keyidx *)a, *y = (const keyidx *)b;
    if (x->key > y->key) return -1;
    if (x->key < y->key) return 1;
    return (x->idx > y->idx) - (x->idx < y->idx);
}

/* The w smallest dissimilarities, ordered (g ascending, cluster id ascending). */
void oracle_select_clusters(const float *g, int32_t L, int32_t w, int32_t *sel, float *sel_g)
{
    keyidx *t = (keyidx *)malloc(sizeof(keyidx) * (size_t)L);
    for (int32_t l = 0; l < L; ++l) { t[l].key = g[l]; t[l].idx = l; }
    qsort(t, (size_t)L, sizeof(keyidx), cmp_key_asc);
    for (int32_t j = 0; j < w; ++j) { sel[j] = (int32_t)t[j].idx; if (sel_g) sel_g[j] = t[j].key; }
    free(t);
}

/* ---- Step 3 (Sec. 3.3 absmax quantization of the query): codes = rint(c_x q'), c_x = 127 / |q'|_inf. ---- */
void oracle_quantize_query(const float *qp, int32_t dp, int8_t *q8, float *dx)
{
    float a = 0.0f;
    for (int32_t i = 0; i < dp; ++i) { float v = fabsf(qp[i]); if (v > a) a = v; }
    if (!(a > 0.0f)) { memset(q8, 0, (size_t)dp); *dx = 0.0f; return; }
    float cx = 127.0f / a;
    for (int32_t i = 0; i < dp; ++i) {
        float s = qp[i] * cx;
        int v = (int)rintf(s);
        if (v > 127) v = 127;
        if (v < -127) v = -127;
        q8[i] = (int8_t)v;
    }
    *dx = a / 127.0f;
}

/* ---- Step 4 (Sec. 3.3, first 8-bit product and re-quantization) for one (query, cluster) pair. ---- */
/* R_j = sum_i q8[i] A_c[i][j] exactly; M = max|R_j|; z_j = sign(R_j) floor((254|R_j| + M) / (2M));
 * sigma = M/127 * Delta_x * DeltaA_c * DeltaB_c evaluated left to right in double, rounded once. */
void oracle_stage_a(const int8_t *q8, int32_t dp, int32_t r, const int8_t *A_c /* [r][dp] */, float dx,
                    float dA, float dB, int32_t *R, int8_t *z, float *sigma)
{
    int64_t M = 0;
    for (int32_t j = 0; j < r; ++j) {
        int32_t acc = 0;
        const int8_t *col = A_c + (size_t)j * dp;
        for (int32_t i = 0; i < dp; ++i) acc += (int32_t)q8[i] * (int32_t)col[i];
        R[j] = acc;
        int64_t a = acc < 0 ? -(int64_t)acc : (int64_t)acc;
        if (a > M) M = a;
    }
    if (M == 0) { memset(z, 0, (size_t)r); *sigma = 0.0f; return; }
    for (int32_t j = 0; j < r; ++j) {
        int64_t a = R[j] < 0 ? -(int64_t)R[j] : (int64_t)R[j];
        int64_t v = (254 * a + M) / (2 * M);
        z[j] = (int8_t)(R[j] < 0 ? -v : v);
    }
    *sigma = (float)((double)M / 127.0 * (double)dx * (double)dA * (double)dB);
}

/* Step 4 with one step size per column of A_c (Sec. 3.3 as printed): the float approximation of r = x^T A is
 * rho_j = R_j * (Delta_x * DeltaA_cj) - the paper's s (.) r_i32 with s_j = 1 / (c_x c_Aj) - and it is re-quantized
 * like any vector: z = rint(rho * 127 / |rho|_inf), step size sigma = |rho|_inf / 127.  Every operation is one
 * IEEE float operation in the order written. */
void oracle_stage_a_columns(const int8_t *q8, int32_t dp, int32_t r, const int8_t *A_c /* [r][dp] */, float dx,
                            const float *dA /* [r] */, int32_t *R, int8_t *z, float *sigma)
{
    float *rho = (float *)malloc(sizeof(float) * (size_t)r);
    for (int32_t j = 0; j < r; ++j) {
        int32_t acc = 0;
        const int8_t *col = A_c + (size_t)j * dp;
        for (int32_t i = 0; i < dp; ++i) acc += (int32_t)q8[i] * (int32_t)col[i];
        R[j] = acc;
        volatile float sj = dx * dA[j];            /* volatile: no contraction of the two multiplications */
        rho[j] = (float)acc * sj;
    }
    oracle_quantize_query(rho, r, z, sigma);
    free(rho);
}

/* Estimated score with one step size per column of B_c (i.e. per corpus point): the multiplier of the integer
 * score is sigma' * DeltaB_t rounded to float (sigma' = sigma, or 2 sigma for Euclidean), then ONE fused
 * multiply-add as in oracle_score. */
float oracle_score_columns(int32_t Y, float sigma, float dB_t, int32_t metric, float sqnorm)
{
    if (metric == ORACLE_L2) { volatile float mult = (2.0f * sigma) * dB_t; return fmaf((float)Y, mult, -sqnorm); }
    volatile float mult = sigma * dB_t;
    return fmaf((float)Y, mult, -0.0f);
}

/* ---- Mixed-precision decomposition (Sec. 4.2): x = (x_0, x_rest), r = (r_0, r_rest). ----
 * Only x_rest and r_rest are quantized (absmax over the rest alone, code 0 in the first position, so that the
 * integer products skip it whatever the matrices hold there); x_0 meets the float first row of A_c, r_0 the float
 * first row of B_c.  Every operation is one IEEE float operation (fmaf = one rounding) in the order written. */
void oracle_quantize_query_mixed(const float *qp, int32_t dp, int8_t *q8, float *dx)
{
    q8[0] = 0;
    oracle_quantize_query(qp + 1, dp - 1, q8 + 1, dx);
}

/* r_j ~= rho_j = x_0 A_c[0][j] + R_j (Delta_x DeltaA_cj) with R_j over the quantized rest; rho_0 stays a float,
 * (rho_1..) is re-quantized like a query. */
void oracle_stage_a_mixed(const int8_t *q8, float x0, int32_t dp, int32_t r, const int8_t *A_c /* [r][dp] */, float dx,
                          const float *dA /* [r] */, const float *A0 /* [r] first row of A_c */, int32_t *R, int8_t *z,
                          float *sigma, float *rho0)
{
    float *rho = (float *)calloc((size_t)(r > 0 ? r : 1), sizeof(float));
    for (int32_t j = 0; j < r; ++j) {
        int32_t acc = 0;
        const int8_t *col = A_c + (size_t)j * dp;
        for (int32_t i = 1; i < dp; ++i) acc += (int32_t)q8[i] * (int32_t)col[i];
        R[j] = acc;
        volatile float sj = dx * dA[j];
        volatile float quantized_part = (float)acc * sj;
        rho[j] = fmaf(x0, A0[j], quantized_part);
    }
    *rho0 = rho[0];
    z[0] = 0;
    if (r > 1) oracle_quantize_query(rho + 1, r - 1, z + 1, sigma); else *sigma = 0.0f;
    free(rho);
}

/* Estimated score: the float rank-one term r_0 B_c[0][t] on top of the quantized rest (as oracle_score_columns);
 * for Euclidean both parts carry the factor 2 of Sec. 3.1 (doubling is exact). */
float oracle_score_mixed(int32_t Y, float sigma, float dB_t, float rho0, float B0_t, int32_t metric, float sqnorm)
{
    const float rest = oracle_score_columns(Y, sigma, dB_t, metric, sqnorm);
    return fmaf(metric == ORACLE_L2 ? 2.0f * rho0 : rho0, B0_t, rest);
}

/* ---- Step 5 (Sec. 3.2 prediction y = (x^T A) B in its 8-bit form, Sec. 3.1 Euclidean reduction). ---- */
/* int32 accumulators of one pair: Y_j = sum_t z_t B[row_j][t]. */
void oracle_pair_accumulators(const int8_t *z, int32_t r, const int8_t *B_c /* [m_c][r] */, int64_t m_c, int32_t *Y)
{
    for (int64_t j = 0; j < m_c; ++j) {
        int32_t acc = 0;
        const int8_t *code = B_c + (size_t)j * r;
        for (int32_t t = 0; t < r; ++t) acc += (int32_t)z[t] * (int32_t)code[t];
        Y[j] = acc;
    }
}

/* Squared norm of a corpus row: double accumulation over i ascending, rounded to float. */
float oracle_row_sqnorm(const float *c, int32_t d)
{
    double acc = 0.0;
    for (int32_t i = 0; i < d; ++i) acc += (double)c[i] * (double)c[i];
    return (float)acc;
}

void oracle_corpus_sqnorms(const float *corpus, int64_t n, int32_t d, float *out)
{
    for (int64_t j = 0; j < n; ++j) out[j] = oracle_row_sqnorm(corpus + (size_t)j * d, d);
}

/* Estimated score (higher = better): inner product / cosine: sigma * Y; Euclidean: 2 sigma Y - |c|^2,
 * each as ONE fused multiply-add in float. */
float oracle_score(int32_t Y, float sigma, int32_t metric, float sqnorm)
{
    if (metric == ORACLE_L2) return fmaf((float)Y, 2.0f * sigma, -sqnorm);
    return fmaf((float)Y, sigma, -0.0f);
}

/* ---- Step 7 (Sec. 2.1 dissimilarities; Sec. 4.1: the original d-dimensional query is used). ---- */
float oracle_exact_dissim(const float *q, const float *c, int32_t d, int32_t metric)
{
    double acc = 0.0;
    if (metric == ORACLE_L2) {
        for (int32_t i = 0; i < d; ++i) { double t = (double)q[i] - (double)c[i]; acc += t * t; }
        return (float)acc;
    }
    for (int32_t i = 0; i < d; ++i) acc += (double)q[i] * (double)c[i];
    if (metric == ORACLE_IP) return (float)(-acc);
    double qn = 0.0;
    for (int32_t i = 0; i < d; ++i) qn += (double)q[i] * (double)q[i];
    if (!(qn > 0.0)) return 1.0f;
    return (float)(1.0 - acc / sqrt(qn));
}

/* ---- The whole query phase for one query (steps 1-7). ---- */
/* rerank = 0 is the variant without the final re-ranking step (Sec. 7.1 memory usage, App. D.3: the original
 * vectors are then not needed): the k points of highest estimated score are the answer (ties at the boundary
 * toward the lower corpus row, as in step 6), reported with dissimilarity = -score and ordered like every other
 * result (dissimilarity ascending, id ascending); m plays no role. */
static void search_one(const oracle_index *ix, const float *q, int32_t k, int32_t w, int32_t m,
                       int64_t *out_ids, float *out_dists, const oracle_dump *dump, int64_t qi, int rerank)
{
    const int32_t d = ix->d, dp = ix->dp, r = ix->r, L = ix->L;
    float *qp = (float *)malloc(sizeof(float) * (size_t)dp);
    float *g = (float *)malloc(sizeof(float) * (size_t)L);
    int32_t *sel = (int32_t *)malloc(sizeof(int32_t) * (size_t)w);
    float *sel_g = (float *)malloc(sizeof(float) * (size_t)w);
    int8_t *q8 = (int8_t *)malloc((size_t)dp);
    int32_t *R = (int32_t *)malloc(sizeof(int32_t) * (size_t)r);
    int8_t *z = (int8_t *)malloc((size_t)r);
    float dx, sigma, rho0 = 0.0f;
    const int columns = ix->col_scale_A && ix->pt_scale_B;
    const int mixed = columns && ix->first_row_A && ix->first_row_B;

    oracle_project(q, d, dp, ix->P, qp);                                   /* step 1 */
    oracle_centroid_dissim(qp, dp, ix->centroids, L, ix->metric, g);       /* step 2 */
    oracle_select_clusters(g, L, w, sel, sel_g);
    if (mixed) oracle_quantize_query_mixed(qp, dp, q8, &dx);               /* step 3 */
    else oracle_quantize_query(qp, dp, q8, &dx);

    int64_t total = 0, max_mc = 0;
    for (int32_t j = 0; j < w; ++j) {
        int64_t mc = ix->offsets[sel[j] + 1] - ix->offsets[sel[j]];
        total += mc;
        if (mc > max_mc) max_mc = mc;
    }
    keyidx *sc = (keyidx *)malloc(sizeof(keyidx) * (size_t)(total > 0 ? total : 1));
    int32_t *Y = (int32_t *)malloc(sizeof(int32_t) * (size_t)(max_mc > 0 ? max_mc : 1));
    int64_t pos = 0;
    for (int32_t j = 0; j < w; ++j) {                                      /* steps 4-5 per selected cluster */
        const int32_t c = sel[j];
        const int64_t off = ix->offsets[c], mc = ix->offsets[c + 1] - off;
        if (mixed) oracle_stage_a_mixed(q8, qp[0], dp, r, ix->A + (size_t)c * r * dp, dx, ix->col_scale_A + (size_t)c * r,
                                        ix->first_row_A + (size_t)c * r, R, z, &sigma, &rho0);
        else if (columns) oracle_stage_a_columns(q8, dp, r, ix->A + (size_t)c * r * dp, dx, ix->col_scale_A + (size_t)c * r, R, z, &sigma);
        else oracle_stage_a(q8, dp, r, ix->A + (size_t)c * r * dp, dx, ix->scale_A[c], ix->scale_B[c], R, z, &sigma);
        if (dump) {
            if (dump->R) memcpy(dump->R + ((size_t)qi * w + j) * r, R, sizeof(int32_t) * (size_t)r);
            if (dump->z) memcpy(dump->z + ((size_t)qi * w + j) * r, z, (size_t)r);
            if (dump->sigma) dump->sigma[(size_t)qi * w + j] = sigma;
            if (dump->rho0) dump->rho0[(size_t)qi * w + j] = rho0;
        }
        oracle_pair_accumulators(z, r, ix->B + (size_t)off * r, mc, Y);
        float best = -INFINITY;
        for (int64_t t = 0; t < mc; ++t) {
            float sq = 0.0f;   /* Sec. 3.1: the norms |c_j|^2 may be computed ahead of the search */
            if (ix->metric == ORACLE_L2)
                sq = ix->sqnorms ? ix->sqnorms[off + t] : oracle_row_sqnorm(ix->corpus + (size_t)(off + t) * d, d);
            sc[pos].key = mixed ? oracle_score_mixed(Y[t], sigma, ix->pt_scale_B[off + t], rho0, ix->first_row_B[off + t], ix->metric, sq)
                        : columns ? oracle_score_columns(Y[t], sigma, ix->pt_scale_B[off + t], ix->metric, sq)
                                  : oracle_score(Y[t], sigma, ix->metric, sq);
            sc[pos].idx = off + t;
            if (sc[pos].key > best) best = sc[pos].key;
            ++pos;
        }
        if (dump && dump->pair_best) dump->pair_best[(size_t)qi * w + j] = best;
    }
    /* step 6: the m highest estimated scores, order (score descending, row ascending) */
    qsort(sc, (size_t)total, sizeof(keyidx), cmp_key_desc);
    if (!rerank) m = k;
    int64_t nc = total < m ? total : m;
    keyidx *fin = (keyidx *)malloc(sizeof(keyidx) * (size_t)(nc > 0 ? nc : 1));
    for (int64_t t = 0; t < nc; ++t) {                                     /* step 7: exact re-rank */
        int64_t row = sc[t].idx;
        fin[t].key = rerank ? oracle_exact_dissim(q, ix->corpus + (size_t)row * d, d, ix->metric) : -sc[t].key;
        fin[t].idx = ix->ids ? ix->ids[row] : row;
    }
    qsort(fin, (size_t)nc, sizeof(keyidx), cmp_key_asc);
    for (int32_t t = 0; t < k; ++t) {
        if (t < nc) { out_ids[t] = fin[t].idx; out_dists[t] = fin[t].key; }
        else { out_ids[t] = -1; out_dists[t] = INFINITY; }
    }
    if (dump) {
        if (dump->qproj) memcpy(dump->qproj + (size_t)qi * dp, qp, sizeof(float) * (size_t)dp);
        if (dump->q8) memcpy(dump->q8 + (size_t)qi * dp, q8, (size_t)dp);
        if (dump->dx) dump->dx[qi] = dx;
        if (dump->sel) memcpy(dump->sel + (size_t)qi * w, sel, sizeof(int32_t) * (size_t)w);
        if (dump->sel_g) memcpy(dump->sel_g + (size_t)qi * w, sel_g, sizeof(float) * (size_t)w);
        for (int32_t t = 0; t < m; ++t) {
            if (dump->cand_rows) dump->cand_rows[(size_t)qi * m + t] = t < nc ? sc[t].idx : -1;
            if (dump->cand_scores) dump->cand_scores[(size_t)qi * m + t] = t < nc ? sc[t].key : 0.0f;
        }
    }
    free(fin); free(Y); free(sc); free(z); free(R); free(q8); free(sel_g); free(sel); free(g); free(qp);
}

/* Search a batch.  Parallel over queries only; each query runs the sequential algorithm above.
 * Returns 0, or -1 on invalid arguments. */
int oracle_search(const oracle_index *ix, const float *Q, int64_t nq, int32_t k, int32_t w, int32_t m,
                  int64_t *out_ids, float *out_dists, const oracle_dump *dump, int32_t threads)
{
    if (!ix || !Q || nq < 0 || k < 1 || m < 1 || k > m || w < 1 || w > ix->L || !out_ids || !out_dists) return -1;
    if (!ix->P && ix->dp != ix->d) return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t qi = 0; qi < nq; ++qi)
        search_one(ix, Q + (size_t)qi * ix->d, k, w, m, out_ids + (size_t)qi * k, out_dists + (size_t)qi * k, dump, qi, 1);
    return 0;
}

/* The same without the final re-ranking step (see search_one); ix->corpus is only read for the row norms of
 * the Euclidean score when ix->sqnorms is NULL. */
int oracle_search_no_rerank(const oracle_index *ix, const float *Q, int64_t nq, int32_t k, int32_t w,
                            int64_t *out_ids, float *out_dists, int32_t threads)
{
    if (!ix || !Q || nq < 0 || k < 1 || w < 1 || w > ix->L || !out_ids || !out_dists) return -1;
    if (!ix->P && ix->dp != ix->d) return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 4) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t qi = 0; qi < nq; ++qi)
        search_one(ix, Q + (size_t)qi * ix->d, k, w, k, out_ids + (size_t)qi * k, out_dists + (size_t)qi * k, NULL, qi, 0);
    return 0;
}

/* ---- Exact k-NN by exhaustive evaluation (Sec. 2.1, Eq. 1): ground truth for recall. ---- */
int oracle_exact_knn(const float *corpus, int64_t n, int32_t d, int32_t metric, const int64_t *ids, const float *Q,
                     int64_t nq, int32_t k, int64_t *out_ids, float *out_dists, int32_t threads)
{
    if (!corpus || !Q || n < 0 || nq < 0 || k < 1) return -1;
#ifdef _OPENMP
#pragma omp parallel for schedule(dynamic, 1) num_threads(threads > 0 ? threads : 1)
#endif
    for (int64_t qi = 0; qi < nq; ++qi) {
        keyidx *t = (keyidx *)malloc(sizeof(keyidx) * (size_t)(n > 0 ? n : 1));
        for (int64_t j = 0; j < n; ++j) {
            t[j].key = oracle_exact_dissim(Q + (size_t)qi * d, corpus + (size_t)j * d, d, metric);
            t[j].idx = ids ? ids[j] : j;
        }
        qsort(t, (size_t)n, sizeof(keyidx), cmp_key_asc);
        for (int32_t j = 0; j < k; ++j) {
            out_ids[(size_t)qi * k + j] = j < n ? t[j].idx : -1;
            out_dists[(size_t)qi * k + j] = j < n ? t[j].key : INFINITY;
        }
        free(t);
    }
    return 0;
}

/* ---- Unquantized prediction y = (x^T A) B (Sec. 3.2) in double, for the full-rank and Theorem-1 checks. ---- */
void oracle_rrr_predict_f64(const double *x, int32_t s, int32_t r, const double *A /* [s][r] */,
                            const double *B /* [r][m_c] */, int64_t m_c, double *y)
{
    double *t = (double *)malloc(sizeof(double) * (size_t)r);
    for (int32_t j = 0; j < r; ++j) {
        double acc = 0.0;
        for (int32_t i = 0; i < s; ++i) acc += x[i] * A[(size_t)i * r + j];
        t[j] = acc;
    }
    for (int64_t c = 0; c < m_c; ++c) {
        double acc = 0.0;
        for (int32_t j = 0; j < r; ++j) acc += t[j] * B[(size_t)j * m_c + c];
        y[c] = acc;
    }
    free(t);
}


/* ------------------------------------------------------------------------------------------------------------
 * The serialized index file (written by the harness, read here and - by code of its own - by the library).
 * Little-endian.  Header of 64 bytes: "LRNIDX01", int32 metric, d, dp, r, L, flags (bit 0: P present, bit 1:
 * ids present), int64 n at offset 32.  Then, each at the next multiple of 64 bytes: cluster_offsets
 * int64[L+1], ids int64[n] (if present), centroids float[L][dp], P float[d][dp] (if present), A int8[L][r][dp],
 * B int8[n][r], scale_A float[L], scale_B float[L], corpus float[n][d].
 * oracle_load_file returns a heap-allocated index that owns its arrays (NULL on any error);
 * oracle_free_loaded releases it.
 * ------------------------------------------------------------------------------------------------------------ */
static void *read_array(FILE *f, long long *pos, size_t bytes)
{
    long long at = (*pos + 63) / 64 * 64;
    void *buf = malloc(bytes ? bytes : 1);
    if (!buf) return NULL;
    if (fseeko(f, (off_t)at, SEEK_SET) != 0 || fread(buf, 1, bytes, f) != bytes) { free(buf); return NULL; }
    *pos = at + (long long)bytes;
    return buf;
}

void oracle_free_loaded(oracle_index *ix)
{
    if (!ix) return;
    free((void *)ix->centroids); free((void *)ix->P); free((void *)ix->A); free((void *)ix->B);
    free((void *)ix->scale_A); free((void *)ix->scale_B); free((void *)ix->offsets); free((void *)ix->corpus);
    free((void *)ix->ids); free((void *)ix->sqnorms);
    free(ix);
}

oracle_index *oracle_load_file(const char *path)
{
    FILE *f = fopen(path, "rb");
    if (!f) return NULL;
    unsigned char head[64];
    oracle_index *ix = NULL;
    if (fread(head, 1, 64, f) == 64 && memcmp(head, "LRNIDX01", 8) == 0) {
        int32_t hv[6];
        int64_t n;
        memcpy(hv, head + 8, sizeof hv);
        memcpy(&n, head + 32, sizeof n);
        ix = (oracle_index *)calloc(1, sizeof *ix);
        if (ix && n >= 1 && hv[1] >= 1 && hv[2] >= 1 && hv[3] >= 1 && hv[4] >= 1) {
            const int flags = hv[5];
            long long pos = 64;
            int ok = 1;
            ix->metric = hv[0]; ix->d = hv[1]; ix->dp = hv[2]; ix->r = hv[3]; ix->L = hv[4]; ix->n = n;
            ok = ok && (ix->offsets = (const int64_t *)read_array(f, &pos, ((size_t)ix->L + 1) * 8)) != NULL;
            if (flags & 2) ok = ok && (ix->ids = (const int64_t *)read_array(f, &pos, (size_t)n * 8)) != NULL;
            ok = ok && (ix->centroids = (const float *)read_array(f, &pos, (size_t)ix->L * ix->dp * 4)) != NULL;
            if (flags & 1) ok = ok && (ix->P = (const float *)read_array(f, &pos, (size_t)ix->d * ix->dp * 4)) != NULL;
            ok = ok && (ix->A = (const int8_t *)read_array(f, &pos, (size_t)ix->L * ix->r * ix->dp)) != NULL;
            ok = ok && (ix->B = (const int8_t *)read_array(f, &pos, (size_t)n * ix->r)) != NULL;
            ok = ok && (ix->scale_A = (const float *)read_array(f, &pos, (size_t)ix->L * 4)) != NULL;
            ok = ok && (ix->scale_B = (const float *)read_array(f, &pos, (size_t)ix->L * 4)) != NULL;
            ok = ok && (ix->corpus = (const float *)read_array(f, &pos, (size_t)n * ix->d * 4)) != NULL;
            if (ok && !(flags & 1) && ix->dp != ix->d) ok = 0;          /* no projection means identity */
            if (ok && (ix->offsets[0] != 0 || ix->offsets[ix->L] != n)) ok = 0;
            if (ok && ix->metric == ORACLE_L2) {
                float *sq = (float *)malloc((size_t)n * sizeof(float));
                if (sq) { oracle_corpus_sqnorms(ix->corpus, n, ix->d, sq); ix->sqnorms = sq; } else ok = 0;
            }
            if (!ok) { oracle_free_loaded(ix); ix = NULL; }
        } else {
            free(ix); ix = NULL;
        }
    }
    fclose(f);
    return ix;
}
