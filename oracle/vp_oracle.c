/*
 * CPU oracle for clustered vocabulary projection (arxiv 2208.06874).
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain definition that the
 * GPU library is checked against.  Nothing in the product path may call it;
 * only the tests, the smoke check and the benchmark's cpu_baseline leg do.
 * It shares no code, header, table or helper with the HIP library.
 *
 * Inputs are IEEE binary16 bit patterns (uint16_t), the same bits the GPU
 * receives.  Every value is widened exactly to double and all arithmetic is
 * double precision.  Summation over the embedding dimension always runs
 * i = 0, 1, ..., d-1 for each output element.
 *
 * Notation (paper, section 2.1 / 2.3): W is d x V (one column per token),
 * b has V entries, a hidden row h has d entries, C_j is centroid j (K of
 * them), A_j is the ascending list of active token ids of cluster j.
 *
 * Pins (see tests): nearest centroid vs brute-force Euclidean distance,
 * full-list candidate sets reproduce the full projection, full projection vs
 * a library log_softmax(h W + b), sum of exp(logp) over the candidates = 1,
 * hand-computed integer case, tie-break cases; the batch-union form against the
 * paper's worked example of the boolean list and against the per-cluster form
 * when all rows share a cluster.  The paper prints no logits,
 * probabilities or cluster ids, so no value here is pinned to a number
 * printed in the paper.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* Exact widening of an IEEE 754 binary16 bit pattern to double. */
double vpo_half_to_double(uint16_t bits)
{
    int sign = (bits >> 15) & 1;
    int expo = (bits >> 10) & 0x1f;
    int frac = bits & 0x3ff;
    double v;
    if (expo == 0) {
        v = ldexp((double)frac, -24);            /* zero and subnormals */
    } else if (expo == 31) {
        v = frac ? NAN : INFINITY;
    } else {
        v = ldexp((double)(frac | 0x400), expo - 25);
    }
    return sign ? -v : v;
}

/* Section 2.3: the term C_j^2 that is precomputed per centroid is the squared
 * Euclidean norm of C_j. */
void vpo_cnorm(const uint16_t *C, int K, int d, double *cnorm)
{
    for (int j = 0; j < K; ++j) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i) {
            double c = vpo_half_to_double(C[(size_t)j * d + i]);
            acc += c * c;
        }
        cnorm[j] = acc;
    }
}

/* Eq. 2 (section 2.3), read as the signed scalar ||C_j||^2 - 2 <h, C_j>
 * (which is ||h - C_j||^2 minus the constant ||h||^2): the cluster of a row
 * is the j in [0, K) that minimises it; the first minimum wins a tie.
 * scores (optional, N*K) receives every s[r, j]. */
void vpo_assign(const uint16_t *H, int N, int d, const uint16_t *C, int K,
                const double *cnorm, int32_t *g, double *scores)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < N; ++r) {
        int best = -1;
        double best_s = 0.0;
        for (int j = 0; j < K; ++j) {
            double dot = 0.0;
            for (int i = 0; i < d; ++i)
                dot += vpo_half_to_double(H[(size_t)r * d + i]) *
                       vpo_half_to_double(C[(size_t)j * d + i]);
            double s = cnorm[j] - 2.0 * dot;
            if (scores) scores[(size_t)r * K + j] = s;
            if (best < 0 || s < best_s) { best = j; best_s = s; }
        }
        g[r] = best;
    }
}

/* Eq. 1 (section 2.1) restricted to the listed columns (step 3 of the
 * inference list in section 2.3): z[c] = sum_i W[i, ids[c]] * h[i] + b[ids[c]].
 * ids == NULL means the identity list 0..n-1 (the full vocabulary).
 * The loop nest is i-outer so that W is walked row by row; each z[c] still
 * receives its d products in the order i = 0..d-1, then the bias. */
void vpo_logits_row(const uint16_t *W, const uint16_t *b, int d, int V,
                    const uint16_t *h, const int32_t *ids, int n, double *z)
{
    for (int c = 0; c < n; ++c) z[c] = 0.0;
    for (int i = 0; i < d; ++i) {
        double hi = vpo_half_to_double(h[i]);
        const uint16_t *Wi = W + (size_t)i * V;
        if (ids) {
            for (int c = 0; c < n; ++c) z[c] += vpo_half_to_double(Wi[ids[c]]) * hi;
        } else {
            for (int c = 0; c < n; ++c) z[c] += vpo_half_to_double(Wi[c]) * hi;
        }
    }
    for (int c = 0; c < n; ++c)
        z[c] += vpo_half_to_double(b[ids ? ids[c] : c]);
}

/* Steps 4-5 of the inference list (section 2.3): tokens outside the set are
 * at -infinity, so the softmax normalises over the listed candidates only.
 * Returns the log of the normaliser; logp may be NULL. */
double vpo_log_softmax(const double *z, int n, double *logp)
{
    double m = z[0];
    for (int c = 1; c < n; ++c) if (z[c] > m) m = z[c];
    double sum = 0.0;
    for (int c = 0; c < n; ++c) sum += exp(z[c] - m);
    double lse = m + log(sum);
    if (logp) for (int c = 0; c < n; ++c) logp[c] = z[c] - lse;
    return lse;
}

/* Section 2.1: the search consumes the candidates in descending order of
 * probability.  Selects the k best positions by (z descending, position
 * ascending); positions are ascending token ids, so ties go to the smaller
 * token id.  Positions beyond n are reported as -1. */
void vpo_topk(const double *z, int n, int k, int32_t *pos)
{
    char *taken = (char *)calloc((size_t)(n > 0 ? n : 1), 1);
    for (int t = 0; t < k; ++t) {
        int best = -1;
        for (int c = 0; c < n; ++c) {
            if (taken[c]) continue;
            if (best < 0 || z[c] > z[best]) best = c;
        }
        pos[t] = best;
        if (best >= 0) taken[best] = 1;
    }
    free(taken);
}

/*
 * The whole clustered path for N rows.
 *   cand_off[K+1], cand_ids[]: the active sets A_j, ascending ids.
 *   forced_g: NULL, or per-row cluster ids to use instead of Eq. 2 (entries
 *             < 0 fall back to Eq. 2).
 * Outputs (any may be NULL except out_g):
 *   out_g[N], out_ids[N*k] (token ids, -1 padding), out_logp[N*k]
 *   (-inf padding), out_z[N*k] (logit of each selected token),
 *   out_lse[N], all_off[N+1] + all_z[] (every candidate logit of every row,
 *   row r at all_off[r] .. all_off[r+1]; all_z must hold sum_r n_{g[r]}).
 */
void vpo_project(const uint16_t *W, const uint16_t *b, int d, int V,
                 const uint16_t *C, int K,
                 const int64_t *cand_off, const int32_t *cand_ids,
                 const uint16_t *H, int N, int k, const int32_t *forced_g,
                 int32_t *out_g, int32_t *out_ids, double *out_logp,
                 double *out_z, double *out_lse,
                 const int64_t *all_off, double *all_z)
{
    double *cnorm = (double *)malloc(sizeof(double) * (size_t)K);
    vpo_cnorm(C, K, d, cnorm);
    vpo_assign(H, N, d, C, K, cnorm, out_g, NULL);
    free(cnorm);
    if (forced_g)
        for (int r = 0; r < N; ++r) if (forced_g[r] >= 0) out_g[r] = forced_g[r];

#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < N; ++r) {
        int j = out_g[r];
        const int32_t *ids = cand_ids + cand_off[j];
        int n = (int)(cand_off[j + 1] - cand_off[j]);
        double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        vpo_logits_row(W, b, d, V, H + (size_t)r * d, ids, n, z);
        double lse = n > 0 ? vpo_log_softmax(z, n, NULL) : -INFINITY;
        vpo_topk(z, n, k, pos);
        for (int t = 0; t < k; ++t) {
            int p = pos[t];
            if (out_ids)  out_ids[(size_t)r * k + t]  = p >= 0 ? ids[p] : -1;
            if (out_logp) out_logp[(size_t)r * k + t] = p >= 0 ? z[p] - lse : -INFINITY;
            if (out_z)    out_z[(size_t)r * k + t]    = p >= 0 ? z[p] : -INFINITY;
        }
        if (out_lse) out_lse[r] = lse;
        if (all_off && all_z) memcpy(all_z + all_off[r], z, sizeof(double) * (size_t)n);
        free(pos);
        free(z);
    }
}

/* The default projection of section 2.1 (Eq. 1, softmax, descending order)
 * over all V tokens.  It calls the same per-row routines as vpo_project with
 * the identity candidate list.  all_z (optional) is N*V. */
void vpo_project_full(const uint16_t *W, const uint16_t *b, int d, int V,
                      const uint16_t *H, int N, int k,
                      int32_t *out_ids, double *out_logp, double *out_z,
                      double *out_lse, double *all_z)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < N; ++r) {
        double *z = (double *)malloc(sizeof(double) * (size_t)V);
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        vpo_logits_row(W, b, d, V, H + (size_t)r * d, NULL, V, z);
        double lse = vpo_log_softmax(z, V, NULL);
        vpo_topk(z, V, k, pos);
        for (int t = 0; t < k; ++t) {
            int p = pos[t];
            if (out_ids)  out_ids[(size_t)r * k + t]  = p;
            if (out_logp) out_logp[(size_t)r * k + t] = p >= 0 ? z[p] - lse : -INFINITY;
            if (out_z)    out_z[(size_t)r * k + t]    = p >= 0 ? z[p] : -INFINITY;
        }
        if (out_lse) out_lse[r] = lse;
        if (all_z) memcpy(all_z + (size_t)r * V, z, sizeof(double) * (size_t)V);
        free(pos);
        free(z);
    }
}

/*
 * The paper's own batched form of the inference list (section 2.3): the active
 * sets of the predicted clusters of ALL rows of the batch are united (a
 * boolean list over the vocabulary, switched on for every active token of
 * every predicted cluster; the reduced column set U is where it is 1, in
 * ascending order), every row is projected onto U (step 3), tokens outside U
 * are at -infinity (step 4) and the softmax (step 5) therefore normalises over
 * U for every row.
 *   flags[V] (optional) receives the boolean list, U[V] the reduced column
 *   set (first *nU entries).  all_z (optional) is N * (*nU) logits, row-major.
 */
void vpo_project_union(const uint16_t *W, const uint16_t *b, int d, int V,
                       const uint16_t *C, int K,
                       const int64_t *cand_off, const int32_t *cand_ids,
                       const uint16_t *H, int N, int k, const int32_t *forced_g,
                       int32_t *out_g, uint8_t *flags, int32_t *U, int32_t *nU,
                       int32_t *out_ids, double *out_logp, double *out_z,
                       double *out_lse, double *all_z)
{
    double *cnorm = (double *)malloc(sizeof(double) * (size_t)K);
    vpo_cnorm(C, K, d, cnorm);
    vpo_assign(H, N, d, C, K, cnorm, out_g, NULL);
    free(cnorm);
    if (forced_g)
        for (int r = 0; r < N; ++r) if (forced_g[r] >= 0) out_g[r] = forced_g[r];

    uint8_t *fl = flags ? flags : (uint8_t *)malloc((size_t)V);
    memset(fl, 0, (size_t)V);
    for (int r = 0; r < N; ++r) {
        int j = out_g[r];
        for (int64_t c = cand_off[j]; c < cand_off[j + 1]; ++c) fl[cand_ids[c]] = 1;
    }
    int n = 0;
    for (int v = 0; v < V; ++v) if (fl[v]) U[n++] = v;
    *nU = n;
    if (!flags) free(fl);

#pragma omp parallel for schedule(dynamic, 1)
    for (int r = 0; r < N; ++r) {
        double *z = (double *)malloc(sizeof(double) * (size_t)(n > 0 ? n : 1));
        int32_t *pos = (int32_t *)malloc(sizeof(int32_t) * (size_t)k);
        vpo_logits_row(W, b, d, V, H + (size_t)r * d, U, n, z);
        double lse = n > 0 ? vpo_log_softmax(z, n, NULL) : -INFINITY;
        vpo_topk(z, n, k, pos);
        for (int t = 0; t < k; ++t) {
            int p = pos[t];
            if (out_ids)  out_ids[(size_t)r * k + t]  = p >= 0 ? U[p] : -1;
            if (out_logp) out_logp[(size_t)r * k + t] = p >= 0 ? z[p] - lse : -INFINITY;
            if (out_z)    out_z[(size_t)r * k + t]    = p >= 0 ? z[p] : -INFINITY;
        }
        if (out_lse) out_lse[r] = lse;
        if (all_z) memcpy(all_z + (size_t)r * n, z, sizeof(double) * (size_t)n);
        free(pos);
        free(z);
    }
}

/* Logit of single tokens of single rows (Eq. 1), for spot checks at sizes
 * where whole rows are too slow: z[q] = W[:, tok[q]] . H[row[q]] + b[tok[q]]. */
void vpo_logit_points(const uint16_t *W, const uint16_t *b, int d, int V,
                      const uint16_t *H, const int32_t *row, const int32_t *tok,
                      int nq, double *z)
{
    for (int q = 0; q < nq; ++q) {
        double acc = 0.0;
        for (int i = 0; i < d; ++i)
            acc += vpo_half_to_double(W[(size_t)i * V + tok[q]]) *
                   vpo_half_to_double(H[(size_t)row[q] * d + i]);
        z[q] = acc + vpo_half_to_double(b[tok[q]]);
    }
}
