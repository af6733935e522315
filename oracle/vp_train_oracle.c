/*
 * CPU oracle for the offline training of the clusters (arxiv 2208.06874,
 * section 2.2 "Offline Training of Clusters" and the cluster training settings
 * of section 3.1: k-means over recorded hidden vectors, 20 iterations; the
 * active set of a cluster is the union of the K recorded likely tokens of all
 * of its members).
 *
 * TEST INFRASTRUCTURE ONLY, like vp_oracle.c: nothing in the product path may
 * call it, and it shares no code, header, table or helper with the HIP library.
 *
 * k-means is Lloyd's algorithm written out: every vector goes to its nearest
 * centroid in squared Euclidean distance (ties to the lowest index), every
 * centroid becomes the arithmetic mean of its members, a cluster without
 * members keeps its centroid.  All arithmetic is double precision over exactly
 * widened binary16 inputs.  With round_half != 0 each new centroid coordinate is
 * rounded to binary16 (nearest, ties to even) before the next assignment, which
 * is the precision the projection library stores centroids in; with
 * round_half == 0 the routine is the textbook iteration and is pinned to
 * library implementations of it.
 *
 * Pins (see tests): the rounding routine against every binary16 value, its
 * midpoints and a library cast; one Lloyd step against a hand-computed case;
 * several steps against two library k-means routines started from the same
 * centroids; nearest-centroid membership against brute force; monotone
 * objective; the active-set union against the worked example printed in
 * section 2.2 and against sets built in Python.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

double vpo_half_to_double(uint16_t bits);   /* vp_oracle.c */

/* double -> IEEE 754 binary16, round to nearest, ties to even; overflow gives
 * infinity.  rint() rounds to nearest-even in the default rounding mode. */
uint16_t vpo_double_to_half(double v)
{
    uint16_t sign = signbit(v) ? 0x8000u : 0u;
    double a = fabs(v);
    if (isnan(v)) return 0x7e00u;
    if (a >= 65520.0) return (uint16_t)(sign | 0x7c00u);   /* at or above the midpoint to 2^16 */
    if (a < ldexp(1.0, -14)) {
        /* subnormal range: multiples of 2^-24; 1024 of them is the least normal number */
        double q = rint(ldexp(a, 24));
        return (uint16_t)(sign | (uint16_t)q);
    }
    int e;
    double m = frexp(a, &e);            /* a = m 2^e, 0.5 <= m < 1  =>  a = (2m) 2^(e-1) */
    double q = rint(ldexp(m, 11));      /* 2m scaled to 10 fraction bits: 1024 .. 2048 */
    int expo = e - 1;
    if (q == 2048.0) {
        q = 1024.0;
        expo += 1;
    }
    if (expo + 15 >= 31) return (uint16_t)(sign | 0x7c00u);
    return (uint16_t)(sign | ((expo + 15) << 10) | ((int)q - 1024));
}

/* One Lloyd iteration from the centroids C (K x d, double).
 * forced (may be NULL): membership to use instead of the nearest centroid, per
 * vector, where >= 0.  Outputs: assign[n], counts[K], Cnew[K x d] (may alias
 * nothing), *objective = sum over vectors of the squared distance to the
 * centroid they were assigned to (before the update). */
void vpo_kmeans_step(const uint16_t *X, int n, int d, const double *C, int K, const int32_t *forced,
                     int32_t *assign, int32_t *counts, double *Cnew, double *objective)
{
    double obj = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : obj)
    for (int r = 0; r < n; ++r) {
        int best = -1;
        double best_d = INFINITY;
        for (int j = 0; j < K; ++j) {
            double s = 0.0;
            for (int i = 0; i < d; ++i) {
                double t = vpo_half_to_double(X[(size_t)r * d + i]) - C[(size_t)j * d + i];
                s += t * t;
            }
            if (s < best_d) {   /* strict: ties stay with the lowest j */
                best_d = s;
                best = j;
            }
        }
        if (forced && forced[r] >= 0 && forced[r] != best) {
            int j = forced[r];
            double s = 0.0;
            for (int i = 0; i < d; ++i) {
                double t = vpo_half_to_double(X[(size_t)r * d + i]) - C[(size_t)j * d + i];
                s += t * t;
            }
            best = j;
            best_d = s;
        }
        assign[r] = best;
        obj += best_d;
    }
    if (objective) *objective = obj;
    memset(counts, 0, sizeof(int32_t) * (size_t)K);
    for (int r = 0; r < n; ++r) counts[assign[r]] += 1;
    if (!Cnew) return;
    for (size_t e = 0; e < (size_t)K * d; ++e) Cnew[e] = 0.0;
    for (int r = 0; r < n; ++r) {
        const int j = assign[r];
        for (int i = 0; i < d; ++i) Cnew[(size_t)j * d + i] += vpo_half_to_double(X[(size_t)r * d + i]);
    }
    for (int j = 0; j < K; ++j) {
        for (int i = 0; i < d; ++i) {
            if (counts[j] > 0)
                Cnew[(size_t)j * d + i] /= (double)counts[j];
            else
                Cnew[(size_t)j * d + i] = C[(size_t)j * d + i];   /* no members: centroid unchanged */
        }
    }
}

/* Optional remedy for clusters that lost all their members (the paper names no remedy; k-means
 * libraries usually split a big cluster).  Deterministic form: the clusters without members are
 * taken in ascending order; each takes the cluster that currently has the most members (ties: lowest
 * index; it must have at least two), whose centroid c is replaced by c (1 - eps) and whose copy
 * c (1 + eps) becomes the empty cluster's centroid, eps = 2^-10; the member count is shared out
 * (half, rounded down, goes to the new cluster) so that the next empty cluster sees the new sizes.
 * With round_half the two products are rounded to binary16. */
void vpo_split_empty(double *C, int32_t *counts, int K, int d, int round_half)
{
    const double eps = ldexp(1.0, -10);
    for (int j = 0; j < K; ++j) {
        if (counts[j] != 0) continue;
        int big = 0;
        for (int i = 1; i < K; ++i)
            if (counts[i] > counts[big]) big = i;
        if (counts[big] < 2) return;
        for (int e = 0; e < d; ++e) {
            const double c = C[(size_t)big * d + e];
            double up = c * (1.0 + eps), down = c * (1.0 - eps);
            if (round_half) {
                up = vpo_half_to_double(vpo_double_to_half(up));
                down = vpo_half_to_double(vpo_double_to_half(down));
            }
            C[(size_t)j * d + e] = up;
            C[(size_t)big * d + e] = down;
        }
        counts[j] = counts[big] / 2;
        counts[big] -= counts[j];
    }
}

/* iters Lloyd iterations from the binary16 centroids C0, then one more
 * assignment against the final centroids (the membership used to build the
 * active sets).  C_out (double, K x d) and C_out_bits (binary16, may be NULL
 * unless round_half) receive the final centroids; objective[t] is the value
 * at the start of iteration t (t < iters) and objective[iters] that of the
 * final assignment. */
void vpo_kmeans(const uint16_t *X, int n, int d, const uint16_t *C0, int K, int iters, int round_half,
                int split_empty, double *C_out, uint16_t *C_out_bits, int32_t *assign, int32_t *counts,
                double *objective)
{
    double *C = (double *)malloc(sizeof(double) * (size_t)K * d);
    double *Cn = (double *)malloc(sizeof(double) * (size_t)K * d);
    for (size_t e = 0; e < (size_t)K * d; ++e) C[e] = vpo_half_to_double(C0[e]);
    for (int t = 0; t < iters; ++t) {
        vpo_kmeans_step(X, n, d, C, K, NULL, assign, counts, Cn, objective ? objective + t : NULL);
        for (size_t e = 0; e < (size_t)K * d; ++e)
            C[e] = round_half ? vpo_half_to_double(vpo_double_to_half(Cn[e])) : Cn[e];
        if (split_empty) vpo_split_empty(C, counts, K, d, round_half);
    }
    vpo_kmeans_step(X, n, d, C, K, NULL, assign, counts, NULL, objective ? objective + iters : NULL);
    for (size_t e = 0; e < (size_t)K * d; ++e) {
        C_out[e] = C[e];
        if (C_out_bits) C_out_bits[e] = vpo_double_to_half(C[e]);
    }
    free(C);
    free(Cn);
}

/* Active sets (section 2.2): A_j = union over the members r of cluster j of
 * the T recorded tokens top[r][0..T), ascending.  Entries < 0 are "no token".
 * cand_off[K+1] is always written; cand_ids only when not NULL (call once with
 * NULL to size it).  Returns the total number of entries. */
int64_t vpo_active_sets(const int32_t *top, int n, int T, const int32_t *assign, int K, int V,
                        int64_t *cand_off, int32_t *cand_ids)
{
    unsigned char *flag = (unsigned char *)malloc((size_t)V);
    int64_t total = 0;
    for (int j = 0; j < K; ++j) {
        memset(flag, 0, (size_t)V);
        for (int r = 0; r < n; ++r) {
            if (assign[r] != j) continue;
            for (int t = 0; t < T; ++t) {
                const int v = top[(size_t)r * T + t];
                if (v >= 0 && v < V) flag[v] = 1;
            }
        }
        cand_off[j] = total;
        for (int v = 0; v < V; ++v) {
            if (flag[v]) {
                if (cand_ids) cand_ids[total] = v;
                total += 1;
            }
        }
    }
    cand_off[K] = total;
    free(flag);
    return total;
}
