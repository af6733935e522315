/* Runs every entry of the C oracle on small seeded cases with exactly sized heap buffers.  Built by
 * tests/test_oracle_sanitizers.py with -fsanitize=address,undefined: an access outside a buffer, a
 * signed overflow or a misaligned access in the oracle ends the run with a report.  It also checks a
 * few invariants of the results so that the calls cannot be optimised away. */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

double vpo_half_to_double(uint16_t bits);
uint16_t vpo_double_to_half(double v);
void vpo_project(const uint16_t *W, const uint16_t *b, int d, int V, const uint16_t *C, int K, const int64_t *cand_off,
                 const int32_t *cand_ids, const uint16_t *H, int N, int k, const int32_t *forced_g, int32_t *out_g,
                 int32_t *out_ids, double *out_logp, double *out_z, double *out_lse, const int64_t *all_off,
                 double *all_z);
void vpo_project_full(const uint16_t *W, const uint16_t *b, int d, int V, const uint16_t *H, int N, int k,
                      int32_t *out_ids, double *out_logp, double *out_z, double *out_lse, double *all_z);
void vpo_project_union(const uint16_t *W, const uint16_t *b, int d, int V, const uint16_t *C, int K,
                       const int64_t *cand_off, const int32_t *cand_ids, const uint16_t *H, int N, int k,
                       const int32_t *forced_g, int32_t *out_g, uint8_t *flags, int32_t *U, int32_t *nU,
                       int32_t *out_ids, double *out_logp, double *out_z, double *out_lse, double *all_z);
void vpo_kmeans(const uint16_t *X, int n, int d, const uint16_t *C0, int K, int iters, int round_half, int split_empty,
                double *C_out, uint16_t *C_out_bits, int32_t *assign, int32_t *counts, double *objective);
int64_t vpo_active_sets(const int32_t *top, int n, int T, const int32_t *assign, int K, int V, int64_t *cand_off,
                        int32_t *cand_ids);
void vpo_beam_step(const int32_t *cand_ids, const float *cand_logp, const float *scores, int S, int B, int k,
                   float *out_scores, int32_t *out_parent, int32_t *out_token);

static uint64_t state = 0x9E3779B97F4A7C15ull;
static double uniform(void)
{
    state = state * 6364136223846793005ull + 1442695040888963407ull;
    return (double)(state >> 11) / 9007199254740992.0;
}
static uint16_t *random_halves(size_t n, double scale)
{
    uint16_t *p = (uint16_t *)malloc(sizeof(uint16_t) * n);
    for (size_t e = 0; e < n; ++e) p[e] = vpo_double_to_half((uniform() * 2.0 - 1.0) * scale);
    return p;
}
#define CHECK(c) do { if (!(c)) { fprintf(stderr, "check failed: %s (line %d)\n", #c, __LINE__); return 1; } } while (0)

int main(void)
{
    const int d = 24, V = 97, K = 5, N = 7, k = 6;
    uint16_t *W = random_halves((size_t)d * V, 0.5), *b = random_halves(V, 0.3);
    uint16_t *C = random_halves((size_t)K * d, 1.0), *H = random_halves((size_t)N * d, 1.0);
    /* active sets of 0, 3, 40, 97 and 1 tokens (ascending ids) */
    const int sizes[5] = {0, 3, 40, 97, 1};
    int64_t off[6] = {0};
    for (int j = 0; j < K; ++j) off[j + 1] = off[j] + sizes[j];
    int32_t *ids = (int32_t *)malloc(sizeof(int32_t) * (size_t)off[K]);
    for (int j = 0; j < K; ++j)
        for (int c = 0; c < sizes[j]; ++c) ids[off[j] + c] = (int32_t)((int64_t)c * V / sizes[j]);
    int32_t forced[7] = {0, 1, 2, 3, 4, -1, 2};

    int32_t *g = (int32_t *)malloc(sizeof(int32_t) * N), *oi = (int32_t *)malloc(sizeof(int32_t) * N * k);
    double *ol = (double *)malloc(sizeof(double) * N * k), *oz = (double *)malloc(sizeof(double) * N * k);
    double *lse = (double *)malloc(sizeof(double) * N);
    vpo_project(W, b, d, V, C, K, off, ids, H, N, k, forced, g, oi, ol, oz, lse, NULL, NULL);
    int64_t all_off[8] = {0};
    for (int r = 0; r < N; ++r) all_off[r + 1] = all_off[r] + sizes[g[r]];
    double *all_z = (double *)malloc(sizeof(double) * (size_t)(all_off[N] > 0 ? all_off[N] : 1));
    int32_t same[7];
    memcpy(same, g, sizeof(same));
    vpo_project(W, b, d, V, C, K, off, ids, H, N, k, same, g, oi, ol, oz, lse, all_off, all_z);
    CHECK(memcmp(same, g, sizeof(same)) == 0);
    CHECK(oi[0] == -1 && isinf(ol[0]));                       /* row 0: empty set */
    CHECK(oi[1 * k + 3] == -1 && oi[1 * k + 2] >= 0);           /* row 1: three tokens, k = 6 */
    CHECK(oi[4 * k] == ids[off[4]] && fabs(ol[4 * k]) < 1e-12); /* row 4: one token, log-prob 0 */
    for (int r = 0; r < N; ++r) {
        double p = 0.0;
        for (int64_t c = all_off[r]; c < all_off[r + 1]; ++c) p += exp(all_z[c] - lse[r]);
        CHECK(sizes[g[r]] == 0 || fabs(p - 1.0) < 1e-9);
    }

    double *fz = (double *)malloc(sizeof(double) * (size_t)N * V);
    vpo_project_full(W, b, d, V, H, N, k, oi, ol, oz, lse, fz);
    CHECK(oi[0] >= 0 && oi[0] < V && ol[0] <= 0.0);

    uint8_t *flags = (uint8_t *)malloc((size_t)V);
    int32_t *U = (int32_t *)malloc(sizeof(int32_t) * V), nU = -1;
    int32_t g12[7] = {1, 2, 1, 4, 2, 1, 4};
    vpo_project_union(W, b, d, V, C, K, off, ids, H, N, k, g12, g, flags, U, &nU, oi, ol, oz, lse, NULL);
    CHECK(nU > 0 && nU <= 3 + 40 + 1);
    double *uz = (double *)malloc(sizeof(double) * (size_t)N * nU);
    vpo_project_union(W, b, d, V, C, K, off, ids, H, N, k, g12, g, NULL, U, &nU, oi, ol, oz, lse, uz);
    int32_t g0[7] = {0, 0, 0, 0, 0, 0, 0};
    vpo_project_union(W, b, d, V, C, K, off, ids, H, N, k, g0, g, flags, U, &nU, oi, ol, oz, lse, NULL);
    CHECK(nU == 0 && oi[0] == -1);

    /* training: 60 vectors, 6 clusters two of which start far away (they lose their members) */
    const int n = 60, Kt = 6, iters = 4, T = 3;
    uint16_t *X = random_halves((size_t)n * d, 1.0), *C0 = random_halves((size_t)Kt * d, 1.0);
    for (int i = 0; i < d; ++i) C0[4 * d + i] = C0[5 * d + i] = vpo_double_to_half(50.0);
    double *Cout = (double *)malloc(sizeof(double) * Kt * d), obj[5];
    uint16_t *Cbits = (uint16_t *)malloc(sizeof(uint16_t) * Kt * d);
    int32_t *assign = (int32_t *)malloc(sizeof(int32_t) * n), counts[6];
    for (int split = 0; split < 2; ++split) {
        vpo_kmeans(X, n, d, C0, Kt, iters, 1, split, Cout, Cbits, assign, counts, obj);
        int total = 0;
        for (int j = 0; j < Kt; ++j) total += counts[j];
        CHECK(total == n && obj[iters] <= obj[0] + 1e-9);
        if (split) CHECK(counts[4] + counts[5] > 0);
    }
    int32_t *top = (int32_t *)malloc(sizeof(int32_t) * n * T);
    for (int e = 0; e < n * T; ++e) top[e] = (int32_t)(uniform() * (V + 6)) - 3;   /* some outside [0, V) */
    int64_t aoff[7];
    const int64_t total = vpo_active_sets(top, n, T, assign, Kt, V, aoff, NULL);
    int32_t *aids = (int32_t *)malloc(sizeof(int32_t) * (size_t)(total > 0 ? total : 1));
    CHECK(vpo_active_sets(top, n, T, assign, Kt, V, aoff, aids) == total && aoff[Kt] == total);

    /* one beam step: 2 sentences, 3 hypotheses, 4 candidates each, some candidates missing */
    const int S = 2, B = 3, kb = 4;
    int32_t cid[2 * 3 * 4];
    float clp[2 * 3 * 4], sc[2 * 3] = {0.f, -1.f, -INFINITY, -0.5f, -0.5f, -2.f}, os[6];
    int32_t op[6], ot[6];
    for (int e = 0; e < S * B * kb; ++e) {
        cid[e] = e % 5 == 4 ? -1 : e * 7 % V;
        clp[e] = cid[e] < 0 ? -INFINITY : (float)(-uniform() * 3.0);
    }
    vpo_beam_step(cid, clp, sc, S, B, kb, os, op, ot);
    CHECK(os[0] >= os[1] && os[1] >= os[2] && op[0] >= 0 && op[0] < B);

    free(W); free(b); free(C); free(H); free(ids); free(g); free(oi); free(ol); free(oz); free(lse); free(all_z);
    free(fz); free(flags); free(U); free(uz); free(X); free(C0); free(Cout); free(Cbits); free(assign); free(top);
    free(aids);
    puts("oracle sanitizer run ok");
    return 0;
}
