/*
 * CPU oracle of the toy search consumer: one beam-search step over the sorted
 * candidates the projection returns (arxiv 2208.06874, section 2.1: the sorted
 * probabilities feed beam search, greedy search or sampling).
 *
 * TEST INFRASTRUCTURE ONLY, like the other oracle files: no code shared with
 * the HIP library, never called by the product path.
 *
 * The step is the textbook one.  For a sentence with B live hypotheses, each
 * with an accumulated log-probability score[b] and k candidate continuations
 * (token id, log-prob), the B best of the B*k sums score[b] + logp[b][j]
 * become the next hypotheses.  Order: sum descending, then hypothesis index
 * ascending, then candidate rank ascending.  Candidates with id < 0 do not
 * exist.  The sum is one single-precision addition (the precision the library
 * computes it in; a single IEEE addition is the same on both sides), the
 * ranking is done on that float.  Missing hypotheses: score -inf, parent -1,
 * token -1.
 *
 * Pins (see tests): a hand-computed step, numpy's lexsort on random inputs,
 * B = 1 (greedy: the best candidate of the only hypothesis), ties.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>

typedef struct {
    float sum;
    int b, j;
} vpo_cont;

static int cont_before(const vpo_cont *x, const vpo_cont *y)
{
    if (x->sum != y->sum) return x->sum > y->sum;
    if (x->b != y->b) return x->b < y->b;
    return x->j < y->j;
}

void vpo_beam_step(const int32_t *cand_ids, const float *cand_logp, const float *scores, int S, int B, int k,
                   float *out_scores, int32_t *out_parent, int32_t *out_token)
{
    vpo_cont *c = (vpo_cont *)malloc(sizeof(vpo_cont) * (size_t)B * k);
    for (int s = 0; s < S; ++s) {
        int n = 0;
        for (int b = 0; b < B; ++b) {
            for (int j = 0; j < k; ++j) {
                const size_t at = ((size_t)s * B + b) * k + j;
                if (cand_ids[at] < 0) continue;
                c[n].sum = scores[(size_t)s * B + b] + cand_logp[at];   /* one float addition */
                c[n].b = b;
                c[n].j = j;
                ++n;
            }
        }
        /* selection sort of the first B places: plain and obviously right */
        for (int t = 0; t < B; ++t) {
            const size_t o = (size_t)s * B + t;
            int best = -1;
            for (int i = t; i < n; ++i)
                if (best < 0 || cont_before(&c[i], &c[best])) best = i;
            if (best < 0 || isnan(c[best].sum) || c[best].sum == -INFINITY) {
                out_scores[o] = -INFINITY;
                out_parent[o] = -1;
                out_token[o] = -1;
                /* everything left is -inf too (or nothing is left) */
                for (int u = t + 1; u < B; ++u) {
                    out_scores[(size_t)s * B + u] = -INFINITY;
                    out_parent[(size_t)s * B + u] = -1;
                    out_token[(size_t)s * B + u] = -1;
                }
                break;
            }
            vpo_cont tmp = c[t];
            c[t] = c[best];
            c[best] = tmp;
            out_scores[o] = c[t].sum;
            out_parent[o] = c[t].b;
            out_token[o] = cand_ids[((size_t)s * B + c[t].b) * k + c[t].j];
        }
    }
    free(c);
}
