// Toy search consumer: one beam-search step over the sorted candidates the
// projection returns (section 2.1: the sorted probabilities feed beam search,
// greedy search or sampling).  For every sentence the B best of the B * k sums
// score[b] + logp[b][j] become the next hypotheses; order: sum descending, then
// hypothesis index, then candidate rank.  One workgroup per sentence keeps all
// continuations in registers and selects B times.
#include <hip/hip_runtime.h>

#include "vp.h"
#include "vp_kernels.h"
#include "wave_ops.h"

namespace {

constexpr int BEAM_THREADS = 256;
constexpr int BEAM_PER_THREAD = 8;   // B * k <= 2048

// (without short-circuit evaluation: compares and selects instead of branches around the tie case)
__device__ inline bool cont_before(float v, int c, float v2, int c2) { return (v > v2) | ((v == v2) & (c < c2)); }

__global__ __launch_bounds__(BEAM_THREADS) void beam_step_kernel(
    const int32_t *__restrict__ cand_ids, const float *__restrict__ cand_logp, const float *__restrict__ scores, int B,
    int k, float *__restrict__ out_scores, int32_t *__restrict__ out_parent, int32_t *__restrict__ out_token)
{
    const int s = blockIdx.x;
    const int n = B * k;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const size_t base = (size_t)s * n;
    float sum[BEAM_PER_THREAD];
#pragma unroll
    for (int u = 0; u < BEAM_PER_THREAD; ++u) {
        const int c = threadIdx.x + u * BEAM_THREADS;   // continuation number b * k + j
        sum[u] = -__builtin_inff();
        if (c < n && cand_ids[base + c] >= 0) sum[u] = scores[(size_t)s * B + c / k] + cand_logp[base + c];
    }
    __shared__ float wv[4];
    __shared__ int wc[4];
    __shared__ float win_v[BEAM_THREADS * BEAM_PER_THREAD];   // the winners of the B rounds (B <= B * k <= 2048)
    __shared__ int win_c[BEAM_THREADS * BEAM_PER_THREAD];
    float pv = __builtin_inff();
    int pc = -1;
    for (int t = 0; t < B; ++t) {
        float bv = -__builtin_inff();
        int bc = 0x7fffffff;
#pragma unroll
        for (int u = 0; u < BEAM_PER_THREAD; ++u) {
            const int c = threadIdx.x + u * BEAM_THREADS;
            const bool after_prev = (sum[u] < pv) | ((sum[u] == pv) & (c > pc));
            const bool take = (c < n) & after_prev & cont_before(sum[u], c, bv, bc);
            bv = take ? sum[u] : bv;
            bc = take ? c : bc;
        }
        wave_best_entry(bv, bc);   // (sum descending, continuation ascending)
        __syncthreads();   // the previous round's wv / wc have been read
        if (lane == 0) {
            wv[wave] = bv;
            wc[wave] = bc;
        }
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const bool take = cont_before(wv[w], wc[w], bv, bc);
            bv = take ? wv[w] : bv;
            bc = take ? wc[w] : bc;
        }
        if (threadIdx.x == 0) {
            win_v[t] = bv;
            win_c[t] = bc;
        }
        pv = bv;
        pc = bc;
    }
    // the outputs, one thread per hypothesis: the token look-ups are in flight together instead of
    // one memory latency per round
    __syncthreads();
    for (int t = threadIdx.x; t < B; t += BEAM_THREADS) {
        const float bv = win_v[t];
        const int bc = win_c[t];
        const size_t o = (size_t)s * B + t;
        const bool none = bc == 0x7fffffff || bv == -__builtin_inff();
        out_scores[o] = none ? -__builtin_inff() : bv;
        out_parent[o] = none ? -1 : bc / k;
        out_token[o] = none ? -1 : cand_ids[base + bc];
    }
}

}  // namespace

extern "C" vp_status vp_beam_step(const int32_t *cand_ids, const float *cand_logp, const float *scores, int32_t S,
                                  int32_t B, int32_t k, float *out_scores, int32_t *out_parent, int32_t *out_token,
                                  void *hip_stream)
{
    if (S < 0 || B < 1 || k < 1 || k > VP_MAX_TOPK || (long)B * k > BEAM_THREADS * BEAM_PER_THREAD)
        return (vp_status)vpi_fail(VP_ERR_UNSUPPORTED, "vp_beam_step: S = %d, B = %d, k = %d (need B * k <= %d, k <= %d)", S, B, k,
                                   BEAM_THREADS * BEAM_PER_THREAD, VP_MAX_TOPK);
    if (S == 0) return VP_OK;
    if (!cand_ids || !cand_logp || !scores || !out_scores || !out_parent || !out_token)
        return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "vp_beam_step: null pointer argument");
    hipLaunchKernelGGL(beam_step_kernel, dim3(S), dim3(BEAM_THREADS), 0, (hipStream_t)hip_stream, cand_ids, cand_logp,
                       scores, B, k, out_scores, out_parent, out_token);
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (vp_status)vpi_fail(VP_ERR_HIP, "vp_beam_step: %s", hipGetErrorString(e));
    return VP_OK;
}
