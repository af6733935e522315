// Per-row merge of the partial results of the projection kernel: the
// log-sum-exp over the row's whole active set (steps 4-5 of the inference list
// in section 2.3: only listed tokens contribute) and the k best candidates in
// descending order (section 2.1), mapped back to token ids.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int MERGE_THREADS = 256;

__device__ inline float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * LOG2E); }
__device__ inline bool entry_before(float v, int i, float v2, int i2) { return v > v2 || (v == v2 && i < i2); }

__global__ __launch_bounds__(MERGE_THREADS) void merge_kernel(
    VpSlabSet set, const int32_t *__restrict__ perm, const int32_t *__restrict__ g,
    const int32_t *__restrict__ row_item0, const int32_t *__restrict__ row_stride,
    const int32_t *__restrict__ row_nit, const VpItem *__restrict__ items,
    const float *__restrict__ partials, int k, int32_t *__restrict__ out_ids, float *__restrict__ out_logp)
{
    const int p = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int row = perm[p];
    const int cluster = g ? g[row] : 0;
    const int item0 = row_item0[p];
    const int stride = row_stride[p];
    const int nit = row_nit[p];
    const int nloc = p - items[item0].perm_start;
    const int PFL = vp_partial_floats(k);
    const float *base = partials + ((size_t)item0 * VP_ROWS_PER_ITEM + nloc) * PFL;
    const size_t part_stride = (size_t)stride * VP_ROWS_PER_ITEM * PFL;

    __shared__ float red_v[MERGE_THREADS / 64];
    __shared__ float red_s[MERGE_THREADS / 64];
    __shared__ int red_i[MERGE_THREADS / 64];

    // log-sum-exp over all parts
    float m = VP_NEG_BIG, s = 0.f;
    for (int c = tid; c < nit; c += MERGE_THREADS) {
        const float *pp = base + c * part_stride;
        const float m2 = pp[0], s2 = pp[1];
        const float mn = fmaxf(m, m2);
        s = s * fast_exp(m - mn) + s2 * fast_exp(m2 - mn);
        m = mn;
    }
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        const float m2 = __shfl_xor(m, off), s2 = __shfl_xor(s, off);
        const float mn = fmaxf(m, m2);
        s = s * fast_exp(m - mn) + s2 * fast_exp(m2 - mn);
        m = mn;
    }
    if (lane == 0) {
        red_v[wave] = m;
        red_s[wave] = s;
    }
    __syncthreads();
    float M = red_v[0];
#pragma unroll
    for (int w = 1; w < MERGE_THREADS / 64; ++w) M = fmaxf(M, red_v[w]);
    float S = 0.f;
#pragma unroll
    for (int w = 0; w < MERGE_THREADS / 64; ++w) S += red_s[w] * fast_exp(red_v[w] - M);
    const float lse = M + __builtin_amdgcn_logf(S) * LN2;
    __syncthreads();

    const int32_t *ids = set.ids ? set.ids + (size_t)set.tile_off[cluster] * VP_TILE_ITEMS : nullptr;

    // k rounds: the best entry that comes after the previous winner.  Every part
    // lists its entries in that order already, so its first such entry is its best.
    float pv = __builtin_inff();
    int pi = -1;
    for (int t = 0; t < k; ++t) {
        float bv = -__builtin_inff();
        int bi = VP_IDX_NONE;
        for (int c = tid; c < nit; c += MERGE_THREADS) {
            const float *pp = base + c * part_stride;
            for (int e = 0; e < k; ++e) {
                const float v = pp[2 + e];
                const int i = __float_as_int(pp[2 + k + e]);
                if (v < pv || (v == pv && i > pi)) {
                    if (entry_before(v, i, bv, bi)) {
                        bv = v;
                        bi = i;
                    }
                    break;
                }
            }
        }
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float v2 = __shfl_xor(bv, off);
            const int i2 = __shfl_xor(bi, off);
            if (entry_before(v2, i2, bv, bi)) {
                bv = v2;
                bi = i2;
            }
        }
        if (lane == 0) {
            red_v[wave] = bv;
            red_i[wave] = bi;
        }
        __syncthreads();
        bv = red_v[0];
        bi = red_i[0];
#pragma unroll
        for (int w = 1; w < MERGE_THREADS / 64; ++w) {
            if (entry_before(red_v[w], red_i[w], bv, bi)) {
                bv = red_v[w];
                bi = red_i[w];
            }
        }
        __syncthreads();
        if (tid == 0) {
            const bool real = bi != VP_IDX_NONE;
            out_ids[(size_t)row * k + t] = real ? (ids ? ids[bi] : bi) : -1;
            out_logp[(size_t)row * k + t] = real ? bv - lse : -__builtin_inff();
        }
        pv = bv;
        pi = bi;
    }
}

}  // namespace

void vpk_merge(const VpSlabSet &set, const int32_t *perm, const int32_t *g, const int32_t *row_item0,
               const int32_t *row_stride, const int32_t *row_nit, const VpItem *items, const float *partials,
               int k, int N, int32_t *out_ids, float *out_logp, hipStream_t st)
{
    hipLaunchKernelGGL(merge_kernel, dim3(N), dim3(MERGE_THREADS), 0, st, set, perm, g, row_item0, row_stride,
                       row_nit, items, partials, k, out_ids, out_logp);
}
