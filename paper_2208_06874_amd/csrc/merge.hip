// Per-row merge of the partial results of the projection kernel: the
// log-sum-exp over the row's whole active set (steps 4-5 of the inference list
// in section 2.3: only listed tokens contribute) and the k best candidates in
// descending order (section 2.1), mapped back to token ids.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"
#include "wave_ops.h"

namespace {

constexpr float LOG2E = 1.4426950408889634f;
constexpr float LN2 = 0.6931471805599453f;
constexpr int MERGE_THREADS = 256;
constexpr int VP_MAX_TOPK_SLOTS = 32;   // largest k of the C ABI (checked on the host)

__device__ inline float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * LOG2E); }
// (without short-circuit evaluation: compares and selects instead of branches around the tie case)
__device__ inline bool entry_before(float v, int i, float v2, int i2) { return (v > v2) | ((v == v2) & (i < i2)); }

// One workgroup per row.  Thread t owns the parts t, t + 256, ...  The entries
// of its first part are copied to LDS in one batch of loads; every part lists
// its entries in (logit descending, position ascending) order, so a part only
// ever offers its first entry not yet taken, and a round is one workgroup-wide
// arg-max over those offers.
__global__ __launch_bounds__(MERGE_THREADS) void merge_kernel(
    VpSlabSet set, const VpRowPlan *__restrict__ rowplan, const VpPlanHeader *__restrict__ hdr,
    const float *__restrict__ partials, int k,
    int32_t *__restrict__ out_ids, float *__restrict__ out_logp)
{
    const VpRowPlan rp = rowplan[blockIdx.x];
    const int rpi = hdr->rows_per_item;
    const int tid = threadIdx.x;
    if (hdr->overflow) {
        // The plan did not fit its item list (a bound of the host side is wrong): rows would silently
        // lose candidates.  Make the call's results unusable instead; the flag stays in the workspace.
        if (tid < k) {
            out_ids[(size_t)rp.row * k + tid] = -1;
            out_logp[(size_t)rp.row * k + tid] = __builtin_nanf("");
        }
        return;
    }
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int nit = rp.nit;
    const int PFL = vp_partial_floats(k);
    const float *base = partials + ((size_t)rp.item0 * rpi + rp.local) * PFL;
    const size_t part_stride = (size_t)rp.stride * rpi * PFL;

    extern __shared__ float staged[];            // [2k][256]: entries of each thread's first part
    __shared__ float red_v[MERGE_THREADS / 64];
    __shared__ float red_s[MERGE_THREADS / 64];
    __shared__ float rnd_v[2][MERGE_THREADS / 64];    // the wavefronts' offers of a round; rounds alternate between
    __shared__ int rnd_i[2][MERGE_THREADS / 64];      // two sets, so one barrier per round is enough
    __shared__ float win_v[VP_MAX_TOPK_SLOTS];        // the winners of the k rounds, written out together at the end
    __shared__ int win_i[VP_MAX_TOPK_SLOTS];

    float m = VP_NEG_BIG, s = 0.f;
    if (tid < nit) {
        const float *pp = base + tid * part_stride;
        m = pp[0];
        s = pp[1];
        for (int e = 0; e < 2 * k; ++e) staged[e * MERGE_THREADS + tid] = pp[2 + e];
    }
    for (int c = tid + MERGE_THREADS; c < nit; c += MERGE_THREADS) {
        const float *pp = base + c * part_stride;
        const float m2 = pp[0], s2 = pp[1];
        const float mn = fmaxf(m, m2);
        s = s * fast_exp(m - mn) + s2 * fast_exp(m2 - mn);
        m = mn;
    }
    // log-sum-exp over all parts
    wave_log_sum_exp(m, s);
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
    const float lse = M + __builtin_amdgcn_logf(S) * LN2;   // (red_v / red_s are not written again)

    // (in the masked full projection candidate positions are token ids already)
    const int32_t *ids = (set.ids && hdr->mode == 0) ? set.ids + rp.ids_off : nullptr;

    int pos = 0;                                  // entries of the first part already taken
    float cv = -__builtin_inff();
    int ci = VP_IDX_NONE;
    if (tid < nit) {
        cv = staged[tid];
        ci = __float_as_int(staged[k * MERGE_THREADS + tid]);
    }
    float pv = __builtin_inff();
    int pi = -1;
    for (int t = 0; t < k; ++t) {
        float bv = cv;
        int bi = ci;
        // parts beyond the first of this thread (only when a row has more than 256 parts)
        for (int c = tid + MERGE_THREADS; c < nit; c += MERGE_THREADS) {
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
        wave_best_entry(bv, bi);
        const float *rv = rnd_v[t & 1];
        const int *ri = rnd_i[t & 1];
        if (lane == 0) {
            rnd_v[t & 1][wave] = bv;
            rnd_i[t & 1][wave] = bi;
        }
        __syncthreads();   // (the set written next round was last read before this barrier)
        bv = rv[0];
        bi = ri[0];
#pragma unroll
        for (int w = 1; w < MERGE_THREADS / 64; ++w) {
            const bool take = entry_before(rv[w], ri[w], bv, bi);
            bv = take ? rv[w] : bv;
            bi = take ? ri[w] : bi;
        }
        if (tid == 0) {
            win_v[t] = bv;
            win_i[t] = bi;
        }
        if (bi != VP_IDX_NONE && ci == bi) {      // my first part won: offer its next entry
            ++pos;
            cv = pos < k ? staged[pos * MERGE_THREADS + tid] : -__builtin_inff();
            ci = pos < k ? __float_as_int(staged[(k + pos) * MERGE_THREADS + tid]) : VP_IDX_NONE;
        }
        pv = bv;
        pi = bi;
    }
    // Positions to token ids and the outputs, one thread per slot: the k look-ups are in flight
    // together (inside the rounds each would be waited for, k memory latencies one after the other:
    // 9 us instead of 3.5 us for a top-8 merge).
    __syncthreads();
    if (tid < k) {
        const float bv = win_v[tid];
        const int bi = win_i[tid];
        const bool real = bi != VP_IDX_NONE;
        out_ids[(size_t)rp.row * k + tid] = real ? (ids ? ids[bi] : bi) : -1;
        out_logp[(size_t)rp.row * k + tid] = real ? bv - lse : -__builtin_inff();
    }
}

}  // namespace

size_t vpk_merge_lds_bytes(int k) { return (size_t)2 * k * MERGE_THREADS * sizeof(float); }

hipError_t vpk_merge_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(merge_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024);
}

void vpk_merge(const VpSlabSet &set, const VpRowPlan *rowplan, const VpPlanHeader *hdr, const float *partials, int k,
               int N,
               int32_t *out_ids, float *out_logp, hipStream_t st)
{
    hipLaunchKernelGGL(merge_kernel, dim3(N), dim3(MERGE_THREADS), vpk_merge_lds_bytes(k), st, set, rowplan,
                       hdr, partials, k, out_ids, out_logp);
}
