// The paper's own batched form of the inference list (section 2.3): the active
// sets of the predicted clusters of all rows of the batch are united and every
// row is projected onto the union.
//
// As in the paper, the union is formed with a boolean list over the vocabulary
// (bit-packed here): it starts all zero, threads switch on the bits of every
// active token of every predicted cluster (by OR-ing the clusters' membership
// bit lists), and a prefix scan over the list yields the reduced column set U in
// ascending order.  The columns of U are
// then gathered from the packed copy of W into a slab in the workspace, and
// the projection / log-softmax / top-k kernels run on that slab with all rows
// in one bucket, so every row is normalised over U (tokens outside U are at
// -infinity, steps 4-5).
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "vp_kernels.h"
#include "plan_common.h"
#include "wave_ops.h"

namespace {

constexpr int UNION_THREADS = 1024;

// Finishes Eq. 2 (minimum over the centroid parts), lists the occupied clusters
// and clears the boolean list.
__global__ __launch_bounds__(UNION_THREADS) void union_prepare_kernel(
    const int2 *__restrict__ cpart, int parts, int N, int K, int mask_words, int32_t *__restrict__ g,
    int32_t *__restrict__ out_cluster, int32_t *__restrict__ occ, VpUnionHeader *__restrict__ uh,
    unsigned int *__restrict__ mask, int32_t *__restrict__ zero_g)
{
    extern __shared__ int seen[];   // [K]
    __shared__ int n_occ;
    const int tid = threadIdx.x;
    for (int j = tid; j < K; j += UNION_THREADS) seen[j] = 0;
    for (int w = tid; w < mask_words; w += UNION_THREADS) mask[w] = 0;
    if (tid == 0) n_occ = 0;
    __syncthreads();
    for (int r = tid; r < N; r += UNION_THREADS) {
        float bs = __builtin_inff();
        int bj = VP_IDX_NONE;
        for (int p = 0; p < parts; ++p) {
            const int2 e = cpart[(size_t)r * parts + p];
            const float s = __int_as_float(e.x);
            if (s < bs || (s == bs && e.y < bj)) {
                bs = s;
                bj = e.y;
            }
        }
        if (bj < 0 || bj >= K) bj = 0;
        g[r] = bj;
        if (out_cluster) out_cluster[r] = bj;
        zero_g[r] = 0;   // every row reads the one boolean list when the union is projected as a masked full projection
        seen[bj] = 1;
    }
    __syncthreads();
    for (int j = tid; j < K; j += UNION_THREADS)
        if (seen[j]) occ[atomicAdd(&n_occ, 1)] = j;   // any order: the boolean list does not care
    __syncthreads();
    if (tid == 0) uh->n_occ = n_occ;
}

// Switches on the bits of the active tokens of every occupied cluster: the index keeps one
// membership bit list per cluster, so the boolean list is the OR of the occupied clusters'
// lists.  A thread owns one 32-bit word; blockIdx.y splits the clusters.
constexpr int UNION_OR_SPLIT = 8;
constexpr int UNION_BLOCK_WORDS = 256;   // words of the boolean list per workgroup of the scan kernels

__global__ __launch_bounds__(256) void union_flag_kernel(const int32_t *__restrict__ occ,
                                                         const VpUnionHeader *__restrict__ uh,
                                                         const uint32_t *__restrict__ bitmaps, int bm_words,
                                                         int mask_words, unsigned int *__restrict__ mask)
{
    const int w = blockIdx.x * 256 + threadIdx.x;
    if (w >= mask_words) return;
    const int n_occ = uh->n_occ;
    unsigned int acc = 0;
    int c = blockIdx.y;
    for (; c + 3 * UNION_OR_SPLIT < n_occ; c += 4 * UNION_OR_SPLIT) {   // four lists in flight
        const int j0 = occ[c], j1 = occ[c + UNION_OR_SPLIT], j2 = occ[c + 2 * UNION_OR_SPLIT],
                  j3 = occ[c + 3 * UNION_OR_SPLIT];
        const unsigned int b0 = bitmaps[(size_t)j0 * bm_words + w], b1 = bitmaps[(size_t)j1 * bm_words + w],
                           b2 = bitmaps[(size_t)j2 * bm_words + w], b3 = bitmaps[(size_t)j3 * bm_words + w];
        acc |= (b0 | b1) | (b2 | b3);
    }
    for (; c < n_occ; c += UNION_OR_SPLIT) acc |= bitmaps[(size_t)occ[c] * bm_words + w];
    if (acc) atomicOr(&mask[w], acc);
}

// Prefix scan over the boolean list in three steps: set bits per block of the list, scan of
// the block counts (with the plan of the projection over U), and the ascending ids.
__global__ __launch_bounds__(256) void union_count_kernel(const unsigned int *__restrict__ mask, int mask_words,
                                                          int32_t *__restrict__ bsum)
{
    __shared__ int part[4];
    const int w = blockIdx.x * UNION_BLOCK_WORDS + threadIdx.x;
    int c = w < mask_words ? __popc(mask[w]) : 0;
    c = wave_sum(c);
    if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = c;
    __syncthreads();
    if (threadIdx.x == 0) bsum[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

__global__ __launch_bounds__(UNION_THREADS) void union_compact_kernel(
    int32_t *__restrict__ bsum, int blocks, int N, int rpi, int target_items, int min_items, int max_items,
    int32_t *__restrict__ uids, VpUnionHeader *__restrict__ uh, int32_t *__restrict__ out_union_size,
    int32_t *__restrict__ perm, VpRowPlan *__restrict__ rowplan, unsigned int *__restrict__ floors,
    VpItem *__restrict__ items, VpPlanHeader *__restrict__ hdr, int allow_full, int V, int vtiles, int k,
    VpCostModel cost, int max_items_full)
{
    __shared__ int wsum[UNION_THREADS / 64 + 1];
    __shared__ int carry_s;
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    if (tid == 0) carry_s = 0;
    __syncthreads();
    // exclusive scan of the block counts, in place
    for (int base = 0; base < blocks; base += UNION_THREADS) {
        const int b = base + tid;
        const int v = b < blocks ? bsum[b] : 0;
        const int inc = wave_inclusive_sum(v);
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        if (tid == 0) {
            int run = carry_s;
            for (int w = 0; w < UNION_THREADS / 64; ++w) {
                const int t = wsum[w];
                wsum[w] = run;
                run += t;
            }
            wsum[UNION_THREADS / 64] = run;
        }
        __syncthreads();
        if (b < blocks) bsum[b] = wsum[wave] + inc - v;
        __syncthreads();
        if (tid == 0) carry_s = wsum[UNION_THREADS / 64];
        __syncthreads();
    }
    const int nU = carry_s;
    const int tiles = (nU + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS;
    for (int c = nU + tid; c < tiles * VP_TILE_ITEMS; c += UNION_THREADS) uids[c] = -1;   // pad the last group
    if (tid == 0) {
        uh->n_union = nU;
        uh->tiles = tiles;
        if (out_union_size) *out_union_size = nU;
    }
    // A large union is cheaper projected in place: the full projection with the boolean list as
    // every row's mask streams W once and gathers nothing (same results: tokens outside U are at
    // -infinity either way).  Per candidate group the projection costs the same in both forms.
    if (allow_full) {
        const int rgs = ceil_div(N, rpi);
        const float per_group = rpi >= 64 ? (1.f / cost.bw_full + (rgs - 1) / cost.bw_gemm) * (1.f + k * 0.0625f)
                                          : fmaxf(1.f / cost.bw_full, rgs / cost.bw_l2) * (1.f + k * 0.125f);
        const float t_union = cost.t_gather + tiles * (1.f / cost.bw_gather + per_group);
        const float t_full = vtiles * per_group;
        if (t_full < t_union) {
            __syncthreads();   // uh->tiles = 0 below must come after the write above
            if (tid == 0) uh->tiles = 0;   // nothing to gather
            vp_plan_single_bucket(N, V, vtiles, rpi, target_items, min_items, max_items_full, perm, rowplan, floors,
                                  items, hdr, nullptr, tid, UNION_THREADS);
            if (tid == 0) hdr->mode = 1;
            return;
        }
    }
    vp_plan_single_bucket(N, nU, tiles, rpi, target_items, min_items, max_items, perm, rowplan, floors, items, hdr,
                          nullptr, tid, UNION_THREADS);
}

// U in ascending order: every block of the list writes its ids behind those of the blocks before it.
__global__ __launch_bounds__(256) void union_emit_kernel(const unsigned int *__restrict__ mask, int mask_words,
                                                         const int32_t *__restrict__ boff, int32_t *__restrict__ uids)
{
    __shared__ int part[4];
    const int w = blockIdx.x * UNION_BLOCK_WORDS + threadIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    unsigned int bits = w < mask_words ? mask[w] : 0u;
    const int c = __popc(bits);
    const int inc = wave_inclusive_sum(c);
    if (lane == 63) part[wave] = inc;
    __syncthreads();
    int pos = boff[blockIdx.x] + inc - c;
    for (int x = 0; x < wave; ++x) pos += part[x];
    while (bits) {
        const int b = __ffs(bits) - 1;
        bits &= bits - 1;
        uids[pos++] = w * 32 + b;
    }
}

// Gathers the columns of U into the union slab (packed tile layout), with their bias.  The
// columns come from the token-major copy of W, where a token's k-values are one contiguous row
// (in the packed tiles they are interleaved with those of 15 other tokens, and a gather from
// there fetches four to eight times the bytes it uses).  A workgroup takes groups of 16 union
// tokens in turn.
__global__ __launch_bounds__(256) void union_gather_kernel(
    const uint4 *__restrict__ wt, const float *__restrict__ bias_full, int kt_count,
    const int32_t *__restrict__ uids, const VpUnionHeader *__restrict__ uh, uint4 *__restrict__ slab,
    float *__restrict__ ubias)
{
    const int tiles = uh->tiles;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int q = lane >> 4;
    for (int group = blockIdx.x; group < tiles; group += gridDim.x) {
        const int v = uids[group * VP_TILE_ITEMS + (lane & 15)];
        if (threadIdx.x < 16) ubias[group * VP_TILE_ITEMS + lane] = v >= 0 ? bias_full[v] : 0.f;
        const uint4 *row = wt + (size_t)(v >= 0 ? v : 0) * (kt_count * 4) + q;
        for (int kt = wave; kt < kt_count; kt += VP_WG_WAVES) {
            uint4 o = make_uint4(0, 0, 0, 0);
            if (v >= 0) o = row[kt * 4];
            slab[((size_t)group * kt_count + kt) * 64 + lane] = o;
        }
    }
}

}  // namespace

hipError_t vpk_union_prepare()
{
    return hipFuncSetAttribute(reinterpret_cast<const void *>(union_prepare_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 32 * 1024);
}

void vpk_union_mark(const void *cpart, int parts, int N, int K, int mask_words, int32_t *g, int32_t *out_cluster,
                    int32_t *occ, VpUnionHeader *uh, unsigned int *mask, int32_t *zero_g, hipStream_t st)
{
    hipLaunchKernelGGL(union_prepare_kernel, dim3(1), dim3(UNION_THREADS), (size_t)K * sizeof(int), st,
                       (const int2 *)cpart, parts, N, K, mask_words, g, out_cluster, occ, uh, mask, zero_g);
}

void vpk_union_flags(const int32_t *occ, const VpUnionHeader *uh, const uint32_t *bitmaps, int bm_words,
                     int mask_words, unsigned int *mask, hipStream_t st)
{
    dim3 grid((mask_words + 255) / 256, UNION_OR_SPLIT);
    hipLaunchKernelGGL(union_flag_kernel, grid, dim3(256), 0, st, occ, uh, bitmaps, bm_words, mask_words, mask);
}

int vpk_union_blocks(int mask_words) { return (mask_words + UNION_BLOCK_WORDS - 1) / UNION_BLOCK_WORDS; }

void vpk_union_compact(const unsigned int *mask, int mask_words, int32_t *bsum, int N, int rpi, int target_items,
                       int min_items, int max_items, int32_t *uids, VpUnionHeader *uh, int32_t *out_union_size,
                       int32_t *perm, VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr,
                       int allow_full, int V, int vtiles, int k, const VpCostModel &cost, int max_items_full,
                       hipStream_t st)
{
    const int blocks = vpk_union_blocks(mask_words);
    hipLaunchKernelGGL(union_count_kernel, dim3(blocks), dim3(256), 0, st, mask, mask_words, bsum);
    hipLaunchKernelGGL(union_compact_kernel, dim3(1), dim3(UNION_THREADS), 0, st, bsum, blocks, N, rpi, target_items,
                       min_items, max_items, uids, uh, out_union_size, perm, rowplan, floors, items, hdr, allow_full, V,
                       vtiles, k, cost, max_items_full);
    hipLaunchKernelGGL(union_emit_kernel, dim3(blocks), dim3(256), 0, st, mask, mask_words, bsum, uids);
}

void vpk_union_gather(const void *wt, const float *bias_full, int kt, const int32_t *uids, const VpUnionHeader *uh,
                      int max_groups, void *slab, float *ubias, hipStream_t st)
{
    const int grid = max_groups < 4096 ? max_groups : 4096;   // |U| is not known here
    hipLaunchKernelGGL(union_gather_kernel, dim3(grid), dim3(256), 0, st, (const uint4 *)wt, bias_full, kt, uids,
                       uh, (uint4 *)slab, ubias);
}
