// The paper's own batched form of the inference list (section 2.3): the active
// sets of the predicted clusters of all rows of the batch are united and every
// row is projected onto the union.
//
// As in the paper, the union is formed with a boolean list over the vocabulary
// (bit-packed here): the bits of every active token of every predicted cluster
// are switched on (by OR-ing the clusters' membership bit lists), and a prefix
// scan over the list yields the reduced column set U in ascending order.  Two
// launches do all of that (clusters + list + counts; scan + ids + plan).  The projection /
// log-softmax / top-k kernels then run with all rows in one bucket over the columns of U, so
// every row is normalised over U (tokens outside U are at -infinity, steps 4-5): the 64-row
// kernel reads the columns in place from the copy of W that holds one contiguous row per
// token; where that kernel is not built they are first gathered into a slab in the workspace.
#include <hip/hip_runtime.h>
#include <hip/hip_fp16.h>
#include "vp_kernels.h"
#include "plan_common.h"
#include "wave_ops.h"

namespace {

constexpr int UNION_THREADS = 256;
constexpr int UNION_BLOCK_WORDS = 256;   // words of the boolean list per workgroup
constexpr int UNION_LISTS_IN_FLIGHT = 32;

// Steps 1-2 of the inference list in one launch.  Every workgroup owns 256 words of the boolean
// list and builds them from scratch: it finishes Eq. 2 for all rows itself (minimum over the
// centroid parts; a few kilobytes, cheaper than a kernel of its own and a trip through memory),
// marks the occupied clusters in LDS, ORs the occupied clusters' membership lists word by word
// (no atomics, nothing to clear beforehand), and leaves the number of set bits of its block for
// the prefix scan.  Workgroup 0 also writes the clusters.
__global__ __launch_bounds__(UNION_THREADS) void union_mark_kernel(
    const int2 *__restrict__ cpart, int parts, int N, int K, const uint32_t *__restrict__ bitmaps, int bm_words,
    int mask_words, int32_t *__restrict__ g, int32_t *__restrict__ out_cluster, int32_t *__restrict__ zero_g,
    unsigned int *__restrict__ mask, int32_t *__restrict__ bsum)
{
    extern __shared__ int sm[];
    int *seen = sm;            // [K]
    int *occ = sm + K;         // [min(N, K)] occupied clusters, any order
    __shared__ int n_occ_s;
    __shared__ int part[UNION_THREADS / 64];
    const int tid = threadIdx.x;
    for (int j = tid; j < K; j += UNION_THREADS) seen[j] = 0;
    if (tid == 0) n_occ_s = 0;
    __syncthreads();
    const bool first = blockIdx.x == 0;
    vp_finish_eq2(cpart, parts, N, K, tid, UNION_THREADS, [&](int r, int j) {
        seen[j] = 1;
        if (first) {
            g[r] = j;
            if (out_cluster) out_cluster[r] = j;
            zero_g[r] = 0;   // every row reads the one boolean list when the union is projected as a masked full projection
        }
    });
    __syncthreads();
    for (int j = tid; j < K; j += UNION_THREADS)
        if (seen[j]) occ[atomicAdd(&n_occ_s, 1)] = j;   // any order: the boolean list does not care
    __syncthreads();
    const int n_occ = n_occ_s;
    const int w = blockIdx.x * UNION_BLOCK_WORDS + tid;
    unsigned int acc = 0;
    if (w < mask_words) {
        int c = 0;
        for (; c + UNION_LISTS_IN_FLIGHT <= n_occ; c += UNION_LISTS_IN_FLIGHT) {
            unsigned int b[UNION_LISTS_IN_FLIGHT];
#pragma unroll
            for (int u = 0; u < UNION_LISTS_IN_FLIGHT; ++u) b[u] = bitmaps[(size_t)occ[c + u] * bm_words + w];
#pragma unroll
            for (int u = 0; u < UNION_LISTS_IN_FLIGHT; ++u) acc |= b[u];
        }
        for (; c < n_occ; ++c) acc |= bitmaps[(size_t)occ[c] * bm_words + w];
        mask[w] = acc;
    }
    const int cnt = wave_sum(__popc(acc));
    if ((tid & 63) == 0) part[tid >> 6] = cnt;
    __syncthreads();
    if (tid == 0) bsum[blockIdx.x] = part[0] + part[1] + part[2] + part[3];
}

// The prefix scan over the boolean list and U in ascending order, in one launch: every block of
// the list adds up the counts of the blocks before it itself (a few hundred numbers) and writes
// its ids behind theirs.  The last block then knows |U|: it pads U's last group, decides between
// the gathered and the in-place form and plans the projection.
__global__ __launch_bounds__(UNION_THREADS) void union_emit_kernel(
    const unsigned int *__restrict__ mask, int mask_words, const int32_t *__restrict__ bsum, int N, int rpi,
    int target_items, int min_items, int max_items, int32_t *__restrict__ uids, VpUnionHeader *__restrict__ uh,
    int32_t *__restrict__ out_union_size, int32_t *__restrict__ perm, VpRowPlan *__restrict__ rowplan,
    unsigned int *__restrict__ floors, VpItem *__restrict__ items, VpPlanHeader *__restrict__ hdr, int allow_full,
    int V, int vtiles, int k, VpCostModel cost, int max_items_full, const float *__restrict__ bias_full,
    float *__restrict__ ubias)
{
    __shared__ int part[UNION_THREADS / 64];
    __shared__ int before[UNION_THREADS / 64];
    const int tid = threadIdx.x;
    const int lane = tid & 63, wave = tid >> 6;
    int mine = 0;
    for (int b = tid; b < (int)blockIdx.x; b += UNION_THREADS) mine += bsum[b];
    mine = wave_sum(mine);
    const int w = blockIdx.x * UNION_BLOCK_WORDS + tid;
    unsigned int bits = w < mask_words ? mask[w] : 0u;
    const int c = __popc(bits);
    const int inc = wave_inclusive_sum(c);
    if (lane == 63) part[wave] = inc;
    if (lane == 0) before[wave] = mine;
    __syncthreads();
    const int boff = before[0] + before[1] + before[2] + before[3];
    int pos = boff + inc - c;
    for (int x = 0; x < wave; ++x) pos += part[x];
    while (bits) {
        const int b = __ffs(bits) - 1;
        bits &= bits - 1;
        uids[pos] = w * 32 + b;
        ubias[pos] = bias_full[w * 32 + b];   // step 3 substitutes the reduced bias too
        ++pos;
    }
    if (blockIdx.x != gridDim.x - 1) return;

    const int nU = boff + part[0] + part[1] + part[2] + part[3];
    const int tiles = (nU + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS;
    for (int e = nU + tid; e < tiles * VP_TILE_ITEMS; e += UNION_THREADS) {   // pad the last group
        uids[e] = -1;
        ubias[e] = 0.f;
    }
    if (tid == 0 && out_union_size) *out_union_size = nU;
    // A large union is cheaper projected in place: the full projection with the boolean list as
    // every row's mask streams W once and gathers nothing (same results: tokens outside U are at
    // -infinity either way).  Per candidate group the projection costs the same in both forms.
    if (allow_full) {
        const int rgs = ceil_div(N, rpi);
        const float per_group = rpi >= 48 ? fmaxf(1.f / cost.bw_full, rgs / cost.bw_gemm) * (1.f + k * 0.0125f)
                                          : fmaxf(1.f / cost.bw_full, rgs / cost.bw_l2) * (1.f + k * 0.125f);
        const float t_union = cost.t_gather + tiles * (1.f / cost.bw_gather + per_group);
        const float t_full = vtiles * per_group;
        if (t_full < t_union) {
            if (tid == 0) {
                uh->n_union = nU;
                uh->tiles = 0;   // nothing to gather
            }
            vp_plan_single_bucket(N, V, vtiles, rpi, target_items, min_items, max_items_full, perm, rowplan, floors,
                                  items, hdr, nullptr, tid, UNION_THREADS);
            __syncthreads();   // the header's mode after the planner's own write of it
            if (tid == 0) hdr->mode = 1;
            return;
        }
    }
    if (tid == 0) {
        uh->n_union = nU;
        uh->tiles = tiles;
    }
    vp_plan_single_bucket(N, nU, tiles, rpi, target_items, min_items, max_items, perm, rowplan, floors, items, hdr,
                          nullptr, tid, UNION_THREADS);
}

// Gathers the columns of U into the union slab (packed tile layout), for the projection kernels
// that want a packed slab (items of 16 or 32 rows, k-extents beyond d_pad = 1024).  The
// columns come from the token-major copy of W, where a token's k-values are one contiguous row
// (in the packed tiles they are interleaved with those of 15 other tokens, and a gather from
// there fetches four to eight times the bytes it uses).  A workgroup takes groups of 16 union
// tokens in turn.
__global__ __launch_bounds__(256) void union_gather_kernel(
    const uint4 *__restrict__ wt, int kt_count, const int32_t *__restrict__ uids,
    const VpUnionHeader *__restrict__ uh, uint4 *__restrict__ slab)
{
    const int tiles = uh->tiles;
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    const int q = lane >> 4;
    for (int group = blockIdx.x; group < tiles; group += gridDim.x) {
        const int v = uids[group * VP_TILE_ITEMS + (lane & 15)];
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
    return hipFuncSetAttribute(reinterpret_cast<const void *>(union_mark_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 64 * 1024);
}

int vpk_union_blocks(int mask_words) { return (mask_words + UNION_BLOCK_WORDS - 1) / UNION_BLOCK_WORDS; }

// steps 1-2: clusters, boolean list (OR of the occupied clusters' membership lists), set bits per block
void vpk_union_mark(const void *cpart, int parts, int N, int K, const uint32_t *bitmaps, int bm_words, int mask_words,
                    int32_t *g, int32_t *out_cluster, int32_t *zero_g, unsigned int *mask, int32_t *bsum,
                    hipStream_t st)
{
    const int blocks = vpk_union_blocks(mask_words);
    const size_t lds = (size_t)(K + (N < K ? N : K)) * sizeof(int);
    hipLaunchKernelGGL(union_mark_kernel, dim3(blocks), dim3(UNION_THREADS), lds, st, (const int2 *)cpart, parts, N, K,
                       bitmaps, bm_words, mask_words, g, out_cluster, zero_g, mask, bsum);
}

// prefix scan, U ascending, choice of the form, plan of the projection
void vpk_union_compact(const unsigned int *mask, int mask_words, const int32_t *bsum, int N, int rpi, int target_items,
                       int min_items, int max_items, int32_t *uids, VpUnionHeader *uh, int32_t *out_union_size,
                       int32_t *perm, VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr,
                       int allow_full, int V, int vtiles, int k, const VpCostModel &cost, int max_items_full,
                       const float *bias_full, float *ubias, hipStream_t st)
{
    const int blocks = vpk_union_blocks(mask_words);
    hipLaunchKernelGGL(union_emit_kernel, dim3(blocks), dim3(UNION_THREADS), 0, st, mask, mask_words, bsum, N, rpi,
                       target_items, min_items, max_items, uids, uh, out_union_size, perm, rowplan, floors, items, hdr,
                       allow_full, V, vtiles, k, cost, max_items_full, bias_full, ubias);
}

void vpk_union_gather(const void *wt, int kt, const int32_t *uids, const VpUnionHeader *uh, int max_groups, void *slab,
                      hipStream_t st)
{
    const int grid = max_groups < 4096 ? max_groups : 4096;   // |U| is not known here
    hipLaunchKernelGGL(union_gather_kernel, dim3(grid), dim3(256), 0, st, (const uint4 *)wt, kt, uids, uh,
                       (uint4 *)slab);
}
