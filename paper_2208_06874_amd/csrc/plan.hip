// Row bucketing by cluster and work planning (one workgroup, all in LDS).
//
// The paper unions the active sets of a batch (section 2.3); here each row is
// instead projected against its own cluster's slab, so rows are first grouped
// by cluster: histogram of the cluster ids -> exclusive prefix scan -> scatter
// of the row numbers into bucket order.  The same kernel finishes Eq. 2 (it
// reduces the per-part minima of the centroid kernel) and cuts the projection
// work into items of equal slab bytes: (bucket, group of up to 16 rows, range
// of candidate tiles).  The number of tiles per item adapts to the total work
// so that any batch, from one row to thousands, yields about `target_items`
// items.  The order of rows inside a bucket is the order in which the LDS
// atomics happen to be served; each row's result is independent of its slot.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"
#include "plan_common.h"
#include "wave_ops.h"

namespace {

constexpr int PLAN_THREADS = 1024;

// Exclusive prefix sum over the workgroup; returns this thread's prefix and the
// total to everyone.  wsum: LDS scratch of PLAN_THREADS / 64 + 1 elements.
template <typename T>
__device__ T block_exscan(T v, T *total, T *wsum)
{
    const int lane = threadIdx.x & 63;
    const int wave = threadIdx.x >> 6;
    T inc = v;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        T up = __shfl_up(inc, off);
        if (lane >= off) inc += up;
    }
    __syncthreads();   // wsum may still be read from a previous call
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    if (wave == 0) {
        const int nw = blockDim.x >> 6;
        T w = lane < nw ? wsum[lane] : T(0);
        T winc = w;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            T up = __shfl_up(winc, off);
            if (lane >= off) winc += up;
        }
        if (lane < nw) wsum[lane] = winc - w;
        if (lane == nw - 1) wsum[nw] = winc;
    }
    __syncthreads();
    *total = wsum[blockDim.x >> 6];
    return wsum[wave] + inc - v;
}


// The same scan for ints, two barriers: every wavefront scans the wavefront totals itself.
__device__ inline int block_exscan_int(int v, int *total, int *wsum)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    const int inc = wave_inclusive_sum(v);
    __syncthreads();   // wsum may still be read from a previous call
    if (lane == 63) wsum[wave] = inc;
    __syncthreads();
    const int w = lane < nw ? wsum[lane] : 0;
    const int winc = wave_inclusive_sum(w);
    *total = __builtin_amdgcn_readlane(winc, nw - 1);
    return __builtin_amdgcn_readlane(winc - w, wave) + inc - v;
}

// Sums of three per-thread values over the workgroup, to every thread.  wsum3: 3 x 16 ints.
__device__ inline void block_sum3(int a, int b, int c, int *ta, int *tb, int *tc, int *wsum3)
{
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int nw = blockDim.x >> 6;
    a = wave_inclusive_sum(a);
    b = wave_inclusive_sum(b);
    c = wave_inclusive_sum(c);
    __syncthreads();
    if (lane == 63) {
        wsum3[wave] = a;
        wsum3[16 + wave] = b;
        wsum3[32 + wave] = c;
    }
    __syncthreads();
    *ta = __builtin_amdgcn_readlane(wave_inclusive_sum(lane < nw ? wsum3[lane] : 0), nw - 1);
    *tb = __builtin_amdgcn_readlane(wave_inclusive_sum(lane < nw ? wsum3[16 + lane] : 0), nw - 1);
    *tc = __builtin_amdgcn_readlane(wave_inclusive_sum(lane < nw ? wsum3[32 + lane] : 0), nw - 1);
}

__global__ __launch_bounds__(PLAN_THREADS) void plan_kernel(
    const int2 *__restrict__ cpart, int parts, int N, int K, const int32_t *__restrict__ n_cand,
    const int32_t *__restrict__ tile_off, int target_items, int min_items, int max_items, int32_t *__restrict__ g,
    int32_t *__restrict__ out_cluster, int32_t *__restrict__ perm, VpRowPlan *__restrict__ rowplan,
    unsigned int *__restrict__ floors, VpItem *__restrict__ items, VpPlanHeader *__restrict__ hdr,
    int64_t *__restrict__ dbg_row_off, int dispatch, VpCostModel cost, int k, int V, int vtiles,
    int full_target_items, int full_min_items, int max_items_full)
{
    extern __shared__ int lds[];
    int *cnt = lds;             // [K]   rows per cluster, later the scatter cursor
    int *off = cnt + K;         // [K+1] first perm position of each bucket
    int *ioff = off + K + 1;    // [K+1] first item of each bucket
    int *tl = ioff + K + 1;     // [K]   candidate tiles of each cluster
    __shared__ int wsum[PLAN_THREADS / 64 + 1];
    __shared__ long long wsum64[PLAN_THREADS / 64 + 1];
    __shared__ int wsum3[48];
    __shared__ int max_rgs;     // most row groups any bucket has
    const int tid = threadIdx.x;

    if (tid == 0) max_rgs = 0;
    for (int j = tid; j < K; j += PLAN_THREADS) {
        cnt[j] = 0;
        tl[j] = tile_off[j + 1] - tile_off[j];
    }
    __syncthreads();

    // finish Eq. 2: minimum over the centroid parts, ties to the lowest index
    vp_finish_eq2(cpart, parts, N, K, tid, PLAN_THREADS, [&](int r, int j) {
        g[r] = j;
        if (out_cluster) out_cluster[r] = j;
        atomicAdd(&cnt[j], 1);
    });
    __threadfence_block();   // the scatter below reads g[] written by other threads of this workgroup
    __syncthreads();

    // exclusive scan of the histogram -> bucket offsets; total candidate tiles of all row groups
    int carry = 0;
    int my_tiles = 0, my_occ_tiles = 0, my_units = 0;
    for (int base = 0; base < K; base += PLAN_THREADS) {
        const int j = base + tid;
        const int c = j < K ? cnt[j] : 0;
        int tot;
        const int ex = block_exscan_int(c, &tot, wsum);
        if (j < K) {
            off[j] = carry + ex;
            my_tiles += ceil_div(c, VP_ROWS_PER_ITEM) * tl[j];
            my_units += ceil_div(c, VP_ROWS_PER_ITEM);
            if (c > 4 * VP_ROWS_PER_ITEM) atomicMax(&max_rgs, ceil_div(c, VP_ROWS_PER_ITEM));
            if (c > 0) my_occ_tiles += tl[j];
        }
        carry += tot;
    }
    if (tid == 0) off[K] = carry;
    int total_tiles, units, occ_tiles;
    block_sum3(my_tiles, my_units, my_occ_tiles, &total_tiles, &units, &occ_tiles, wsum3);

    // both forms give the same results, so the cheaper one is taken (cost model in plan_common.h)
    if (dispatch) {
        const int rpi_full = dispatch;   // rows per item of the masked projection (16 or 64)
        if (vp_full_is_cheaper(occ_tiles, total_tiles, N, rpi_full, vtiles, k, cost)) {
            __syncthreads();
            vp_plan_single_bucket(N, V, vtiles, rpi_full, full_target_items, full_min_items, max_items_full, perm,
                                  rowplan, floors, items, hdr, nullptr, tid, PLAN_THREADS);
            if (tid == 0) hdr->mode = 1;
            return;
        }
    }
    const int tpw = vp_tiles_per_wave_units(total_tiles, units, target_items, min_items);
    const int tpi = tpw * VP_WG_WAVES;

    // items per bucket -> item offsets
    carry = 0;
    for (int base = 0; base < K; base += PLAN_THREADS) {
        const int j = base + tid;
        int c = 0;
        if (j < K) c = ceil_div(cnt[j], VP_ROWS_PER_ITEM) * ceil_div(tl[j], tpi);
        int tot;
        const int ex = block_exscan_int(c, &tot, wsum);
        if (j < K) ioff[j] = carry + ex;
        carry += tot;
    }
    if (tid == 0) ioff[K] = carry;
    __syncthreads();
    const int total_items = min(ioff[K], max_items);

    // scatter rows into bucket order (cnt becomes the per-bucket cursor) and tell the
    // merge kernel where the partial results of each row will be
    for (int j = tid; j < K; j += PLAN_THREADS) cnt[j] = 0;
    __syncthreads();
    for (int r = tid; r < N; r += PLAN_THREADS) {
        const int j = g[r];
        const int local = atomicAdd(&cnt[j], 1);
        const int p = off[j] + local;
        perm[p] = r;
        floors[r] = VP_FLOOR_NONE;   // no lower bound of the row's k-th best logit known yet
        VpRowPlan rp;
        rp.row = r;
        rp.cluster = j;
        rp.item0 = ioff[j] + local / VP_ROWS_PER_ITEM;
        rp.stride = ceil_div(off[j + 1] - off[j], VP_ROWS_PER_ITEM);
        rp.nit = ceil_div(tl[j], tpi);
        rp.local = local % VP_ROWS_PER_ITEM;
        rp.ids_off = tile_off[j] * VP_TILE_ITEMS;
        rp.pad = 0;
        rowplan[p] = rp;
    }

    // the items: for each bucket, candidate ranges outermost and row groups
    // innermost, so items that re-read the same tiles sit next to each other
    for (int it = tid; it < total_items; it += PLAN_THREADS) {
        int lo = 0, hi = K;   // largest j with ioff[j] <= it (empty buckets have empty ranges)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (ioff[mid] <= it) lo = mid; else hi = mid;
        }
        const int j = lo;
        const int rows = off[j + 1] - off[j];
        const int rgs = ceil_div(rows, VP_ROWS_PER_ITEM);
        const int local = it - ioff[j];
        const int ch = local / rgs;
        const int rg = local - ch * rgs;
        VpItem v;
        v.cluster = j;
        v.perm_start = off[j] + rg * VP_ROWS_PER_ITEM;
        v.nrows = min(VP_ROWS_PER_ITEM, rows - rg * VP_ROWS_PER_ITEM);
        v.tile0 = ch * tpi;
        v.ntiles = min(tpi, tl[j] - ch * tpi);
        v.shared = rgs > 1;
        v.tile_off = tile_off[j];
        v.ncand = n_cand[j];
        items[it] = v;
    }
    if (tid == 0) {
        hdr->total_items = total_items;
        hdr->tiles_per_wave = tpw;
        hdr->overflow = ioff[K] > max_items;
        hdr->total_tiles = total_tiles;
        // buckets of five row groups and more: keep the row groups of a candidate range on one XCD
        hdr->swz_rgs = max_rgs > 4 ? -VP_XCD_BLOCK_ITEMS : 0;
        hdr->swz_chunks = 0;
        hdr->rows_per_item = VP_ROWS_PER_ITEM;
        hdr->mode = 0;
    }

    // debug entry only: where each row's candidate logits start
    if (dbg_row_off) {
        __syncthreads();
        long long carry64 = 0;
        for (int base = 0; base < N; base += PLAN_THREADS) {
            const int r = base + tid;
            const long long c = r < N ? (long long)n_cand[g[r]] : 0;
            long long tot;
            const long long ex = block_exscan<long long>(c, &tot, wsum64);
            if (r < N) dbg_row_off[r] = carry64 + ex;
            carry64 += tot;
        }
        if (tid == 0) dbg_row_off[N] = carry64;
    }
}

// Plan of the full-vocabulary projection: one bucket holding every row in
// order, one slab holding every token.  Nothing depends on device data.
__global__ __launch_bounds__(256) void plan_full_kernel(
    int N, int V, int vtiles, int rpi, int target_items, int min_items, int max_items, int32_t *__restrict__ perm,
    VpRowPlan *__restrict__ rowplan, unsigned int *__restrict__ floors, VpItem *__restrict__ items,
    VpPlanHeader *__restrict__ hdr, int64_t *__restrict__ dbg_row_off)
{
    vp_plan_single_bucket(N, V, vtiles, rpi, target_items, min_items, max_items, perm, rowplan, floors, items, hdr,
                          dbg_row_off, blockIdx.x * blockDim.x + threadIdx.x, gridDim.x * blockDim.x);
}

}  // namespace

size_t vpk_plan_lds_bytes(int K) { return (size_t)(4 * K + 2) * sizeof(int); }

hipError_t vpk_plan_prepare()
{
    // clusters up to VP_MAX_CLUSTERS need a little over 64 KiB of dynamic LDS; allow it explicitly
    return hipFuncSetAttribute(reinterpret_cast<const void *>(plan_kernel),
                               hipFuncAttributeMaxDynamicSharedMemorySize, 72 * 1024);
}

void vpk_plan(const void *cpart, int parts, int N, int K, const int32_t *n_cand, const int32_t *tile_off,
              int target_items, int min_items, int max_items, int32_t *g, int32_t *out_cluster, int32_t *perm,
              VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr, int64_t *dbg_row_off,
              int dispatch, const VpCostModel &cost, int k, int V, int vtiles, int full_target_items,
              int full_min_items, int max_items_full, hipStream_t st)
{
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(PLAN_THREADS), vpk_plan_lds_bytes(K), st, (const int2 *)cpart,
                       parts, N, K, n_cand, tile_off, target_items, min_items, max_items, g, out_cluster, perm, rowplan, floors,
                       items, hdr, dbg_row_off, dispatch, cost, k, V, vtiles, full_target_items, full_min_items, max_items_full);
}

void vpk_plan_full(int N, int V, int vtiles, int rpi, int target_items, int min_items, int max_items, int32_t *perm,
                   VpRowPlan *rowplan, unsigned int *floors, VpItem *items, VpPlanHeader *hdr,
                   int64_t *dbg_row_off, hipStream_t st)
{
    const int work = max(N, max_items);
    const int blocks = min(64, (work + 255) / 256);
    hipLaunchKernelGGL(plan_full_kernel, dim3(blocks), dim3(256), 0, st, N, V, vtiles, rpi, target_items, min_items, max_items,
                       perm, rowplan, floors, items, hdr, dbg_row_off);
}
