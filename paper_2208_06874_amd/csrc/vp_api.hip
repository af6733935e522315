// Host side of the C ABI declared in include/vp.h: argument validation, arena
// and workspace carving, kernel sequencing.  No device memory is allocated
// here; every buffer is carved from memory the caller supplies.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <mutex>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>
#include <utility>
#include <vector>

#include "vp.h"
#include "vp_kernels.h"

// Scratch of vp_project_static: a call's workspace for callers that cannot allocate.  In host
// code this name is only a handle of the symbol; the array's address on a device comes from
// hipGetSymbolAddress with that device current (static_scratch_of_current_device).
static __device__ __align__(256) unsigned char scratch[VP_STATIC_SCRATCH_BYTES];

namespace {

thread_local char g_err[512] = "";

vp_status fail(vp_status st, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

static_assert(VP_MAX_TOPK == 32, "merge_kernel keeps the winners of at most 32 rounds");
constexpr size_t ALIGN = 256;

constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES] = {};   // per device: where its copy of the array lives

// The current device's copy of the scratch array; resolved once per device.  Allocates nothing.
vp_status static_scratch_of_current_device(const char *fn, void **out)
{
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return fail(VP_ERR_HIP, "%s: hipGetDevice: %s", fn, hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES)
        return fail(VP_ERR_UNSUPPORTED, "%s: device %d out of range", fn, dev);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !p)
            return fail(VP_ERR_HIP, "%s: hipGetSymbolAddress: %s", fn, hipGetErrorString(e));
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return VP_OK;
}
constexpr size_t LDS_LIMIT = 160 * 1024;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

// Byte offsets of the index sections inside the arena.
struct ArenaLayout {
    int d_pad, kt, vtiles, ctiles;
    long total_groups;     // candidate groups (of 16) over all clusters
    long n_total;
    int n_min, n_max, max_tiles;
    size_t wp, wt, biasf, cp, cnorm, full_meta, tile_off, n_cand, ids_pad, sbias, bitmaps, slabs, total;
    int bm_words;
};

}  // namespace

int vpi_fail(int status, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return status;
}

// Event pairs around the projection kernel (benchmark aid, see vp_get_profile).
struct VpProfile {
    bool on = false;
    std::vector<std::pair<hipEvent_t, hipEvent_t>> pool;   // created on demand, reused
    size_t used = 0;
};

struct vp_index {
    int d, V, K, k_max;
    ArenaLayout L;
    char *arena;
    VpSlabSet clusters;
    VpSlabSet full;
    const void *cp;
    const float *cnorm;
    int target_items, full_target_items, rstar;
    int min_items;   // resident workgroup slots of the projection kernel on this GPU
    int cus;         // compute units of this GPU
    int wide_items;  // 1: single-bucket projections of more than 16 rows use items of 32 rows
    int gemm_target_items;   // work items of the GEMM-shaped kernel: its resident workgroup slots
    int gemm_lds;        // 1: many-row items use the kernel that holds the rows in LDS where it is built (d_pad <= 1536, k <= 32)
    int gemm_lds_items;  // its work items: one per compute unit
    int gemm_min_rows;   // single-bucket projections of at least this many rows use the GEMM-shaped kernel (0: never)
    int dispatch;    // 1: the planner may choose the masked full projection (same results)
    VpCostModel cost;
    const uint32_t *bitmaps;
    int union_dispatch;   // 1: vp_project_union may project a large union as a masked full projection
    bool has_token_major;   // the copy of W vp_project_union reads is part of the arena
    int small_path;   // 1: batches of at most 16 rows are planned by the projection workgroups themselves
    int small_pf;     // 1 KiB loads a wavefront of that path keeps in flight (0: chosen from the batch size)
    int raw_logits;   // 1: short items of small top-k >= 4 calls keep raw logits instead of lists (see run_clustered)
    // [n] = candidate groups of the n longest active sets together, n = 0 .. K: the most slab
    // bytes n rows can occupy (host-side bound of the planner's choice)
    std::vector<int64_t> longest_tiles;
    VpProfile *prof;
};

namespace {

// Checks everything in the description that lives on the host and computes the layout.
vp_status plan_arena(const vp_build_desc *D, bool check_ids, ArenaLayout *L)
{
    if (!D) return fail(VP_ERR_INVALID_ARG, "vp_build: null description");
    if (D->flags & ~VP_BUILD_NO_UNION) return fail(VP_ERR_INVALID_ARG, "vp_build: unknown flag bits %#x", D->flags);
    if (D->d < 8 || D->d > VP_MAX_DIM || D->d % 8 != 0)
        return fail(VP_ERR_UNSUPPORTED, "vp_build: d = %d must be a multiple of 8 in [8, %d]", D->d, VP_MAX_DIM);
    if (D->K < 1 || D->K > VP_MAX_CLUSTERS)
        return fail(VP_ERR_UNSUPPORTED, "vp_build: K = %d must be in [1, %d]", D->K, VP_MAX_CLUSTERS);
    if (D->V < 1 || D->V > 2147483647 - 16) return fail(VP_ERR_UNSUPPORTED, "vp_build: V = %d out of range", D->V);
    if (D->k_max < 1 || D->k_max > VP_MAX_TOPK)
        return fail(VP_ERR_UNSUPPORTED, "vp_build: k_max = %d must be in [1, %d]", D->k_max, VP_MAX_TOPK);
    if (!D->cand_offsets || !D->cand_ids) return fail(VP_ERR_INVALID_ARG, "vp_build: null candidate lists");
    if (D->cand_offsets[0] != 0) return fail(VP_ERR_INVALID_ARG, "vp_build: cand_offsets[0] must be 0");

    L->d_pad = (D->d + VP_KPAD - 1) / VP_KPAD * VP_KPAD;
    L->kt = L->d_pad / VP_TILE_K;
    if (vpk_project_lds_bytes(L->kt, D->k_max, 1) > LDS_LIMIT)
        return fail(VP_ERR_UNSUPPORTED, "vp_build: d = %d with k_max = %d needs more than %zu bytes of LDS", D->d,
                    D->k_max, LDS_LIMIT);
    L->vtiles = ceil_div(D->V, VP_TILE_ITEMS);
    L->ctiles = ceil_div(D->K, VP_TILE_ITEMS);
    long groups = 0, total = 0;
    int n_min = 2147483647, n_max = 0;
    for (int j = 0; j < D->K; ++j) {
        const int64_t a = D->cand_offsets[j], b = D->cand_offsets[j + 1];
        if (b < a) return fail(VP_ERR_INVALID_ARG, "vp_build: cand_offsets decreases at cluster %d", j);
        const int64_t n = b - a;
        if (n > D->V) return fail(VP_ERR_INVALID_ARG, "vp_build: cluster %d lists %lld > V tokens", j, (long long)n);
        if (check_ids && n > 0) {
            const int32_t *ids = D->cand_ids + a;
            if (ids[0] < 0 || ids[n - 1] >= D->V)
                return fail(VP_ERR_INVALID_ARG, "vp_build: cluster %d has a token id outside [0, V)", j);
            for (int64_t c = 1; c < n; ++c)
                if (ids[c] <= ids[c - 1])
                    return fail(VP_ERR_INVALID_ARG,
                                "vp_build: active set of cluster %d is not strictly ascending at position %lld", j,
                                (long long)c);
        }
        groups += (n + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS;
        total += n;
        n_min = std::min<int64_t>(n_min, n);
        n_max = std::max<int64_t>(n_max, n);
    }
    if (groups > (1L << 27)) return fail(VP_ERR_UNSUPPORTED, "vp_build: active sets too large in total");
    if (groups == 0) return fail(VP_ERR_UNSUPPORTED, "vp_build: every active set is empty");
    L->total_groups = groups;
    L->n_total = total;
    L->n_min = n_min;
    L->n_max = n_max;
    L->max_tiles = ceil_div(n_max, VP_TILE_ITEMS);

    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    const size_t group_bytes = (size_t)L->kt * VP_TILE_BYTES;
    L->wp = take((size_t)L->vtiles * group_bytes);
    // token-major copy for the batch-union form (left out on request)
    L->wt = take((D->flags & VP_BUILD_NO_UNION) ? 0 : (size_t)D->V * L->d_pad * 2);
    L->biasf = take((size_t)L->vtiles * VP_TILE_ITEMS * sizeof(float));
    L->cp = take((size_t)L->ctiles * group_bytes);
    L->cnorm = take((size_t)L->ctiles * VP_TILE_ITEMS * sizeof(float));
    L->full_meta = take(4 * sizeof(int32_t));
    L->tile_off = take((size_t)(D->K + 1) * sizeof(int32_t));
    L->n_cand = take((size_t)D->K * sizeof(int32_t));
    L->ids_pad = take((size_t)groups * VP_TILE_ITEMS * sizeof(int32_t));
    L->sbias = take((size_t)groups * VP_TILE_ITEMS * sizeof(float));
    L->bm_words = (ceil_div((long)L->vtiles * VP_TILE_ITEMS, 32) + 1) & ~1;   // even: a list's words pair up into aligned 64-bit loads
    L->bitmaps = take((size_t)D->K * L->bm_words * sizeof(uint32_t));
    L->slabs = take((size_t)groups * group_bytes);
    L->total = o;
    return VP_OK;
}

// Byte offsets of the per-call scratch inside the workspace.
struct WsLayout {
    int max_items;
    size_t hdr, cpart, g, perm, rowplan, floors, items, partials, total;
};

int max_items_clustered(const vp_index *I, int N)
{
    return I->target_items + ceil_div(N, VP_ROWS_PER_ITEM) + std::min(N, I->K) + 2;
}
// (the grid of the full projection is padded to 8 candidate ranges at a time, one per XCD)
int max_items_full(const vp_index *I, int N)
{
    // (the kernel with the rows in LDS takes up to eight rounds of its one item per compute unit)
    return std::max(I->full_target_items, std::max(I->gemm_target_items, 8 * I->gemm_lds_items)) +
           8 * ceil_div(N, VP_ROWS_PER_ITEM) + 2;
}

WsLayout plan_workspace(const vp_index *I, int N)
{
    WsLayout W;
    W.max_items = std::max(max_items_clustered(I, N), max_items_full(I, N));
    size_t o = 0;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    const size_t n = (size_t)std::max(N, 1);
    W.hdr = take(sizeof(VpPlanHeader));
    W.cpart = take(n * I->L.ctiles * 8);
    W.g = take(n * 4);
    W.perm = take(n * 4);
    W.rowplan = take(n * sizeof(VpRowPlan));
    W.floors = take(n * 4 * (1 + VP_BOUND_SETS));   // [N] bounds of the 16-row kernels, then [N][sets] of the GEMM kernel
    // (workgroups read the record at their own index before they know the item count)
    W.items = take((size_t)(W.max_items + 8 * VP_XCD_BLOCK_ITEMS) * sizeof(VpItem));
    // one partial result per (item, row slot): 16 slots in the clustered plan, up to 64 in single-bucket plans
    const size_t slots = std::max((size_t)max_items_clustered(I, N) * VP_ROWS_PER_ITEM,
                                  (size_t)max_items_full(I, N) * VP_MAX_ROWS_PER_ITEM);
    W.partials = take(slots * vp_partial_floats(I->k_max) * sizeof(float));
    W.total = o;
    return W;
}

vp_status check_call(const char *fn, const vp_index *I, const void *hidden, int N, int k, const void *out_ids,
                     const void *out_logp, const void *ws, size_t ws_bytes, bool need_outputs)
{
    if (!I) return fail(VP_ERR_INVALID_ARG, "%s: null index", fn);
    if (N < 0 || N > VP_MAX_ROWS) return fail(VP_ERR_INVALID_ARG, "%s: N = %d must be in [0, %d]", fn, N, VP_MAX_ROWS);
    if (k < 1 || k > I->k_max)
        return fail(VP_ERR_UNSUPPORTED, "%s: k = %d must be in [1, k_max = %d]", fn, k, I->k_max);
    if (N == 0) return VP_OK;
    if (!hidden || !aligned(hidden, 16)) return fail(VP_ERR_INVALID_ARG, "%s: hidden is null or not 16-byte aligned", fn);
    if (need_outputs && (!out_ids || !out_logp)) return fail(VP_ERR_INVALID_ARG, "%s: null output pointer", fn);
    if (!ws || !aligned(ws, ALIGN)) return fail(VP_ERR_INVALID_ARG, "%s: workspace is null or not 256-byte aligned", fn);
    const WsLayout W = plan_workspace(I, N);
    if (ws_bytes < W.total)
        return fail(VP_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed for N = %d", fn, ws_bytes, W.total, N);
    return VP_OK;
}

vp_status launch_status(const char *fn)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return fail(VP_ERR_HIP, "%s: kernel launch failed: %s", fn, hipGetErrorString(e));
    return VP_OK;
}

constexpr size_t PROFILE_MAX = 16384;

// Returns the event pair to bracket the next projection kernel with, or null.
std::pair<hipEvent_t, hipEvent_t> *profile_slot(const vp_index *I)
{
    VpProfile *P = I->prof;
    if (!P || !P->on || P->used >= PROFILE_MAX) return nullptr;
    if (P->used == P->pool.size()) {
        hipEvent_t a, b;
        if (hipEventCreate(&a) != hipSuccess) return nullptr;
        if (hipEventCreate(&b) != hipSuccess) {
            (void)hipEventDestroy(a);
            return nullptr;
        }
        P->pool.emplace_back(a, b);
    }
    return &P->pool[P->used++];
}

// Row tiles per item for projections that keep all rows in one bucket (full, masked, union).
// From gemm_min_rows rows on (default 17: measured faster than two 16-row passes from there): 4,
// the GEMM-shaped kernels (64 rows per item, every loaded slab tile feeds four MFMAs), or 3 where
// the one that keeps the rows in LDS has room for 48 only.  Where
// neither is built for the k-extent, two row tiles per loaded slab tile pay off
// (measured: -10 % at top-1, N = 256) only while the top-k lists are short.
int single_bucket_row_tiles(const vp_index *I, int N, int k)
{
    if (I->gemm_min_rows > 0 && N >= I->gemm_min_rows) {
        // (the kernel that keeps the rows in LDS has room for three row tiles at d_pad = 1536)
        if (I->gemm_lds && vpk_project_rows_lds_supported(I->L.kt, k)) return vpk_project_rows_lds_row_tiles(I->L.kt);
        if (vpk_project_gemm_supported(I->L.kt)) return 4;
    }
    if (!I->wide_items || k > 2 || N <= VP_ROWS_PER_ITEM || I->L.kt % 16 != 0) return 1;
    return vpk_project_lds_bytes(I->L.kt, k, 2) <= LDS_LIMIT / 2 ? 2 : 1;
}

// Item count bounds (target, minimum) of a single-bucket plan with this many row tiles.
inline bool use_gemm_lds(const vp_index *I, int row_tiles, int k)
{
    return row_tiles >= 3 && I->gemm_lds && vpk_project_rows_lds_supported(I->L.kt, k) &&
           row_tiles == vpk_project_rows_lds_row_tiles(I->L.kt);
}
// Item count of the kernel that keeps an item's rows in LDS: whole rounds of its one workgroup per
// compute unit (vp_rounds_item_count).
inline int gemm_lds_item_count(const vp_index *I, int N, int row_tiles)
{
    return vp_rounds_item_count(ceil_div(N, VP_ROWS_PER_ITEM * row_tiles), I->gemm_lds_items, I->L.vtiles);
}
inline int sb_target(const vp_index *I, int N, int row_tiles, int k)
{
    return use_gemm_lds(I, row_tiles, k) ? gemm_lds_item_count(I, N, row_tiles)
                                         : row_tiles >= 3 ? I->gemm_target_items : I->full_target_items;
}
inline int sb_min(const vp_index *I, int N, int row_tiles, int k)
{
    return use_gemm_lds(I, row_tiles, k) ? gemm_lds_item_count(I, N, row_tiles)
                                         : row_tiles >= 3 ? I->gemm_target_items : I->min_items;
}
// candidate tiles per wavefront of a single-bucket plan (the split the planning kernels make)
inline int sb_tiles_per_wave(const vp_index *I, int N, int rgs, int row_tiles, int k)
{
    return vp_tiles_per_wave((long long)rgs * I->L.vtiles, sb_target(I, N, row_tiles, k), sb_min(I, N, row_tiles, k));
}

// Launches the projection kernel that goes with the plan's rows per item.
void launch_single_bucket(const VpSlabSet &set, const vp_index *I, const void *hidden, const int32_t *perm,
                          const VpItem *items, const VpPlanHeader *hdr, int N, int grid_items, int row_tiles, int k, int rstar,
                          float *partials, unsigned int *floors, float *dbg_logits, const int64_t *dbg_row_off,
                          hipStream_t st)
{
    if (use_gemm_lds(I, row_tiles, k))
        vpk_project_rows_lds(set, hidden, I->d, perm, items, hdr, grid_items, k, partials, floors, nullptr, false, st);
    else if (row_tiles == 4)
        vpk_project_gemm(set, hidden, I->d, perm, items, hdr, grid_items, k, partials, floors + N, nullptr, st);
    else
        vpk_project(set, hidden, I->d, perm, items, hdr, grid_items, row_tiles, k, rstar, partials, floors, dbg_logits,
                    dbg_row_off, 0, st);
}

// Eq. 2 for a decode batch: up to VP_KSPLIT_ROWS rows with one workgroup per (centroid tile, row
// tile) and the k-extent split over its wavefronts (every load in flight at once: 4.6 us instead
// of 9.3 at 64 rows; at 256 rows its thousand small workgroups take 9.2 us against 7-8), beyond
// that the kernel whose workgroups walk several centroid tiles.  Returns the number of per-row
// minima left in cpart.
constexpr int VP_KSPLIT_ROWS = 64;
int launch_eq2(const vp_index *I, const void *hidden, int N, void *cpart, hipStream_t st)
{
    if (N <= VP_KSPLIT_ROWS) {
        vpk_centroid_small(hidden, N, I->d, I->cp, I->cnorm, I->K, I->L.kt, I->L.ctiles, cpart, st);
        return I->L.ctiles;
    }
    const int row_tiles = ceil_div(N, 16);
    int parts = std::min(ceil_div(I->L.ctiles, 4), std::max(1, 2048 / (4 * row_tiles)));
    const int tpw_c = ceil_div(I->L.ctiles, parts * 4);
    parts = ceil_div(I->L.ctiles, tpw_c * 4);
    vpk_centroid(hidden, N, I->d, I->cp, I->cnorm, I->K, I->L.kt, I->L.ctiles, tpw_c, parts, cpart, st);
    return parts;
}

// The kernel sequence shared by vp_project and the clustered debug entry.
vp_status run_clustered(const char *fn, const vp_index *I, const void *hidden, int N, int k, int32_t *out_ids,
                        float *out_logp, int32_t *out_cluster, char *ws, int64_t *dbg_row_off, float *dbg_logits,
                        hipStream_t st)
{
    const WsLayout W = plan_workspace(I, N);
    VpPlanHeader *hdr = reinterpret_cast<VpPlanHeader *>(ws + W.hdr);
    void *cpart = ws + W.cpart;
    int32_t *g = reinterpret_cast<int32_t *>(ws + W.g);
    int32_t *perm = reinterpret_cast<int32_t *>(ws + W.perm);
    VpRowPlan *rowplan = reinterpret_cast<VpRowPlan *>(ws + W.rowplan);
    unsigned int *floors = reinterpret_cast<unsigned int *>(ws + W.floors);
    VpItem *items = reinterpret_cast<VpItem *>(ws + W.items);
    float *partials = reinterpret_cast<float *>(ws + W.partials);

    const int row_tiles = ceil_div(N, 16);
    const int max_items = max_items_clustered(I, N);
    // the debug entry lays its logits out per cluster list, so it always takes the slabs
    // with dispatch: rows per item of the masked full projection the planner may choose
    const int rt_single = single_bucket_row_tiles(I, N, VP_MAX_TOPK);
    const int rt_masked = rt_single >= 3 ? rt_single : 1;
    int dispatch = (I->dispatch && !dbg_logits) ? VP_ROWS_PER_ITEM * rt_masked : 0;
    const int max_full = max_items_full(I, N);
    // the tile counts of the cost model are in tiles of kt KiB: fold that into the constants
    VpCostModel cost = I->cost;
    const float tile_bytes = (float)I->L.kt * VP_TILE_BYTES;
    cost.bw_slab /= tile_bytes;
    cost.bw_full /= tile_bytes;
    cost.bw_l2 /= tile_bytes;
    if (rt_masked >= 3 && !use_gemm_lds(I, rt_masked, k)) cost.bw_gemm = cost.bw_gemm_split;
    cost.bw_gemm /= tile_bytes;
    const long row_groups = (long)row_tiles + std::min(N, I->K);
    const long by_tiles = row_groups * ceil_div(I->L.max_tiles, VP_WG_WAVES);
    // (+ one round of blocks: the XCD swizzle of plans with heavy buckets rounds the grid up)
    const int grid_items = (int)std::min<long>(max_items, by_tiles) + 8 * VP_XCD_BLOCK_ITEMS;
    // If the slabs are the cheaper form even when every row sits in a cluster of its own and those
    // are the clusters with the longest lists (the planner's cost model on that worst case), the planner has nothing to
    // decide and the masked full projection is not launched at all (learned active sets of a
    // fraction of a percent of V: the common case).
    if (dispatch) {
        const int buckets = std::min(N, I->K);
        const float occ = (float)I->longest_tiles[buckets];
        const float total = occ + (float)row_tiles * I->L.max_tiles;
        const float t_slab = occ / cost.bw_slab + (total - occ) / cost.bw_l2 + N * cost.t_row_slab;
        const int rgs_full = ceil_div(N, dispatch);
        const float t_full = dispatch >= 48
            ? std::max(I->L.vtiles / cost.bw_full, rgs_full * (I->L.vtiles / cost.bw_gemm)) * (1.f + k * 0.0125f)
            : std::max(I->L.vtiles / cost.bw_full, (float)rgs_full * I->L.vtiles / cost.bw_l2) * (1.f + k * 0.125f);
        if (t_slab <= t_full) dispatch = 0;
    }
    // Batches of a few rows: no planning kernel; the projection workgroups find their own work
    // (project_small_kernel) - unless the planner has a choice to make.
    const bool small = I->small_path && N <= VP_SMALL_ROWS && !dbg_row_off && !dbg_logits && !dispatch;
    const int raw_ok_all = I->raw_logits && !dbg_logits && k >= 4 && (long)N * I->L.max_tiles <= 8192;
    if (small) {
        VpSmallArgs a = {};
        a.cpart = reinterpret_cast<const int32_t *>(cpart);
        a.parts = launch_eq2(I, hidden, N, cpart, st);
        a.N = N;
        a.K = I->K;
        a.tile_off = I->clusters.tile_off;
        a.n_cand = I->clusters.n_cand;
        a.target_items = I->target_items;
        a.min_items = I->min_items;
        a.g = g;
        a.out_cluster = out_cluster;
        a.rowplan = rowplan;
        a.hdr = hdr;
        // items: at most one per tiles_per_wave * 4 tiles of a bucket plus a partly filled one per
        // bucket; tiles_per_wave is 1 only while that gives at most min_items items
        const long worst_tiles = (long)N * I->L.max_tiles;
        const long eff = std::max<long>(I->min_items, std::min<long>(I->target_items, worst_tiles / (4 * VP_WG_WAVES)));
        const int grid_small = (int)std::min<long>((long)N * ceil_div(I->L.max_tiles, VP_WG_WAVES), eff + N);
        // loads in flight per wavefront: 16 (three wavefronts per SIMD) measured best or within 2 %
        // of the best from 1 to 16 rows, top-1 and top-8 (32: no faster even for one row, whose
        // wavefronts then hold their whole share in flight; 8: 13 % slower at 4 rows, top-8)
        int pf = I->small_pf;
        if (pf == 0) pf = I->L.kt % 16 == 0 ? 16 : 8;
        // resident workgroups of the kernel with that many loads in flight (2, 3 or 4 wavefronts per SIMD)
        const int per_cu = std::max(1, I->min_items / I->cus);
        a.min_items = I->cus * std::min(per_cu, pf == 32 ? 2 : pf == 16 ? 3 : 4);
        auto *ev = profile_slot(I);
        if (ev) (void)hipEventRecord(ev->first, st);
        vpk_project_small(I->clusters, hidden, I->d, a, grid_small, k, I->rstar, partials, raw_ok_all, pf, st);
        if (ev) (void)hipEventRecord(ev->second, st);
        vpk_merge(I->clusters, rowplan, hdr, partials, k, N, out_ids, out_logp, st);
        return launch_status(fn);
    }
    const int parts = launch_eq2(I, hidden, N, cpart, st);
    vpk_plan(cpart, parts, N, I->K, I->clusters.n_cand, I->clusters.tile_off, I->target_items, I->min_items, max_items, g,
             out_cluster, perm, rowplan, floors, items, hdr, dbg_row_off, dispatch, cost, k, I->V, I->L.vtiles,
             sb_target(I, N, rt_masked, k), sb_min(I, N, rt_masked, k), max_full, st);

    auto *ev = profile_slot(I);
    if (ev) (void)hipEventRecord(ev->first, st);
    // Few rows against short lists: at most 8,192 tiles in all, which the default item sizing cuts
    // into items of one or two tiles per wavefront (unless the plan lands just past one round of
    // workgroups and its items are lengthened; the kernel checks the plan's figure itself).
    // For those, keeping raw logits beats building top-k lists from k = 4 on (measured: N = 1,
    // top-8: 50 -> 40 us per call; top-1: no gain, so the lists stay).
    const int raw_ok = raw_ok_all;
    vpk_project(I->clusters, hidden, I->d, perm, items, hdr, grid_items, 1, k, I->rstar, partials, floors, dbg_logits,
                dbg_row_off, raw_ok, st);
    if (dispatch) {
        // launched as well; exactly one of the two does the work, as the planner decided
        const int rgs = ceil_div(N, dispatch);
        const int tpw = sb_tiles_per_wave(I, N, rgs, rt_masked, k);
        const int chunks = ceil_div(I->L.vtiles, (long)tpw * VP_WG_WAVES);
        const int grid_full = (rgs > 1 && chunks >= 8) ? ceil_div(chunks, 8) * 8 * rgs : chunks * rgs;
        const VpMaskInfo mask = {g, I->bitmaps, I->L.bm_words};
        if (use_gemm_lds(I, rt_masked, k))
            vpk_project_rows_lds(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors, &mask, false, st);
        else if (rt_masked == 4)
            vpk_project_gemm(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors + N, &mask, st);
        else
            vpk_project_masked(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors, mask, st);
    }
    if (ev) (void)hipEventRecord(ev->second, st);
    if (out_ids)
        vpk_merge(I->clusters, rowplan, hdr, partials, k, N, out_ids, out_logp, st);
    return launch_status(fn);
}

vp_status run_full(const char *fn, const vp_index *I, const void *hidden, int N, int k, int32_t *out_ids,
                   float *out_logp, char *ws, int64_t *dbg_row_off, float *dbg_logits, hipStream_t st)
{
    const WsLayout W = plan_workspace(I, N);
    VpPlanHeader *hdr = reinterpret_cast<VpPlanHeader *>(ws + W.hdr);
    int32_t *perm = reinterpret_cast<int32_t *>(ws + W.perm);
    VpRowPlan *rowplan = reinterpret_cast<VpRowPlan *>(ws + W.rowplan);
    unsigned int *floors = reinterpret_cast<unsigned int *>(ws + W.floors);
    VpItem *items = reinterpret_cast<VpItem *>(ws + W.items);
    float *partials = reinterpret_cast<float *>(ws + W.partials);

    // rows per item: 16, 32 or (GEMM-shaped kernel) 64; the debug entry always takes 16
    const int row_tiles = dbg_logits ? 1 : single_bucket_row_tiles(I, N, k);
    const int rpi = VP_ROWS_PER_ITEM * row_tiles;
    const int max_items = max_items_full(I, N);
    vpk_plan_full(N, I->V, I->L.vtiles, rpi, sb_target(I, N, row_tiles, k), sb_min(I, N, row_tiles, k), max_items, perm, rowplan,
                  floors, items, hdr, dbg_row_off, st);
    // the same split the planning kernel makes; with several row groups the projection kernel
    // deals candidate ranges to the XCDs, which needs the grid padded to 8 ranges at a time
    const int rgs = ceil_div(N, rpi);
    const int tpw = sb_tiles_per_wave(I, N, rgs, row_tiles, k);
    const int chunks = ceil_div(I->L.vtiles, (long)tpw * VP_WG_WAVES);
    const int grid_items = (rgs > 1 && chunks >= 8) ? ceil_div(chunks, 8) * 8 * rgs : chunks * rgs;
    auto *ev = profile_slot(I);
    if (ev) (void)hipEventRecord(ev->first, st);
    launch_single_bucket(I->full, I, hidden, perm, items, hdr, N, grid_items, row_tiles, k, N <= I->rstar ? I->rstar : 0,
                         partials, floors, dbg_logits, dbg_row_off, st);
    if (ev) (void)hipEventRecord(ev->second, st);
    if (out_ids)
        vpk_merge(I->full, rowplan, hdr, partials, k, N, out_ids, out_logp, st);
    return launch_status(fn);
}

// Extra workspace of the batch-union form, placed after the common part.
struct UnionLayout {
    size_t base, uh, mask, zero_g, bsum, uids, ubias, uslab, total;
    int mask_words;
};

UnionLayout plan_union_workspace(const vp_index *I, int N)
{
    UnionLayout U;
    U.base = plan_workspace(I, N).total;
    size_t o = U.base;
    auto take = [&](size_t bytes) { size_t at = o; o = align_up(o + bytes); return at; };
    U.mask_words = I->L.bm_words;   // one bit per token, padded like the per-cluster membership lists
    const size_t vpad = (size_t)I->L.vtiles * VP_TILE_ITEMS;
    U.uh = take(sizeof(VpUnionHeader));
    U.mask = take((size_t)U.mask_words * 4);
    U.zero_g = take((size_t)std::max(N, 1) * 4);
    U.bsum = take((size_t)vpk_union_blocks(U.mask_words) * 4);
    U.uids = take(vpad * 4);
    U.ubias = take(vpad * 4);
    U.uslab = take((size_t)I->L.vtiles * I->L.kt * VP_TILE_BYTES);
    U.total = o;
    return U;
}

}  // namespace

extern "C" {

const char *vp_last_error(void) { return g_err; }

size_t vp_build_bytes(const vp_build_desc *desc)
{
    ArenaLayout L;
    if (plan_arena(desc, false, &L) != VP_OK) return 0;
    return L.total;
}

vp_status vp_build(const vp_build_desc *D, void *hip_stream, vp_index **out)
{
    if (!out) return fail(VP_ERR_INVALID_ARG, "vp_build: null output handle");
    *out = nullptr;
    ArenaLayout L;
    vp_status s = plan_arena(D, true, &L);
    if (s != VP_OK) return s;
    if (!D->W || !D->bias || !D->centroids) return fail(VP_ERR_INVALID_ARG, "vp_build: null W, bias or centroids");
    if (!aligned(D->W, 2) || !aligned(D->bias, 2) || !aligned(D->centroids, 16))
        return fail(VP_ERR_INVALID_ARG, "vp_build: W/bias must be 2-byte and centroids 16-byte aligned");
    if (!D->arena || !aligned(D->arena, ALIGN)) return fail(VP_ERR_INVALID_ARG, "vp_build: arena is null or not 256-byte aligned");
    if (D->arena_bytes < L.total)
        return fail(VP_ERR_WORKSPACE, "vp_build: arena of %zu bytes, %zu needed", D->arena_bytes, L.total);

    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    hipError_t e = vpk_plan_prepare();
    if (e == hipSuccess) e = vpk_project_prepare();
    if (e == hipSuccess) e = vpk_merge_prepare();
    if (e == hipSuccess) e = vpk_union_prepare();
    if (e == hipSuccess) e = vpk_project_gemm_prepare();
    if (e == hipSuccess) e = vpk_project_rows_lds_prepare();
    if (e != hipSuccess) return fail(VP_ERR_HIP, "vp_build: cannot configure kernels: %s", hipGetErrorString(e));

    // host-side metadata: candidate groups per cluster, ids padded to whole groups
    std::vector<int32_t> tile_off(D->K + 1), n_cand(D->K);
    std::vector<int32_t> ids_pad((size_t)L.total_groups * VP_TILE_ITEMS, -1);
    tile_off[0] = 0;
    for (int j = 0; j < D->K; ++j) {
        const int64_t a = D->cand_offsets[j];
        const int n = (int)(D->cand_offsets[j + 1] - a);
        n_cand[j] = n;
        tile_off[j + 1] = tile_off[j] + (n + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS;
        std::memcpy(ids_pad.data() + (size_t)tile_off[j] * VP_TILE_ITEMS, D->cand_ids + a, (size_t)n * sizeof(int32_t));
    }
    const int32_t full_meta[4] = {0, L.vtiles, D->V, 0};   // tile_off[2], n_cand[1]

    char *A = static_cast<char *>(D->arena);
    auto up = [&](size_t at, const void *src, size_t bytes) {
        if (e == hipSuccess) e = hipMemcpyAsync(A + at, src, bytes, hipMemcpyHostToDevice, st);
    };
    up(L.tile_off, tile_off.data(), tile_off.size() * sizeof(int32_t));
    up(L.n_cand, n_cand.data(), n_cand.size() * sizeof(int32_t));
    up(L.ids_pad, ids_pad.data(), ids_pad.size() * sizeof(int32_t));
    up(L.full_meta, full_meta, sizeof(full_meta));
    if (e != hipSuccess) return fail(VP_ERR_HIP, "vp_build: upload failed: %s", hipGetErrorString(e));

    vpk_pack_w(D->W, D->d, D->V, L.kt, A + L.wp, st);
    if (!(D->flags & VP_BUILD_NO_UNION)) vpk_token_major(A + L.wp, D->V, L.kt, A + L.wt, st);
    vpk_bias_full(D->bias, D->V, L.vtiles * VP_TILE_ITEMS, reinterpret_cast<float *>(A + L.biasf), st);
    vpk_pack_rows(D->centroids, D->K, D->d, L.kt, A + L.cp, st);
    vpk_cnorm(D->centroids, D->K, D->d, L.ctiles * VP_TILE_ITEMS, reinterpret_cast<float *>(A + L.cnorm), st);
    vpk_gather_slabs(A + L.wp, D->bias, L.kt, reinterpret_cast<const int32_t *>(A + L.ids_pad), L.total_groups,
                     A + L.slabs, reinterpret_cast<float *>(A + L.sbias), st);
    e = hipMemsetAsync(A + L.bitmaps, 0, (size_t)D->K * L.bm_words * sizeof(uint32_t), st);
    if (e != hipSuccess) return fail(VP_ERR_HIP, "vp_build: %s", hipGetErrorString(e));
    vpk_bitmaps(reinterpret_cast<const int32_t *>(A + L.ids_pad), reinterpret_cast<const int32_t *>(A + L.tile_off),
                D->K, L.total_groups, L.bm_words, reinterpret_cast<uint32_t *>(A + L.bitmaps), st);
    s = launch_status("vp_build");
    if (s != VP_OK) return s;
    e = hipStreamSynchronize(st);
    if (e != hipSuccess) return fail(VP_ERR_HIP, "vp_build: %s", hipGetErrorString(e));

    vp_index *I = new (std::nothrow) vp_index();
    if (!I) return fail(VP_ERR_INVALID_ARG, "vp_build: out of host memory");
    I->d = D->d;
    I->V = D->V;
    I->K = D->K;
    I->k_max = D->k_max;
    I->L = L;
    I->arena = A;
    I->cp = A + L.cp;
    I->cnorm = reinterpret_cast<const float *>(A + L.cnorm);
    I->clusters.tiles = A + L.slabs;
    I->clusters.bias = reinterpret_cast<const float *>(A + L.sbias);
    I->clusters.ids = reinterpret_cast<const int32_t *>(A + L.ids_pad);
    I->clusters.tile_off = reinterpret_cast<const int32_t *>(A + L.tile_off);
    I->clusters.n_cand = reinterpret_cast<const int32_t *>(A + L.n_cand);
    I->clusters.entries = D->K;
    I->clusters.kt = L.kt;
    I->full.tiles = A + L.wp;
    I->full.bias = reinterpret_cast<const float *>(A + L.biasf);
    I->full.ids = nullptr;
    I->full.tile_off = reinterpret_cast<const int32_t *>(A + L.full_meta);
    I->full.n_cand = reinterpret_cast<const int32_t *>(A + L.full_meta) + 2;
    I->full.entries = 1;
    I->full.kt = L.kt;
    try {
        I->longest_tiles.assign((size_t)D->K + 1, 0);
        for (int j = 0; j < D->K; ++j)
            I->longest_tiles[j + 1] = ceil_div((long)(D->cand_offsets[j + 1] - D->cand_offsets[j]), VP_TILE_ITEMS);
        std::sort(I->longest_tiles.begin() + 1, I->longest_tiles.end(), [](int64_t a, int64_t b) { return a > b; });
        for (int j = 0; j < D->K; ++j) I->longest_tiles[j + 1] += I->longest_tiles[j];
    } catch (...) {
        delete I;
        return fail(VP_ERR_INVALID_ARG, "vp_build: out of host memory");
    }
    I->target_items = 8192;
    I->full_target_items = 2048;
    I->rstar = 0;
    I->wide_items = 1;
    I->gemm_min_rows = 17;
    I->gemm_target_items = 512;
    I->gemm_lds = 1;
    I->gemm_lds_items = 256;
    // The planner takes whichever of the two forms of the clustered projection its cost model says
    // is cheaper (same results): per-cluster slabs, or the full projection masked to every row's own
    // active set.
    I->dispatch = 1;
    // measured on MI355X at d = 1024, V = 250,000: bytes per second of the regimes of the cost model.
    // Slabs stream at 6.8 TB/s, and a row costs about 60 ns beyond its bytes (512 rows against 32
    // short lists: 72 us for 10 us of bytes).  The masked full projection with 64-row items takes
    // about 100 us for one pass over W from HBM (5.1 TB/s) or, with more row groups, 35 us per row
    // group on the matrix cores (14 TB/s of W; the split-k kernel at d = 1536: 98 us per row group
    // over 0.77 GB, 8 TB/s); with 16-row items every row group re-reads W through the L2 at 17 TB/s.
    I->cost.bw_slab = 6.8e12f;
    I->cost.bw_full = 5.1e12f;
    I->cost.bw_l2 = 17.0e12f;
    I->cost.bw_gemm = 14.0e12f;
    I->cost.bw_gemm_split = 8.0e12f;
    I->cost.t_row_slab = 60.0e-9f;
    // batch-union form: the gather of U's columns from the token-major copy into the union slab
    // (fitted to the measured crossover at |U| = 28 % of V for 64 rows) and the kernels only the
    // gathered form needs
    I->cost.bw_gather = 2.4e12f;
    I->cost.t_gather = 12.0e-6f;
    I->union_dispatch = 1;
    I->has_token_major = !(D->flags & VP_BUILD_NO_UNION);
    I->bitmaps = reinterpret_cast<const uint32_t *>(A + L.bitmaps);
    I->small_path = 1;
    I->small_pf = 0;
    I->raw_logits = 1;
    {
        // workgroups of the projection kernel that fit on the chip at once (LDS-limited)
        int dev = 0, cus = 256;
        if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        const size_t lds = vpk_project_lds_bytes(L.kt, D->k_max, 1);
        const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(8, LDS_LIMIT / lds));
        I->min_items = std::max(1, cus) * per_cu;
        I->cus = std::max(1, cus);
        I->gemm_lds_items = I->cus;
    }
    I->prof = new (std::nothrow) VpProfile();
    // resolve this device's scratch array now, so that vp_project_static's first call does not have to
    {
        void *p = nullptr;
        if (static_scratch_of_current_device("vp_build", &p) != VP_OK) {
            vp_destroy(I);
            return VP_ERR_HIP;
        }
    }
    *out = I;
    return VP_OK;
}

vp_status vp_get_info(const vp_index *I, vp_index_info *info)
{
    if (!I || !info) return fail(VP_ERR_INVALID_ARG, "vp_get_info: null argument");
    info->d = I->d;
    info->V = I->V;
    info->K = I->K;
    info->k_max = I->k_max;
    info->d_pad = I->L.d_pad;
    info->n_min = I->L.n_min;
    info->n_max = I->L.n_max;
    info->n_total = I->L.n_total;
    info->slab_bytes = (int64_t)I->L.total_groups * I->L.kt * VP_TILE_BYTES;
    info->full_bytes = (int64_t)I->L.vtiles * I->L.kt * VP_TILE_BYTES;
    info->arena_bytes_used = (int64_t)I->L.total;
    return VP_OK;
}

vp_status vp_set_option(vp_index *I, const char *name, int64_t value)
{
    if (!I || !name) return fail(VP_ERR_INVALID_ARG, "vp_set_option: null argument");
    // one row per option: where it lives, its range, and for the rates of the cost model the
    // factor from the option's unit (GB/s) to bytes per second
    struct Option {
        const char *name;
        int vp_index::*field;
        float VpCostModel::*rate;
        int64_t lo, hi;
    };
    static const Option table[] = {
        {"target_items", &vp_index::target_items, nullptr, 1, 1 << 20},
        {"full_target_items", &vp_index::full_target_items, nullptr, 1, 1 << 20},
        {"gemm_target_items", &vp_index::gemm_target_items, nullptr, 1, 1 << 20},
        {"gemm_min_rows", &vp_index::gemm_min_rows, nullptr, 0, VP_MAX_ROWS},
        {"gemm_lds", &vp_index::gemm_lds, nullptr, 0, 1},
        {"gemm_lds_items", &vp_index::gemm_lds_items, nullptr, 1, 1 << 20},
        {"rstar", &vp_index::rstar, nullptr, 0, VP_GEMV_MAX_ROWS},
        {"wide_items", &vp_index::wide_items, nullptr, 0, 1},
        {"dispatch", &vp_index::dispatch, nullptr, 0, 1},
        {"union_dispatch", &vp_index::union_dispatch, nullptr, 0, 1},
        {"small_path", &vp_index::small_path, nullptr, 0, 1},
        {"small_pf", &vp_index::small_pf, nullptr, 0, 32},
        {"raw_logits", &vp_index::raw_logits, nullptr, 0, 1},
        {"cost_bw_slab_gbs", nullptr, &VpCostModel::bw_slab, 1, 1000000},
        {"cost_bw_full_gbs", nullptr, &VpCostModel::bw_full, 1, 1000000},
        {"cost_bw_l2_gbs", nullptr, &VpCostModel::bw_l2, 1, 1000000},
        {"cost_bw_gemm_gbs", nullptr, &VpCostModel::bw_gemm, 1, 1000000},
        {"cost_bw_gemm_split_gbs", nullptr, &VpCostModel::bw_gemm_split, 1, 1000000},
        {"cost_bw_gather_gbs", nullptr, &VpCostModel::bw_gather, 1, 1000000},
        {"cost_row_slab_ns", nullptr, &VpCostModel::t_row_slab, 0, 100000},
    };
    if (!std::strcmp(name, "profile")) {
        if (value != 0 && value != 1) return fail(VP_ERR_INVALID_ARG, "vp_set_option: profile must be 0 or 1");
        if (!I->prof) return fail(VP_ERR_INVALID_ARG, "vp_set_option: profiling unavailable");
        I->prof->on = value == 1;
        return VP_OK;
    }
    for (const Option &o : table) {
        if (std::strcmp(name, o.name) != 0) continue;
        if (value < o.lo || value > o.hi)
            return fail(VP_ERR_INVALID_ARG, "vp_set_option: %s = %lld must be in [%lld, %lld]", name, (long long)value,
                        (long long)o.lo, (long long)o.hi);
        if (o.field == &vp_index::small_pf && value != 0 && value != 8 && value != 16 && value != 32)
            return fail(VP_ERR_INVALID_ARG, "vp_set_option: small_pf must be 0, 8, 16 or 32");
        if (o.field) I->*o.field = (int)value;
        else if (o.rate == &VpCostModel::t_row_slab) I->cost.t_row_slab = (float)value * 1e-9f;
        else I->cost.*o.rate = (float)value * 1e9f;
        return VP_OK;
    }
    return fail(VP_ERR_INVALID_ARG, "vp_set_option: unknown option '%s'", name);
}

size_t vp_workspace_bytes(const vp_index *I, int32_t N_max)
{
    if (!I || N_max < 0 || N_max > VP_MAX_ROWS) {
        fail(VP_ERR_INVALID_ARG, "vp_workspace_bytes: bad index or N_max");
        return 0;
    }
    return plan_workspace(I, N_max).total;
}

vp_status vp_project(const vp_index *I, const void *hidden, int32_t N, int32_t k, int32_t *out_ids, float *out_logp,
                     int32_t *out_cluster, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    vp_status s = check_call("vp_project", I, hidden, N, k, out_ids, out_logp, workspace, workspace_bytes, true);
    if (s != VP_OK || N == 0) return s;
    return run_clustered("vp_project", I, hidden, N, k, out_ids, out_logp, out_cluster, static_cast<char *>(workspace),
                         nullptr, nullptr, reinterpret_cast<hipStream_t>(hip_stream));
}

vp_status vp_project_static(const vp_index *I, const void *hidden, int32_t N, int32_t k, int32_t *out_ids,
                            float *out_logp, int32_t *out_cluster, void *hip_stream)
{
    const char *fn = "vp_project_static";
    if (!I) return fail(VP_ERR_INVALID_ARG, "%s: null index", fn);
    if (N < 0 || N > VP_MAX_ROWS) return fail(VP_ERR_INVALID_ARG, "%s: N = %d must be in [0, %d]", fn, N, VP_MAX_ROWS);
    const size_t need = plan_workspace(I, N).total;
    if (need > (size_t)VP_STATIC_SCRATCH_BYTES)
        return fail(VP_ERR_WORKSPACE, "%s: N = %d needs %zu bytes of scratch, the library's array holds %zu", fn, N,
                    need, (size_t)VP_STATIC_SCRATCH_BYTES);
    void *ptr = nullptr;   // the array's address on this device (never the symbol's name)
    vp_status s = static_scratch_of_current_device(fn, &ptr);
    if (s != VP_OK) return s;
    s = check_call(fn, I, hidden, N, k, out_ids, out_logp, ptr, VP_STATIC_SCRATCH_BYTES, true);
    if (s != VP_OK || N == 0) return s;
    return run_clustered(fn, I, hidden, N, k, out_ids, out_logp, out_cluster, static_cast<char *>(ptr), nullptr,
                         nullptr, reinterpret_cast<hipStream_t>(hip_stream));
}

vp_status vp_project_full(const vp_index *I, const void *hidden, int32_t N, int32_t k, int32_t *out_ids,
                          float *out_logp, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    vp_status s = check_call("vp_project_full", I, hidden, N, k, out_ids, out_logp, workspace, workspace_bytes, true);
    if (s != VP_OK || N == 0) return s;
    return run_full("vp_project_full", I, hidden, N, k, out_ids, out_logp, static_cast<char *>(workspace), nullptr,
                    nullptr, reinterpret_cast<hipStream_t>(hip_stream));
}

vp_status vp_project_debug_logits(const vp_index *I, const void *hidden, int32_t N, int32_t full,
                                  int32_t *out_cluster, int64_t *out_row_offsets, float *out_logits,
                                  size_t out_logits_capacity, void *workspace, size_t workspace_bytes,
                                  void *hip_stream)
{
    const char *fn = "vp_project_debug_logits";
    vp_status s = check_call(fn, I, hidden, N, 1, nullptr, nullptr, workspace, workspace_bytes, false);
    if (s != VP_OK) return s;
    if (!out_row_offsets || (N > 0 && !out_logits)) return fail(VP_ERR_INVALID_ARG, "%s: null output pointer", fn);
    if (!full && !out_cluster) return fail(VP_ERR_INVALID_ARG, "%s: out_cluster is required when full == 0", fn);
    if (N == 0) return VP_OK;
    const size_t need = (size_t)N * (full ? (size_t)I->V : (size_t)I->L.n_max);
    if (out_logits_capacity < need)
        return fail(VP_ERR_WORKSPACE, "%s: out_logits holds %zu elements, %zu needed", fn, out_logits_capacity, need);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    if (full) return run_full(fn, I, hidden, N, 1, nullptr, nullptr, static_cast<char *>(workspace), out_row_offsets, out_logits, st);
    return run_clustered(fn, I, hidden, N, 1, nullptr, nullptr, out_cluster, static_cast<char *>(workspace),
                         out_row_offsets, out_logits, st);
}

vp_status vp_get_profile(vp_index *I, double *kernel_ms_total, int64_t *launches)
{
    if (!I || !kernel_ms_total || !launches) return fail(VP_ERR_INVALID_ARG, "vp_get_profile: null argument");
    *kernel_ms_total = 0.0;
    *launches = 0;
    VpProfile *P = I->prof;
    if (!P) return VP_OK;
    for (size_t i = 0; i < P->used; ++i) {
        hipError_t e = hipEventSynchronize(P->pool[i].second);
        float ms = 0.f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, P->pool[i].first, P->pool[i].second);
        if (e != hipSuccess) {
            P->used = 0;
            return fail(VP_ERR_HIP, "vp_get_profile: %s", hipGetErrorString(e));
        }
        *kernel_ms_total += ms;
        *launches += 1;
    }
    P->used = 0;
    return VP_OK;
}

vp_status vp_measure_ceilings(const void *buf, size_t bytes, int32_t repeats, double *read_gbs, double *mfma_tflops,
                              void *hip_stream)
{
    const char *fn = "vp_measure_ceilings";
    if (!buf || !aligned(buf, ALIGN) || !read_gbs || !mfma_tflops) return fail(VP_ERR_INVALID_ARG, "%s: null or misaligned argument", fn);
    if (bytes < (64u << 20) || repeats < 1 || repeats > 100)
        return fail(VP_ERR_INVALID_ARG, "%s: bytes must be at least 64 MiB and repeats in [1, 100]", fn);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    void *sink = nullptr;
    vp_status s = static_scratch_of_current_device(fn, &sink);
    if (s != VP_OK) return s;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) == hipSuccess) (void)hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
    cus = std::max(1, cus);
    hipEvent_t e0, e1;
    if (hipEventCreate(&e0) != hipSuccess) return fail(VP_ERR_HIP, "%s: cannot create events", fn);
    if (hipEventCreate(&e1) != hipSuccess) {
        (void)hipEventDestroy(e0);
        return fail(VP_ERR_HIP, "%s: cannot create events", fn);
    }
    *read_gbs = 0.0;
    *mfma_tflops = 0.0;
    hipError_t e = hipSuccess;
    const int mfma_iters = 4096;
    for (int r = 0; r <= repeats && e == hipSuccess; ++r) {   // (the first pass warms up and is not counted)
        float ms = 0.f;
        (void)hipEventRecord(e0, st);
        const size_t read = vpk_ceiling_read(buf, bytes, cus, sink, st);
        (void)hipEventRecord(e1, st);
        e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && r > 0 && ms > 0.f) *read_gbs = std::max(*read_gbs, (double)read / (ms * 1e-3) / 1e9);
        (void)hipEventRecord(e0, st);
        const double flops = vpk_ceiling_mfma(mfma_iters, cus, sink, st);
        (void)hipEventRecord(e1, st);
        if (e == hipSuccess) e = hipEventSynchronize(e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess && r > 0 && ms > 0.f) *mfma_tflops = std::max(*mfma_tflops, flops / (ms * 1e-3) / 1e12);
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (e != hipSuccess) return fail(VP_ERR_HIP, "%s: %s", fn, hipGetErrorString(e));
    return launch_status(fn);
}

size_t vp_union_workspace_bytes(const vp_index *I, int32_t N_max)
{
    if (!I || N_max < 0 || N_max > VP_MAX_ROWS) {
        fail(VP_ERR_INVALID_ARG, "vp_union_workspace_bytes: bad index or N_max");
        return 0;
    }
    return plan_union_workspace(I, N_max).total;
}

vp_status vp_project_union(const vp_index *I, const void *hidden, int32_t N, int32_t k, int32_t *out_ids,
                           float *out_logp, int32_t *out_cluster, int32_t *out_union_size, void *workspace,
                           size_t workspace_bytes, void *hip_stream)
{
    const char *fn = "vp_project_union";
    vp_status s = check_call(fn, I, hidden, N, k, out_ids, out_logp, workspace, workspace_bytes, true);
    if (s != VP_OK) return s;
    if (!I->has_token_major) return fail(VP_ERR_UNSUPPORTED, "%s: the index was built with VP_BUILD_NO_UNION", fn);
    if (N == 0) return VP_OK;
    const UnionLayout U = plan_union_workspace(I, N);
    if (workspace_bytes < U.total)
        return fail(VP_ERR_WORKSPACE, "%s: workspace of %zu bytes, %zu needed for N = %d", fn, workspace_bytes,
                    U.total, N);
    hipStream_t st = reinterpret_cast<hipStream_t>(hip_stream);
    char *ws = static_cast<char *>(workspace);
    const WsLayout W = plan_workspace(I, N);
    VpPlanHeader *hdr = reinterpret_cast<VpPlanHeader *>(ws + W.hdr);
    void *cpart = ws + W.cpart;
    int32_t *g = reinterpret_cast<int32_t *>(ws + W.g);
    int32_t *perm = reinterpret_cast<int32_t *>(ws + W.perm);
    VpRowPlan *rowplan = reinterpret_cast<VpRowPlan *>(ws + W.rowplan);
    unsigned int *floors = reinterpret_cast<unsigned int *>(ws + W.floors);
    VpItem *items = reinterpret_cast<VpItem *>(ws + W.items);
    float *partials = reinterpret_cast<float *>(ws + W.partials);
    VpUnionHeader *uh = reinterpret_cast<VpUnionHeader *>(ws + U.uh);
    unsigned int *mask = reinterpret_cast<unsigned int *>(ws + U.mask);
    int32_t *bsum = reinterpret_cast<int32_t *>(ws + U.bsum);
    int32_t *uids = reinterpret_cast<int32_t *>(ws + U.uids);
    float *ubias = reinterpret_cast<float *>(ws + U.ubias);
    void *uslab = ws + U.uslab;

    // step 1: predicted centroids (Eq. 2)
    const int parts = launch_eq2(I, hidden, N, cpart, st);
    // step 2: boolean list over the vocabulary -> reduced column set U
    int32_t *zero_g = reinterpret_cast<int32_t *>(ws + U.zero_g);
    vpk_union_mark(cpart, parts, N, I->K, I->bitmaps, I->L.bm_words, U.mask_words, g, out_cluster, zero_g, mask, bsum, st);
    const int max_items = max_items_full(I, N);
    const int row_tiles_u = single_bucket_row_tiles(I, N, k);
    // the masked full projection exists for items of 16 rows and of 48 / 64 rows
    int allow_full = I->union_dispatch && (row_tiles_u == 1 || row_tiles_u >= 3);
    VpCostModel cost = I->cost;
    const float tile_bytes = (float)I->L.kt * VP_TILE_BYTES;
    cost.bw_full /= tile_bytes;
    cost.bw_l2 /= tile_bytes;
    if (row_tiles_u >= 3 && !use_gemm_lds(I, row_tiles_u, k)) cost.bw_gemm = cost.bw_gemm_split;
    cost.bw_gemm /= tile_bytes;
    cost.bw_gather /= tile_bytes;
    if (allow_full) {
        // the in-place form cannot win if the gathered form is cheaper even for the largest union this
        // batch can have (every row in a cluster of its own with the longest list): then it is not launched
        const int rpi_u = VP_ROWS_PER_ITEM * row_tiles_u;
        const int rgs_u = ceil_div(N, rpi_u);
        const float per_group = rpi_u >= 48 ? std::max(1.f / cost.bw_full, rgs_u / cost.bw_gemm) * (1.f + k * 0.0125f)
                                            : std::max(1.f / cost.bw_full, rgs_u / cost.bw_l2) * (1.f + k * 0.125f);
        const long u_max = std::min<long>(I->V, (long)std::min(N, I->K) * I->L.n_max);
        const float tiles_max = (float)ceil_div(u_max, VP_TILE_ITEMS);
        if (cost.t_gather + tiles_max * (1.f / cost.bw_gather + per_group) <= I->L.vtiles * per_group) allow_full = 0;
    }
    vpk_union_compact(mask, U.mask_words, bsum, N, VP_ROWS_PER_ITEM * row_tiles_u, sb_target(I, N, row_tiles_u, k), sb_min(I, N, row_tiles_u, k), max_items, uids, uh,
                      out_union_size, perm, rowplan, floors, items, hdr, allow_full, I->V, I->L.vtiles, k, cost, max_items, I->full.bias, ubias, st);
    // step 3: the reduced weight matrix and Eq. 1 over it; steps 4-5 fused (no [N, V] array).  With
    // the items of the rows-in-LDS kernel the columns of U are read where they lie, through U,
    // from the token-major copy of W (the bias of U's tokens was collected with U); otherwise they
    // are first gathered into a packed slab in the workspace.
    const bool fused_gather = use_gemm_lds(I, row_tiles_u, k) && (long)I->V * I->L.kt * 4 < (1L << 31);
    VpSlabSet uset = I->full;
    uset.bias = ubias;
    uset.ids = uids;
    // grid: the largest split the planner can choose for |U| <= V
    const int rgs = ceil_div(N, VP_ROWS_PER_ITEM * row_tiles_u);
    const int grid_items = std::min(max_items, ceil_div(rgs * (long)ceil_div(I->L.vtiles, VP_WG_WAVES), 8) * 8 + 8 * rgs);
    if (fused_gather) {
        uset.tiles = I->arena + I->L.wt;
        vpk_project_rows_lds(uset, hidden, I->d, perm, items, hdr, grid_items, k, partials, floors, nullptr, true, st);
    } else {
        vpk_union_gather(I->arena + I->L.wt, I->L.kt, uids, uh, I->L.vtiles, uslab, st);
        uset.tiles = uslab;
        launch_single_bucket(uset, I, hidden, perm, items, hdr, N, grid_items, row_tiles_u, k, 0, partials, floors,
                             nullptr, nullptr, st);
    }
    if (allow_full) {
        // launched as well; exactly one of the two does the work, as the planner decided
        const int tpw = sb_tiles_per_wave(I, N, rgs, row_tiles_u, k);
        const int chunks = ceil_div(I->L.vtiles, (long)tpw * VP_WG_WAVES);
        const int grid_full = (rgs > 1 && chunks >= 8) ? ceil_div(chunks, 8) * 8 * rgs : chunks * rgs;
        const VpMaskInfo umask = {zero_g, mask, 0};   // every row reads list 0: the boolean list of the batch
        if (use_gemm_lds(I, row_tiles_u, k))
            vpk_project_rows_lds(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors, &umask, false, st);
        else if (row_tiles_u == 4)
            vpk_project_gemm(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors + N, &umask, st);
        else
            vpk_project_masked(I->full, hidden, I->d, perm, items, hdr, grid_full, k, partials, floors, umask, st);
    }
    vpk_merge(uset, rowplan, hdr, partials, k, N, out_ids, out_logp, st);
    return launch_status(fn);
}

void vp_destroy(vp_index *I)
{
    if (!I) return;
    if (I->prof) {
        for (auto &p : I->prof->pool) {
            (void)hipEventDestroy(p.first);
            (void)hipEventDestroy(p.second);
        }
        delete I->prof;
    }
    delete I;
}

}  // extern "C"
