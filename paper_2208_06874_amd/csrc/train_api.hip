// Host side of the cluster-training entry points of include/vp.h (section 2.2):
// argument validation, workspace carving, kernel sequencing.  No device memory
// is allocated here.
#include <hip/hip_runtime.h>

#include <algorithm>

#include "vp.h"
#include "vp_kernels.h"

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t x) { return (x + ALIGN - 1) / ALIGN * ALIGN; }
inline bool aligned(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline int ceil_div(long a, long b) { return (int)((a + b - 1) / b); }

constexpr int CHUNK_ROWS = 65536;   // vectors per launch of the Eq. 2 kernel

struct KmeansLayout {
    int d_pad, kt, ctiles, K_pad, parts, tpw;
    size_t cp, cnorm, cpart, start, cursor, perm, acc, total;
};

vp_status kmeans_layout(int64_t n, int d, int K, KmeansLayout *L)
{
    if (d < 8 || d > VP_MAX_DIM || d % 8) return (vp_status)vpi_fail(VP_ERR_UNSUPPORTED, "d = %d: need 8 <= d <= %d, d %% 8 == 0", d, VP_MAX_DIM);
    if (K < 1 || K > VP_MAX_CLUSTERS) return (vp_status)vpi_fail(VP_ERR_UNSUPPORTED, "K = %d: need 1 <= K <= %d", K, VP_MAX_CLUSTERS);
    if (n < 1 || n >= (1ll << 31)) return (vp_status)vpi_fail(VP_ERR_UNSUPPORTED, "n = %lld: need 1 <= n < 2^31", (long long)n);
    L->d_pad = ceil_div(d, VP_KPAD) * VP_KPAD;
    L->kt = L->d_pad / VP_TILE_K;
    L->ctiles = ceil_div(K, VP_TILE_ITEMS);
    L->K_pad = L->ctiles * VP_TILE_ITEMS;
    const int chunk = (int)std::min<int64_t>(n, CHUNK_ROWS);
    const int row_tiles = ceil_div(chunk, 16);
    int parts = std::min(ceil_div(L->ctiles, 4), std::max(1, 2048 / (4 * row_tiles)));
    L->tpw = ceil_div(L->ctiles, parts * 4);
    L->parts = ceil_div(L->ctiles, L->tpw * 4);
    size_t o = 0;
    L->cp = o;      o += align_up((size_t)L->K_pad * L->d_pad * 2);
    L->cnorm = o;   o += align_up((size_t)L->K_pad * 4);
    L->cpart = o;   o += align_up((size_t)chunk * L->parts * 8);
    L->start = o;   o += align_up((size_t)(K + 1) * 4);
    L->cursor = o;  o += align_up((size_t)K * 4);
    L->perm = o;    o += align_up((size_t)n * 4);
    L->acc = o;     o += align_up((size_t)K * d * 8);
    L->total = o;
    return VP_OK;
}

}  // namespace

extern "C" {

uint16_t vp_round_to_half(double v) { return vpk_round_to_half(v); }

size_t vp_kmeans_workspace_bytes(int64_t n, int32_t d, int32_t K)
{
    KmeansLayout L;
    if (kmeans_layout(n, d, K, &L) != VP_OK) return 0;
    return L.total;
}

vp_status vp_kmeans(const void *x, int64_t n, int32_t d, int32_t K, int32_t iters, uint32_t flags, void *centroids,
                    int32_t *assign, int32_t *counts, void *workspace, size_t workspace_bytes,
                    void *hip_stream)
{
    if (flags & ~(uint32_t)VP_KMEANS_SPLIT_EMPTY) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "vp_kmeans: unknown flags 0x%x", flags);
    KmeansLayout L;
    vp_status s = kmeans_layout(n, d, K, &L);
    if (s != VP_OK) return s;
    if (iters < 0 || iters > 1000) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "iters = %d: need 0 <= iters <= 1000", iters);
    if (!x || !centroids || !assign || !counts || !workspace) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "null pointer argument");
    if (!aligned(x, 16) || !aligned(centroids, 16)) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "x and centroids must be 16-byte aligned");
    if (!aligned(workspace, ALIGN)) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (workspace_bytes < L.total) return (vp_status)vpi_fail(VP_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, L.total);
    hipStream_t st = (hipStream_t)hip_stream;
    char *ws = (char *)workspace;
    void *cp = ws + L.cp;
    float *cnorm = (float *)(ws + L.cnorm);
    void *cpart = ws + L.cpart;
    int32_t *start = (int32_t *)(ws + L.start), *cursor = (int32_t *)(ws + L.cursor), *perm = (int32_t *)(ws + L.perm);
    void *acc = ws + L.acc;
    // clusters x splits workgroups of the summing kernel: a few thousand
    const int splits = std::max(1, std::min(64, 2048 / K));

    vpk_fill_u32(acc, (size_t)K * d * 2, 0u, st);
    for (int it = 0; it <= iters; ++it) {
        // Eq. 2 operands of the current centroids
        vpk_pack_rows(centroids, K, d, L.kt, cp, st);
        vpk_cnorm(centroids, K, d, L.K_pad, cnorm, st);
        vpk_fill_u32(counts, (size_t)K, 0u, st);
        // memberships: the GEMM-shaped kernel when there are enough vectors to fill the chip with
        // 64-vector workgroups, else (or for k-extents it is not built for) the decode-time kernel
        const bool gemm = n >= 4096 && vpk_kmeans_assign_gemm(x, (long)n, d, cp, cnorm, K, L.kt, L.ctiles, assign, counts, st);
        for (int64_t r0 = 0; !gemm && r0 < n; r0 += CHUNK_ROWS) {
            const int rows = (int)std::min<int64_t>(CHUNK_ROWS, n - r0);
            vpk_centroid((const char *)x + (size_t)r0 * d * 2, rows, d, cp, cnorm, K, L.kt, L.ctiles, L.tpw, L.parts,
                         cpart, st);
            vpk_kmeans_assign(cpart, L.parts, rows, K, assign + r0, counts, st);
        }
        if (it == iters) break;   // the last pass only assigns
        vpk_kmeans_bucket(assign, (long)n, counts, K, start, cursor, perm, st);
        vpk_kmeans_update(x, d, perm, start, counts, K, splits, acc, centroids, st);
        if (flags & VP_KMEANS_SPLIT_EMPTY) vpk_kmeans_split(counts, K, d, centroids, st);
    }
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess) return (vp_status)vpi_fail(VP_ERR_HIP, "vp_kmeans: %s", hipGetErrorString(e));
    return VP_OK;
}

size_t vp_active_sets_workspace_bytes(int32_t K, int32_t V)
{
    if (K < 1 || K > VP_MAX_CLUSTERS || V < 1) {
        vpi_fail(VP_ERR_UNSUPPORTED, "K = %d, V = %d out of range", K, V);
        return 0;
    }
    const size_t words = (size_t)ceil_div(V, 32);
    return align_up((size_t)K * words * 4) + align_up((size_t)K * 4);
}

vp_status vp_active_sets(const int32_t *top_ids, const int32_t *assign, int64_t n, int32_t T, int32_t K,
                         int32_t V, int64_t *cand_offsets, int32_t *cand_ids, int64_t capacity,
                         int64_t *total, void *workspace, size_t workspace_bytes, void *hip_stream)
{
    const size_t need = vp_active_sets_workspace_bytes(K, V);
    if (!need) return VP_ERR_UNSUPPORTED;
    if (n < 0 || n >= (1ll << 31) || T < 1 || T > VP_MAX_TOPK) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "n = %lld, T = %d out of range", (long long)n, T);
    if ((n > 0 && (!top_ids || !assign)) || !cand_offsets || !total || !workspace || capacity < 0 || (capacity > 0 && !cand_ids))
        return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "null pointer argument");
    if (!aligned(workspace, ALIGN)) return (vp_status)vpi_fail(VP_ERR_INVALID_ARG, "workspace must be 256-byte aligned");
    if (workspace_bytes < need) return (vp_status)vpi_fail(VP_ERR_WORKSPACE, "workspace of %zu bytes, %zu needed", workspace_bytes, need);
    hipStream_t st = (hipStream_t)hip_stream;
    const int words = ceil_div(V, 32);
    uint32_t *bitmaps = (uint32_t *)workspace;
    int32_t *sizes = (int32_t *)((char *)workspace + align_up((size_t)K * words * 4));
    vpk_aset_flags(top_ids, assign, (long)n, T, K, V, words, bitmaps, sizes, cand_offsets, st);
    int64_t tot = 0;
    hipError_t e = hipMemcpyAsync(&tot, cand_offsets + K, sizeof(tot), hipMemcpyDeviceToHost, st);
    if (e == hipSuccess) e = hipStreamSynchronize(st);
    if (e != hipSuccess) return (vp_status)vpi_fail(VP_ERR_HIP, "vp_active_sets: %s", hipGetErrorString(e));
    *total = tot;
    if (tot > capacity) return (vp_status)vpi_fail(VP_ERR_WORKSPACE, "cand_ids holds %lld entries, %lld needed", (long long)capacity, (long long)tot);
    if (tot > 0) vpk_aset_emit(bitmaps, words, K, cand_offsets, cand_ids, st);
    e = hipGetLastError();
    if (e != hipSuccess) return (vp_status)vpi_fail(VP_ERR_HIP, "vp_active_sets: %s", hipGetErrorString(e));
    return VP_OK;
}

}  // extern "C"
