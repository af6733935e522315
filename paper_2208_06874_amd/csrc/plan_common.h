// Device code shared by the planning kernels.
#pragma once
#include <hip/hip_runtime.h>
#include "vp_layout.h"

__device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

// Finishes Eq. 2 for rows 0 .. N-1: the minimum over a row's `parts` per-part minima (score bits,
// centroid index), ties to the lowest index.  Called by all `nthreads` threads of a workgroup (a
// multiple of 64).  With few rows several lanes share a row (a power of two, at most a wavefront,
// each taking every T-th part) so that the loads of a row are in flight together instead of one
// batch after the other; emit(r, j) is called once per row, by the first of its lanes.
template <typename Emit>
__device__ inline void vp_finish_eq2(const int2 *__restrict__ cpart, int parts, int N, int K, int tid, int nthreads,
                                     Emit emit)
{
    int T = 1;
    while (T < 64 && 2 * T * N <= nthreads && 2 * T <= parts) T *= 2;
    const int rows_per_pass = nthreads / T;
    const int sub = tid & (T - 1);
    for (int r0 = 0; r0 < N; r0 += rows_per_pass) {
        const int r = r0 + tid / T;
        float bs = __builtin_inff();
        int bj = VP_IDX_NONE;
        if (r < N) {
            const int2 *cp = cpart + (size_t)r * parts;
            for (int p0 = sub; p0 < parts; p0 += 8 * T) {
                int2 e[8];
#pragma unroll
                for (int v = 0; v < 8; ++v) e[v] = p0 + v * T < parts ? cp[p0 + v * T] : make_int2(0x7f800000, VP_IDX_NONE);
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float s = __int_as_float(e[v].x);
                    const bool take = (s < bs) | ((s == bs) & (e[v].y < bj));
                    bs = take ? s : bs;
                    bj = take ? e[v].y : bj;
                }
            }
        }
        for (int off = 1; off < T; off <<= 1) {   // (T is the same in every lane)
            const float s2 = __shfl_xor(bs, off);
            const int j2 = __shfl_xor(bj, off);
            const bool take = (s2 < bs) | ((s2 == bs) & (j2 < bj));
            bs = take ? s2 : bs;
            bj = take ? j2 : bj;
        }
        if (r < N && sub == 0) emit(r, (bj < 0 || bj >= K) ? 0 : bj);   // non-finite scores: keep every index in range
    }
}

// Plan for one bucket that holds all N rows in their own order against one slab
// of ncand candidates in vtiles tiles (the full vocabulary, or the union of the
// batch's active sets), rpi (16, 32 or 64) rows per item.  Called by every thread gtid of
// gsize cooperating threads.
__device__ inline void vp_plan_single_bucket(int N, int ncand, int vtiles, int rpi, int target_items, int min_items,
                                             int max_items, int32_t *__restrict__ perm,
                                             VpRowPlan *__restrict__ rowplan, unsigned int *__restrict__ floors,
                                             VpItem *__restrict__ items, VpPlanHeader *__restrict__ hdr,
                                             int64_t *__restrict__ dbg_row_off, int gtid, int gsize)
{
    const int rgs = ceil_div(N, rpi);
    const long long total_tiles = (long long)rgs * vtiles;
    const int tpw = vp_tiles_per_wave(total_tiles, target_items, min_items);
    const int tpi = tpw * VP_WG_WAVES;
    const int chunks = ceil_div(vtiles, tpi);
    const int total_items = min(chunks * rgs, max_items);
    for (int p = gtid; p < N; p += gsize) {
        perm[p] = p;
        floors[p] = VP_FLOOR_NONE;
        for (int j = 0; j < VP_BOUND_SETS; ++j) floors[N + p * VP_BOUND_SETS + j] = VP_FLOOR_NONE;
        VpRowPlan rp;
        rp.row = p;
        rp.cluster = 0;
        rp.item0 = p / rpi;
        rp.stride = rgs;
        rp.nit = chunks;
        rp.local = p % rpi;
        rp.ids_off = 0;
        rp.pad = 0;
        rowplan[p] = rp;
        if (dbg_row_off) dbg_row_off[p] = (int64_t)p * ncand;
    }
    for (int it = gtid; it < total_items; it += gsize) {
        const int ch = it / rgs;
        const int rg = it - ch * rgs;
        VpItem v;
        v.cluster = 0;
        v.perm_start = rg * rpi;
        v.nrows = min(rpi, N - rg * rpi);
        v.tile0 = ch * tpi;
        v.ntiles = min(tpi, vtiles - ch * tpi);
        v.shared = rgs > 1;
        v.tile_off = 0;
        v.ncand = ncand;
        items[it] = v;
    }
    if (gtid == 0) {
        hdr->total_items = total_items;
        hdr->tiles_per_wave = tpw;
        hdr->overflow = chunks * rgs > max_items;
        hdr->total_tiles = (int)min(total_tiles, 2147483647LL);
        // candidate ranges are dealt to the 8 XCDs only when there are enough of them to go round
        hdr->swz_rgs = (rgs > 1 && chunks >= 8) ? rgs : 0;
        hdr->swz_chunks = chunks;
        hdr->rows_per_item = rpi;
        hdr->mode = 0;
        if (dbg_row_off) dbg_row_off[N] = (int64_t)N * ncand;
    }
}

// Cost model of the planner.  Slabs: the occupied slabs are streamed once from HBM, further row
// groups of a bucket re-read them through the L2, and every row costs a little beyond its bytes
// (staging, top-k lists, partial results: what a batch of many rows against short lists is made
// of).  Masked full projection with 64-row items: one pass over W from HBM, or the matrix cores'
// time for all row groups, whichever is longer (W is then served by the L2; the rate of the
// matrix cores is expressed in bytes of W per second).  With 16-row items every row group
// re-reads W through the L2.  The top-k lists cost the full projection more than the slabs
// (every lane of every wavefront is busy there): a margin that grows with k keeps the choice on
// the safe side (64-row items: top-8 measured 10 % over top-1).  Tile counts are in candidate
// groups; the rates are groups per second.
__device__ inline bool vp_full_is_cheaper(int occ_tiles, int total_tiles, int N, int rpi_full, int vtiles, int k,
                                          const VpCostModel &cost)
{
    const int rgs_full = ceil_div(N, rpi_full);
    const float t_slab = occ_tiles / cost.bw_slab + (total_tiles - occ_tiles) / cost.bw_l2 + N * cost.t_row_slab;
    const float t_full = rpi_full >= 48
        ? fmaxf(vtiles / cost.bw_full, rgs_full * (vtiles / cost.bw_gemm)) * (1.f + k * 0.0125f)
        : fmaxf(vtiles / cost.bw_full, (float)rgs_full * vtiles / cost.bw_l2) * (1.f + k * 0.125f);
    return t_full < t_slab;
}
