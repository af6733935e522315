// Device code shared by the planning kernels.
#pragma once
#include <hip/hip_runtime.h>
#include "vp_layout.h"

__device__ inline int ceil_div(int a, int b) { return (a + b - 1) / b; }

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
    const float t_full = rpi_full == 64
        ? fmaxf(vtiles / cost.bw_full, rgs_full * (vtiles / cost.bw_gemm)) * (1.f + k * 0.0125f)
        : fmaxf(vtiles / cost.bw_full, (float)rgs_full * vtiles / cost.bw_l2) * (1.f + k * 0.125f);
    return t_full < t_slab;
}
