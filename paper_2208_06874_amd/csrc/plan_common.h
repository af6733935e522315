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

// Cost model of the planner: the occupied slabs are streamed once from HBM and further row
// groups of a bucket re-read them through the L2; the masked full projection streams W once
// and pays for every further row group.  The top-k lists cost the full projection more than
// the slabs (every lane of every wavefront is busy there): a margin that grows with k keeps
// the choice on the safe side.  64-row items: one pass from HBM, each further row group at
// the measured rate of the GEMM-shaped kernel.  16-row items: every row group re-reads W
// through the L2.  Tile counts are in candidate groups; the constants are groups per second.
__device__ inline bool vp_full_is_cheaper(int occ_tiles, int total_tiles, int N, int rpi_full, int vtiles, int k,
                                          const VpCostModel &cost)
{
    const int rgs_full = ceil_div(N, rpi_full);
    const float t_slab = occ_tiles / cost.bw_slab + (total_tiles - occ_tiles) / cost.bw_l2;
    const float t_full = rpi_full == 64
        ? (vtiles / cost.bw_full + (rgs_full - 1) * (vtiles / cost.bw_gemm)) * (1.f + k * 0.0625f)
        : fmaxf(vtiles / cost.bw_full, (float)rgs_full * vtiles / cost.bw_l2) * (1.f + k * 0.125f);
    return t_full < t_slab;
}

constexpr int VP_PLAN_SMALL_THREADS = 256;

// The planner for batches of at most 64 rows, run by one workgroup of 256 threads: lane r of
// every wavefront stands for row r, buckets are found by comparing cluster ids across the
// lanes, so nothing depends on the number of clusters and there are three barriers in all.
// Same plan as plan_kernel's, with the rows of a bucket in ascending order.  cpart is read
// with device-scope loads: the workgroups that wrote it may sit on other XCDs.
__device__ inline void vp_plan_small(const int2 *cpart, int parts, int N, int K, const VpPlanArgs &a)
{
    __shared__ float ps[4][VP_PLAN_SMALL_ROWS];
    __shared__ int pj[4][VP_PLAN_SMALL_ROWS];
    __shared__ int tab[VP_PLAN_SMALL_ROWS][8];   // per bucket: cluster, first perm slot, rows, tiles, first item, tile_off, n_cand
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int r = lane;

    // finish Eq. 2: each wavefront takes a quarter of the parts of every row
    {
        float bs = __builtin_inff();
        int bj = VP_IDX_NONE;
        if (r < N) {
            const int *cp = reinterpret_cast<const int *>(cpart + (size_t)r * parts);
            for (int p0 = wave; p0 < parts; p0 += 32) {
                int ex[8], ey[8];
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const int p = p0 + v * 4;
                    ex[v] = 0x7f800000;
                    ey[v] = VP_IDX_NONE;
                    if (p < parts) {
                        ex[v] = __hip_atomic_load(cp + 2 * p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                        ey[v] = __hip_atomic_load(cp + 2 * p + 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                    }
                }
#pragma unroll
                for (int v = 0; v < 8; ++v) {
                    const float s = __int_as_float(ex[v]);
                    const bool take = (s < bs) | ((s == bs) & (ey[v] < bj));   // (selects, no branches)
                    bs = take ? s : bs;
                    bj = take ? ey[v] : bj;
                }
            }
        }
        ps[wave][r] = bs;
        pj[wave][r] = bj;
    }
    __syncthreads();
    int j = VP_IDX_NONE;
    if (r < N) {
        float bs = ps[0][r];
        j = pj[0][r];
#pragma unroll
        for (int w = 1; w < 4; ++w) {
            const float s = ps[w][r];
            const int jj = pj[w][r];
            const bool take = (s < bs) | ((s == bs) & (jj < j));
            bs = take ? s : bs;
            j = take ? jj : j;
        }
        if (j < 0 || j >= K) j = 0;   // non-finite scores: keep every index in range
    }
    int tl = 0, to = 0, nc = 0;
    if (r < N) {
        to = a.tile_off[j];
        tl = a.tile_off[j + 1] - to;
        nc = a.n_cand[j];
    }
    if (wave == 0 && r < N) {
        a.g[r] = j;
        if (a.out_cluster) a.out_cluster[r] = j;
    }

    // position of every row in bucket order, size of its bucket
    int before = 0, same_before = 0, same_total = 0;
    for (int s = 0; s < N; ++s) {
        const int js = __builtin_amdgcn_readlane(j, s);   // s is the same in every lane: a lane read, no shuffle
        before += (js < j || (js == j && s < r)) ? 1 : 0;
        same_before += (js == j && s < r) ? 1 : 0;
        same_total += (js == j) ? 1 : 0;
    }
    const bool leader = r < N && same_before == 0;
    const int rgs = ceil_div(same_total, VP_ROWS_PER_ITEM);
    int total_tiles = leader ? rgs * tl : 0;
    int occ_tiles = leader ? tl : 0;
    int units = leader ? rgs : 0;
#pragma unroll
    for (int off = 1; off < 64; off <<= 1) {
        total_tiles += __shfl_xor(total_tiles, off);
        occ_tiles += __shfl_xor(occ_tiles, off);
        units += __shfl_xor(units, off);
    }
    if (a.dispatch && vp_full_is_cheaper(occ_tiles, total_tiles, N, a.dispatch, a.vtiles, a.k, a.cost)) {
        vp_plan_single_bucket(N, a.V, a.vtiles, a.dispatch, a.full_target_items, a.full_min_items, a.max_items_full,
                              a.perm, a.rowplan, a.floors, a.items, a.hdr, nullptr, tid, VP_PLAN_SMALL_THREADS);
        if (tid == 0) a.hdr->mode = 1;
        return;
    }
    const int tpw = vp_tiles_per_wave_units(total_tiles, units, a.target_items, a.min_items);
    const int tpi = tpw * VP_WG_WAVES;
    const int nit = ceil_div(tl, tpi);
    const int c = leader ? rgs * nit : 0;
    int ioff = 0, brank = 0, all_items = 0, nb = 0;
    for (int s = 0; s < N; ++s) {
        const int js = __builtin_amdgcn_readlane(j, s);
        const int cs = __builtin_amdgcn_readlane(c, s);
        const int ls = __builtin_amdgcn_readlane(leader ? 1 : 0, s);
        const bool lower = ls && js < j;
        ioff += lower ? cs : 0;
        brank += lower ? 1 : 0;
        all_items += cs;
        nb += ls;
    }
    if (wave == 0 && r < N) {
        const int p = before;
        a.perm[p] = r;
        a.floors[r] = VP_FLOOR_NONE;   // no lower bound of the row's k-th best logit known yet
        VpRowPlan rp;
        rp.row = r;
        rp.cluster = j;
        rp.item0 = ioff + same_before / VP_ROWS_PER_ITEM;
        rp.stride = rgs;
        rp.nit = nit;
        rp.local = same_before % VP_ROWS_PER_ITEM;
        rp.ids_off = to * VP_TILE_ITEMS;
        rp.pad = 0;
        a.rowplan[p] = rp;
        if (leader) {
            tab[brank][0] = j;
            tab[brank][1] = before;
            tab[brank][2] = same_total;
            tab[brank][3] = tl;
            tab[brank][4] = ioff;
            tab[brank][5] = to;
            tab[brank][6] = nc;
        }
    }
    __syncthreads();
    const int total_items = min(all_items, a.max_items);
    // the items: for each bucket, candidate ranges outermost and row groups innermost
    for (int it = tid; it < total_items; it += VP_PLAN_SMALL_THREADS) {
        int lo = 0, hi = nb;   // largest bucket whose first item is <= it (buckets without items have empty ranges)
        while (hi - lo > 1) {
            const int mid = (lo + hi) >> 1;
            if (tab[mid][4] <= it) lo = mid; else hi = mid;
        }
        const int rows = tab[lo][2];
        const int brgs = ceil_div(rows, VP_ROWS_PER_ITEM);
        const int local = it - tab[lo][4];
        const int ch = local / brgs;
        const int rg = local - ch * brgs;
        VpItem v;
        v.cluster = tab[lo][0];
        v.perm_start = tab[lo][1] + rg * VP_ROWS_PER_ITEM;
        v.nrows = min(VP_ROWS_PER_ITEM, rows - rg * VP_ROWS_PER_ITEM);
        v.tile0 = ch * tpi;
        v.ntiles = min(tpi, tab[lo][3] - ch * tpi);
        v.shared = brgs > 1;
        v.tile_off = tab[lo][5];
        v.ncand = tab[lo][6];
        a.items[it] = v;
    }
    if (tid == 0) {
        a.hdr->total_items = total_items;
        a.hdr->tiles_per_wave = tpw;
        a.hdr->overflow = all_items > a.max_items;
        a.hdr->total_tiles = total_tiles;
        a.hdr->swz_rgs = 0;
        a.hdr->swz_chunks = 0;
        a.hdr->rows_per_item = VP_ROWS_PER_ITEM;
        a.hdr->mode = 0;
    }
}
