// Internal layout definitions shared by the host API and the HIP kernels.
//
// Packed tile layout.  All matrices the hot kernels stream (per-cluster slabs,
// the whole-W copy, the centroids) are stored as 1 KiB tiles of 16 "items"
// (candidate tokens, or centroids) x 32 k-values, in the operand order of
// v_mfma_f32_16x16x32_f16: lane l of a wavefront owns item (l % 16) and the 8
// consecutive k-values starting at (l / 16) * 8, stored as 16 contiguous bytes
// at byte l * 16 of the tile.  The tiles of one group of 16 items follow each
// other along k (KT = d_pad / 32 tiles), so a group is one contiguous run of
// KT KiB, and consecutive groups are contiguous too: a wavefront that streams
// a range of items reads one linear range of memory, 1 KiB per load.
#pragma once
#include <stdint.h>

#define VP_TILE_ITEMS 16
#define VP_TILE_K 32
#define VP_TILE_BYTES 1024
#define VP_KPAD 256            // d is padded (with zeros) to a multiple of this
#define VP_WG_THREADS 256      // projection kernel: 4 wavefronts per workgroup
#define VP_WG_WAVES 4
#define VP_ROWS_PER_ITEM 16    // rows one work item projects (one MFMA row tile)
#define VP_BOUND_SETS 8          // per row: candidate-range sets whose best logits bound the k-th best (GEMM kernel)
#define VP_MAX_ROWS_PER_ITEM 64  // four row tiles: the GEMM-shaped kernel of single-bucket projections
#define VP_GEMV_MAX_ROWS 4
#define VP_RAW_TILES 2           // slab items of at most this many tiles per wavefront keep raw logits, no top-k lists
#define VP_XCD_BLOCK_ITEMS 32    // clustered plans with heavy buckets: consecutive items one XCD takes at a time

// One unit of projection work: up to 16 rows of one bucket against a range of
// candidate tiles of that bucket's slab.
struct VpItem {
    int32_t cluster;     // slab set entry (cluster id; 0 for the full-vocabulary set)
    int32_t perm_start;  // first position in perm[] of this item's rows
    int32_t nrows;       // 1..16
    int32_t tile0;       // first candidate tile, counted within the entry's slab
    int32_t ntiles;      // candidate tiles of this item (split among the 4 wavefronts)
    int32_t shared;      // 1 if other items (further row groups of the bucket) read the same tiles
    int32_t tile_off;    // first tile of the entry's slab within the slab set (copy of tile_off[cluster])
    int32_t ncand;       // candidates of the entry (copy of n_cand[cluster])
};

// Where the merge kernel finds everything about the row at one position of
// the bucket order: partial results sit at items item0, item0 + stride, ...
// (nit of them), in row slot `local` of each.
struct VpRowPlan {
    int32_t row;        // row number in the caller's batch
    int32_t cluster;
    int32_t item0;
    int32_t stride;
    int32_t nit;
    int32_t local;
    int32_t ids_off;    // first entry of the cluster's token-id list
    int32_t pad;
};

// Header the planning kernel leaves for the projection and merge kernels.
struct VpPlanHeader {
    int32_t total_items;
    int32_t tiles_per_wave;
    int32_t overflow;        // set if the item list did not fit (never expected)
    int32_t total_tiles;
    // Workgroup -> item swizzle.  > 1: a single bucket whose row groups share tiles (the
    // full-vocabulary projection): the number of row groups, with swz_chunks candidate ranges.
    // < 0: a clustered plan with buckets of many row groups: -(items per block), blocks of
    // consecutive items are dealt to the 8 XCDs in turn and every XCD starts at another place
    // of the list (see item_of_workgroup).  0: none.
    int32_t swz_rgs;
    int32_t swz_chunks;
    int32_t rows_per_item;   // row slots per item in the partial results (16, or 32 with two row tiles)
    int32_t mode;            // 0: per-cluster slabs; 1: masked full projection chosen by the planner
    int32_t pad[56];
};

// State of one batch-union projection (see union.hip).
struct VpUnionHeader {
    int32_t n_occ;     // occupied clusters
    int32_t n_union;   // |U|
    int32_t tiles;     // candidate groups of 16 in the union slab
    int32_t pad[61];
};

// A set of packed slabs: the K clusters, or the single whole-vocabulary slab.
struct VpSlabSet {
    const void *tiles;        // packed fp16 tiles of all entries back to back
    const float *bias;        // fp32 bias per candidate, padded to 16 per entry
    const int32_t *ids;       // token id per candidate (-1 in padding); NULL = identity
    const int32_t *tile_off;  // [entries + 1] cumulative candidate tiles
    const int32_t *n_cand;    // [entries] candidates per entry
    int32_t entries;
    int32_t kt;               // k-tiles per candidate group (d_pad / 32)
};

// Tiles per wavefront for a projection of total_tiles candidate tiles (counted once
// per row group): about target_items items when there is plenty of work; with little
// work, fewer and longer items (at least ~4 tiles per wavefront while that still
// leaves min_items items, one per resident workgroup slot), because a short item
// spends most of its life staging rows and waiting for its first loads.
static inline __host__ __device__ int vp_tiles_per_wave(long long total_tiles, int target_items, int min_items)
{
    long long eff = total_tiles / (4 * VP_WG_WAVES);
    if (eff < min_items) eff = min_items;
    if (eff > target_items) eff = target_items;
    if (eff < 1) eff = 1;
    const long long per = (long long)VP_WG_WAVES * eff;
    const long long tpw = (total_tiles + per - 1) / per;
    return (int)(tpw > 1 ? tpw : 1);
}

// Items of a single-bucket plan for the kernel that keeps an item's rows in LDS and runs one
// workgroup per compute unit (`slots` at a time): row groups x candidate ranges as close below a
// multiple of the slots as up to eight rounds allow, so that no round is left nearly empty (86 row
// groups on 256 slots: three ranges each would be 258 items, a second round for two of them; 23
// ranges are 7.7 rounds).  At least one range per row group.
static inline __host__ __device__ int vp_rounds_item_count(int rgs, int slots, int vtiles)
{
    if (slots < 1) slots = 1;
    int best = rgs;
    double best_fill = 0.0;
    for (int rounds = 1; rounds <= 8; ++rounds) {
        long long ranges = (long long)rounds * slots / rgs;
        if (ranges > vtiles) ranges = vtiles;
        if (ranges < 1) continue;
        const long long items = (long long)rgs * ranges;
        const long long full = (items + slots - 1) / slots * slots;
        const double fill = (double)items / (double)full;
        if (fill > best_fill + 1e-9) {
            best_fill = fill;
            best = (int)items;
        }
        if (fill > 0.97) break;
    }
    return best;
}

// The same for the clustered plan, which also knows its number of (bucket, row group) units:
// every unit ends with a partly filled item, so the plan has at most total / (4 tpw) + units
// items.  When that lies between one and two times the resident workgroup slots (min_items),
// the second round of workgroups would leave most of the chip idle (measured: 63 % against
// 72 % of the HBM peak at 1.4 rounds), so the items are made just long enough for one round.
static inline __host__ __device__ int vp_tiles_per_wave_units(long long total_tiles, int units, int target_items,
                                                              int min_items)
{
    const int tpw = vp_tiles_per_wave(total_tiles, target_items, min_items);
    const long long per = (long long)VP_WG_WAVES * tpw;
    const long long items_ub = (total_tiles + per - 1) / per + units;
    if (items_ub <= min_items || items_ub > 2LL * min_items || 2 * units >= min_items) return tpw;
    const long long room = (long long)VP_WG_WAVES * (min_items - units);
    const long long one_round = (total_tiles + room - 1) / room;
    return (int)(one_round > tpw ? one_round : tpw);
}

// The workgroup -> item maps behind VpPlanHeader.swz_rgs (wg = the workgroup's index in the grid;
// workgroups are handed to the 8 XCDs in turn).  Every item in [0, total_items) is taken by exactly
// one workgroup of a grid that is large enough (total_items + 8 blocks for the first map, the chunk
// count rounded up to 8 times the row groups for the second); the others get -1.
static inline __host__ __device__ int vp_item_of_workgroup(int wg, int total_items, int swz_rgs, int swz_chunks)
{
    const int xcd = wg & 7;
    if (swz_rgs < 0) {
        const int B = -swz_rgs;          // items per block
        const int l = wg >> 3;           // this XCD's l-th workgroup
        // Every XCD starts an eighth of the list further on (and wraps round), so that the
        // workgroups in flight at any time come from eight places of the list: a heavy bucket's
        // items, served by the L2, then overlap with items that stream from HBM on the other XCDs
        // instead of forming a phase of their own on the whole chip (skewed workload: 70 -> 77 %
        // of the HBM peak; most of it from this overlap, blocks of 8 to 32 items do equally well).
        const int nbx = ((total_items + B - 1) / B + 7) >> 3;   // blocks per XCD
        int i = l / B;
        if (i >= nbx) return -1;
        i = (i + xcd * ((nbx + 7) >> 3)) % nbx;
        const int it = (i * 8 + xcd) * B + l % B;
        return it < total_items ? it : -1;
    }
    if (swz_rgs > 1) {
        const int t = wg >> 3;
        const int chl = t / swz_rgs;
        const int ch = chl * 8 + xcd;
        if (ch >= swz_chunks) return -1;
        return ch * swz_rgs + (t - chl * swz_rgs);
    }
    return wg;
}

// What the masked full projection needs besides the slab set: each row's cluster
// and the per-cluster membership bit lists over the vocabulary.
struct VpMaskInfo {
    const int32_t *g;          // [N] cluster of each row (NULL: no masking)
    const uint32_t *bitmaps;   // [K][words]
    int32_t words;             // 32-bit words per cluster
};

// Machine constants of the planner's cost model (bytes per second).
struct VpCostModel {
    float bw_slab;   // slabs streamed once from HBM
    float bw_full;   // one pass over the packed W from HBM
    float bw_l2;     // further passes over tiles already in the L2 (16-row items)
    float bw_gemm;   // further passes over W by the 48- / 64-row items of the GEMM-shaped kernel (rows in LDS)
    float bw_gemm_split;   // the same for the split-k kernel (k-extents beyond d_pad = 1536, k > 32)
    float bw_gather; // batch-union form: columns of U gathered from the packed W into the union slab
    float t_gather;  // ... and the fixed time of the kernels only that gather needs (seconds)
    float t_row_slab;  // per-cluster slabs: time per row beyond the bytes (staging, lists, partial results; seconds)
};

#define VP_SMALL_ROWS 16   // batches up to this size are planned by the projection workgroups themselves

// What a workgroup of the small-batch projection needs to find its own work (project.hip).
struct VpSmallArgs {
    const int32_t *cpart;       // [N][parts][2] per-part (score bits, index) minima of Eq. 2
    int parts, N, K;
    const int32_t *tile_off;    // per cluster: first candidate tile of its slab
    const int32_t *n_cand;      // per cluster: candidates
    int target_items, min_items;
    int32_t *g;                 // [N] cluster of each row (out)
    int32_t *out_cluster;       // [N] or null
    VpRowPlan *rowplan;         // [N] the merge kernel's records, indexed by row (out)
    VpPlanHeader *hdr;          // (out)
};

// Size in floats of one partial result: running max, sum of exponentials, then
// k logits and k candidate positions.
static inline __host__ __device__ int vp_partial_floats(int k) { return 2 + 2 * k; }

#define VP_NEG_BIG (-3.0e38f)
#define VP_IDX_NONE 0x7fffffff
#define VP_FLOOR_NONE 0x007fffffu   // order-preserving key of -infinity (float_key in project.hip)
