// Gathered per-cluster projection with the fused candidate log-softmax / top-k.
//
// For each work item (up to 16 rows of one bucket x a range of candidate tiles
// of that bucket's slab) this computes Eq. 1 of section 2.1 restricted to the
// cluster's active tokens (step 3 of the inference list in section 2.3),
//     z[r, c] = sum_i h[r, i] * S_j[c, i] + b_j[c],
// and folds the logits straight into the pieces of steps 4-5 (softmax over the
// listed tokens only; the rest are at -infinity) and of the descending sort of
// section 2.1: a running maximum, a running sum of exponentials and the k best
// (logit, candidate position) pairs.  Logits never leave the registers.
//
// Each of the 4 wavefronts streams its own contiguous run of packed tiles
// (vp_layout.h) with 1 KiB loads, 8 loads in flight.  Two inner loops share
// everything else:
//   MFMA: v_mfma_f32_16x16x32_f16 with the slab tile as the A operand and the
//         16 hidden rows (staged once in LDS, in operand order) as B.  Lane l
//         then owns row l % 16 and candidates 4 * (l / 16) .. + 3 of the tile.
//   GEMV: buckets of at most `rstar` (<= 4) rows: v_dot2_f32_f16 against the
//         rows held row-major in LDS, partial sums of the four k-slices added
//         with cross-lane shuffles.
// Both stream the slab exactly once at full load width; which is faster for a
// given bucket size is a measured choice.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"
#include "project_common.h"
#include "wave_ops.h"

namespace {

// PF = 1 KiB tile loads a wavefront keeps in flight.  RT = row tiles of 16 rows per
// item: 1 everywhere except in single-bucket projections (full, union) of more than
// 16 rows, where RT = 2 feeds every loaded slab tile to two MFMAs (half the L2-to-CU
// traffic per row) and, with half as many wavefronts per CU, keeps twice the loads in
// flight per wavefront.
template <bool NT, int RT, int PF, bool MASKED>
__device__ inline void project_item(
    const VpSlabSet &set, const uint4 *__restrict__ hidden, int d, int row_of_tid,
    const VpItem &item, int it, int tpw, int k, int rstar,
    float *__restrict__ partials, unsigned int *__restrict__ floors, float *__restrict__ dbg_logits,
    const int64_t *__restrict__ dbg_row_off, const VpMaskInfo &mask, bool raw_ok = false)
{
    // row_of_tid: for threads tid < 16 * RT, the batch row in row slot tid of the item (-1: none)
    constexpr int ROWS = 16 * RT;               // row slots of an item
    const int KT = set.kt;
    const int X = KT * 4;                       // 16-byte pieces per padded row
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int n = lane & 15;                    // this lane owns row slots n, 16 + n, ... in the epilogue
    const int q = lane >> 4;
    const bool gemv = RT == 1 && item.nrows <= rstar;

    extern __shared__ uint4 lds[];
    uint4 *ldsA = lds;                                                       // RT * KT KiB: the hidden rows
    float *list_val = reinterpret_cast<float *>(lds + (size_t)RT * KT * 64);  // [4 waves][k][ROWS]
    int *list_idx = reinterpret_cast<int *>(list_val + VP_WG_WAVES * k * ROWS);
    float *hdr_m = reinterpret_cast<float *>(list_idx + VP_WG_WAVES * k * ROWS);   // [4][16]
    float *hdr_s = hdr_m + VP_WG_WAVES * ROWS;
    int *rowid = reinterpret_cast<int *>(hdr_s + VP_WG_WAVES * ROWS);             // [ROWS]
    unsigned int *wg_floor = reinterpret_cast<unsigned int *>(rowid + ROWS);      // [ROWS]
    int *rowcl = reinterpret_cast<int *>(wg_floor + ROWS);                        // [ROWS] (masked projection)
    // Items of at most two tiles per wavefront (a handful of rows against few candidates: the whole
    // call is a few tens of microseconds) keep no top-k lists while they stream.  A list that has
    // seen fewer than a few dozen candidates takes almost every one of them, one LDS insertion
    // after the other, which cost more than the streaming itself; instead the logits (at most 32
    // per row and wavefront) go to LDS as they are and the epilogue selects among them.
    const bool raw = RT == 1 && raw_ok && tpw <= VP_RAW_TILES;
    float *raw_val = reinterpret_cast<float *>(rowcl + ROWS);   // [4 waves][32 slots][16 rows], only if raw_ok

    // this wavefront's run of tiles; its first loads go out before anything else
    const int ncand = item.ncand;
    const int toff = item.tile_off;
    const uint4 *slab = reinterpret_cast<const uint4 *>(set.tiles) + (size_t)toff * KT * 64;
    const float *bias = set.bias + (size_t)toff * VP_TILE_ITEMS;
    const int tb = item.tile0 + wave * tpw;
    const int te = min(tb + tpw, item.tile0 + item.ntiles);
    const uint4 *sp = slab + (size_t)tb * KT * 64 + lane;
    uint4 buf[PF];
    float4 bcur = make_float4(0.f, 0.f, 0.f, 0.f);
    if (tb < te) {
#pragma unroll
        for (int u = 0; u < PF; ++u) buf[u] = load_piece<NT>(sp + (size_t)u * 64);
        bcur = *reinterpret_cast<const float4 *>(bias + tb * VP_TILE_ITEMS + q * 4);
    }

    if (tid < ROWS) {
        const int row = row_of_tid;
        rowid[tid] = row;
        // buckets walked by several row groups hand their bound from workgroup to workgroup
        wg_floor[tid] = (item.shared && row >= 0) ? floors[row] : VP_FLOOR_NONE;
        if (MASKED) rowcl[tid] = row >= 0 ? mask.g[row] : 0;
    }
    for (int e = tid; e < VP_WG_WAVES * k * ROWS; e += VP_WG_THREADS) {
        list_val[e] = -__builtin_inff();
        list_idx[e] = VP_IDX_NONE;
    }
    if (raw)
        for (int e = tid; e < VP_WG_WAVES * VP_RAW_TILES * VP_TILE_ITEMS * 16; e += VP_WG_THREADS) raw_val[e] = -__builtin_inff();
    __syncthreads();

    // Stage the item's hidden rows: MFMA operand order, or row-major for the GEMV loop.
    // Row slots beyond nrows are left as they are: an MFMA output column depends on its
    // own operand column only, and those columns are never looked at.
    // (four pieces per thread are fetched together: a full item's 8 to 12 pieces per thread cost two or
    // three trips to the L2, not one each)
    {
        const int pieces_per_row = d >> 3;
        const int total = item.nrows * X;
        for (int e0 = tid; e0 < total; e0 += 4 * VP_WG_THREADS) {
            uint4 v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * VP_WG_THREADS;
                const int r = e / X;
                const int x = e - r * X;
                v[u] = make_uint4(0, 0, 0, 0);
                if (e < total && x < pieces_per_row) v[u] = hidden[(size_t)rowid[r] * pieces_per_row + x];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * VP_WG_THREADS;
                const int r = e / X;
                const int x = e - r * X;
                if (e < total) {
                    if (gemv) ldsA[r * X + x] = v[u];
                    else ldsA[((r >> 4) * KT + (x >> 2)) * 64 + (x & 3) * 16 + (r & 15)] = v[u];
                }
            }
        }
    }
    __syncthreads();

    RowState st[RT];
    RowList list[RT];
    bool row_valid[RT];
    int64_t dbg_base[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        const int slot = rt * 16 + n;
        row_valid[rt] = slot < item.nrows;
        st[rt].m = VP_NEG_BIG;
        st[rt].s = 0.f;
        st[rt].thr = row_valid[rt] ? -__builtin_inff() : __builtin_inff();
        list[rt].val = list_val + wave * k * ROWS + slot;
        list[rt].idx = list_idx + wave * k * ROWS + slot;
        list[rt].stride = ROWS;
        dbg_base[rt] = (dbg_logits && row_valid[rt]) ? dbg_row_off[rowid[slot]] : 0;
    }

    // masked full projection: the 4 membership bits of this lane's candidates, per row tile,
    // fetched a tile ahead like the bias (4 consecutive tokens never straddle a 32-bit word)
    const uint32_t *mrow[RT];
    uint32_t mcur[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        mrow[rt] = MASKED ? mask.bitmaps + (size_t)rowcl[rt * 16 + n] * mask.words : nullptr;
        mcur[rt] = 0xffffffffu;
        if (MASKED && tb < te) mcur[rt] = mrow[rt][(tb * VP_TILE_ITEMS + q * 4) >> 5];
    }

    // top-1 without lists (not for the masked projection, whose register budget is tight)
    const bool top1 = !MASKED && k == 1 && !raw;
    float b1v[RT];
    int b1i[RT];
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
        b1v[rt] = -__builtin_inff();
        b1i[rt] = VP_IDX_NONE;
    }
    const bool exchange = item.shared && wave == 0 && q == 0 && !top1;
    unsigned int pending[RT];
    bool has_pending = false;
    if (tb < te) {
        const int S = (te - tb) * KT;   // 1 KiB steps; KT % 8 == 0
        int kt = 0;
        int tile = tb;
        floatx4 acc[RT];                              // MFMA: 4 candidates of row slot rt * 16 + n
#pragma unroll
        for (int rt = 0; rt < RT; ++rt) acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
        float ga[VP_GEMV_MAX_ROWS] = {0.f, 0.f, 0.f, 0.f};   // GEMV: candidate n, k-slice q, rows 0..3

        for (int s0 = 0; s0 < S; s0 += PF) {
#pragma unroll
            for (int u = 0; u < PF; ++u) {
                Frag a;
                a.u = buf[u];
                const int nx = s0 + PF + u;
                if (nx < S) buf[u] = load_piece<NT>(sp + (size_t)nx * 64);
                if (!gemv) {
#pragma unroll
                    for (int rt = 0; rt < RT; ++rt) {
                        Frag b;
                        b.u = ldsA[(rt * KT + kt + u) * 64 + lane];
                        acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, b.h, acc[rt], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int r = 0; r < VP_GEMV_MAX_ROWS; ++r) {
                        if (r < item.nrows) {
                            Frag b;
                            b.u = ldsA[r * X + (kt + u) * 4 + q];
#pragma unroll
                            for (int e = 0; e < 4; ++e) ga[r] = __builtin_amdgcn_fdot2(a.p[e], b.p[e], ga[r], false);
                        }
                    }
                }
            }
            kt += PF;
            if (kt == KT) {
                // a group of 16 candidates is complete for all rows
                const int c0 = tile * VP_TILE_ITEMS + q * 4;
                const float bz[4] = {bcur.x, bcur.y, bcur.z, bcur.w};
#pragma unroll
                for (int rt = 0; rt < RT; ++rt) {
                    float z[4];
                    if (!gemv) {
                        z[0] = acc[rt][0]; z[1] = acc[rt][1]; z[2] = acc[rt][2]; z[3] = acc[rt][3];
                        acc[rt] = floatx4{0.f, 0.f, 0.f, 0.f};
                    } else {
                        float full[VP_GEMV_MAX_ROWS];
#pragma unroll
                        for (int r = 0; r < VP_GEMV_MAX_ROWS; ++r) {
                            float t = ga[r];
                            t += __shfl_xor(t, 16);
                            t += __shfl_xor(t, 32);
                            full[r] = t;     // every lane with the same (lane & 15) holds candidate (lane & 15) of row r
                            ga[r] = 0.f;
                        }
                        // hand lane (n, q) the logits of row n for candidates 4q .. 4q+3
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const int src = q * 4 + i;
                            const float t0 = __shfl(full[0], src);
                            const float t1 = __shfl(full[1], src);
                            const float t2 = __shfl(full[2], src);
                            const float t3 = __shfl(full[3], src);
                            z[i] = n == 0 ? t0 : n == 1 ? t1 : n == 2 ? t2 : t3;
                        }
                    }
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const bool member = !MASKED || ((mcur[rt] >> ((c0 & 31) + i)) & 1u);
                        z[i] = (c0 + i < ncand && member) ? z[i] + bz[i] : -__builtin_inff();
                    }
                    if (dbg_logits && row_valid[rt]) {
#pragma unroll
                        for (int i = 0; i < 4; ++i)
                            if (c0 + i < ncand) dbg_logits[dbg_base[rt] + c0 + i] = z[i];
                    }
                    if (raw) {
                        const float tmax = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
                        const float mn = fmaxf(st[rt].m, tmax);
                        st[rt].s = st[rt].s * fast_exp(st[rt].m - mn) + fast_exp(z[0] - mn) + fast_exp(z[1] - mn) +
                                   fast_exp(z[2] - mn) + fast_exp(z[3] - mn);
                        st[rt].m = mn;
                        float *slot = raw_val + ((wave * VP_RAW_TILES + (tile - tb)) * VP_TILE_ITEMS + q * 4) * 16 + n;
#pragma unroll
                        for (int i = 0; i < 4; ++i) slot[i * 16] = z[i];
                    } else if (top1) {
                        // greedy search: the best (logit, position) of this lane's stream stays in registers;
                        // positions ascend along the stream, so a strict comparison keeps the smaller one
                        const float tmax = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
                        const float mn = fmaxf(st[rt].m, tmax);
                        st[rt].s = st[rt].s * fast_exp(st[rt].m - mn) + fast_exp(z[0] - mn) + fast_exp(z[1] - mn) +
                                   fast_exp(z[2] - mn) + fast_exp(z[3] - mn);
                        st[rt].m = mn;
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const bool take = z[i] > b1v[rt];
                            b1v[rt] = take ? z[i] : b1v[rt];
                            b1i[rt] = take ? c0 + i : b1i[rt];
                        }
                    } else {
                        fold_logits(z, c0, q, k, st[rt], list[rt], wg_floor + rt * 16 + n);
                    }
                }
                if (exchange) {
                    // Every fourth tile the first wavefront trades bounds with the other workgroups
                    // that walk this bucket: one atomicMax per row publishes ours and returns
                    // theirs, which is folded into the LDS copy a tile later (no wait here).
                    if (has_pending) {
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt)
                            if (row_valid[rt]) atomicMax(wg_floor + rt * 16 + n, pending[rt]);
                        has_pending = false;
                    }
                    if (((tile - tb) & 3) == 3) {
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt)
                            if (row_valid[rt])
                                pending[rt] = atomicMax(floors + rowid[rt * 16 + n],
                                                        __hip_atomic_load(wg_floor + rt * 16 + n, __ATOMIC_RELAXED,
                                                                          __HIP_MEMORY_SCOPE_WORKGROUP));
                        has_pending = true;
                    }
                }
                kt = 0;
                ++tile;
                if (tile < te) {
                    bcur = *reinterpret_cast<const float4 *>(bias + tile * VP_TILE_ITEMS + q * 4);
                    if (MASKED) {
#pragma unroll
                        for (int rt = 0; rt < RT; ++rt) mcur[rt] = mrow[rt][(tile * VP_TILE_ITEMS + q * 4) >> 5];
                    }
                }
            }
        }
    }

    // the four lanes that own a row (one per candidate quarter) -> one (m, s)
#pragma unroll
    for (int rt = 0; rt < RT; ++rt) {
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float m2 = __shfl_xor(st[rt].m, off);
            const float s2 = __shfl_xor(st[rt].s, off);
            const float mn = fmaxf(st[rt].m, m2);
            st[rt].s = st[rt].s * fast_exp(st[rt].m - mn) + s2 * fast_exp(m2 - mn);
            st[rt].m = mn;
        }
        if (q == 0) {
            hdr_m[wave * ROWS + rt * 16 + n] = st[rt].m;
            hdr_s[wave * ROWS + rt * 16 + n] = st[rt].s;
        }
        if (top1) {
            // the row's four lanes -> this wavefront's one-entry list
#pragma unroll
            for (int off = 16; off <= 32; off <<= 1) {
                const float v2 = __shfl_xor(b1v[rt], off);
                const int i2 = __shfl_xor(b1i[rt], off);
                const bool take = (v2 > b1v[rt]) | ((v2 == b1v[rt]) & (i2 < b1i[rt]));
                b1v[rt] = take ? v2 : b1v[rt];
                b1i[rt] = take ? i2 : b1i[rt];
            }
            if (q == 0 && row_valid[rt]) {
                list_val[wave * k * ROWS + rt * 16 + n] = b1v[rt];
                list_idx[wave * k * ROWS + rt * 16 + n] = b1i[rt];
            }
        }
    }
    __syncthreads();

    // Combine the workgroup's four lists per row (one per wavefront) into one partial
    // result per (item, row): k rounds of "best entry after the previous winner".
    const int PFL = vp_partial_floats(k);
    for (int r = wave; r < item.nrows; r += VP_WG_WAVES) {
        float M = hdr_m[r];
#pragma unroll
        for (int w = 1; w < VP_WG_WAVES; ++w) M = fmaxf(M, hdr_m[w * ROWS + r]);
        float Ssum = 0.f;
#pragma unroll
        for (int w = 0; w < VP_WG_WAVES; ++w) Ssum += hdr_s[w * ROWS + r] * fast_exp(hdr_m[w * ROWS + r] - M);
        float *out = partials + ((size_t)it * ROWS + r) * PFL;
        if (lane == 0) {
            out[0] = M;
            out[1] = Ssum;
        }
        // lane -> one of the 4 source lists and a residue class (mod 16) of its slots
        const float *sv = list_val + (lane & 3) * k * ROWS + r;
        const int *si = list_idx + (lane & 3) * k * ROWS + r;
        // without lists: this lane's two of the row's 4 x 32 stored logits and their candidate positions
        float rv[2] = {-__builtin_inff(), -__builtin_inff()};
        int ri[2] = {VP_IDX_NONE, VP_IDX_NONE};
        if (raw) {
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int e = lane + u * 64;   // wavefront e / 32 of the item, its slot e % 32
                rv[u] = raw_val[e * 16 + r];
                if (rv[u] > -__builtin_inff())
                    ri[u] = (item.tile0 + (e / (VP_RAW_TILES * VP_TILE_ITEMS)) * tpw) * VP_TILE_ITEMS +
                            e % (VP_RAW_TILES * VP_TILE_ITEMS);
            }
        }
        float pv = __builtin_inff();
        int pi = -1;
        for (int t = 0; t < k; ++t) {
            float bv = -__builtin_inff();
            int bi = VP_IDX_NONE;
            if (raw) {
#pragma unroll
                for (int u = 0; u < 2; ++u) {
                    const bool after_prev = rv[u] < pv || (rv[u] == pv && ri[u] > pi);
                    if (after_prev && entry_before(rv[u], ri[u], bv, bi)) {
                        bv = rv[u];
                        bi = ri[u];
                    }
                }
            } else
            for (int p = lane >> 2; p < k; p += 16) {
                const float v = sv[p * ROWS];
                const int i = si[p * ROWS];
                const bool after_prev = v < pv || (v == pv && i > pi);
                if (after_prev && entry_before(v, i, bv, bi)) {
                    bv = v;
                    bi = i;
                }
            }
            wave_best_entry(bv, bi);
            if (lane == 0) {
                out[2 + t] = bv;
                out[2 + k + t] = __int_as_float(bi);
            }
            pv = bv;
            pi = bi;
        }
    }
    if (item.shared && tid < item.nrows) atomicMax(floors + rowid[tid], wg_floor[tid]);
}

// The batch row in row slot threadIdx.x of an item of the planner's list (-1: no such slot).
__device__ inline int row_of_slot(const int32_t *__restrict__ perm, const VpItem &item, int slots)
{
    const int tid = threadIdx.x;
    return (tid < slots && tid < item.nrows) ? perm[item.perm_start + tid] : -1;
}

__global__ __launch_bounds__(VP_WG_THREADS) void project_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, const int32_t *__restrict__ perm,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k, int rstar,
    float *__restrict__ partials, unsigned int *__restrict__ floors, float *__restrict__ dbg_logits,
    const int64_t *__restrict__ dbg_row_off, int raw_ok)
{
    // without the swizzle the item record does not depend on the header: both loads go out
    // together (the grid never exceeds the item array; records past total_items are unused)
    const VpItem probe = items[blockIdx.x];
    const int total_items = hdr->total_items;
    const int tpw = hdr->tiles_per_wave;
    if (hdr->mode != 0) return;   // the planner chose the masked full projection for this batch
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = it == (int)blockIdx.x ? probe : items[it];
    const VpMaskInfo none = {nullptr, nullptr, 0};
    if (item.shared)
        project_item<false, 1, 8, false>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, rstar, partials, floors, dbg_logits,
                                         dbg_row_off, none, raw_ok != 0);
    else
        project_item<true, 1, 8, false>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, rstar, partials, floors, dbg_logits,
                                        dbg_row_off, none, raw_ok != 0);
}

// Batches of at most 16 rows: no planning kernel, no item list.  Every workgroup reduces the
// per-part minima of Eq. 2 itself (lane l: row l / 4, every fourth part; the row's cluster id ends
// up in all four of its lanes), finds the buckets by comparing cluster ids across lanes, sizes the
// items with the planner's own rule and takes the item with its own number: bucket = cluster (in
// ascending order of the cluster id), range of candidate tiles = its chunk of that cluster's slab.
// The plan is therefore the one plan_kernel would write - same buckets, same item boundaries, same
// partial results - but nothing waits for a planner, and the only loads in front of the first slab
// byte are the minima and two words of the cluster's metadata.  The first workgroup of a bucket
// leaves the merge kernel's records of the bucket's rows, workgroup 0 the header and the clusters.
template <int PF>
__device__ inline void project_small(const VpSlabSet &set, const uint4 *__restrict__ hidden, int d, const VpSmallArgs &a,
                                     int k, int rstar, float *__restrict__ partials, int raw_ok)
{
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int r = lane >> 2;     // the row this lane stands for
    const int sub = lane & 3;
    const int N = a.N;

    // finish Eq. 2: minimum over the centroid parts, ties to the lowest index
    float bs = __builtin_inff();
    int bj = VP_IDX_NONE;
    if (r < N) {
        const int2 *cp = reinterpret_cast<const int2 *>(a.cpart) + (size_t)r * a.parts;
        // (up to 64 parts in one batch of loads: one round trip, not one per four parts)
        for (int p0 = 0; p0 < a.parts; p0 += 64) {
            int2 e[16];
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const int p = p0 + 4 * u + sub;
                e[u] = p < a.parts ? cp[p] : make_int2(0x7f800000, VP_IDX_NONE);
            }
#pragma unroll
            for (int u = 0; u < 16; ++u) {
                const float s = __int_as_float(e[u].x);
                const bool take = (s < bs) | ((s == bs) & (e[u].y < bj));
                bs = take ? s : bs;
                bj = take ? e[u].y : bj;
            }
        }
    }
#define VP_QUAD_MIN(ctrl)                                                                                        \
    {                                                                                                            \
        const float s2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(bs), ctrl, 0xf, 0xf, false)); \
        const int j2 = __builtin_amdgcn_update_dpp(0, bj, ctrl, 0xf, 0xf, false);                                \
        const bool take = (s2 < bs) | ((s2 == bs) & (j2 < bj));                                                  \
        bs = take ? s2 : bs;                                                                                     \
        bj = take ? j2 : bj;                                                                                     \
    }
    VP_QUAD_MIN(0xB1)   // quad_perm [1, 0, 3, 2]
    VP_QUAD_MIN(0x4E)   // quad_perm [2, 3, 0, 1]
#undef VP_QUAD_MIN
    int j = -1;          // rows beyond N match no bucket
    int to = 0, nc = 0;
    if (r < N) {
        j = (bj < 0 || bj >= a.K) ? 0 : bj;   // non-finite scores: keep every index in range
        to = a.tile_off[j];
        nc = a.n_cand[j];
    }
    const int tl = (nc + VP_TILE_ITEMS - 1) / VP_TILE_ITEMS;

    // position of every row among the rows of its cluster
    int same_before = 0, same_total = 0;
    for (int s = 0; s < N; ++s) {
        const int js = __builtin_amdgcn_readlane(j, 4 * s);
        same_before += (js == j && s < r) ? 1 : 0;
        same_total += (js == j) ? 1 : 0;
    }
    const bool leader = r < N && sub == 0 && same_before == 0;   // one lane per bucket
    const int total_tiles = wave_sum(leader ? tl : 0);
    const int units = wave_sum(leader ? 1 : 0);
    const int tpw = vp_tiles_per_wave_units(total_tiles, units, a.target_items, a.min_items);
    const int tpi = tpw * VP_WG_WAVES;
    const int nit = (tl + tpi - 1) / tpi;
    const int c = leader ? nit : 0;
    int ioff = 0, all_items = 0;
    for (int s = 0; s < N; ++s) {
        const int js = __builtin_amdgcn_readlane(j, 4 * s);
        const int cs = __builtin_amdgcn_readlane(c, 4 * s);
        ioff += js < j ? cs : 0;
        all_items += cs;
    }

    const int it = blockIdx.x;
    if (it == 0 && tid < 64) {
        if (sub == 0 && r < N) {
            a.g[r] = j;
            if (a.out_cluster) a.out_cluster[r] = j;
            if (tl == 0) {   // a cluster without candidates has no items: its rows' records come from here
                VpRowPlan rp = {r, j, 0, 1, 0, 0, to * VP_TILE_ITEMS, 0};
                a.rowplan[r] = rp;
            }
        }
        if (tid == 0) {
            a.hdr->total_items = all_items;
            a.hdr->tiles_per_wave = tpw;
            a.hdr->overflow = all_items > (int)gridDim.x;
            a.hdr->total_tiles = total_tiles;
            a.hdr->swz_rgs = 0;
            a.hdr->swz_chunks = 0;
            a.hdr->rows_per_item = VP_ROWS_PER_ITEM;
            a.hdr->mode = 0;
        }
    }
    if (it >= all_items) return;

    // the bucket this workgroup's item belongs to
    const unsigned long long owner = __ballot(leader && it >= ioff && it < ioff + c);
    const int src = __ffsll((long long)owner) - 1;
    const int jb = __builtin_amdgcn_readlane(j, src);
    const int ioff_b = __builtin_amdgcn_readlane(ioff, src);
    VpItem item;
    item.cluster = jb;
    item.perm_start = 0;
    item.nrows = __builtin_amdgcn_readlane(same_total, src);
    item.tile0 = (it - ioff_b) * tpi;
    item.ntiles = min(tpi, __builtin_amdgcn_readlane(tl, src) - item.tile0);
    item.shared = 0;
    item.tile_off = __builtin_amdgcn_readlane(to, src);
    item.ncand = __builtin_amdgcn_readlane(nc, src);
    if (it == ioff_b && tid < 64 && sub == 0 && j == jb) {
        VpRowPlan rp = {r, j, ioff_b, 1, nit, same_before, to * VP_TILE_ITEMS, 0};
        a.rowplan[r] = rp;
    }
    // row slot s of the item holds the bucket's s-th row
    int row_of_tid = -1;
    {
        int cnt = 0;
        for (int s = 0; s < N; ++s) {
            if (__builtin_amdgcn_readlane(j, 4 * s) == jb) {
                if (tid == cnt) row_of_tid = s;
                ++cnt;
            }
        }
    }
    const VpMaskInfo none = {nullptr, nullptr, 0};
    project_item<true, 1, PF, false>(set, hidden, d, row_of_tid, item, it, tpw, k, rstar, partials, nullptr, nullptr,
                                     nullptr, none, raw_ok != 0);
}

template <int PF>
__global__ __launch_bounds__(VP_WG_THREADS) void project_small_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, VpSmallArgs a, int k, int rstar,
    float *__restrict__ partials, int raw_ok)
{
    project_small<PF>(set, hidden, d, a, k, rstar, partials, raw_ok);
}

// The same with 16 loads in flight per wavefront, for k-extents whose staged rows leave room
// for fewer than four workgroups per CU (d_pad >= 1280): fewer wavefronts, deeper queues
// (skewed workload, d = 1536: 68.4 % -> 69.9 % of the HBM peak).
__global__ __launch_bounds__(VP_WG_THREADS) void project_pf16_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, const int32_t *__restrict__ perm,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k, int rstar,
    float *__restrict__ partials, unsigned int *__restrict__ floors, float *__restrict__ dbg_logits,
    const int64_t *__restrict__ dbg_row_off)
{
    const VpItem probe = items[blockIdx.x];
    const int total_items = hdr->total_items;
    const int tpw = hdr->tiles_per_wave;
    if (hdr->mode != 0) return;
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = it == (int)blockIdx.x ? probe : items[it];
    const VpMaskInfo none = {nullptr, nullptr, 0};
    if (item.shared)
        project_item<false, 1, 16, false>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, rstar, partials, floors, dbg_logits,
                                          dbg_row_off, none);
    else
        project_item<true, 1, 16, false>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, rstar, partials, floors, dbg_logits,
                                         dbg_row_off, none);
}

// Items of up to 32 rows, all sharing their tiles with other row groups: single-bucket
// projections (full, union) of more than 16 rows.
__global__ __launch_bounds__(VP_WG_THREADS) void project2_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, const int32_t *__restrict__ perm,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k,
    float *__restrict__ partials, unsigned int *__restrict__ floors, float *__restrict__ dbg_logits,
    const int64_t *__restrict__ dbg_row_off)
{
    const int total_items = hdr->total_items;
    const int tpw = hdr->tiles_per_wave;
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = items[it];
    const VpMaskInfo none = {nullptr, nullptr, 0};
    project_item<false, 2, 16, false>(set, hidden, d, row_of_slot(perm, item, 32), item, it, tpw, k, 0, partials, floors, dbg_logits,
                                      dbg_row_off, none);
}

// The full projection with every row masked to its own cluster's active set: the same
// results as the per-cluster slabs (token ids as candidate positions), for batches whose
// occupied slabs outweigh one pass over W.  Runs only when the planner chose it.
__global__ __launch_bounds__(VP_WG_THREADS) void project_masked_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, const int32_t *__restrict__ perm,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k,
    float *__restrict__ partials, unsigned int *__restrict__ floors, VpMaskInfo mask)
{
    if (hdr->mode != 1) return;
    const int total_items = hdr->total_items;
    const int tpw = hdr->tiles_per_wave;
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = items[it];
    if (item.shared)
        project_item<false, 1, 8, true>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, 0, partials, floors, nullptr, nullptr,
                                        mask);
    else
        project_item<true, 1, 8, true>(set, hidden, d, row_of_slot(perm, item, 16), item, it, tpw, k, 0, partials, floors, nullptr, nullptr,
                                       mask);
}

}  // namespace

size_t vpk_project_lds_bytes(int kt, int k, int row_tiles)
{
    const size_t rows = 16 * (size_t)row_tiles;
    return (size_t)row_tiles * kt * VP_TILE_BYTES + (size_t)VP_WG_WAVES * k * rows * 8 + VP_WG_WAVES * rows * 8 +
           rows * 12;
}

hipError_t vpk_project_prepare()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project2_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_pf16_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_masked_kernel),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_small_kernel<8>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_small_kernel<16>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_small_kernel<32>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e;
}

// raw_ok: the plan may consist of items short enough to keep raw logits (see project_item); the
// workgroups then get 8 KiB more LDS for them
void vpk_project(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                 const VpPlanHeader *hdr, int grid_items, int row_tiles, int k, int rstar, float *partials,
                 unsigned int *floors, float *dbg_logits, const int64_t *dbg_row_off, int raw_ok, hipStream_t st)
{
    if (row_tiles == 2) {
        hipLaunchKernelGGL(project2_kernel, dim3(grid_items), dim3(VP_WG_THREADS),
                           vpk_project_lds_bytes(set.kt, k, 2), st, set, (const uint4 *)hidden, d, perm, items, hdr, k,
                           partials, floors, dbg_logits, dbg_row_off);
        return;
    }
    const size_t lds = vpk_project_lds_bytes(set.kt, k, 1);
    if (set.kt % 16 == 0 && lds * 4 > 160 * 1024) {
        hipLaunchKernelGGL(project_pf16_kernel, dim3(grid_items), dim3(VP_WG_THREADS), lds, st, set,
                           (const uint4 *)hidden, d, perm, items, hdr, k, rstar, partials, floors, dbg_logits,
                           dbg_row_off);
        return;
    }
    const size_t raw_bytes = (size_t)VP_WG_WAVES * VP_RAW_TILES * VP_TILE_ITEMS * 16 * sizeof(float);
    if (lds + raw_bytes > 160 * 1024) raw_ok = 0;
    hipLaunchKernelGGL(project_kernel, dim3(grid_items), dim3(VP_WG_THREADS), lds + (raw_ok ? raw_bytes : 0), st,
                       set, (const uint4 *)hidden, d, perm, items, hdr, k, rstar, partials, floors, dbg_logits,
                       dbg_row_off, raw_ok);
}

// pf: 1 KiB loads a wavefront keeps in flight (8, 16 or 32; the k-tile count must be a multiple)
void vpk_project_small(const VpSlabSet &set, const void *hidden, int d, const VpSmallArgs &a, int grid_items, int k,
                       int rstar, float *partials, int raw_ok, int pf, hipStream_t st)
{
    const size_t lds = vpk_project_lds_bytes(set.kt, k, 1);
    const size_t raw_bytes = (size_t)VP_WG_WAVES * VP_RAW_TILES * VP_TILE_ITEMS * 16 * sizeof(float);
    if (lds + raw_bytes > 160 * 1024) raw_ok = 0;
    const size_t bytes = lds + (raw_ok ? raw_bytes : 0);
    if (pf == 32 && set.kt % 32 == 0)
        hipLaunchKernelGGL(project_small_kernel<32>, dim3(grid_items), dim3(VP_WG_THREADS), bytes, st, set,
                           (const uint4 *)hidden, d, a, k, rstar, partials, raw_ok);
    else if (pf >= 16 && set.kt % 16 == 0)
        hipLaunchKernelGGL(project_small_kernel<16>, dim3(grid_items), dim3(VP_WG_THREADS), bytes, st, set,
                           (const uint4 *)hidden, d, a, k, rstar, partials, raw_ok);
    else
        hipLaunchKernelGGL(project_small_kernel<8>, dim3(grid_items), dim3(VP_WG_THREADS), bytes, st, set,
                           (const uint4 *)hidden, d, a, k, rstar, partials, raw_ok);
}

void vpk_project_masked(const VpSlabSet &full, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                        const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *floors,
                        const VpMaskInfo &mask, hipStream_t st)
{
    hipLaunchKernelGGL(project_masked_kernel, dim3(grid_items), dim3(VP_WG_THREADS),
                       vpk_project_lds_bytes(full.kt, k, 1), st, full, (const uint4 *)hidden, d, perm, items, hdr, k,
                       partials, floors, mask);
}
