// Projection of many rows against one run of slab tiles with the rows held in LDS: the
// GEMM-shaped case of Eq. 1 (section 2.1) for single-bucket plans (the full projection, the
// masked full projection, the batch-union form) of more than 16 rows and k-extents up to
// d_pad = 1536.
//
// An item is 64 rows (48 at d_pad = 1536, where 64 do not fit) x a range of candidate groups, one
// workgroup of eight wavefronts.  The rows are staged once in LDS in MFMA operand order (4 or 3
// row tiles x KT KiB) and never move again.  The range is cut into steps of four candidate groups (64 candidates); wavefront w
// takes steps w, w + 8, ...  A step streams the four groups' tiles straight into registers
// (a ring of four k-tiles ahead, crossing step boundaries, so the loads never drain), and per
// k-tile feeds each loaded 1 KiB slab tile to one v_mfma_f32_16x16x32_f16 per row tile,
// whose row operands are read from LDS (one 1 KiB read per four MFMAs: four groups per step).  No wavefront waits
// for another inside the loop: there is no split of the k-extent, so nothing is exchanged and
// there is no barrier between the staging of the rows and the end of the item.
//
// After the 32 x 16 MFMAs of a step a lane holds, for each of the four row tiles, the 16 logits
// of one row (its quarter of each of the four groups).  They are folded in one go: bias,
// validity and membership mask, one online log-sum-exp update per row (steps 4-5 of the
// inference list of section 2.3), and the top-k (section 2.1).  Top-1 stays in registers.  For
// k >= 2 the workgroup keeps ONE list per row in LDS, shared by all eight wavefronts: k 64-bit
// keys (the logit's bits made monotone above the complemented position, so a larger key is an
// earlier entry in (logit descending, position ascending) order), always sorted.  A candidate is
// inserted without locks or turns by a cascade of LDS atomic maxima: slot 0 takes max(slot, key)
// and hands the smaller of the two to slot 1, and so on; every step keeps the multiset of keys
// (slots plus keys on their way) and the order of the slots, slots only ever grow, and a key
// leaves the far end only if k others are ahead of it - so whatever the interleaving of the
// lanes and wavefronts, the list ends as the k best keys in order.  The last slot is at all
// times a lower bound of the row's k-th best: a lane offers only candidates that are not below
// it (nor below the bound the workgroups that hold the same rows trade through global memory),
// best first, re-reading the bound after every insertion - so even the first step, which finds
// the list empty, costs a lane one or two insertions rather than sixteen.
#include <hip/hip_runtime.h>
#include <type_traits>
#include "vp_kernels.h"
#include "project_common.h"
#include "wave_ops.h"

namespace {

constexpr int L_NW = 8;        // wavefronts per workgroup
constexpr int L_G = 4;         // candidate groups per step
// row tiles per item: four (64 rows), or three where four do not fit the LDS (d_pad = 1536: 48 rows, 144 KiB)
constexpr int lds_row_tiles(int kt) { return kt == 48 ? 3 : 4; }
constexpr int L_PF = 4;        // k-tiles of the four groups kept in flight
constexpr int VP_MAX_TOPK_LANES = 32;   // the epilogue writes a row's list with one lane per entry

// (logit descending, position ascending), without branches
__device__ inline bool before_entry(float v, int i, float v2, int i2) { return (v > v2) | ((v == v2) & (i < i2)); }

template <int KT, bool MASKED, bool NT, bool TOP1, bool GATHER>
__device__ inline void gemm_lds_item(const VpSlabSet &set, const uint4 *__restrict__ hidden, int d,
                                     const VpItem &item, int it, int k,
                                     float *__restrict__ partials, unsigned int *__restrict__ floors,
                                     const VpMaskInfo &mask)
{
    constexpr int L_RT = lds_row_tiles(KT);
    constexpr int L_ROWS = 16 * L_RT;
    const int tid = threadIdx.x;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);   // (uniform: step numbers and tile offsets stay in scalar registers)
    const int lane = tid & 63;
    const int n = lane & 15;
    const int q = lane >> 4;

    extern __shared__ uint4 lds[];
    uint4 *ldsB = lds;                                                          // [L_RT][KT][64]: the rows
    unsigned long long *lkey = reinterpret_cast<unsigned long long *>(lds + L_RT * KT * 64);   // [k][64]: the rows' lists
    unsigned int *wg_floor = reinterpret_cast<unsigned int *>(lkey + k * L_ROWS);               // [64]
    // after the loop, in place of the rows:
    float *hdr_m = reinterpret_cast<float *>(lds);                              // [L_NW][64]
    float *hdr_s = hdr_m + L_NW * L_ROWS;

    const int ncand = item.ncand;
    const int gb = item.tile0;
    const int ge = item.tile0 + item.ntiles;
    const int nsteps = (item.ntiles + L_G - 1) / L_G;
    // Where the slab operands come from.  Packed slab: group after group of KT tiles of 1 KiB, lane l
    // at piece l of a tile.  GATHER (the batch-union form without a gathered copy, as the paper's
    // gathered GEMM reads its columns): the candidate's row of the token-major copy of W, whose
    // k-tile kt holds this lane's 16 bytes at piece kt * 4 + q; the candidates' token ids are U.
    constexpr int KSTEP = GATHER ? 4 : 64;   // pieces from one k-tile to the next
    const uint4 *slab = GATHER ? reinterpret_cast<const uint4 *>(set.tiles)
                               : reinterpret_cast<const uint4 *>(set.tiles) + (size_t)item.tile_off * KT * 64 + lane;
    const float *bias = set.bias + (size_t)item.tile_off * VP_TILE_ITEMS + q * 4;
    const int32_t *tokens = GATHER ? set.ids + (size_t)item.tile_off * VP_TILE_ITEMS + n : nullptr;

    // offsets (in 16-byte pieces) of the four groups of a step; groups past the item's end repeat
    // its last group (loaded, never looked at)
    auto group_off = [&](int step, unsigned int (&off)[L_G]) {
#pragma unroll
        for (int j = 0; j < L_G; ++j) {
            const int g = min(gb + step * L_G + j, ge - 1);
            if (GATHER) {
                const int tok = tokens[(size_t)g * VP_TILE_ITEMS];   // -1 in the padding of U's last group
                off[j] = (unsigned int)max(tok, 0) * (KT * 4) + q;
            } else {
                off[j] = (unsigned int)g * (KT * 64);
            }
        }
    };

    // The rows of this item -> LDS, MFMA operand order (row slots beyond nrows: zeros).  A
    // single-bucket plan keeps the rows in their own order: slot r of the item is row perm_start + r.
    // All of a thread's pieces are fetched in one batch, in front of the first slab loads (loads
    // return in order: behind them, the rows would wait for bytes from HBM they do not depend on).
    constexpr int X = KT * 4;   // 16-byte pieces per padded row
    constexpr int PER = L_ROWS * X / (L_NW * 64);   // pieces per thread
    static_assert(PER * L_NW * 64 == L_ROWS * X, "the rows' pieces divide evenly over the threads");
    uint4 piece[PER];
    {
        const int pieces_per_row = d >> 3;
#pragma unroll
        for (int i = 0; i < PER; ++i) {
            const int e = tid + i * (L_NW * 64);
            const int r = e / X;
            const int x = e - r * X;
            piece[i] = make_uint4(0, 0, 0, 0);
            if (r < item.nrows && x < pieces_per_row) piece[i] = hidden[(size_t)(item.perm_start + r) * pieces_per_row + x];
        }
    }

    uint4 ring[L_PF][L_G];
    unsigned int cur[L_G], nxt[L_G];
    int step = wave;
    const bool active = step < nsteps;
    if (active) {
        group_off(step, cur);
#pragma unroll
        for (int p = 0; p < L_PF; ++p)
#pragma unroll
            for (int j = 0; j < L_G; ++j) ring[p][j] = load_piece<NT>(slab + cur[j] + p * KSTEP);
    }

#pragma unroll
    for (int i = 0; i < PER; ++i) {
        const int e = tid + i * (L_NW * 64);
        const int r = e / X;
        const int x = e - r * X;
        ldsB[((r >> 4) * KT + (x >> 2)) * 64 + (x & 3) * 16 + (r & 15)] = piece[i];
    }
    for (int e = tid; e < k * L_ROWS; e += L_NW * 64) lkey[e] = 0ull;   // below the key of every logit
    // this lane's row in each row tile
    int myrow[L_RT];
    bool row_valid[L_RT];
#pragma unroll
    for (int rt = 0; rt < L_RT; ++rt) {
        const int slot = rt * 16 + n;
        row_valid[rt] = slot < item.nrows;
        myrow[rt] = row_valid[rt] ? item.perm_start + slot : -1;
    }
    if (tid < L_ROWS) wg_floor[tid] = (!TOP1 && tid < item.nrows) ? floors[item.perm_start + tid] : VP_FLOOR_NONE;
    __syncthreads();

    // per row tile: running maximum, sum of exponentials, k-th best of this wavefront's list
    float m_run[L_RT], s_run[L_RT];
    float b1v[L_RT];
    int b1i[L_RT];
    unsigned int moff[L_RT];   // first word of the row's membership list
#pragma unroll
    for (int rt = 0; rt < L_RT; ++rt) {
        m_run[rt] = VP_NEG_BIG;
        s_run[rt] = 0.f;
        b1v[rt] = -__builtin_inff();
        b1i[rt] = VP_IDX_NONE;
        moff[rt] = MASKED ? (unsigned int)(row_valid[rt] ? mask.g[myrow[rt]] : 0) * (unsigned int)mask.words : 0u;
    }
    constexpr bool top1 = TOP1;   // k == 1: the best entry stays in registers, no list traffic in the loop
    unsigned int pending[L_RT];
    int pending_rt = -1;
    int done_steps = 0;

    uint4 bnext[L_RT];   // the rows' operands of the k-tile to come
#pragma unroll
    for (int rt = 0; rt < L_RT; ++rt) bnext[rt] = ldsB[(rt * KT) * 64 + lane];

    while (step < nsteps) {
        const int g0 = gb + step * L_G;
        const int next_step = step + L_NW;
        group_off(next_step < nsteps ? next_step : step, nxt);
        // bias and membership words of the step, wanted only after its MFMAs
        float4 bz[L_G];
#pragma unroll
        for (int j = 0; j < L_G; ++j) bz[j] = *reinterpret_cast<const float4 *>(bias + (size_t)min(g0 + j, ge - 1) * VP_TILE_ITEMS);
        uint2 mw[L_RT];
        if (MASKED) {
            // the step's 64 candidates start at a multiple of 64: one aligned pair of 32-bit words (the
            // lists are padded to an even number of words)
#pragma unroll
            for (int rt = 0; rt < L_RT; ++rt)
                mw[rt] = *reinterpret_cast<const uint2 *>(mask.bitmaps + (moff[rt] + ((g0 * VP_TILE_ITEMS) >> 5)));
        }

        floatx4 acc[L_RT][L_G];
#pragma unroll
        for (int rt = 0; rt < L_RT; ++rt)
#pragma unroll
            for (int j = 0; j < L_G; ++j) acc[rt][j] = floatx4{0.f, 0.f, 0.f, 0.f};
        // L_PF k-tiles per pass of the loop body: pass b consumes the ring and refills it with
        // k-tiles (b + 1) * L_PF ... of this step, the last pass with the first k-tiles of the
        // wavefront's next step
#pragma unroll 1
        for (int b = 0; b < KT / L_PF; ++b) {
            const bool last = b == KT / L_PF - 1;
            unsigned int src[L_G];
#pragma unroll
            for (int j = 0; j < L_G; ++j) src[j] = last ? nxt[j] : cur[j] + (b + 1) * (L_PF * KSTEP);
#pragma unroll
            for (int u = 0; u < L_PF; ++u) {
                // The rows' operands of the next k-tile are read while this one's MFMAs run (after a
                // step's last k-tile: the first one again; the rows never change), and a ring slot is
                // refilled as soon as its MFMAs have been issued: the loads then have three quarters
                // of a pass, and the other wavefront's share of the matrix cores, to come back.  The
                // scheduling barrier keeps that order (left alone, the compiler sinks all loads of a
                // pass to its end, right in front of their first use).
                Frag bf[L_RT];
                const int kt_next = (b * L_PF + u + 1) == KT ? 0 : b * L_PF + u + 1;
#pragma unroll
                for (int rt = 0; rt < L_RT; ++rt) {
                    bf[rt].u = bnext[rt];
                    bnext[rt] = ldsB[(rt * KT + kt_next) * 64 + lane];
                }
#pragma unroll
                for (int rt = 0; rt < L_RT; ++rt)
#pragma unroll
                    for (int j = 0; j < L_G; ++j) {
                        Frag a;
                        a.u = ring[u][j];
                        acc[rt][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, bf[rt].h, acc[rt][j], 0, 0, 0);
                    }
#pragma unroll
                for (int j = 0; j < L_G; ++j) ring[u][j] = load_piece<NT>(slab + src[j] + u * KSTEP);
                __builtin_amdgcn_sched_barrier(0);
            }
        }

        // fold the 16 logits of each of this lane's four rows
        const int c_first = g0 * VP_TILE_ITEMS + q * 4;           // position of z[0] (j = 0, i = 0) in the slab
        const bool ragged = (g0 + L_G) * VP_TILE_ITEMS > ncand || g0 + L_G > ge;   // (wavefront-uniform)
        if (pending_rt >= 0) {
            // bounds read from the other workgroups a step ago
#pragma unroll
            for (int rt = 0; rt < L_RT; ++rt)
                if (rt == pending_rt && q == 0 && row_valid[rt]) atomicMax(wg_floor + rt * 16 + n, pending[rt]);
            pending_rt = -1;
        }
        // (written per row tile with the tile's number a compile-time constant: the accumulators
        // and the per-tile state must stay in registers)
        auto fold_row_tile = [&](auto rt_const) {
            constexpr int rt = decltype(rt_const)::value;
            float z[L_G * 4];
#pragma unroll
            for (int j = 0; j < L_G; ++j) {
                z[j * 4 + 0] = acc[rt][j][0] + bz[j].x;
                z[j * 4 + 1] = acc[rt][j][1] + bz[j].y;
                z[j * 4 + 2] = acc[rt][j][2] + bz[j].z;
                z[j * 4 + 3] = acc[rt][j][3] + bz[j].w;
            }
            if (ragged) {
#pragma unroll
                for (int j = 0; j < L_G; ++j)
#pragma unroll
                    for (int i = 0; i < 4; ++i)
                        if (g0 + j >= ge || c_first + j * VP_TILE_ITEMS + i >= ncand) z[j * 4 + i] = -__builtin_inff();
            }
            if (MASKED) {
                // a token outside the row's active set is at -infinity (steps 4-5 of section 2.3's list):
                // the membership bit, spread over a word, keeps the logit's bits or takes -infinity's
#pragma unroll
                for (int j = 0; j < L_G; ++j) {
                    const uint32_t w = (j >> 1) ? mw[rt].y : mw[rt].x;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const uint32_t keep = (uint32_t)__builtin_amdgcn_sbfe((int)w, (j & 1) * 16 + q * 4 + i, 1);   // 0 or ~0
                        z[j * 4 + i] = __uint_as_float((__float_as_uint(z[j * 4 + i]) & keep) | (0xff800000u & ~keep));
                    }
                }
            }
            float tmax = z[0];
#pragma unroll
            for (int e = 1; e < L_G * 4; ++e) tmax = fmaxf(tmax, z[e]);
            const float mn = fmaxf(m_run[rt], tmax);
            float sum = 0.f;
#pragma unroll
            for (int e = 0; e < L_G * 4; ++e) sum += fast_exp(z[e] - mn);
            s_run[rt] = s_run[rt] * fast_exp(m_run[rt] - mn) + sum;
            m_run[rt] = mn;

            if (top1) {
                // positions ascend along a lane's own stream: a strict comparison keeps the smaller one
#pragma unroll
                for (int e = 0; e < L_G * 4; ++e) {
                    const bool take = z[e] > b1v[rt];
                    b1v[rt] = take ? z[e] : b1v[rt];
                    b1i[rt] = take ? c_first + (e >> 2) * VP_TILE_ITEMS + (e & 3) : b1i[rt];
                }
                return;
            }
            const int slot = rt * 16 + n;
            unsigned long long *list = lkey + slot;              // + p * L_ROWS
            const float far_floor = key_float(__hip_atomic_load(wg_floor + slot, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
            auto row_floor = [&]() {
                const unsigned long long kth = __hip_atomic_load(list + (k - 1) * L_ROWS, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
                return fmaxf(far_floor, kth ? key_float((unsigned int)(kth >> 32)) : -__builtin_inff());
            };
            float floor = row_floor();
            const bool want = row_valid[rt] & (tmax >= floor) & (tmax > -__builtin_inff());
            if (__ballot(want) != 0) {
                if (want) {
                    // this lane's candidates, best first, until one is below the bound (the others,
                    // which are not better, then are too)
                    while (true) {
                        float v = z[0];
                        int e_best = 0;
#pragma unroll
                        for (int e = 1; e < L_G * 4; ++e) {
                            const bool take = z[e] > v;   // strict: of equal logits the smaller position
                            v = take ? z[e] : v;
                            e_best = take ? e : e_best;
                        }
                        if (!((v >= floor) & (v > -__builtin_inff()))) break;
                        const unsigned int c = (unsigned int)(c_first + (e_best >> 2) * VP_TILE_ITEMS + (e_best & 3));
                        // (-0 becomes +0: equal as logits, they must tie and be ordered by position)
                        unsigned long long carry = ((unsigned long long)float_key(v + 0.f) << 32) | (unsigned int)~c;
                        for (int p = 0; p < k && carry != 0ull; ++p) {
                            const unsigned long long old = __hip_atomic_fetch_max(list + p * L_ROWS, carry, __ATOMIC_RELAXED,
                                                                                  __HIP_MEMORY_SCOPE_WORKGROUP);
                            carry = old < carry ? old : carry;
                        }
#pragma unroll
                        for (int e = 0; e < L_G * 4; ++e) z[e] = e == e_best ? -__builtin_inff() : z[e];
                        floor = row_floor();
                    }
                }
            }
        };
        fold_row_tile(std::integral_constant<int, 0>{});
        fold_row_tile(std::integral_constant<int, 1>{});
        fold_row_tile(std::integral_constant<int, 2>{});
        if constexpr (L_RT > 3) fold_row_tile(std::integral_constant<int, 3>{});
        // every second step of a wavefront, one row tile in turn: trade bounds with the other
        // workgroups that project the same rows onto other candidate ranges (one atomicMax
        // publishes ours and returns theirs, folded into the LDS copy a step later: no wait here)
        ++done_steps;
        if (!top1 && (done_steps & 1) == 0) {
            const int rt_x = ((done_steps >> 1) + wave) % L_RT;
#pragma unroll
            for (int rt = 0; rt < L_RT; ++rt)
                if (rt == rt_x && q == 0 && row_valid[rt]) {
                    const unsigned long long kth = __hip_atomic_load(lkey + (k - 1) * L_ROWS + rt * 16 + n, __ATOMIC_RELAXED,
                                                                     __HIP_MEMORY_SCOPE_WORKGROUP);
                    const unsigned int mine = max((unsigned int)(kth >> 32),
                                                  __hip_atomic_load(wg_floor + rt * 16 + n, __ATOMIC_RELAXED,
                                                                    __HIP_MEMORY_SCOPE_WORKGROUP));
                    pending[rt] = atomicMax(floors + myrow[rt], max(mine, (unsigned int)VP_FLOOR_NONE));
                }
            pending_rt = rt_x;
        }
#pragma unroll
        for (int j = 0; j < L_G; ++j) cur[j] = nxt[j];
        step = next_step;
    }

    // the row's four lanes (one per quarter of every group) -> one (m, s); top-1: one entry
#pragma unroll
    for (int rt = 0; rt < L_RT; ++rt) {
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float m2 = __shfl_xor(m_run[rt], off);
            const float s2 = __shfl_xor(s_run[rt], off);
            const float mn = fmaxf(m_run[rt], m2);
            s_run[rt] = s_run[rt] * fast_exp(m_run[rt] - mn) + s2 * fast_exp(m2 - mn);
            m_run[rt] = mn;
            if (top1) {
                const float v2 = __shfl_xor(b1v[rt], off);
                const int i2 = __shfl_xor(b1i[rt], off);
                const bool take = before_entry(v2, i2, b1v[rt], b1i[rt]);
                b1v[rt] = take ? v2 : b1v[rt];
                b1i[rt] = take ? i2 : b1i[rt];
            }
        }
        if (top1 && q == 0 && row_valid[rt] && b1i[rt] != VP_IDX_NONE)
            __hip_atomic_fetch_max(lkey + rt * 16 + n,
                                   ((unsigned long long)float_key(b1v[rt] + 0.f) << 32) | (unsigned int)~(unsigned int)b1i[rt],
                                   __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP);
    }
    __syncthreads();   // nobody reads the rows any more: their LDS becomes the (m, s) exchange
#pragma unroll
    for (int rt = 0; rt < L_RT; ++rt) {
        if (q == 0) {
            hdr_m[wave * L_ROWS + rt * 16 + n] = m_run[rt];
            hdr_s[wave * L_ROWS + rt * 16 + n] = s_run[rt];
        }
    }
    if (!top1 && tid < item.nrows) {
        const unsigned int kth = (unsigned int)(lkey[(k - 1) * L_ROWS + tid] >> 32);
        atomicMax(floors + item.perm_start + tid, max(max(kth, wg_floor[tid]), (unsigned int)VP_FLOOR_NONE));
    }
    __syncthreads();

    // one partial result per (item, row): the row's list is in order already; wavefront w takes
    // row slots w, w + 8, ...
    const int PFL = vp_partial_floats(k);
    for (int r = wave; r < item.nrows; r += L_NW) {
        float M = hdr_m[r];
#pragma unroll
        for (int w = 1; w < L_NW; ++w) M = fmaxf(M, hdr_m[w * L_ROWS + r]);
        float S = 0.f;
#pragma unroll
        for (int w = 0; w < L_NW; ++w) S += hdr_s[w * L_ROWS + r] * fast_exp(hdr_m[w * L_ROWS + r] - M);
        float *out = partials + ((size_t)it * L_ROWS + r) * PFL;
        if (lane == 0) {
            out[0] = M;
            out[1] = S;
        }
        if (lane < k) {
            const unsigned long long key = lkey[lane * L_ROWS + r];
            out[2 + lane] = key ? key_float((unsigned int)(key >> 32)) : -__builtin_inff();
            out[2 + k + lane] = __int_as_float(key ? (int)~(unsigned int)key : VP_IDX_NONE);
        }
    }
}

template <int KT, bool MASKED, bool TOP1, bool GATHER>
__global__ __launch_bounds__(L_NW * 64) void project_gemm_lds_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k,
    float *__restrict__ partials, unsigned int *__restrict__ floors, VpMaskInfo mask)
{
    if (MASKED ? hdr->mode != 1 : hdr->mode != 0) return;   // the planner chose the other form
    const int total_items = hdr->total_items;
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = items[it];
    if (item.shared || GATHER)
        gemm_lds_item<KT, MASKED, false, TOP1, GATHER>(set, hidden, d, item, it, TOP1 ? 1 : k, partials, floors, mask);
    else
        gemm_lds_item<KT, MASKED, true, TOP1, false>(set, hidden, d, item, it, TOP1 ? 1 : k, partials, floors, mask);
}

template <int KT, bool MASKED, bool GATHER>
void launch_lds(const VpSlabSet &set, const void *hidden, int d, const VpItem *items,
                const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *floors,
                const VpMaskInfo &mask, hipStream_t st)
{
    if (k == 1)
        hipLaunchKernelGGL((project_gemm_lds_kernel<KT, MASKED, true, GATHER>), dim3(grid_items), dim3(L_NW * 64),
                           vpk_project_rows_lds_bytes(k, KT), st, set, (const uint4 *)hidden, d, items, hdr, k,
                           partials, floors, mask);
    else
        hipLaunchKernelGGL((project_gemm_lds_kernel<KT, MASKED, false, GATHER>), dim3(grid_items), dim3(L_NW * 64),
                           vpk_project_rows_lds_bytes(k, KT), st, set, (const uint4 *)hidden, d, items, hdr, k,
                           partials, floors, mask);
}

template <int KT>
hipError_t allow_lds_bytes()
{
    const void *fns[] = {reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, false, false, false>),
                         reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, false, true, false>),
                         reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, true, false, false>),
                         reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, true, true, false>),
                         reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, false, false, true>),
                         reinterpret_cast<const void *>(project_gemm_lds_kernel<KT, false, true, true>)};
    for (const void *f : fns) {
        const hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
        if (e != hipSuccess) return e;
    }
    return hipSuccess;
}

}  // namespace

size_t vpk_project_rows_lds_bytes(int k, int kt)
{
    const int rows = 16 * lds_row_tiles(kt);
    return (size_t)rows * kt * (VP_TILE_BYTES / 16) + (size_t)k * rows * 8 + rows * 4;
}

// built for d_pad = 256, 512, 1024 and 1536 (the rows of an item must fit the LDS beside its lists)
bool vpk_project_rows_lds_supported(int kt, int k)
{
    return (kt == 8 || kt == 16 || kt == 32 || kt == 48) && k >= 1 && k <= VP_MAX_TOPK_LANES;
}
// row tiles of an item of that kernel
int vpk_project_rows_lds_row_tiles(int kt) { return lds_row_tiles(kt); }

hipError_t vpk_project_rows_lds_prepare()
{
    hipError_t e = allow_lds_bytes<8>();
    if (e == hipSuccess) e = allow_lds_bytes<16>();
    if (e == hipSuccess) e = allow_lds_bytes<32>();
    if (e == hipSuccess) e = allow_lds_bytes<48>();
    return e;
}

// mask: nullptr, or the membership lists of the masked full projection.  gather: the set's tiles
// are the token-major copy of W and its ids the batch's union U (no mask then); the slab operands
// are read through U instead of from a packed copy.  (perm is not read: a single-bucket plan keeps
// the rows in their own order.)
void vpk_project_rows_lds(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                          const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *floors,
                          const VpMaskInfo *mask, bool gather, hipStream_t st)
{
    const VpMaskInfo none = {nullptr, nullptr, 0};
#define VP_LDS_CASE(KT)                                                                                                   \
    case KT:                                                                                                              \
        if (mask) launch_lds<KT, true, false>(set, hidden, d, items, hdr, grid_items, k, partials, floors, *mask, st); \
        else if (gather) launch_lds<KT, false, true>(set, hidden, d, items, hdr, grid_items, k, partials, floors, none, st); \
        else launch_lds<KT, false, false>(set, hidden, d, items, hdr, grid_items, k, partials, floors, none, st);     \
        break;
    switch (set.kt) {
        VP_LDS_CASE(8)
        VP_LDS_CASE(16)
        VP_LDS_CASE(32)
        VP_LDS_CASE(48)
        default: break;   // callers check vpk_project_rows_lds_supported
    }
#undef VP_LDS_CASE
}
