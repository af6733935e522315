// Projection of many rows against one run of slab tiles: the GEMM-shaped case
// of Eq. 1 (section 2.1), used when a single bucket holds all rows (the full
// projection, the masked full projection, the batch-union form) and there are
// more rows than one 16-row item takes.
//
// An item is 64 rows x a range of candidate groups.  The k-extent is split over
// the wavefronts of the workgroup (four up to d_pad = 1024, eight beyond, so that a
// slice of the rows still fits the registers twice per SIMD): wavefront w keeps
// k-slice w of all 64 rows in registers, already in
// MFMA operand order, and streams only its slice of every slab tile group, so
// each 1 KiB slab load feeds four v_mfma_f32_16x16x32_f16 (one per row tile) and
// the hidden rows cost no LDS traffic in the loop.  Per candidate group the four
// partial accumulators of a row tile are exchanged through LDS (double
// buffered, one barrier per group) and wavefront w finishes row tile w: bias,
// online log-sum-exp and the top-k.
//
// Top-k here: every lane keeps the k best of the candidates it has seen itself
// (its row, its quarter of every group) in a private, unsorted LDS buffer and
// remembers the buffer's worst entry.  A better candidate overwrites the worst
// entry and one pass over the k slots finds the new worst: two LDS round trips
// per insertion, no shifting, no turn taking between lanes.  The four lanes of
// a row tell each other their worst kept logit, the largest of which bounds the
// row's k-th best from below and filters the others' candidates.  At the end of
// the item the four buffers of a row are merged into one sorted list.
#include <hip/hip_runtime.h>
#include "vp_kernels.h"
#include "project_common.h"

namespace {

constexpr int G_RT = 4;                    // row tiles per item
constexpr int G_ROWS = 16 * G_RT;          // row slots per item

template <int NW, int KW, bool MASKED, bool NT>
__device__ inline void gemm_item(const VpSlabSet &set, const uint4 *__restrict__ hidden, int d,
                                 const int32_t *__restrict__ perm, const VpItem &item, int it, int k,
                                 float *__restrict__ partials, unsigned int *__restrict__ bounds, int set_id,
                                 const VpMaskInfo &mask)
{
    constexpr int KT = KW * NW;   // NW wavefronts split the k-extent; the first four also finish a row tile each
    const int tid = threadIdx.x;
    const int wave = tid >> 6;
    const int lane = tid & 63;
    const int n = lane & 15;
    const int q = lane >> 4;

    extern __shared__ uint4 lds[];
    floatx4 *xbuf = reinterpret_cast<floatx4 *>(lds);                             // [2][G_RT][NW waves][64 lanes]
    const int k4 = (k + 3) & ~3;                                                   // slots per lane, padded
    float *keep_val = reinterpret_cast<float *>(xbuf + 2 * G_RT * NW * 64);        // [4 finishing waves][k4][64 lanes]
    int *keep_idx = reinterpret_cast<int *>(keep_val + G_RT * k4 * 64);

    const int ncand = item.ncand;
    const int toff = item.tile_off;
    const uint4 *slab = reinterpret_cast<const uint4 *>(set.tiles) + (size_t)toff * KT * 64 + (size_t)wave * KW * 64 + lane;
    const float *bias = set.bias + (size_t)toff * VP_TILE_ITEMS + q * 4;
    const int gb = item.tile0;
    const int ge = item.tile0 + item.ntiles;

    Frag X[KW], Y[KW];
    auto issue = [&](Frag(&buf)[KW], int g) {
        const uint4 *p = slab + (size_t)g * KT * 64;
#pragma unroll
        for (int i = 0; i < KW; ++i) buf[i].u = load_piece<NT>(p + i * 64);
    };
    // the first slab loads go out before anything else
    if (gb < ge) issue(X, gb);
    if (gb + 1 < ge) issue(Y, gb + 1);

    // this wavefront's k-slice of the 64 rows, in MFMA operand order
    Frag B[G_RT][KW];
    const int pieces_per_row = d >> 3;
#pragma unroll
    for (int rt = 0; rt < G_RT; ++rt) {
        const int slot = rt * 16 + n;
        const int row = slot < item.nrows ? perm[item.perm_start + slot] : -1;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            const int piece = (wave * KW + i) * 4 + q;
            B[rt][i].u = make_uint4(0, 0, 0, 0);
            if (row >= 0 && piece < pieces_per_row) B[rt][i].u = hidden[(size_t)row * pieces_per_row + piece];
        }
    }

    // the rows this wavefront finishes: row tile `wave` (wavefronts 4 .. NW-1 only contribute
    // their k-slices)
    const bool finisher = NW == G_RT || wave < G_RT;
    const int fw = finisher ? wave : 0;
    const int slot = fw * 16 + n;
    const bool row_valid = finisher && slot < item.nrows;
    const int myrow = row_valid ? perm[item.perm_start + slot] : -1;
    // this lane's buffer: slot s at mine[s * 64]; slots k .. k4-1 are padding that never loses
    float *my_val = keep_val + (size_t)fw * k4 * 64 + lane;
    int *my_idx = keep_idx + (size_t)fw * k4 * 64 + lane;
    if (finisher) {
        for (int s = 0; s < k4; ++s) {
            my_val[s * 64] = s < k ? -__builtin_inff() : __builtin_inff();
            my_idx[s * 64] = VP_IDX_NONE;
        }
    }
    float m_run = VP_NEG_BIG;                 // running maximum and sum of exponentials
    float s_run = 0.f;
    float worst = row_valid ? -__builtin_inff() : __builtin_inff();   // this lane's worst kept logit ...
    int worst_slot = 0;                                                // ... and where it is
    // Bound from the other workgroups that project the same rows onto other candidate ranges.
    // The ranges are dealt into VP_BOUND_SETS sets; bounds[row][s] is the best logit any
    // workgroup of set s has seen for the row so far.  Sets are disjoint, so the k-th largest of
    // the values stands for k different candidates: the row's k-th best cannot be below it.
    unsigned int *my_bounds = (row_valid && k <= VP_BOUND_SETS) ? bounds + (size_t)myrow * VP_BOUND_SETS : nullptr;
    float far_floor = -__builtin_inff();

    const uint32_t *mrow = nullptr;
    uint32_t mnext = 0xffffffffu;
    if (MASKED) {
        mrow = mask.bitmaps + (size_t)(row_valid ? mask.g[myrow] : 0) * mask.words;
        if (gb < ge) mnext = mrow[(gb * VP_TILE_ITEMS + q * 4) >> 5];
    }
    float4 bnext = make_float4(0.f, 0.f, 0.f, 0.f);
    if (gb < ge) bnext = *reinterpret_cast<const float4 *>(bias + gb * VP_TILE_ITEMS);

    floatx4 acc[G_RT];

    // all MFMAs of one candidate group; every consumed buffer slot is refilled with the
    // same slice of the group two ahead
    auto compute = [&](Frag(&buf)[KW], int gnext) {
        const bool more = gnext < ge;
        const uint4 *p = slab + (size_t)gnext * KT * 64;
#pragma unroll
        for (int i = 0; i < KW; ++i) {
            Frag a;
            a.u = buf[i].u;
            if (more) buf[i].u = load_piece<NT>(p + i * 64);
            // the first MFMA of a group starts from zero: the accumulators are dead between groups
#pragma unroll
            for (int rt = 0; rt < G_RT; ++rt)
                acc[rt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a.h, B[rt][i].h,
                                                                 i == 0 ? floatx4{0.f, 0.f, 0.f, 0.f} : acc[rt], 0, 0, 0);
        }
    };

    // k-slices of group g -> LDS, barrier, this wavefront's row tile summed and folded
    auto finish = [&](int g, int par) {
        floatx4 *xw = xbuf + (size_t)par * G_RT * NW * 64;
#pragma unroll
        for (int rt = 0; rt < G_RT; ++rt) {
            xw[(rt * NW + wave) * 64 + lane] = acc[rt];
        }
        const float4 bz4 = bnext;
        const uint32_t mcur = mnext;
        if (finisher && g + 1 < ge) {
            bnext = *reinterpret_cast<const float4 *>(bias + (g + 1) * VP_TILE_ITEMS);
            if (MASKED) mnext = mrow[((g + 1) * VP_TILE_ITEMS + q * 4) >> 5];
        }
        __syncthreads();
        if (!finisher) return;   // wavefronts beyond the fourth go on with the next group's k-slices
        // fixed order of the partial sums: pairs, then pairs of pairs
        floatx4 sum;
        {
            const floatx4 *pw = xw + (size_t)(fw * NW) * 64 + lane;
            floatx4 part[NW];
#pragma unroll
            for (int w = 0; w < NW; ++w) part[w] = pw[w * 64];
#pragma unroll
            for (int step = 1; step < NW; step <<= 1) {
#pragma unroll
                for (int w = 0; w < NW; w += 2 * step) part[w] = part[w] + part[w + step];
            }
            sum = part[0];
        }
        const int c0 = g * VP_TILE_ITEMS + q * 4;
        const float bz[4] = {bz4.x, bz4.y, bz4.z, bz4.w};
        float z[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) z[i] = sum[i] + bz[i];
        if ((g + 1) * VP_TILE_ITEMS > ncand) {   // the slab's last, partly filled group
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (c0 + i >= ncand) z[i] = -__builtin_inff();
        }
        if (MASKED) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
                if (!((mcur >> ((c0 & 31) + i)) & 1u)) z[i] = -__builtin_inff();
        }
        // log-sum-exp
        const float tmax = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
        const float mn = fmaxf(m_run, tmax);
        s_run = s_run * fast_exp(m_run - mn) + fast_exp(z[0] - mn) + fast_exp(z[1] - mn) + fast_exp(z[2] - mn) +
                fast_exp(z[3] - mn);
        m_run = mn;
        // After 4, 32, 256, ... groups of a long item: publish the row's best logit so far and read
        // the other sets'.  The reads cross the chip (several microseconds) and every workgroup
        // that holds the row makes them, so short items, whose whole life is not much longer, do
        // without, and nothing is read after the item's last groups.
        const int done = g - gb + 1;
        if (k <= VP_BOUND_SETS && ge - gb >= 48 && done + 8 < ge - gb &&
            (done == 4 || done == 32 || done == 256 || done == 2048)) {
            float best = fmaxf(m_run, __shfl_xor(m_run, 16));
            best = fmaxf(best, __shfl_xor(best, 32));
            float kth = -__builtin_inff();
            if (my_bounds && q == 0) {
                atomicMax(my_bounds + set_id, float_key(best));
                float v[VP_BOUND_SETS];
#pragma unroll
                for (int j = 0; j < VP_BOUND_SETS; ++j) {
                    v[j] = key_float(__hip_atomic_load(my_bounds + j, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT));
                    if (j == set_id) v[j] = fmaxf(v[j], best);   // our own value, whether or not the atomic has landed
                }
                for (int t = 0; t < k; ++t) {          // k-th largest of the sets' values
                    kth = v[0];
                    int at = 0;
#pragma unroll
                    for (int j = 1; j < VP_BOUND_SETS; ++j) {
                        if (v[j] > kth) {
                            kth = v[j];
                            at = j;
                        }
                    }
#pragma unroll
                    for (int j = 0; j < VP_BOUND_SETS; ++j)
                        if (j == at) v[j] = -__builtin_inff();
                }
            }
            far_floor = fmaxf(far_floor, __shfl(kth, n));   // lane n holds row n's value
        }
        // top-k: k kept entries >= x in any one buffer prove the row's k-th best is >= x
        float row_floor = fmaxf(worst, __shfl_xor(worst, 16));
        row_floor = fmaxf(fmaxf(row_floor, __shfl_xor(row_floor, 32)), far_floor);
        if (__ballot(tmax > worst && tmax >= row_floor) != 0) {
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                // positions ascend along a lane's stream: on equal logits the kept entry stays
                if (z[i] > worst && z[i] >= row_floor) {
                    my_val[worst_slot * 64] = z[i];
                    my_idx[worst_slot * 64] = c0 + i;
                    float wv = __builtin_inff();
                    int wi = -1, ws = 0;
                    for (int s4 = 0; s4 < k4; s4 += 4) {
                        float v[4];
                        int ix[4];
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            v[u] = my_val[(s4 + u) * 64];
                            ix[u] = my_idx[(s4 + u) * 64];
                        }
#pragma unroll
                        for (int u = 0; u < 4; ++u) {
                            if (v[u] < wv || (v[u] == wv && ix[u] > wi)) {
                                wv = v[u];
                                wi = ix[u];
                                ws = s4 + u;
                            }
                        }
                    }
                    worst = wv;
                    worst_slot = ws;
                }
            }
        }
    };

    int g = gb;
    int par = 0;
    while (g < ge) {
        compute(X, g + 2);
        finish(g, par);
        par ^= 1;
        ++g;
        if (g >= ge) break;
        compute(Y, g + 2);
        finish(g, par);
        par ^= 1;
        ++g;
    }

    if (!finisher) return;   // no barrier follows
    // the four lanes of a row (one per candidate quarter) -> one (m, s)
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {
        const float m2 = __shfl_xor(m_run, off);
        const float s2 = __shfl_xor(s_run, off);
        const float mn = fmaxf(m_run, m2);
        s_run = s_run * fast_exp(m_run - mn) + s2 * fast_exp(m2 - mn);
        m_run = mn;
    }
    // ... and one sorted list: k rounds of "best kept entry after the previous winner" over the
    // row's four buffers (each lane scans its own, two shuffles pick the winner)
    const int PFL = vp_partial_floats(k);
    float *out = partials + ((size_t)it * G_ROWS + slot) * PFL;
    if (row_valid && q == 0) {
        out[0] = m_run;
        out[1] = s_run;
    }
    float pv = __builtin_inff();
    int pi = -1;
    for (int t = 0; t < k; ++t) {
        float bv = -__builtin_inff();
        int bi = VP_IDX_NONE;
        for (int s = 0; s < k; ++s) {
            const float v = my_val[s * 64];
            const int ix = my_idx[s * 64];
            const bool after_prev = v < pv || (v == pv && ix > pi);
            if (after_prev && entry_before(v, ix, bv, bi)) {
                bv = v;
                bi = ix;
            }
        }
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float v2 = __shfl_xor(bv, off);
            const int i2 = __shfl_xor(bi, off);
            if (entry_before(v2, i2, bv, bi)) {
                bv = v2;
                bi = i2;
            }
        }
        if (row_valid && q == (t & 3)) {
            out[2 + t] = bv;
            out[2 + k + t] = __int_as_float(bi);
        }
        pv = bv;
        pi = bi;
    }
}

template <int NW, int KW, bool MASKED>
__global__ __launch_bounds__(NW * 64, (NW == 4 && KW <= 8 ? 2 : 1)) void project_gemm_kernel(
    VpSlabSet set, const uint4 *__restrict__ hidden, int d, const int32_t *__restrict__ perm,
    const VpItem *__restrict__ items, const VpPlanHeader *__restrict__ hdr, int k,
    float *__restrict__ partials, unsigned int *__restrict__ bounds, VpMaskInfo mask)
{
    if (MASKED ? hdr->mode != 1 : hdr->mode != 0) return;   // the planner chose the other form
    const int total_items = hdr->total_items;
    const int it = item_of_workgroup(hdr);
    if (it < 0 || it >= total_items) return;
    const VpItem item = items[it];
    // which set of candidate ranges this item's range belongs to (ranges are 4 * tiles_per_wave groups long)
    const int set_id = (item.tile0 / (hdr->tiles_per_wave * VP_WG_WAVES)) % VP_BOUND_SETS;
    if (item.shared)
        gemm_item<NW, KW, MASKED, false>(set, hidden, d, perm, item, it, k, partials, bounds, set_id, mask);
    else
        gemm_item<NW, KW, MASKED, true>(set, hidden, d, perm, item, it, k, partials, bounds, set_id, mask);
}

template <int NW, int KW, bool MASKED>
void launch(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
            const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *bounds,
            const VpMaskInfo &mask, hipStream_t st)
{
    hipLaunchKernelGGL((project_gemm_kernel<NW, KW, MASKED>), dim3(grid_items), dim3(NW * 64),
                       vpk_project_gemm_lds_bytes(k, NW * KW), st, set, (const uint4 *)hidden, d, perm, items, hdr, k,
                       partials, bounds, mask);
}

}  // namespace

// wavefronts that split the k-extent of kt k-tiles: 4 up to d_pad = 1024, 8 beyond
static int gemm_waves(int kt) { return kt <= 32 ? 4 : 8; }

size_t vpk_project_gemm_lds_bytes(int k, int kt)
{
    const size_t k4 = (size_t)((k + 3) & ~3);
    return (size_t)2 * G_RT * gemm_waves(kt) * 64 * 16 + (size_t)G_RT * k4 * 64 * 8;
}

// k-tile counts the kernel is built for (d_pad = 256, 512, 1024, 1536, 2048)
bool vpk_project_gemm_supported(int kt) { return kt == 8 || kt == 16 || kt == 32 || kt == 48 || kt == 64; }

template <int NW, int KW>
static hipError_t allow_lds()
{
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_gemm_kernel<NW, KW, false>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    if (e == hipSuccess)
        e = hipFuncSetAttribute(reinterpret_cast<const void *>(project_gemm_kernel<NW, KW, true>),
                                hipFuncAttributeMaxDynamicSharedMemorySize, 160 * 1024);
    return e;
}

// more than 64 KiB of dynamic LDS (eight wavefronts, or long top-k lists) has to be allowed explicitly
hipError_t vpk_project_gemm_prepare()
{
    hipError_t e = allow_lds<4, 2>();
    if (e == hipSuccess) e = allow_lds<4, 4>();
    if (e == hipSuccess) e = allow_lds<4, 8>();
    if (e == hipSuccess) e = allow_lds<8, 6>();
    if (e == hipSuccess) e = allow_lds<8, 8>();
    return e;
}

void vpk_project_gemm(const VpSlabSet &set, const void *hidden, int d, const int32_t *perm, const VpItem *items,
                      const VpPlanHeader *hdr, int grid_items, int k, float *partials, unsigned int *bounds,
                      const VpMaskInfo *mask, hipStream_t st)
{
    const VpMaskInfo none = {nullptr, nullptr, 0};
#define VP_GEMM_CASE(NW, KW)                                                                                       \
    case NW * KW:                                                                                                  \
        if (mask) launch<NW, KW, true>(set, hidden, d, perm, items, hdr, grid_items, k, partials, bounds, *mask, st); \
        else launch<NW, KW, false>(set, hidden, d, perm, items, hdr, grid_items, k, partials, bounds, none, st);     \
        break;
    switch (set.kt) {
        VP_GEMM_CASE(4, 2)
        VP_GEMM_CASE(4, 4)
        VP_GEMM_CASE(4, 8)
        VP_GEMM_CASE(8, 6)
        VP_GEMM_CASE(8, 8)
        default: break;   // callers check vpk_project_gemm_supported
    }
#undef VP_GEMM_CASE
}
