// Device helpers shared by the projection kernels: MFMA operand fragments, the
// running softmax / top-k state of a row and its update from four new logits,
// tile loads, and the workgroup -> item map.
#pragma once
#include <hip/hip_runtime.h>
#include "vp_layout.h"

namespace {

typedef _Float16 half8 __attribute__((ext_vector_type(8)));
typedef _Float16 half2v __attribute__((ext_vector_type(2)));
typedef float floatx4 __attribute__((ext_vector_type(4)));

union Frag {
    uint4 u;
    half8 h;
    half2v p[4];
};

constexpr float LOG2E = 1.4426950408889634f;

__device__ inline float fast_exp(float x) { return __builtin_amdgcn_exp2f(x * LOG2E); }

// Per-lane running state of one row over the candidates this lane has seen.
struct RowState {
    float m;     // running maximum of the logits
    float s;     // sum of exp(z - m)
    float thr;   // logit of the row's current k-th best in this wavefront (+inf: lane inactive)
};

// Sorted list of the k best (logit, position) pairs of one row, one list per
// wavefront and row, kept in LDS as [slot][row] (16 rows = 16 different banks).
// The four lanes that own a row share it and take turns (see fold_logits).
struct RowList {
    float *val;
    int *idx;
    int stride;   // row slots of the item (16 or 32)
    __device__ inline float &v(int slot) { return val[slot * stride]; }
    __device__ inline int &i(int slot) { return idx[slot * stride]; }
};

// Orders LDS traffic between lanes of one wavefront: the hardware serves a
// wavefront's LDS instructions in order, this only stops the compiler from
// moving or merging the accesses across it.
__device__ inline void wave_lds_fence()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

// Order-preserving map of a float onto unsigned integers (for atomicMax).
__device__ inline unsigned int float_key(float v)
{
    const unsigned int b = __float_as_uint(v);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ inline float key_float(unsigned int key)
{
    return __uint_as_float((key & 0x80000000u) ? (key & 0x7fffffffu) : ~key);
}

// Folds the four logits a lane holds for its row into the running state.
// z[i] belongs to candidate position c0 + i with c0 = 16 * tile + 4 * q + i.
// The four lanes of a row (q = 0..3) insert into the row's list one after the
// other, in ascending q: positions therefore reach the list in ascending
// order, tile after tile, and on equal logits the entry already listed
// (smaller position = smaller token id) stays ahead.
//
// *floor_key is a lower bound of the row's final k-th best logit shared by the
// workgroup's wavefronts (a list that holds k entries >= x proves the k-th
// best is >= x).  A logit strictly below it cannot be among the k best and
// skips the list.  When bounds get published only changes how much list work
// is saved, never which entries survive the merges.
__device__ inline void fold_logits(const float z[4], int c0, int q, int k, RowState &st, RowList list,
                                   unsigned int *floor_key)
{
    const float tmax = fmaxf(fmaxf(z[0], z[1]), fmaxf(z[2], z[3]));
    const float mn = fmaxf(st.m, tmax);
    st.s = st.s * fast_exp(st.m - mn) + fast_exp(z[0] - mn) + fast_exp(z[1] - mn) + fast_exp(z[2] - mn) +
           fast_exp(z[3] - mn);
    st.m = mn;
    const float floor = key_float(__hip_atomic_load(floor_key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_WORKGROUP));
    const unsigned long long mask = __ballot(tmax > st.thr && tmax >= floor);   // lanes with something to insert
    if (mask != 0) {
        const float thr_before = st.thr;
#pragma unroll
        for (int turn = 0; turn < 4; ++turn) {
            if (((mask >> (turn * 16)) & 0xffffull) == 0) continue;   // nobody in this quarter (wavefront-uniform)
            if (q == turn && tmax > st.thr) {
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const float v = z[i];
                    if (v > st.thr && v >= floor) {
                        int p = k - 1;
                        while (p > 0 && list.v(p - 1) < v) {
                            list.v(p) = list.v(p - 1);
                            list.i(p) = list.i(p - 1);
                            --p;
                        }
                        list.v(p) = v;
                        list.i(p) = c0 + i;
                        st.thr = list.v(k - 1);
                    }
                }
            }
            wave_lds_fence();
            if (st.thr != __builtin_inff()) st.thr = list.v(k - 1);   // the row's other lanes may have raised it
            wave_lds_fence();
        }
        if (q == 0 && st.thr != __builtin_inff() && st.thr > thr_before && st.thr > floor)
            atomicMax(floor_key, float_key(st.thr));
    }
}

// (logit descending, position ascending) order used by every merge level.
__device__ inline bool entry_before(float v, int i, float v2, int i2) { return v > v2 || (v == v2 && i < i2); }

typedef unsigned int uintx4 __attribute__((ext_vector_type(4)));

// One 16-byte piece of a slab tile.  Slabs that only this work item reads are
// loaded with the non-temporal hint: they stream through once and should not
// displace anything; slabs shared by several row groups use plain loads so
// that the later groups find them in the L2.
template <bool NT>
__device__ inline uint4 load_piece(const uint4 *p)
{
    if (NT) {
        const uintx4 v = __builtin_nontemporal_load(reinterpret_cast<const uintx4 *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    }
    return *p;
}

// Which item a workgroup takes.  Workgroups are handed to the 8 XCDs in turn; for a
// single bucket whose row groups share tiles (the full projection) each XCD gets its
// own candidate ranges and all row groups of a range follow each other on that XCD,
// so the range is fetched from HBM once and then served by that XCD's L2.  In a clustered
// plan with heavy buckets (many row groups that read the same candidate ranges, consecutive
// in the item list) every XCD takes blocks of consecutive items in turn and starts an eighth
// of the list after the XCD before it.
__device__ inline int item_of_workgroup(const VpPlanHeader *hdr)
{
    const int swz_rgs = hdr->swz_rgs;
    if (swz_rgs == 0 || swz_rgs == 1) return blockIdx.x;
    return vp_item_of_workgroup(blockIdx.x, hdr->total_items, swz_rgs, hdr->swz_chunks);
}

}  // namespace
