// Wavefront-wide reductions with data-parallel-primitive (DPP) moves in the vector ALU.  A
// cross-lane shuffle goes through the LDS crossbar and costs a round trip of a hundred cycles or
// more; a reduction of (value, index) pairs by shuffles takes twelve of them.  The DPP form walks
// the same tree as an inclusive scan - shifts by 1, 2, 4, 8 inside each row of 16 lanes, then the
// last lane of rows 0 and 2 into rows 1 and 3, then lane 31 into rows 2 and 3 - so lane 63 ends
// with the result over all 64 lanes, which a lane read hands to everyone.
#pragma once
#include <hip/hip_runtime.h>

namespace {

// The entry that comes first in (value descending, index ascending) order, over the wavefront;
// every lane returns with it.  Each entry travels as one 64-bit key - the float's bits made
// monotone above the complemented index - so a step is one 64-bit compare and two selects.
// Written with the two-level comparison on (float, int) the compiler branches around the tie
// case, and a step then costs about 250 cycles in a wavefront that has its SIMD to itself
// (exec-mask bookkeeping in the scalar unit on results of the vector unit); the k rounds of a
// top-8 merge took 14,000 cycles that way.  -0 is turned into +0 first (they compare equal as
// floats and must tie); indices are non-negative.
__device__ inline void wave_best_entry(float &v, int &i)
{
    unsigned int hi = __float_as_uint(v + 0.f);
    hi ^= (hi & 0x80000000u) ? 0xffffffffu : 0x80000000u;   // larger float <=> larger unsigned
    unsigned int lo = ~(unsigned int)i;                      // smaller index <=> larger
#define VP_DPP_BEST(ctrl, rows)                                                                        \
    {                                                                                                  \
        const unsigned int hi2 = (unsigned int)__builtin_amdgcn_update_dpp((int)hi, (int)hi, ctrl, rows, 0xf, false); \
        const unsigned int lo2 = (unsigned int)__builtin_amdgcn_update_dpp((int)lo, (int)lo, ctrl, rows, 0xf, false); \
        const unsigned long long mine = ((unsigned long long)hi << 32) | lo;                           \
        const unsigned long long other = ((unsigned long long)hi2 << 32) | lo2;                        \
        const bool take = other > mine;                                                                \
        hi = take ? hi2 : hi;                                                                          \
        lo = take ? lo2 : lo;                                                                          \
    }
    VP_DPP_BEST(0x111, 0xf)   // row_shr:1
    VP_DPP_BEST(0x112, 0xf)   // row_shr:2
    VP_DPP_BEST(0x114, 0xf)   // row_shr:4
    VP_DPP_BEST(0x118, 0xf)   // row_shr:8
    VP_DPP_BEST(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
    VP_DPP_BEST(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef VP_DPP_BEST
    hi = (unsigned int)__builtin_amdgcn_readlane((int)hi, 63);
    lo = (unsigned int)__builtin_amdgcn_readlane((int)lo, 63);
    hi ^= (hi & 0x80000000u) ? 0x80000000u : 0xffffffffu;
    v = __uint_as_float(hi);
    i = (int)~lo;
}

// Inclusive prefix sum over the 64 lanes of a wavefront (lane 63 ends with the total).
__device__ inline int wave_inclusive_sum(int v)
{
    v += __builtin_amdgcn_update_dpp(0, v, 0x111, 0xf, 0xf, false);   // row_shr:1
    v += __builtin_amdgcn_update_dpp(0, v, 0x112, 0xf, 0xf, false);   // row_shr:2
    v += __builtin_amdgcn_update_dpp(0, v, 0x114, 0xf, 0xf, false);   // row_shr:4
    v += __builtin_amdgcn_update_dpp(0, v, 0x118, 0xf, 0xf, false);   // row_shr:8
    v += __builtin_amdgcn_update_dpp(0, v, 0x142, 0xa, 0xf, false);   // row_bcast:15 -> rows 1, 3
    v += __builtin_amdgcn_update_dpp(0, v, 0x143, 0xc, 0xf, false);   // row_bcast:31 -> rows 2, 3
    return v;
}

// Sum over the wavefront, to every lane.
__device__ inline int wave_sum(int v) { return __builtin_amdgcn_readlane(wave_inclusive_sum(v), 63); }

// Running maximum m and sum of exp(x - m) over the wavefront's (m, s) pairs, to every lane.
__device__ inline void wave_log_sum_exp(float &m, float &s)
{
#define VP_DPP_LSE(ctrl, rows)                                                                                    \
    {                                                                                                             \
        const float m2 = __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(-3.0e38f), __float_as_int(m), ctrl, rows, 0xf, false)); \
        const float s2 = __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(s), ctrl, rows, 0xf, false)); \
        const float mn = fmaxf(m, m2);                                                                            \
        s = s * __builtin_amdgcn_exp2f((m - mn) * 1.4426950408889634f) +                                          \
            s2 * __builtin_amdgcn_exp2f((m2 - mn) * 1.4426950408889634f);                                         \
        m = mn;                                                                                                   \
    }
    VP_DPP_LSE(0x111, 0xf)
    VP_DPP_LSE(0x112, 0xf)
    VP_DPP_LSE(0x114, 0xf)
    VP_DPP_LSE(0x118, 0xf)
    VP_DPP_LSE(0x142, 0xa)
    VP_DPP_LSE(0x143, 0xc)
#undef VP_DPP_LSE
    m = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(m), 63));
    s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(s), 63));
}

}  // namespace
