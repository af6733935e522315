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
// every lane returns with it.
__device__ inline void wave_best_entry(float &v, int &i)
{
#define VP_DPP_BEST(ctrl, rows)                                                                                   \
    {                                                                                                             \
        const float v2 = __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), ctrl, rows, 0xf, false)); \
        const int i2 = __builtin_amdgcn_update_dpp(i, i, ctrl, rows, 0xf, false);                                 \
        if (v2 > v || (v2 == v && i2 < i)) {                                                                      \
            v = v2;                                                                                               \
            i = i2;                                                                                               \
        }                                                                                                         \
    }
    VP_DPP_BEST(0x111, 0xf)   // row_shr:1
    VP_DPP_BEST(0x112, 0xf)   // row_shr:2
    VP_DPP_BEST(0x114, 0xf)   // row_shr:4
    VP_DPP_BEST(0x118, 0xf)   // row_shr:8
    VP_DPP_BEST(0x142, 0xa)   // row_bcast:15 into rows 1 and 3
    VP_DPP_BEST(0x143, 0xc)   // row_bcast:31 into rows 2 and 3
#undef VP_DPP_BEST
    v = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), 63));
    i = __builtin_amdgcn_readlane(i, 63);
}

}  // namespace
