// Host build of the item-sizing rules in csrc/vp_layout.h, for the CPU tests of the host logic
// (the same inline functions run in the planning kernels and in the host API).
#define __host__
#define __device__
#include "vp_layout.h"

extern "C" int shim_tiles_per_wave(long long total_tiles, int target_items, int min_items)
{
    return vp_tiles_per_wave(total_tiles, target_items, min_items);
}

extern "C" int shim_tiles_per_wave_units(long long total_tiles, int units, int target_items, int min_items)
{
    return vp_tiles_per_wave_units(total_tiles, units, target_items, min_items);
}

extern "C" int shim_raw_tiles(void) { return VP_RAW_TILES; }
extern "C" int shim_partial_floats(int k) { return vp_partial_floats(k); }

extern "C" int shim_item_of_workgroup(int wg, int total_items, int swz_rgs, int swz_chunks)
{
    return vp_item_of_workgroup(wg, total_items, swz_rgs, swz_chunks);
}
extern "C" int shim_xcd_block_items(void) { return VP_XCD_BLOCK_ITEMS; }
extern "C" int shim_rounds_item_count(int rgs, int slots, int vtiles) { return vp_rounds_item_count(rgs, slots, vtiles); }
