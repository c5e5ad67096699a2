// The scheduler as the library itself calls it (host code only; defined in difa_worklist.cpp).
#pragma once
#include <stdint.h>

#include "difa.h"

namespace difa {

// difa_schedule_build with two more arguments:
//   die_speed   n_xcd relative speeds of the accelerator dies (NULL: all alike).  Under a heavy load the
//               dies of one chip settle at clocks a few percent apart; a die is given work in
//               proportion to its speed.
//   die_span    receives, per die, the predicted finishing time of its slowest workgroup in the
//               scheduler's cost units at speed 1 (NULL: not wanted).  The caller divides it by the die's
//               measured time to learn the speeds.
difa_status_t schedule_for_dies(const difa_work_item_t* items, int32_t n_items, int32_t n_wg, int32_t n_xcd,
                                const double* die_speed, int64_t* die_span, difa_segment_t* segs,
                                int32_t seg_capacity, int32_t* wg_begin, int32_t* n_segs_out,
                                difa_merge_item_t* merges, int32_t merge_capacity, int32_t* n_merges_out,
                                int32_t* n_slots_out);

}  // namespace difa
