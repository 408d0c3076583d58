// Instantiations of coordinate_median_kernel for every tile variant (see dispatch.h).
#include "dispatch.h"

namespace btard {
namespace {
// [variant][ragged]
#define BTARD_M_ROW(NP, LG) \
    {coordinate_median_kernel<NP, LG, false>, coordinate_median_kernel<NP, LG, true>}
const MedianFn kMedian[kVariants][2] = {BTARD_M_ROW(4, 1),  BTARD_M_ROW(8, 1),  BTARD_M_ROW(16, 1),
                                        BTARD_M_ROW(16, 2), BTARD_M_ROW(16, 4), BTARD_M_ROW(16, 8),
                                        BTARD_M_ROW(16, 16)};
#undef BTARD_M_ROW
}  // namespace

MedianFn median_fn(Variant var, bool ragged) { return kMedian[var][ragged ? 1 : 0]; }

}  // namespace btard
