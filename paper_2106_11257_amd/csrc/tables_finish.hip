// Instantiations of cc_finish_kernel for every tile variant (see dispatch.h).
#include "dispatch.h"

namespace btard {
namespace {
// [variant][ragged][has v0]
#define BTARD_CC_ROW(K, NP, LG)                                                   \
    {{K<NP, LG, false, false>, K<NP, LG, false, true>},                           \
     {K<NP, LG, true, false>, K<NP, LG, true, true>}}
const CcFinishFn kCcFinish[kVariants][2][2] = {
    BTARD_CC_ROW(cc_finish_kernel, 4, 1),  BTARD_CC_ROW(cc_finish_kernel, 8, 1),
    BTARD_CC_ROW(cc_finish_kernel, 16, 1), BTARD_CC_ROW(cc_finish_kernel, 16, 2),
    BTARD_CC_ROW(cc_finish_kernel, 16, 4), BTARD_CC_ROW(cc_finish_kernel, 16, 8),
    BTARD_CC_ROW(cc_finish_kernel, 16, 16)};
#undef BTARD_CC_ROW
}  // namespace

CcFinishFn cc_finish_fn(Variant var, bool ragged, bool based)
{
    return kCcFinish[var][ragged ? 1 : 0][based ? 1 : 0];
}

}  // namespace btard
