// Instantiations of cc_pass_kernel for every tile variant (see dispatch.h).
#include "dispatch.h"

namespace btard {
namespace {
// [variant][ragged: n < NP*LG][has v0]
#define BTARD_PASS_ROW(NP, LG)                                                                  \
    {{cc_pass_kernel<NP, LG, false, false, false>, cc_pass_kernel<NP, LG, false, true, false>},  \
     {cc_pass_kernel<NP, LG, true, false, false>, cc_pass_kernel<NP, LG, true, true, false>}}
const CcPassFn kCcPass[kVariants][2][2] = {
    BTARD_PASS_ROW(4, 1),  BTARD_PASS_ROW(8, 1),  BTARD_PASS_ROW(16, 1), BTARD_PASS_ROW(16, 2),
    BTARD_PASS_ROW(16, 4), BTARD_PASS_ROW(16, 8), BTARD_PASS_ROW(16, 16)};
#undef BTARD_PASS_ROW
// with pre-clipping factors  [variant][ragged][has v0]
#define BTARD_PASS_S(NP, LG)                                                                  \
    {{cc_pass_kernel<NP, LG, false, false, true>, cc_pass_kernel<NP, LG, false, true, true>},  \
     {cc_pass_kernel<NP, LG, true, false, true>, cc_pass_kernel<NP, LG, true, true, true>}}
const CcPassFn kCcPassScaled[kVariants][2][2] = {
    BTARD_PASS_S(4, 1),  BTARD_PASS_S(8, 1),  BTARD_PASS_S(16, 1), BTARD_PASS_S(16, 2),
    BTARD_PASS_S(16, 4), BTARD_PASS_S(16, 8), BTARD_PASS_S(16, 16)};
#undef BTARD_PASS_S
}  // namespace

CcPassFn cc_pass_fn(Variant var, bool ragged, bool based, bool scaled)
{
    return scaled ? kCcPassScaled[var][ragged ? 1 : 0][based ? 1 : 0]
                  : kCcPass[var][ragged ? 1 : 0][based ? 1 : 0];
}

}  // namespace btard
