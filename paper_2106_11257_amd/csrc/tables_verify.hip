// Instantiations of verify_pass_kernel for every tile variant (see dispatch.h).
#include "dispatch.h"

namespace btard {
namespace {
// [scaled: on pre-clipped rows][variant][ragged]
#define BTARD_V_ROW(NP, LG, S) \
    {verify_pass_kernel<NP, LG, false, S>, verify_pass_kernel<NP, LG, true, S>}
const VerifyFn kVerify[2][kVariants][2] = {
    {BTARD_V_ROW(4, 1, false), BTARD_V_ROW(8, 1, false), BTARD_V_ROW(16, 1, false),
     BTARD_V_ROW(16, 2, false), BTARD_V_ROW(16, 4, false), BTARD_V_ROW(16, 8, false),
     BTARD_V_ROW(16, 16, false)},
    {BTARD_V_ROW(4, 1, true), BTARD_V_ROW(8, 1, true), BTARD_V_ROW(16, 1, true),
     BTARD_V_ROW(16, 2, true), BTARD_V_ROW(16, 4, true), BTARD_V_ROW(16, 8, true),
     BTARD_V_ROW(16, 16, true)}};
#undef BTARD_V_ROW
}  // namespace

VerifyFn verify_pass_fn(Variant var, bool ragged, bool scaled)
{
    return kVerify[scaled ? 1 : 0][var][ragged ? 1 : 0];
}

}  // namespace btard
