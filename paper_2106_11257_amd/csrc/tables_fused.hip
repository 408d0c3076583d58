// Instantiations of cc_finish_verify_kernel for every tile variant (see dispatch.h).
#include "dispatch.h"

namespace btard {
namespace {
// [scaled: with pre-clipping factors][variant][ragged]
#define BTARD_F_ROW(NP, LG, S) \
    {cc_finish_verify_kernel<NP, LG, false, S>, cc_finish_verify_kernel<NP, LG, true, S>}
const FusedFn kFused[2][kVariants][2] = {
    {BTARD_F_ROW(4, 1, false), BTARD_F_ROW(8, 1, false), BTARD_F_ROW(16, 1, false),
     BTARD_F_ROW(16, 2, false), BTARD_F_ROW(16, 4, false), BTARD_F_ROW(16, 8, false),
     BTARD_F_ROW(16, 16, false)},
    {BTARD_F_ROW(4, 1, true), BTARD_F_ROW(8, 1, true), BTARD_F_ROW(16, 1, true),
     BTARD_F_ROW(16, 2, true), BTARD_F_ROW(16, 4, true), BTARD_F_ROW(16, 8, true),
     BTARD_F_ROW(16, 16, true)}};
#undef BTARD_F_ROW
}  // namespace

FusedFn fused_pass_fn(Variant var, bool ragged, bool scaled)
{
    return kFused[scaled ? 1 : 0][var][ragged ? 1 : 0];
}

}  // namespace btard
