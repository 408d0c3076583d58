// Which instantiation of each tiled kernel serves a problem.  The instantiations live in
// translation units of their own (tables_*.hip), one per kernel family, so that the library
// builds in parallel; this header is what the host side (btard_api.hip) sees of them.
#pragma once

#include "cc_kernels.h"
#include "fused_kernels.h"
#include "median_kernels.h"
#include "verify_kernels.h"

namespace btard {

// ---- kernel variants: peers per lane group (NP) x lane groups per wavefront (LG)
enum Variant { V4x1, V8x1, V16x1, V16x2, V16x4, V16x8, V16x16, kVariants };

typedef void (*CcPassFn)(CcArgs);
typedef void (*CcFinishFn)(CcFinishArgs);
typedef void (*VerifyFn)(VerifyArgs);
typedef void (*FusedFn)(FusedArgs);
typedef void (*MedianFn)(MedianArgs);

// ragged: n < NP * LG; based: with a start vector v0; scaled: with pre-clipping factors
CcPassFn cc_pass_fn(Variant var, bool ragged, bool based, bool scaled);
CcFinishFn cc_finish_fn(Variant var, bool ragged, bool based);
VerifyFn verify_pass_fn(Variant var, bool ragged, bool scaled);
FusedFn fused_pass_fn(Variant var, bool ragged, bool scaled);
MedianFn median_fn(Variant var, bool ragged);

}  // namespace btard
