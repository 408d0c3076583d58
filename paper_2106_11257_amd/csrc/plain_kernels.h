// A plain streaming kernel with the memory traffic of the method's passes and none of their
// design: the yardstick the measured kernels are set beside.  Not part of the method.
#pragma once
#include "kernels_common.h"

namespace btard {

// Every thread walks the 4-coordinate columns x, x + threads, ... and adds the n rows up in
// fp32; with WRITE the sum goes to v (the traffic of the last pass: n rows read, one
// written), without it nothing is written (the traffic of one CenteredClip pass; the empty
// asm statement keeps the sums, and so the loads, alive).  Non-temporal loads and stores,
// the faster of the two flavours for this kernel as well.  Rows need only be 4-byte
// aligned, as everywhere in this library (the 128-bit accesses are declared so); the
// d mod 4 coordinates at the end are taken one by one.
template <bool WRITE>
__global__ __launch_bounds__(kBlock) void plain_rowsum_kernel(const float *__restrict__ g,
                                                               int64_t ld, int32_t n, int64_t d,
                                                               float *__restrict__ v)
{
    const int64_t threads = (int64_t)gridDim.x * kBlock;
    const int64_t me = (int64_t)blockIdx.x * kBlock + threadIdx.x;
    const int64_t d4 = d / 4;
    for (int64_t x = me; x < d4; x += threads) {
        float s0 = 0.0f, s1 = 0.0f, s2 = 0.0f, s3 = 0.0f;
#pragma unroll 16
        for (int k = 0; k < n; ++k) {
            const f32x4_u t = stream_load((global_f32x4)(g + k * ld + 4 * x));
            s0 += t.x; s1 += t.y; s2 += t.z; s3 += t.w;
        }
        if constexpr (WRITE) {
            f32x4_u o;
            o.x = s0; o.y = s1; o.z = s2; o.w = s3;
            stream_store(v + 4 * x, o);
        } else {
            asm volatile("" : : "v"(s0), "v"(s1), "v"(s2), "v"(s3));
        }
    }
    if (me < d - 4 * d4) {
        const int64_t x = 4 * d4 + me;
        float s = 0.0f;
        for (int k = 0; k < n; ++k) s += g[k * ld + x];
        if constexpr (WRITE) v[x] = s;
        else asm volatile("" : : "v"(s));
    }
}

}  // namespace btard
