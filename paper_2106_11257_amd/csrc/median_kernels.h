// Coordinate-wise median of the n rows (one of the baseline aggregators of Sec. 4.1):
// v[x] = median of g[0][x] .. g[n-1][x], the mean of the two middle values for even n.
// One pass over the slab in the tile geometry of the other kernels: every lane holds the
// values of its 4 coordinates for the NP peers of its lane group.
//   one lane group (n <= 16): a sorting network in registers (Batcher's odd-even merge sort,
//     v_min_f32 / v_max_f32 pairs); absent peers are +inf and sort to the end;
//   several lane groups (n <= 255): the values of a coordinate are spread over LG lanes.
//     Every lane sorts its 16 values with the same network, then the lanes' runs are merged
//     pairwise by bitonic merges whose exchanges across lanes are wavefront shuffles (one
//     shuffle and one v_med3_f32 per value and exchange); the middle ranks are then read
//     from the lane and register they have come to rest in.  About 350 instructions per
//     coordinate at n = 64 (a rank selection bit by bit on integer keys, the first form of
//     this variant, took about 1300): closer to, but still above, the time of reading the
//     rows.
#pragma once

#include "kernels_common.h"

namespace btard {

struct MedianArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    int64_t d;
    float *v;
    uint32_t epoch_mult;     // write bursts of v: 2^32 / ticks per epoch (0: the default)
};

// Batcher's odd-even merge sort of N = 2^m values (ascending), fully unrolled.
template <int N>
__device__ __forceinline__ void sort_network(float (&x)[N])
{
#pragma unroll
    for (int p = 1; p < N; p <<= 1) {
#pragma unroll
        for (int k = p; k >= 1; k >>= 1) {
#pragma unroll
            for (int j = k % p; j + k < N; j += 2 * k) {
#pragma unroll
                for (int i = 0; i < k; ++i) {
                    if (i + j + k < N && (i + j) / (2 * p) == (i + j + k) / (2 * p)) {
                        const float lo = fminf(x[i + j], x[i + j + k]);
                        const float hi = fmaxf(x[i + j], x[i + j + k]);
                        x[i + j] = lo;
                        x[i + j + k] = hi;
                    }
                }
            }
        }
    }
}

template <int NP, int LG, bool RAGGED>
__global__ __launch_bounds__(kBlock) void coordinate_median_kernel(MedianArgs a)
{
    using G = Geo<NP, LG>;
    const int n = a.n;
    const int64_t lo = 0, hi = a.d;
    const int lane = threadIdx.x & 63;
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;
    const int klo = (n - 1) / 2, khi = n / 2;           // ranks of the two middle values

    const TileRange tr = tile_range<G::kW>(lo, hi);
    // (with one lane group the interior tiles of v are parked in LDS and written in bursts)
    __shared__ f32x4_u s_stage[LG == 1 ? kStageSlots : 1];
    TileStage stage;
    stage.begin(s_stage, __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), a.v, tr.xa, tr.stride, a.epoch_mult);
    int64_t staged_next = -1;                           // the tile that would continue the staged run
    for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
        if constexpr (LG == 1) stage.template flush_if_due<64>(lane, 1);
        const int64_t xu = tr.xa + u * G::kW;
        const bool interior = tile_is_interior<G::kW>(xu, lo, hi);
        const int64_t x0 = xu + (int64_t)sub * kVec;
        float val[NP][4];
        load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, interior, val);
        float med[4];
        if constexpr (LG == 1) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                float col[NP];
#pragma unroll
                for (int k = 0; k < NP; ++k) col[k] = (!RAGGED || k < n) ? val[k][e] : INFINITY;
                sort_network<NP>(col);
                float m0 = col[0], m1 = col[0];
#pragma unroll
                for (int k = 0; k < NP; ++k) {          // klo, khi are wavefront-uniform
                    if (k == klo) m0 = col[k];
                    if (k == khi) m1 = col[k];
                }
                med[e] = (float)(0.5 * ((double)m0 + (double)m1));
            }
        } else {
            static_assert(NP == 16, "the merge steps below are written for 16 values per lane");
            // Every lane sorts its 16 values; then runs of 1, 2, 4, .. lane groups are merged
            // pairwise (bitonic merge: the first exchange pairs rank r of the lower run with
            // rank 2R - 1 - r of the upper one, the following ones are half-cleaners at
            // distances R/2 .. 1 lane groups and 8 .. 1 elements).  Afterwards rank r of a
            // coordinate is element r % 16 of lane group r / 16.
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                float col[NP];
#pragma unroll
                for (int k = 0; k < NP; ++k)
                    col[k] = (!RAGGED || lg * NP + k < n) ? val[k][e] : INFINITY;
                sort_network<NP>(col);
#pragma unroll
                for (int k = 0; k < NP; ++k) val[k][e] = col[k];
            }
#pragma unroll
            for (int R = 1; R < LG; R <<= 1) {
                // the first exchange, with the mirrored lane group and the mirrored element
                {
                    const int mask = (2 * R - 1) * G::kLanes;
                    // median of (a, b, -inf) is min(a, b), of (a, b, +inf) max(a, b)
                    const float keep = (lg & R) ? INFINITY : -INFINITY;
#pragma unroll
                    for (int e = 0; e < kVec; ++e) {
                        float other[NP];
#pragma unroll
                        for (int k = 0; k < NP; ++k) other[k] = __shfl_xor(val[NP - 1 - k][e], mask, 64);
#pragma unroll
                        for (int k = 0; k < NP; ++k)
                            val[k][e] = __builtin_amdgcn_fmed3f(val[k][e], other[k], keep);
                    }
                }
                if (!RAGGED && 2 * R == LG) break;     // (the last merge is finished below)
                // half-cleaners across lane groups
#pragma unroll
                for (int s2 = R >> 1; s2 >= 1; s2 >>= 1) {
                    const int mask = s2 * G::kLanes;
                    const float keep = (lg & s2) ? INFINITY : -INFINITY;
#pragma unroll
                    for (int e = 0; e < kVec; ++e)
#pragma unroll
                        for (int k = 0; k < NP; ++k) {
                            const float other = __shfl_xor(val[k][e], mask, 64);
                            val[k][e] = __builtin_amdgcn_fmed3f(val[k][e], other, keep);
                        }
                }
                // and within the lane
#pragma unroll
                for (int e = 0; e < kVec; ++e)
#pragma unroll
                    for (int s2 = NP / 2; s2 >= 1; s2 >>= 1)
#pragma unroll
                        for (int k = 0; k < NP; ++k)
                            if ((k & s2) == 0) {
                                const float lo2 = fminf(val[k][e], val[k + s2][e]);
                                const float hi2 = fmaxf(val[k][e], val[k + s2][e]);
                                val[k][e] = lo2;
                                val[k + s2][e] = hi2;
                            }
            }
            if constexpr (!RAGGED) {
                // n = 16 LG: after the first exchange of the last merge the lower half of the
                // lane groups holds the n / 2 smallest values, and the two middle ranks are
                // the largest of those and the smallest of the others; the halves need not
                // be sorted any further.
                const float keep = (lg & (LG / 2)) ? -INFINITY : INFINITY;    // max below, min above
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    float t = val[0][e];
#pragma unroll
                    for (int k = 1; k < NP; ++k) t = __builtin_amdgcn_fmed3f(t, val[k][e], keep);
#pragma unroll
                    for (int s2 = LG / 4; s2 >= 1; s2 >>= 1)
                        t = __builtin_amdgcn_fmed3f(t, __shfl_xor(t, s2 * G::kLanes, 64), keep);
                    const float m0 = __shfl(t, sub, 64);
                    const float m1 = __shfl(t, (LG / 2) * G::kLanes + sub, 64);
                    med[e] = (float)(0.5 * ((double)m0 + (double)m1));
                }
            } else {
            // the two middle ranks (wavefront-uniform): element, then lane group
            const int elo = klo % NP, ehi = khi % NP;
            const int src_lo = (klo / NP) * G::kLanes + sub, src_hi = (khi / NP) * G::kLanes + sub;
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                float m0 = val[0][e], m1 = val[0][e];
#pragma unroll
                for (int k = 1; k < NP; ++k) {
                    if (k == elo) m0 = val[k][e];
                    if (k == ehi) m1 = val[k][e];
                }
                m0 = __shfl(m0, src_lo, 64);
                m1 = __shfl(m1, src_hi, 64);
                med[e] = (float)(0.5 * ((double)m0 + (double)m1));
            }
            }
        }
        if (lg == 0) {
            if (interior) {
                f32x4_u o;
                o.x = med[0]; o.y = med[1]; o.z = med[2]; o.w = med[3];
                if constexpr (LG == 1) {
                    // (the staged tiles must be `stride` apart: an edge tile in between ends the run)
                    if (stage.count > 0 && u != staged_next) stage.template flush<64>(lane);
                    stage.template put<64>(u, lane, o);
                    staged_next = u + tr.stride;
                } else {
                    stream_store(a.v + x0, o);
                }
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const int64_t x = x0 + e;
                    if (x >= lo && x < hi) a.v[x] = med[e];
                }
            }
        }
    }
    if constexpr (LG == 1) stage.template flush<64>(lane);
}

}  // namespace btard
