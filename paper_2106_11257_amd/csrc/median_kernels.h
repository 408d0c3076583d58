// Coordinate-wise median of the n rows (one of the baseline aggregators of Sec. 4.1):
// v[x] = median of g[0][x] .. g[n-1][x], the mean of the two middle values for even n.
// One pass over the slab in the tile geometry of the other kernels: every lane holds the
// values of its 4 coordinates for the NP peers of its lane group.
//   one lane group (n <= 16): a sorting network in registers (Batcher's odd-even merge sort,
//     v_min_f32 / v_max_f32 pairs); absent peers are +inf and sort to the end;
//   several lane groups (n <= 255): the values of a coordinate are spread over LG lanes, so
//     the k-th smallest is found bit by bit on order-preserving integer keys: for each of
//     the 32 bits, count the keys below the candidate prefix (a count per lane, summed over
//     the lane groups with the 4 coordinates' counts packed into one 32-bit word) and keep
//     the bit if the count does not exceed k.  This variant is bound by the integer ALU
//     (about 40 instructions per bit and coordinate), not by HBM.
#pragma once

#include "kernels_common.h"

namespace btard {

struct MedianArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    int64_t d;
    float *v;
};

// order-preserving map of IEEE-754 binary32 to unsigned integers
__device__ __forceinline__ uint32_t float_key(float x)
{
    const uint32_t b = __float_as_uint(x);
    return b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);
}

__device__ __forceinline__ float key_float(uint32_t k)
{
    const uint32_t b = k ^ ((k >> 31) ? 0x80000000u : 0xFFFFFFFFu);
    return __uint_as_float(b);
}

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
    for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
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
            uint32_t key[NP][4];
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                const bool have = !RAGGED || lg * NP + k < n;
#pragma unroll
                for (int e = 0; e < kVec; ++e) key[k][e] = have ? float_key(val[k][e]) : 0xFFFFFFFFu;
            }
            // the key of rank klo of each of the 4 coordinates
            uint32_t prefix[4] = {0u, 0u, 0u, 0u};
#pragma unroll 1
            for (int bit = 31; bit >= 0; --bit) {
                uint32_t packed = 0;
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const uint32_t cand = prefix[e] | (1u << bit);
                    uint32_t cnt = 0;
#pragma unroll
                    for (int k = 0; k < NP; ++k) cnt += key[k][e] < cand ? 1u : 0u;
                    packed |= cnt << (8 * e);
                }
                // counts of all lane groups (each field stays below 256: n <= 255)
#pragma unroll
                for (int m = G::kLanes; m < 64; m <<= 1) packed += (uint32_t)__shfl_xor((int)packed, m, 64);
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const uint32_t below = (packed >> (8 * e)) & 0xFFu;
                    if (below <= (uint32_t)klo) prefix[e] |= (1u << bit);
                }
            }
            // rank khi: the same value if enough keys are <= it, else the smallest key above
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                uint32_t le = 0, next = 0xFFFFFFFFu;
#pragma unroll
                for (int k = 0; k < NP; ++k) {
                    le += key[k][e] <= prefix[e] ? 1u : 0u;
                    if (key[k][e] > prefix[e] && key[k][e] < next) next = key[k][e];
                }
#pragma unroll
                for (int m = G::kLanes; m < 64; m <<= 1) {
                    le += (uint32_t)__shfl_xor((int)le, m, 64);
                    const uint32_t other = (uint32_t)__shfl_xor((int)next, m, 64);
                    next = other < next ? other : next;
                }
                const uint32_t upper = (le > (uint32_t)khi) ? prefix[e] : next;
                med[e] = (float)(0.5 * ((double)key_float(prefix[e]) + (double)key_float(upper)));
            }
        }
        if (lg == 0) {
            if (interior) {
                f32x4_u o;
                o.x = med[0]; o.y = med[1]; o.z = med[2]; o.w = med[3];
                stream_store(a.v + x0, o);
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const int64_t x = x0 + e;
                    if (x >= lo && x < hi) a.v[x] = med[e];
                }
            }
        }
    }
}

}  // namespace btard
