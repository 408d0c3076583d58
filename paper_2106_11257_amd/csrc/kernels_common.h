// Device-side building blocks shared by the gfx950 kernels: tile geometry,
// row loads that tolerate 4-byte alignment, wavefront (64-lane) reductions.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace btard {

constexpr int kBlock = 256;          // threads per workgroup = 4 wavefronts of 64 lanes
constexpr int kWaves = kBlock / 64;
constexpr int kVec = 4;              // coordinates per lane per tile: one 128-bit load per row

// A 128-bit load that only promises dword alignment: rows of g start at
// arbitrary multiples of 4 bytes (ldg and the partition offsets are not
// multiples of 4 elements in general), and gfx950 serves dword-aligned
// global_load_dwordx4 directly.
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));

// Geometry of one wavefront tile.  A wavefront is cut into LG lane groups of
// LANES = 64/LG lanes.  Lane group lg owns peers [lg*NP, lg*NP + NP); lane
// `sub` of every group owns the same 4 consecutive coordinates, so a tile
// covers W = 4*LANES coordinates and each row is read in LANES*16 contiguous
// bytes.  Quantities that need all peers of a coordinate are combined across
// the lane groups with xor-shuffles.
template <int NP, int LG>
struct Geo {
    static_assert(64 % LG == 0, "lane groups must divide the wavefront");
    static constexpr int kNP = NP;
    static constexpr int kLG = LG;
    static constexpr int kLanes = 64 / LG;
    static constexpr int kW = kLanes * kVec;
    static constexpr int kPeers = NP * LG;   // peers one wavefront can hold
};

// Coordinates are tiled from the partition start rounded DOWN to a multiple of
// 4 in the global numbering, so that a lane's 4 coordinates are always one
// Philox block (floor(x/4)); coordinates outside [lo, hi) are masked.
__device__ __forceinline__ int64_t tile_origin(int64_t lo) { return lo & ~int64_t(kVec - 1); }

__device__ __forceinline__ void load_row4(const float *__restrict__ row, int64_t x0,
                                          int64_t lo, int64_t hi, bool full, float (&out)[4])
{
    if (full) {
        f32x4_u t = *reinterpret_cast<const f32x4_u *>(row + x0);
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    } else {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            const int64_t x = x0 + e;
            out[e] = (x >= lo && x < hi) ? row[x] : 0.0f;
        }
    }
}

// Sum over the lanes of one lane group (xor masks below LANES) ...
template <int LANES>
__device__ __forceinline__ double sum_within_group(double a)
{
#pragma unroll
    for (int m = 1; m < LANES; m <<= 1) a += __shfl_xor(a, m, 64);
    return a;
}

// ... and over the lane groups of a wavefront (xor masks LANES .. 32).  Every
// lane ends with the same value: a + b is commutative in IEEE arithmetic and
// the butterfly pairs the same partial sums on both sides.
template <int LANES>
__device__ __forceinline__ double sum_across_groups(double a)
{
#pragma unroll
    for (int m = LANES; m < 64; m <<= 1) a += __shfl_xor(a, m, 64);
    return a;
}

// Device-wide "last workgroup of this partition" election.  Every workgroup
// calls it after its partial results are stored; exactly one caller per round
// gets true, after all the others' stores are visible to it.
__device__ __forceinline__ bool last_block_of_partition(unsigned int *counter, unsigned int blocks)
{
    __shared__ int s_last;
    __threadfence();            // release this thread's partial results (agent scope)
    __syncthreads();
    if (threadIdx.x == 0) {
        const unsigned int prev = atomicAdd(counter, 1u);
        s_last = (prev == blocks - 1u);
    }
    __syncthreads();
    const bool last = s_last != 0;
    if (last) __threadfence();  // acquire the other workgroups' partial results
    return last;
}

}  // namespace btard
