// Device-side building blocks shared by the gfx950 kernels: tile geometry,
// row loads that tolerate 4-byte alignment, wavefront (64-lane) reductions.
// The kernel headers are included by several translation units (one per family of
// instantiations); kernels that are not templates are therefore declared static, and only
// the unit that launches one keeps its code.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace btard {

constexpr int kBlock = 256;          // threads per workgroup = 4 wavefronts of 64 lanes
constexpr int kWaves = kBlock / 64;
constexpr int kVec = 4;              // coordinates per lane per tile: one 128-bit load per row

// A 128-bit access that only promises dword alignment: rows of g start at
// arbitrary multiples of 4 bytes (ldg and the partition offsets are not
// multiples of 4 elements in general), and gfx950 serves dword-aligned
// global_load_dwordx4 directly.
typedef float f32x4_u __attribute__((ext_vector_type(4), aligned(4)));

// Explicit global-address-space pointer types (the address space survives an empty
// asm statement, which a generic pointer's inferred one does not).
typedef const float __attribute__((address_space(1))) *global_f32;
typedef const char __attribute__((address_space(1))) *global_bytes;
typedef const f32x4_u __attribute__((address_space(1))) *global_f32x4;

// The slab is read once per pass and is far larger than the caches: its loads are marked
// non-temporal so that they do not displace other data (measured: +10 % bandwidth on the
// 84 GB slab, +6 % on the 0.7 GB one).  BTARD_NT_LOADS=0 turns that off for experiments.
#ifndef BTARD_NT_LOADS
#define BTARD_NT_LOADS 1
#endif
__device__ __forceinline__ f32x4_u stream_load(global_f32x4 p)
{
#if BTARD_NT_LOADS
    return __builtin_nontemporal_load(p);
#else
    return *p;
#endif
}

// The aggregate is written once and not read again by the kernel that writes it.
#ifndef BTARD_NT_STORES
#define BTARD_NT_STORES 1
#endif
__device__ __forceinline__ void stream_store(float *p, f32x4_u t)
{
#if BTARD_NT_STORES
    __builtin_nontemporal_store(t, reinterpret_cast<f32x4_u *>(p));
#else
    *reinterpret_cast<f32x4_u *>(p) = t;
#endif
}

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
// 32 in the global numbering: a lane's 4 coordinates are then always one Philox
// block (floor(x/4)), and a wavefront's 1 KiB of v starts on a 128-byte boundary
// when v itself does (whole cache lines are written).  Coordinates outside
// [lo, hi) are masked.
// (Tiles narrower than 32 coordinates start at a multiple of their own width: the
// partition must begin inside tile 0.)
constexpr int kOriginAlign = 32;
__host__ __device__ __forceinline__ int64_t tile_origin_for(int64_t lo, int tile_w)
{
    const int align = tile_w < kOriginAlign ? tile_w : kOriginAlign;
    return lo & ~int64_t(align - 1);
}
template <int W>
__device__ __forceinline__ int64_t tile_origin(int64_t lo)
{
    static_assert(W >= kVec && (W & (W - 1)) == 0, "tile widths are powers of two");
    return tile_origin_for(lo, W);
}

// Which tiles of partition [lo, hi) a wavefront visits.
struct TileRange {
    int64_t xa;        // coordinate of tile 0, lane 0
    int64_t units;     // number of tiles
    int64_t first;     // first tile of this wavefront
    int64_t stride;    // distance to its next tile
};

template <int W>
__device__ __forceinline__ TileRange tile_range(int64_t lo, int64_t hi)
{
    TileRange t;
    t.xa = tile_origin<W>(lo);
    t.units = (hi > lo) ? (hi - t.xa + W - 1) / W : 0;
    // Workgroup b of partition j walks the tiles that workgroup (b + j) mod B would walk
    // in the plain order: where the partitions lie a power of two bytes apart (d = 2^28:
    // 2^27), the same workgroup -- the same XCD -- otherwise reads and writes addresses in all
    // partitions at once that differ in their high bits only (fused last pass of the 8.6 GB
    // slab with 8 peers 1.64 -> 1.61 ms, step of the 64 MiB slab 65.2 -> 63.5 us; other
    // shapes unchanged).
    const uint32_t bx = (blockIdx.x + blockIdx.y) % gridDim.x;
    t.first = (int64_t)bx * kWaves + __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    t.stride = (int64_t)gridDim.x * kWaves;
    return t;
}

// Whether the tile starting at xu lies wholly inside [lo, hi) (wavefront-uniform).  Only
// the first and the last tile of a partition can fail this.
template <int W>
__device__ __forceinline__ bool tile_is_interior(int64_t xu, int64_t lo, int64_t hi)
{
    return (xu >= lo) && (xu + W <= hi);
}

// Whether this wavefront's walk first, first + stride, ... visits tile u.
__device__ __forceinline__ bool owns_tile(const TileRange &t, int64_t u)
{
    return u >= t.first && (u - t.first) % t.stride == 0;
}

// One row, 4 coordinates starting at x0, each guarded against [lo, hi).
__device__ __forceinline__ void load_row4_guarded(const float *__restrict__ row, int64_t x0,
                                                  int64_t lo, int64_t hi, float (&out)[4])
{
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const int64_t x = x0 + e;
        out[e] = (x >= lo && x < hi) ? row[x] : 0.0f;
    }
}

__device__ __forceinline__ void load_row4_vec(const float *__restrict__ p, float (&out)[4])
{
    const f32x4_u t = *reinterpret_cast<const f32x4_u *>(p);
    out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
}

// Walks the NP rows of this lane group over one interior tile, one 128-bit load per row.
// With one lane group the row base is wavefront-uniform and walks from peer to peer in
// scalar registers (the saddr form of global_load_dwordx4 with a 32-bit per-lane byte
// offset); the empty asm pins it there, and, being volatile, keeps the loads in program
// order.  With several lane groups every group starts at its own first peer and the base
// is a per-lane address.  Rows beyond n (RAGGED only) re-read the last valid row; their
// coefficients are zero and their accumulators are ignored.
template <int NP, int LG, bool RAGGED>
struct RowCursor {
    global_bytes row;
    uint32_t lane_bytes;

    __device__ __forceinline__ void begin(const float *__restrict__ g, int64_t ld, int n, int lg,
                                          int sub, int64_t xu)
    {
        lane_bytes = (uint32_t)sub * (uint32_t)(kVec * sizeof(float));
        if constexpr (LG == 1) {
            row = (global_bytes)(g + xu);
        } else {
            int i0 = lg * NP;
            if (RAGGED) i0 = i0 < n ? i0 : n - 1;
            row = (global_bytes)(g + xu) + ((int64_t)i0 * ld * 4 + lane_bytes);
        }
    }

    // row k of the tile (k = 0, 1, ... in this order), then step to the next row
    __device__ __forceinline__ void load(int k, int64_t ld, int n, int lg, float (&out)[4])
    {
        f32x4_u t;
        if constexpr (LG == 1) {
            asm volatile("" : "+s"(row));
            t = stream_load((global_f32x4)(row + lane_bytes));
            if (!RAGGED || k + 1 < n) row += ld * 4;
        } else {
            asm volatile("" : "+v"(row));
            t = stream_load((global_f32x4)row);
            if (!RAGGED) row += ld * 4;
            else row += (lg * NP + k + 1 < n) ? ld * 4 : 0;
        }
        out[0] = t.x; out[1] = t.y; out[2] = t.z; out[3] = t.w;
    }
};

// The tiles u = begin, begin + stride, ... < end of this wavefront that lie wholly inside
// the partition: its walk without tile 0 and tile units - 1 where those are edge tiles.
struct InteriorWalk {
    int64_t begin, end;
};

template <int W>
__device__ __forceinline__ InteriorWalk interior_walk(const TileRange &t, int64_t lo, int64_t hi)
{
    InteriorWalk w;
    w.end = t.units;
    if (t.units > 0 && !tile_is_interior<W>(t.xa + (t.units - 1) * W, lo, hi)) w.end = t.units - 1;
    w.begin = t.first;
    if (t.first == 0 && t.units > 0 && !tile_is_interior<W>(t.xa, lo, hi)) w.begin = t.stride;
    return w;
}

// Loads the 4 coordinates [x0, x0+4) of this lane group's NP peers.
//   interior (wavefront-uniform): the whole tile lies inside [lo, hi): straight-line
//   128-bit loads, all issued before anything waits on them.
//   Rows beyond n (RAGGED only) re-read the last valid row; their coefficients are
//   zero and their accumulators are ignored.
template <int NP, int LG, bool RAGGED>
__device__ __forceinline__ void load_tile(const float *__restrict__ g, int64_t ld, int n, int lg,
                                          int sub, int64_t xu, int64_t lo, int64_t hi,
                                          bool interior, float (&val)[NP][4])
{
    if (interior) {
        RowCursor<NP, LG, RAGGED> cur;
        cur.begin(g, ld, n, lg, sub, xu);
#pragma unroll
        for (int k = 0; k < NP; ++k) cur.load(k, ld, n, lg, val[k]);
    } else {
        // Edge tile (the first or the last of a partition): the same straight-line shape
        // with one 32-bit load per coordinate.  A coordinate outside [lo, hi) reads the
        // nearest one inside instead (lo or hi - 1, both within this tile, so the byte
        // offset from the tile start stays in [0, 4W)) and is then replaced by zero: no
        // branches, and no address outside the partition is touched.
        const int64_t x0 = xu + (int64_t)sub * kVec;
        uint32_t offs[kVec];
        bool inside[kVec];
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            const int64_t x = x0 + e;
            inside[e] = (x >= lo) && (x < hi);
            const int64_t xc = (x < lo) ? lo : ((x >= hi) ? hi - 1 : x);
            offs[e] = (uint32_t)(xc - xu) * (uint32_t)sizeof(float);
        }
        if constexpr (LG == 1) {
            global_f32 row = (global_f32)(g + xu);
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                asm volatile("" : "+s"(row));
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const float t = *(global_f32)((global_bytes)row + offs[e]);
                    val[k][e] = inside[e] ? t : 0.0f;
                }
                if (!RAGGED || k + 1 < n) row += ld;
            }
        } else {
            int i0 = lg * NP;
            if (RAGGED) i0 = i0 < n ? i0 : n - 1;
            global_bytes row = (global_bytes)(g + xu) + (int64_t)i0 * ld * 4;
#pragma unroll
            for (int k = 0; k < NP; ++k) {
                asm volatile("" : "+v"(row));
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const float t = *(global_f32)(row + offs[e]);
                    val[k][e] = inside[e] ? t : 0.0f;
                }
                if (!RAGGED) row += ld * 4;
                else row += (lg * NP + k + 1 < n) ? ld * 4 : 0;
            }
        }
    }
}

// Interior tile with one lane group, for loops that keep the lane's byte offset in one
// register for their whole life (lane_off = 16 * sub, handed back unchanged): every load is
// scalar row base + that 32-bit offset.  The offset is re-declared opaque before each load so
// that it is neither widened to 64 bits nor copied; a register that lives as long as the
// loop is never reused for loaded data, so nothing at the head of the loop has to wait for
// loads still in flight.
template <int NP, bool RAGGED>
__device__ __forceinline__ void load_tile_interior(const float *__restrict__ g, int64_t ld, int n,
                                                   int64_t xu, uint32_t &lane_off,
                                                   float (&val)[NP][4])
{
    global_bytes row = (global_bytes)(g + xu);
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        asm volatile("" : "+s"(row), "+v"(lane_off));
        const f32x4_u t = stream_load((global_f32x4)(row + lane_off));
        if (!RAGGED || k + 1 < n) row += ld * 4;
        val[k][0] = t.x; val[k][1] = t.y; val[k][2] = t.z; val[k][3] = t.w;
    }
}

// Writes of v in bursts.  A few stores sprinkled into a stream of loads cost several times
// their share of the bytes (the memory turns around between reading and writing for every
// handful of them): a pass that writes 4 bytes per coordinate next to 64 read took 30 %
// longer than the same pass without the store.  So a wavefront parks the tiles of v it
// produces in its own LDS area and writes them out together -- when the area is full and,
// which is what keeps the bursts of all wavefronts of the device together however long the
// pass runs, whenever the real-time counter that all of them read (s_memrealtime, 100 MHz)
// enters a new epoch.  What is written and where does not depend on the clock, only when.
constexpr int kStageTiles = 16;              // 16 KiB per wavefront, 64 KiB per workgroup
// The epoch length is the caller's (the host picks half the time a wavefront needs to
// fill its area, between 10 and 80 us); it arrives as the multiplier
// 2^32 / ticks, so that the epoch number is one multiply-high of the counter's low word.
constexpr uint32_t kEpochTicksDefault = 6000;                    // 60 us
__host__ __device__ constexpr uint32_t epoch_multiplier(uint32_t ticks)
{
    return (uint32_t)(0x100000000ull / (ticks < 1 ? 1 : ticks));
}
constexpr int kStageSlots = kWaves * kStageTiles * 64;
constexpr uint32_t kSpinFraction = 3951369912u;                 // 0.92 x 2^32
constexpr int kSpinLooks = 2048;

struct TileStage {
    // wavefront-uniform state (scalar registers); the lane's addresses are formed when used
    f32x4_u *area;        // this wavefront's kStageTiles x 64 slots
    float *base;          // v + the first coordinate of the wavefront's tile 0 (tile u: + u W)
    int64_t first;        // index u of the oldest staged tile; the others follow at `stride`
    int64_t stride;
    int count;
    uint32_t epoch;
    uint32_t multiplier;  // 2^32 / ticks per epoch

    __device__ __forceinline__ uint32_t epoch_now() const
    {
        return __umulhi((uint32_t)__builtin_amdgcn_s_memrealtime(), multiplier);
    }

    // LANES: lanes that hold a tile of v (those of lane group 0), 4 coordinates each; the
    // area then takes 64 / LANES x kStageTiles tiles
    template <int LANES>
    static constexpr int capacity() { return kStageTiles * (64 / LANES); }

    __device__ __forceinline__ void begin(f32x4_u *block_area, int wave, float *v, int64_t xa,
                                          int64_t tile_stride, uint32_t epoch_mult)
    {
        area = block_area + wave * (kStageTiles * 64);
        base = v + xa;
        first = 0;
        stride = tile_stride;
        count = 0;
        multiplier = epoch_mult ? epoch_mult : epoch_multiplier(kEpochTicksDefault);
        epoch = epoch_now();
    }

    // (sub: the lane's index in its lane group; holds: it belongs to lane group 0)
    template <int LANES>
    __device__ __forceinline__ void flush(int sub, bool holds = true)
    {
        if (holds) {
#pragma unroll 1
            for (int t = 0; t < count; ++t)
                stream_store(base + (first + t * stride) * (LANES * kVec) + sub * kVec,
                             area[t * LANES + sub]);
        }
        count = 0;
    }

    // The 4 values of interior tile u; to be called by the whole wavefront, consecutive calls
    // `stride` tiles apart.  The caller makes room first (flush_if_due) at a point of its
    // loop of its choosing.
    template <int LANES>
    __device__ __forceinline__ void put(int64_t u, int sub, f32x4_u o, bool holds = true)
    {
        if (count == 0) first = u;
        if (holds) area[count * LANES + sub] = o;
        ++count;
    }

    // to be called at least once per `room` calls of put: writes the staged tiles out if fewer
    // than `room` more would fit, or if the clock has entered a new epoch
    template <int LANES>
    __device__ __forceinline__ void flush_if_due(int sub, int room, bool holds = true)
    {
        // A wavefront that gets here in the last 8 % of an epoch (and holds tiles) waits for
        // the epoch's end instead of going on for another tile: the bursts of all wavefronts
        // then begin within a narrower window (measured on the 84 GB slab: last pass 14.18
        // against 14.63 ms; windows of 4 %, 6 %, 10 % and 15 %: 14.47, 14.33, 14.35 and
        // 15.1 ms).  The wait is bounded: the clock always advances, and the loop gives up
        // after kSpinLooks looks at it.  The low word of ticks x multiplier is the elapsed
        // fraction of the epoch in units of 2^-32.
        uint32_t ticks = (uint32_t)__builtin_amdgcn_s_memrealtime();
        uint32_t now = __umulhi(ticks, multiplier);
        if (now == epoch && count > 0 && ticks * multiplier > kSpinFraction) {
            for (int look = 0; look < kSpinLooks && now == epoch; ++look) {
                __builtin_amdgcn_s_sleep(1);
                now = epoch_now();
            }
        }
        if (count + room > capacity<LANES>() || now != epoch) flush<LANES>(sub, holds);
        epoch = now;
    }
};

// Makes the compiler forget what it knows about a register value (no instruction is
// emitted).  Used between the two sweeps over a tile so that the fp32 values are
// converted to fp64 again in the second sweep instead of keeping 2x the registers live.
__device__ __forceinline__ void forget(float &x) { asm volatile("" : "+v"(x)); }

// A workgroup-uniform double (the same in every lane) -> scalar registers.
__device__ __forceinline__ double uniform_double(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = __builtin_amdgcn_readfirstlane((uint32_t)b);
    const uint32_t hi = __builtin_amdgcn_readfirstlane((uint32_t)(b >> 32));
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// Pre-clipping factors alpha_ij of this lane group's peers for one partition (scale_j: the
// partition's n factors; a null pointer or an absent peer gives 1).  With one lane group the
// factors are wavefront-uniform and live in scalar registers.
template <int NP, int LG, bool RAGGED>
__device__ __forceinline__ void fetch_scale_factors(const double *__restrict__ scale_j, int n, int lg,
                                                    double (&al)[NP])
{
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = lg * NP + k;
        const bool have = scale_j != nullptr && (!RAGGED || i < n);
        const double f = have ? scale_j[have ? i : 0] : 1.0;
        al[k] = (LG == 1) ? uniform_double(f) : f;
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

// The same for NP independent values at once, step by step, so that the NP shuffles of
// one step are in flight together instead of NP dependent chains one after another.
template <int LANES, int NP>
__device__ __forceinline__ void sum_within_group_all(double (&a)[NP])
{
#pragma unroll
    for (int m = 1; m < LANES; m <<= 1) {
        double other[NP];
#pragma unroll
        for (int k = 0; k < NP; ++k) other[k] = __shfl_xor(a[k], m, 64);
#pragma unroll
        for (int k = 0; k < NP; ++k) a[k] += other[k];
    }
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

// Fixed-order sum of the B workgroups' partial results, pj[b * stride + q] over b, for
// every quantity q < Q (Q <= NT), by all NT threads of the workgroup: the rows b are
// dealt round-robin to `tpq` threads per quantity (independent loads, a few each), whose
// sums are then added in order.  Thread q < Q returns the total of quantity q.  The order
// depends only on (B, Q, NT): results are reproducible.  s_red has NT entries.
// (In two halves, so that a caller can put other work between the loads and the barriers.)
constexpr int kPartialsInFlight = 16;
template <int NT>
__device__ __forceinline__ double reduce_partials_load(const double *__restrict__ pj, int B,
                                                       int stride, int Q)
{
    int tpq = NT / Q;
    if (tpq > 32) tpq = 32;
    const int t = threadIdx.x;
    const int s = t / Q, q = t - s * Q;
    // (kPartialsInFlight loads at a time, added in order: one memory latency per group, not
    // one per row.  A row beyond B counts as 0.0, which changes no sum.)
    double acc = 0.0;
    if (s < tpq) {
        for (int b0 = s; b0 < B; b0 += kPartialsInFlight * tpq) {
            double x[kPartialsInFlight];
#pragma unroll
            for (int k = 0; k < kPartialsInFlight; ++k) {
                const int b = b0 + k * tpq;
                x[k] = (b < B) ? pj[(int64_t)b * stride + q] : 0.0;
            }
#pragma unroll
            for (int k = 0; k < kPartialsInFlight; ++k) acc += x[k];
        }
    }
    return acc;
}

template <int NT>
__device__ __forceinline__ double reduce_partials_combine(double acc, int Q, double *s_red)
{
    int tpq = NT / Q;
    if (tpq > 32) tpq = 32;
    const int t = threadIdx.x;
    __syncthreads();
    s_red[t] = acc;
    __syncthreads();
    double tot = 0.0;
    if (t < Q)
        for (int k = 0; k < tpq; ++k) tot += s_red[k * Q + t];
    return tot;
}

template <int NT>
__device__ __forceinline__ double reduce_partials(const double *__restrict__ pj, int B, int stride,
                                                  int Q, double *s_red)
{
    return reduce_partials_combine<NT>(reduce_partials_load<NT>(pj, B, stride, Q), Q, s_red);
}

}  // namespace btard
