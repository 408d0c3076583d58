// Gram formulation of CenteredClip (coefficient space).
//
// With v^l = sum_i c_i g_i, everything eq. (CenteredClip) needs from the data is in the
// n x n Gram matrix of a partition, Gamma = X X^T (X = the n x d_j slab):
//
//     ||g_i - v||^2 = Gamma_ii - 2 (Gamma c)_i + c^T Gamma c,
//     ||v^{l} - v^{l-1}||^2 = a^T Gamma a        (a = c^l - c^{l-1}).
//
// So ONE pass over the slab (the only dense contraction of the path: fp64 MFMA) replaces
// all the passes of the iteration; the iteration itself then runs on n x n numbers.
//
// The price is cancellation: both quadratic forms subtract numbers of the size of
// ||g||^2 to get something that may be much smaller.  The iteration kernel therefore
// carries a running bound on the error it may have put into v and on the error of the
// step norm it compares with eps, and hands a partition over to the streaming passes
// (which evaluate the same quantities directly, to fp64 rounding) as soon as a decision
// cannot be guaranteed: the state it leaves is exactly what a streaming pass expects, so
// the hand-over costs nothing.  Where residuals are of the size of the gradients (the
// benchmark configurations) the iteration finishes here.
#pragma once

#include "cc_kernels.h"

namespace btard {

typedef double f64x4 __attribute__((ext_vector_type(4)));

constexpr int kGramPeers = 16;                      // one 16 x 16 MFMA block
constexpr int kGramEntries = kGramPeers * kGramPeers;

struct GramArgs {
    const float *g;
    int64_t ld;
    int32_t n;               // <= 16
    const int64_t *off;
    double *gpart;           // [P][B][256] per-workgroup partial Gram matrices
    int32_t stream_permille; // gram_pass_kernel: share of every partition read with non-temporal loads
    // The Gram pass as the first kernel of a call sequence (no cc_begin_kernel before it): the
    // partition offsets come as an argument and workgroup (0, 0) stores them for the
    // kernels that follow.
    int32_t from_args;       // 0: read off[]; 1: read chunk, store it to off_out
    int32_t parts;
    int64_t *off_out;
    OffChunk chunk;
};

__device__ __forceinline__ void gram_partition_range(const GramArgs &a, int j, int64_t &lo, int64_t &hi)
{
    if (a.from_args) {                                   // uniform
        lo = a.chunk.v[j];
        hi = a.chunk.v[j + 1];
        if (blockIdx.x == 0 && blockIdx.y == 0 && (int)threadIdx.x <= a.parts)
            a.off_out[threadIdx.x] = a.chunk.v[threadIdx.x];
    } else {
        lo = a.off[j];
        hi = a.off[j + 1];
    }
}

// Gamma entry held by register r of lane `lane` in the 16x16x4 fp64 MFMA accumulator: row
// lane/16 + 4 r, column lane % 16 (checked against a plain matrix product by the tests; the
// matrix is symmetric, so which of the two is "row" is immaterial).
__device__ __forceinline__ int gram_entry(int lane, int r) { return ((lane >> 4) + 4 * r) * kGramPeers + (lane & 15); }

// 8 < n <= 16.  In the matrix instructions' operands lane (p = lane % 16, q = lane / 16)
// holds peer p's value of one coordinate: in the 16 coordinates 16 s .. 16 s + 15 of a tile
// the lane owns 4 q .. 4 q + 3 and feeds them, one at a time, to v_mfma_f64_4x4x4_4b_f64.
// That instruction multiplies four independent 4 x 4 blocks: block b's first operand is
// held by lanes 16 k + 4 b + i (row i, k-slot k), its second by lanes 16 k + 4 b + j, and its
// result D[b][i][j] by lane 16 i + 4 b + j (checked on the device; the tests compare the
// matrix with a plain product).  The symmetric 16 x 16 matrix has 10 distinct 4 x 4 blocks:
//   - the lane's value as BOTH operands: block b = the diagonal block of peers 4 b ..;
//   - second operand = the value of peer p - 4 (mod 16): block b pairs peers 4 b .. with
//     peers 4 (b - 1) ..: the four blocks next to the diagonal (cyclically: (0, 3) included);
//   - the two remaining blocks, (0, 2) and (1, 3), would fill only half an instruction, so
//     one instruction takes them for TWO coordinates x and y of the lane at once: in its
//     first operand lanes p < 8 hold their own value at x and lanes p >= 8 the value of
//     peer p - 8 at y, in its second lanes p < 8 hold peer p + 8 at x and lanes p >= 8
//     their own value at y; blocks 0, 1 are then (0, 2), (1, 3) summed over x, blocks 2, 3
//     the same two summed over y (added at the end).
// That is 5 instructions per 8 coordinates, every block slot a distinct needed block: 640
// multiply-adds per 4 coordinates where one 16 x 16 x 4 instruction spends 1024 -- and the
// fp64 matrix rate is the same for both shapes (the small instruction issues every 16-17
// cycles).  The operands of other peers come straight out of the wavefront's LDS copy of
// the tile (three 128-bit reads per 4 coordinates: rows p, p - 4, p - 8), each converted
// to fp64 where it is used: no moves between lanes.  Vector and fp64 matrix instructions of
// a SIMD do not overlap on this chip (a tile's arithmetic takes the sum of the two), and
// the pass is bound by their issue, not by memory: with 6 instructions per 8 coordinates
// and lane rotations (DPP, 16 moves per 4 coordinates) it took 13.2 ms on the 84 GB slab,
// with the rotated operands read from LDS 13.15 ms.
// The slab is read row by row (a wavefront's load instruction covers 1 KiB of one peer's
// row, the pattern that reaches the highest bandwidth) and turned into the operand layout
// (16 peers across the lanes) through the wavefront's own LDS area: written row-wise,
// read back as 16 coordinates x 16 peers.  No barrier is involved.  Rows of the LDS copy
// are 16 bytes longer than 1 KiB so that the 16 peers' reads fall into different banks.
#ifndef BTARD_GRAM_LDS_PAD
#define BTARD_GRAM_LDS_PAD 4
#endif
constexpr int kGramLdsRow = 256 + BTARD_GRAM_LDS_PAD;  // floats per LDS row

// `stream` (wavefront-uniform): non-temporal loads, for the part of the slab that will not
// survive in the memory-side cache until the last pass reads it again anyway.
template <bool RAGGED>
__device__ __forceinline__ void gram_fetch_rows(const float *__restrict__ g, int64_t ld, int n, int lane,
                                                int64_t xu, int64_t lo, int64_t hi, bool interior,
                                                bool stream, f32x4_u (&v)[16])
{
    if (interior) {
        // one scalar row base walking from peer to peer (rows beyond n re-read the last one)
        global_bytes row = (global_bytes)(g + xu);
        const uint32_t lane_bytes = (uint32_t)lane * 16u;
        if (stream) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                asm volatile("" : "+s"(row));
                v[r] = __builtin_nontemporal_load((global_f32x4)(row + lane_bytes));
                if (!RAGGED || r + 1 < n) row += ld * 4;
            }
        } else {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                asm volatile("" : "+s"(row));
                v[r] = *(global_f32x4)(row + lane_bytes);
                if (!RAGGED || r + 1 < n) row += ld * 4;
            }
        }
    } else {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const float *rowp = g + (int64_t)((!RAGGED || r < n) ? r : n - 1) * ld;
            float t[4];
            load_row4_guarded(rowp, xu + 4 * lane, lo, hi, t);
            v[r].x = t[0]; v[r].y = t[1]; v[r].z = t[2]; v[r].w = t[3];
        }
    }
}

// One tile: the wavefront's registers -> its LDS area, row-wise ...
__device__ __forceinline__ void gram_stage(float (&tile)[16][kGramLdsRow], int lane, const f32x4_u (&rows)[16])
{
#pragma unroll
    for (int r = 0; r < 16; ++r) *reinterpret_cast<f32x4_u *>(&tile[r][4 * lane]) = rows[r];
}

// ... and read back peer-wise into the matrix instructions.
// acc[0]: diagonal blocks, acc[1]: blocks (b, b - 1), acc[2]: blocks (0, 2), (1, 3) twice;
// two accumulators each, used in turn, so that consecutive instructions do not wait for
// each other.
template <bool RAGGED>
__device__ __forceinline__ void gram_multiply(const float (&tile)[16][kGramLdsRow], int p, int q, int n,
                                              double (&acc)[3][2])
{
    const int p1 = (p + 12) & 15, p2 = (p + 8) & 15;           // peers p - 4 and p - 8 (mod 16)
    const bool low = p < 8;
    const bool have = p < n, have1 = p1 < n, have2 = p2 < n;
    // third block set: lanes p < 8 take coordinates 0, 1 of the lane's four (own value first,
    // peer p + 8 second), lanes p >= 8 coordinates 2, 3 (peer p - 8 first, own value second):
    // the LDS addresses do the selection
    const int pa = low ? p : p2, pb = low ? p2 : p, xo = low ? 0 : 2;
    const bool have_a = low ? have : have2, have_b = low ? have2 : have;
    typedef float f32x2_a __attribute__((ext_vector_type(2), aligned(8)));
#pragma unroll
    for (int s = 0; s < 16; ++s) {
        const f32x4_u t = *reinterpret_cast<const f32x4_u *>(&tile[p][16 * s + 4 * q]);
        const f32x4_u t1 = *reinterpret_cast<const f32x4_u *>(&tile[p1][16 * s + 4 * q]);
        const f32x2_a ta = *reinterpret_cast<const f32x2_a *>(&tile[pa][16 * s + 4 * q + xo]);
        const f32x2_a tb = *reinterpret_cast<const f32x2_a *>(&tile[pb][16 * s + 4 * q + xo]);
        float val[4] = {t.x, t.y, t.z, t.w};
        float val1[4] = {t1.x, t1.y, t1.z, t1.w};
        float va[2] = {ta.x, ta.y}, vb[2] = {tb.x, tb.y};
        if (RAGGED) {
            // (rows of absent peers hold a copy of the last row: replaced by zero)
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                val[e] = have ? val[e] : 0.0f;
                val1[e] = have1 ? val1[e] : 0.0f;
            }
#pragma unroll
            for (int h = 0; h < 2; ++h) {
                va[h] = have_a ? va[h] : 0.0f;
                vb[h] = have_b ? vb[h] : 0.0f;
            }
        }
        // the operands of the group's 10 instructions first, each in registers of its own
        double d[4], d1[4], da[2], db[2];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d[e] = (double)val[e];
            d1[e] = (double)val1[e];
        }
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            da[h] = (double)va[h];
            db[h] = (double)vb[h];
        }
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            acc[0][e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(d[e], d[e], acc[0][e & 1], 0, 0, 0);
            acc[1][e & 1] = __builtin_amdgcn_mfma_f64_4x4x4f64(d[e], d1[e], acc[1][e & 1], 0, 0, 0);
        }
#pragma unroll
        for (int h = 0; h < 2; ++h)
            acc[2][h] = __builtin_amdgcn_mfma_f64_4x4x4f64(da[h], db[h], acc[2][h], 0, 0, 0);
    }
}

template <bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void gram_pass_kernel(GramArgs a)
{
    constexpr int kW = 256;
    __shared__ float tile[kWaves][16][kGramLdsRow];
    __shared__ double sh[kWaves][kGramEntries];
    const int j = blockIdx.y;
    const int n = a.n;
    int64_t lo, hi;
    gram_partition_range(a, j, lo, hi);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = lane & 15, q = lane >> 4;

    // [block set][two independent accumulators: consecutive MFMAs do not wait for each other]
    double acc[3][2];
#pragma unroll
    for (int s = 0; s < 3; ++s) { acc[s][0] = 0.0; acc[s][1] = 0.0; }
    const TileRange tr = tile_range<kW>(lo, hi);
    // the partition's first stream_permille thousandths are read with non-temporal loads
    const int64_t stream_units = tr.units * a.stream_permille / 1000;

    // One register set: while a tile is multiplied out of LDS, the next one's loads travel.
    // (Two sets, loaded two tiles ahead, gain nothing on the 84 GB slab -- 12.85 against
    // 12.89 ms -- and lose on the 0.7 GB one, 126 against 116 us: the pass is not short of
    // requests in flight.)
    f32x4_u rows[16];
    if (tr.first < tr.units) {
        const int64_t xu = tr.xa + tr.first * kW;
        gram_fetch_rows<RAGGED>(a.g, a.ld, n, lane, xu, lo, hi, tile_is_interior<kW>(xu, lo, hi),
                                tr.first < stream_units, rows);
    }
    for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
        gram_stage(tile[wave], lane, rows);
        const int64_t un = u + tr.stride;
        if (un < tr.units) {
            const int64_t xn = tr.xa + un * kW;
            gram_fetch_rows<RAGGED>(a.g, a.ld, n, lane, xn, lo, hi, tile_is_interior<kW>(xn, lo, hi),
                                    un < stream_units, rows);
        }
#ifdef BTARD_PROBE_NO_MULTIPLY
        if (a.n > 100) gram_multiply<RAGGED>(tile[wave], p, q, n, acc);
        asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
#else
        gram_multiply<RAGGED>(tile[wave], p, q, n, acc);
#endif
    }

    // Workgroup partial: the 4 wavefronts' matrices added in order.  Lane 16 i + 4 b + jj holds
    // entry (4 b + i, 4 b + jj) of the diagonal blocks and entry (4 b + i, 4 ((b - 1) mod 4) + jj)
    // of the blocks next to them; of the third set, blocks b = 0, 1 hold entry
    // (4 b + i, 8 + 4 b + jj) summed over one half of the coordinates and blocks b + 2 (8 lanes
    // further on) the same entry summed over the other half.  Transposes are written as well.
    {
        const int i = lane >> 4, b = (lane >> 2) & 3, jj = lane & 3;
        const int r = 4 * b + i;
        sh[wave][r * kGramPeers + 4 * b + jj] = acc[0][0] + acc[0][1];
        const int c1 = 4 * ((b + 3) & 3) + jj;
        const double x1 = acc[1][0] + acc[1][1];
        sh[wave][r * kGramPeers + c1] = x1;
        sh[wave][c1 * kGramPeers + r] = x1;
        double x2 = acc[2][0] + acc[2][1];
        x2 += __shfl_xor(x2, 8, 64);                 // (the same sum in both lanes: a + b = b + a)
        if (b < 2) {
            const int c2 = 8 + 4 * b + jj;
            sh[wave][r * kGramPeers + c2] = x2;
            sh[wave][c2 * kGramPeers + r] = x2;
        }
    }
    __syncthreads();
    const int t = threadIdx.x;
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += sh[w][t];
    a.gpart[((int64_t)j * gridDim.x + blockIdx.x) * kGramEntries + t] = s;
}

// ---------------------------------------------------------------------------
// n <= 8 on the vector ALU.  Gamma is symmetric, so only the pairs (i, i + dl mod NP),
// dl = 0 .. NP/2, are needed: NP (NP/2 + 1) products per coordinate, where a 16 x 16 matrix
// instruction forms 256 of which at most 64 are wanted.  The four wavefronts of a workgroup
// walk the SAME 256-coordinate tiles (a lane holds 4 coordinates) and split the pairs:
// wavefront w takes base rows i = (NP/4) w + k, k < NP/4, for which it needs the
// NP/4 + NP/2 rows i .. i + NP/2 (mod NP) and keeps (NP/4)(NP/2 + 1) accumulators per lane.
// Every row is needed by three of the four wavefronts, so a tile goes through LDS: each
// wavefront loads NP/4 rows of the next tile from memory while the workgroup multiplies the
// current one; two tiles in LDS, one barrier per tile.
// Measured on an 8.6 GB slab with n = 8: 1.24 ms against 1.61 ms for the MFMA form with two
// coordinates per 16-row block.  The template also works for NP = 16, where it was measured
// level with the MFMA kernel (140 against 142-147 us on an 0.7 GB slab) and is not used.
// Two other forms of the same split were slower than the MFMA kernel: every wavefront
// reading its rows from memory (each row three times, twice from the caches), and the four
// rows of 16 lanes of one wavefront taking the four sets of base rows on 64 coordinates.
// ---------------------------------------------------------------------------
template <int NP>
struct GramBand {
    static constexpr int kBase = NP / 4;             // base rows per wavefront = rows it loads
    static constexpr int kDeltas = NP / 2 + 1;       // row distances 0 .. NP/2
    static constexpr int kRows = kBase + NP / 2;     // rows a wavefront multiplies
    static constexpr int kW = 64 * kVec;             // coordinates per tile
};

// Waits for this wavefront's LDS traffic only (loads from memory stay in flight), then the
// workgroup barrier.
__device__ __forceinline__ void lds_barrier()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup", "local");
    __builtin_amdgcn_s_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup", "local");
}

// The wavefront's own rows of the tile at xu: row[m] + xu is wavefront-uniform (a scalar
// base), lane_bytes the lane's 32-bit byte offset.  The compiler must not fold lane_bytes
// into per-row vector addresses outside the loop (two registers and an add per row): the
// value is "changed" in place.
template <int NP>
__device__ __forceinline__ void band_fetch(const global_f32 (&row)[GramBand<NP>::kBase], int64_t xu,
                                           uint32_t &lane_bytes, f32x4_u (&g)[GramBand<NP>::kBase])
{
#pragma unroll
    for (int m = 0; m < GramBand<NP>::kBase; ++m) {
        const char __attribute__((address_space(1))) *base =
            (const char __attribute__((address_space(1))) *)(row[m] + xu);
        g[m] = stream_load((global_f32x4)(base + lane_bytes));
    }
}

template <int NP, bool RAGGED>
__device__ __forceinline__ void band_stage(float (&tile)[NP][GramBand<NP>::kW], int first_row,
                                           const bool (&have)[GramBand<NP>::kBase], int lane,
                                           const f32x4_u (&g)[GramBand<NP>::kBase])
{
#pragma unroll
    for (int m = 0; m < GramBand<NP>::kBase; ++m) {
        f32x4_u t = g[m];
        if (RAGGED && !have[m]) { t.x = 0.0f; t.y = 0.0f; t.z = 0.0f; t.w = 0.0f; }   // absent peer
        *reinterpret_cast<f32x4_u *>(&tile[first_row + m][lane * kVec]) = t;
    }
}

template <int NP>
__device__ __forceinline__ void band_read(const float (&tile)[NP][GramBand<NP>::kW],
                                          const int (&peer)[GramBand<NP>::kRows], int lane,
                                          float (&val)[GramBand<NP>::kRows][4])
{
#pragma unroll
    for (int r = 0; r < GramBand<NP>::kRows; ++r) {
        const f32x4_u t = *reinterpret_cast<const f32x4_u *>(&tile[peer[r]][lane * kVec]);
        val[r][0] = t.x; val[r][1] = t.y; val[r][2] = t.z; val[r][3] = t.w;
    }
}

template <int NP, bool MASKED, int E>
__device__ __forceinline__ void band_accumulate(const float (&val)[GramBand<NP>::kRows][E],
                                                const bool (&have)[GramBand<NP>::kRows],
                                                double (&acc)[GramBand<NP>::kBase][GramBand<NP>::kDeltas])
{
    using B = GramBand<NP>;
#pragma unroll
    for (int e = 0; e < E; ++e) {
        double d[B::kRows];
#pragma unroll
        for (int r = 0; r < B::kRows; ++r) d[r] = (!MASKED || have[r]) ? (double)val[r][e] : 0.0;
#pragma unroll
        for (int k = 0; k < B::kBase; ++k) {
#pragma unroll
            for (int dl = 0; dl < B::kDeltas; ++dl) acc[k][dl] = fma(d[k], d[k + dl], acc[k][dl]);
        }
    }
}

template <int NP, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void gram_pass_band_kernel(GramArgs a)
{
    using B = GramBand<NP>;
    __shared__ float tile[2][NP][B::kW];
    __shared__ double sh[kGramEntries];
    const int j = blockIdx.y;
    const int n = a.n;
    int64_t lo, hi;
    gram_partition_range(a, j, lo, hi);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    sh[threadIdx.x] = 0.0;                           // entries nobody forms (NP < 16) stay 0

    // wavefront-uniform: the rows this wavefront multiplies, and the first kBase of them,
    // which it also loads
    global_f32 row[B::kRows], own[B::kBase];
    bool have[B::kRows], have_own[B::kBase];
    int peer[B::kRows];
#pragma unroll
    for (int r = 0; r < B::kRows; ++r) {
        peer[r] = (B::kBase * wave + r) % NP;
        have[r] = peer[r] < n;
        row[r] = (global_f32)a.g + (int64_t)(have[r] ? peer[r] : n - 1) * a.ld;
    }
#pragma unroll
    for (int m = 0; m < B::kBase; ++m) { own[m] = row[m]; have_own[m] = have[m]; }
    double acc[B::kBase][B::kDeltas];
#pragma unroll
    for (int k = 0; k < B::kBase; ++k) {
#pragma unroll
        for (int dl = 0; dl < B::kDeltas; ++dl) acc[k][dl] = 0.0;
    }

    // the workgroup's interior tiles: begin, begin + stride, ... (count of them; the same
    // for its four wavefronts, which meet at a barrier per tile)
    const int64_t xa = tile_origin<B::kW>(lo);
    const int64_t units = (hi > lo) ? (hi - xa + B::kW - 1) / B::kW : 0;
    const int64_t stride = gridDim.x;
    const int64_t bx = (blockIdx.x + blockIdx.y) % gridDim.x;     // (rotated as in tile_range)
    int64_t begin = bx, end = units;
    if (units > 0 && !tile_is_interior<B::kW>(xa + (units - 1) * B::kW, lo, hi)) end = units - 1;
    if (begin == 0 && units > 0 && !tile_is_interior<B::kW>(xa, lo, hi)) begin = stride;
    const int64_t count = (begin < end) ? (end - begin + stride - 1) / stride : 0;
    uint32_t lane_bytes = (uint32_t)lane * (kVec * (uint32_t)sizeof(float));
    if (count > 0) {
        // Tile t of the walk (t >= count: the last one again -- loads without a condition
        // keep the loop free of joins that would wait for everything in flight).
        const int64_t step = stride * B::kW;
        const int64_t x_first = xa + begin * B::kW, x_last = x_first + (count - 1) * step;
        f32x4_u g[B::kBase];
        float val[B::kRows][4];
        band_fetch<NP>(own, x_first, lane_bytes, g);
        band_stage<NP, RAGGED>(tile[0], B::kBase * wave, have_own, lane, g);
        lds_barrier();
        // here: tile t is in LDS half t % 2; tile t + 1 is loaded while tile t is multiplied
        int64_t x1 = x_first + step;                 // tile t + 1
        for (int64_t t = 0;; t += 2) {
            band_fetch<NP>(own, x1 <= x_last ? x1 : x_last, lane_bytes, g);
            __builtin_amdgcn_sched_barrier(0);
            band_read<NP>(tile[0], peer, lane, val);
            band_accumulate<NP, false, 4>(val, have, acc);
            band_stage<NP, RAGGED>(tile[1], B::kBase * wave, have_own, lane, g);
            lds_barrier();
            if (t + 1 >= count) break;
            x1 += step;
            band_fetch<NP>(own, x1 <= x_last ? x1 : x_last, lane_bytes, g);
            __builtin_amdgcn_sched_barrier(0);
            band_read<NP>(tile[1], peer, lane, val);
            band_accumulate<NP, false, 4>(val, have, acc);
            band_stage<NP, RAGGED>(tile[0], B::kBase * wave, have_own, lane, g);
            lds_barrier();
            if (t + 2 >= count) break;
            x1 += step;
        }
    }
    // the partition's first and last tile where they are not interior: straight from memory
    const int64_t xl = xa + (int64_t)lane * kVec;
#pragma unroll 1
    for (int t = 0; t < 2; ++t) {
        const int64_t u = (t == 0) ? 0 : units - 1;
        if ((t == 1 && units < 2) || u < 0) continue;
        if (u < bx || (u - bx) % stride != 0) continue;
        if (tile_is_interior<B::kW>(xa + u * B::kW, lo, hi)) continue;
        float ve[B::kRows][4];
#pragma unroll
        for (int r = 0; r < B::kRows; ++r) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const int64_t x = xl + u * B::kW + e;
                ve[r][e] = (x >= lo && x < hi) ? row[r][x] : 0.0f;
            }
        }
        band_accumulate<NP, RAGGED, 4>(ve, have, acc);
    }

    // sums over the wavefront's lanes, then entry (i, i + dl) and its mirror image
#pragma unroll
    for (int k = 0; k < B::kBase; ++k) sum_within_group_all<64, B::kDeltas>(acc[k]);
    __syncthreads();                                 // sh is zeroed
    if (lane == 0) {
#pragma unroll
        for (int k = 0; k < B::kBase; ++k) {
            const int i = B::kBase * wave + k;
#pragma unroll
            for (int dl = 0; dl < B::kDeltas; ++dl) {
                // distance NP/2 pairs are formed twice (from i and from i + NP/2) with the
                // same products in the same order: the lower wavefronts write them
                if (dl == NP / 2 && i >= NP / 2) continue;
                const int k2 = (i + dl) % NP;
                sh[i * kGramPeers + k2] = acc[k][dl];
                sh[k2 * kGramPeers + i] = acc[k][dl];
            }
        }
    }
    __syncthreads();
    a.gpart[((int64_t)j * gridDim.x + blockIdx.x) * kGramEntries + threadIdx.x] = sh[threadIdx.x];
}

// ---------------------------------------------------------------------------
// 16 < n <= 64: Gamma is NB x NB blocks of 16 x 16 (NB = ceil(n / 16)), of which the
// NB (NB + 1) / 2 on and above the diagonal are formed: per 4 coordinates one operand
// register per block of peers, and one MFMA per pair of blocks (b <= c) with block b's
// values as the first and block c's as the second operand.  Tiles are 64 coordinates (each
// lane holds 4 coordinates of its peer in each of the NB blocks).  The workgroup's partial
// result is kWidePairs x 256 doubles: pair (b, c) at slot wide_pair(b, c), entry (i, k) of
// the block at i * 16 + k = Gamma[16 b + i][16 c + k] (slots of absent blocks stay unwritten
// and unread).  With 10 MFMAs per 4 coordinates at NB = 4 the pass is bound by the fp64
// MFMA issue rate, about twice the time of reading the slab.
// ---------------------------------------------------------------------------
constexpr int kWideBlocks = 4;                                     // n <= 64
constexpr int kWidePairs = kWideBlocks * (kWideBlocks + 1) / 2;    // 10
constexpr int kWideEntries = kWidePairs * kGramEntries;
__host__ __device__ constexpr int wide_pair(int b, int c) { return b * kWideBlocks - b * (b - 1) / 2 + (c - b); }

// Half a tile: the lane's 8 coordinates (4 at x and 4 at x + 16) of its peer in each block.
template <int NB, int S>
__device__ __forceinline__ void wide_fetch(const global_f32 (&row)[NB], int64_t x,
                                           float (&val)[NB][S][4])
{
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int s = 0; s < S; ++s) {
            const f32x4_u t = *(global_f32x4)(row[b] + x + 16 * s);
            val[b][s][0] = t.x; val[b][s][1] = t.y; val[b][s][2] = t.z; val[b][s][3] = t.w;
        }
    }
}

// Half a tile of 32 coordinates: per 4 of them, one matrix instruction per pair of blocks.
template <int NB, bool RAGGED, int S>
__device__ __forceinline__ void wide_multiply(const float (&val)[NB][S][4], const bool (&have)[NB],
                                              f64x4 (&acc)[NB * (NB + 1) / 2])
{
#pragma unroll
    for (int s = 0; s < S; ++s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            double d[NB];
#pragma unroll
            for (int b = 0; b < NB; ++b) d[b] = (RAGGED && !have[b]) ? 0.0 : (double)val[b][s][e];
            int t = 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int c = b; c < NB; ++c) {
                    acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(d[b], d[c], acc[t], 0, 0, 0);
                    ++t;
                }
            }
        }
    }
}

// The operands of half a tile: fp64, absent peers (RAGGED) as zeros.
template <int NB, bool RAGGED>
__device__ __forceinline__ void wide_convert(float (&val)[NB][2][4], const bool (&have)[NB],
                                             double (&d)[NB][2][4])
{
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int s = 0; s < 2; ++s) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                d[b][s][e] = (RAGGED && !have[b]) ? 0.0 : (double)val[b][s][e];
                // (converted before the loads that follow may overwrite the register)
                asm volatile("" : "+v"(d[b][s][e]));
            }
        }
    }
}

template <int NB>
__device__ __forceinline__ void wide_multiply_f64(const double (&d)[NB][2][4],
                                                  f64x4 (&acc)[NB * (NB + 1) / 2])
{
#pragma unroll
    for (int s = 0; s < 2; ++s) {
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            int t = 0;
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int c = b; c < NB; ++c) {
                    acc[t] = __builtin_amdgcn_mfma_f64_16x16x4f64(d[b][s][e], d[c][s][e], acc[t], 0, 0, 0);
                    ++t;
                }
            }
        }
    }
}

// RAGGED: n < 16 NB (rows beyond n are read from row n - 1 and replaced by zero).
template <int NB, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void gram_pass_wide_kernel(GramArgs a)
{
    constexpr int kW = 64;
    constexpr int kPairs = NB * (NB + 1) / 2;
    __shared__ double sh[kPairs * kGramEntries];
    const int j = blockIdx.y;
    const int n = a.n;
    int64_t lo, hi;
    gram_partition_range(a, j, lo, hi);
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = lane & 15, q = lane >> 4;
    bool have[NB];
    global_f32 row[NB];
#pragma unroll
    for (int b = 0; b < NB; ++b) {
        have[b] = 16 * b + p < n;
        row[b] = (global_f32)a.g + (int64_t)(have[b] ? 16 * b + p : n - 1) * a.ld;
    }

    f64x4 acc[kPairs];
#pragma unroll
    for (int t = 0; t < kPairs; ++t) acc[t] = f64x4{0.0, 0.0, 0.0, 0.0};
    const TileRange tr = tile_range<kW>(lo, hi);
    const InteriorWalk iw = interior_walk<kW>(tr, lo, hi);
    // Interior tiles, half a tile (32 coordinates, 80 matrix instructions at NB = 4) at a
    // time: the half's values are converted to fp64 operands, the loads of the next half are
    // issued into the registers they leave, and then the matrix instructions run -- so the
    // matrix unit does not wait for memory whenever both wavefronts of a SIMD run out of
    // data at about the same time, and nothing is copied.  Vector and fp64 matrix
    // instructions of a SIMD do not overlap on this chip, so every vector instruction saved
    // counts: 4.5 GB slab with 64 peers 1.41 ms with loads issued only when the previous
    // tile is done, 1.33 ms with the next half's loads ahead and a register copy per half,
    // 1.27 ms in this form (a whole tile ahead, 242 registers: 1.40 ms; two loop bodies
    // taking turns make the compiler move the 80 accumulator registers once per round).
    if (iw.begin < iw.end) {
        float val[NB][2][4];
        wide_fetch<NB, 2>(row, tr.xa + iw.begin * kW + 4 * q, val);
        for (int64_t u = iw.begin; u < iw.end; u += tr.stride) {
#pragma unroll 1
            for (int h = 0; h < 2; ++h) {
                // this half's values as fp64 operands, then the next half's loads (the tile's
                // second half, or the next tile's first) into the registers they leave
                double d[NB][2][4];
                wide_convert<NB, RAGGED>(val, have, d);
                const int64_t xn = (h == 0) ? tr.xa + u * kW + 32 : tr.xa + (u + tr.stride) * kW;
                if (h == 0 || u + tr.stride < iw.end) wide_fetch<NB, 2>(row, xn + 4 * q, val);
                wide_multiply_f64<NB>(d, acc);
            }
        }
    }
    // ... then the partition's first and last tile where they are not interior
#pragma unroll 1
    for (int t = 0; t < 2; ++t) {
        const int64_t u = (t == 0) ? 0 : tr.units - 1;
        if ((t == 1 && tr.units < 2) || tr.units < 1 || !owns_tile(tr, u)) continue;
        const int64_t xu = tr.xa + u * kW;
        if (tile_is_interior<kW>(xu, lo, hi)) continue;
#pragma unroll 1
        for (int h = 0; h < 2; ++h) {
            float val[NB][2][4];
#pragma unroll
            for (int b = 0; b < NB; ++b) {
#pragma unroll
                for (int s = 0; s < 2; ++s) {
#pragma unroll
                    for (int e = 0; e < 4; ++e) {
                        const int64_t x = xu + 32 * h + 16 * s + 4 * q + e;
                        val[b][s][e] = (x >= lo && x < hi) ? row[b][x] : 0.0f;
                    }
                }
            }
            wide_multiply<NB, RAGGED, 2>(val, have, acc);
        }
    }

    // workgroup partial: the 4 wavefronts' matrices added in order through one LDS copy
#pragma unroll 1
    for (int w = 0; w < kWaves; ++w) {
        if (wave == w) {
#pragma unroll
            for (int t = 0; t < kPairs; ++t) {
#pragma unroll
                for (int r = 0; r < 4; ++r) {
                    const int idx = t * kGramEntries + gram_entry(lane, r);
                    sh[idx] = (w == 0) ? acc[t][r] : sh[idx] + acc[t][r];
                }
            }
        }
        __syncthreads();
    }
    double *out = a.gpart + ((int64_t)j * gridDim.x + blockIdx.x) * kWideEntries;
    int t = 0;
#pragma unroll
    for (int b = 0; b < NB; ++b) {
#pragma unroll
        for (int c = b; c < NB; ++c) {
            out[wide_pair(b, c) * kGramEntries + threadIdx.x] = sh[t * kGramEntries + threadIdx.x];
            ++t;
        }
    }
}

struct GramIterArgs {
    CcState st;
    const double *gpart;
    int32_t blocks;          // workgroups per partition of gram_pass_kernel
    int32_t n;
    double tau, eps;
    int32_t max_iters;
    double lambda;           // pre-clipping radius (BTARD-Clipped-SGD); <= 0: none
    int32_t nb;              // wide layout only: blocks of 16 peers that were formed
    int32_t fresh;           // 1: no cc_begin_kernel ran: start from c = 1/n and set up what it would have
};

// Relative accuracy assumed for a Gram entry and for a quadratic form in it, in units of
// sum |x_k x_l|: 2^-46 (about 130 roundings; the accumulation per lane is a chain of a few
// hundred fused multiply-adds of exact products, the rest are short fixed-order sums).
constexpr double kGramUnit = 1.4210854715202004e-14;
// The Gram iteration vouches for a squared norm whose error bar is below this fraction of
// it (1e-8 relative on the norm: four orders inside the tolerance of the projections).
constexpr double kGramVouch = 2e-8;
// ... and only if rounding v to fp32 cannot move a norm by 1e-6 of itself (see where they
// are used): squares of 0.34 and of 6e-5.
constexpr double kGramRoundSpread = 0.1156;
constexpr double kGramRoundFloor = 3.6e-9;

// Value of lane `k` (a compile-time constant) for every lane: two v_readlane into scalar
// registers, no LDS traffic.
template <int K>
__device__ __forceinline__ double lane_value(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, K);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), K);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// x of the lane CTRL positions to the left in the same row of 16 lanes (0 if there is none).
template <int CTRL>
__device__ __forceinline__ double row_shift_right(double x)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)b, CTRL, 0xf, 0xf, true);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_update_dpp(0, (int)(uint32_t)(b >> 32), CTRL, 0xf, 0xf, true);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// Sum over lanes 0..15 (row 0 of the wavefront; the other rows hold copies), in a fixed
// order, returned to every lane: DPP row shifts by 1, 2, 4, 8 leave the total in lane 15.
__device__ __forceinline__ double row_sum16(double x)
{
    x += row_shift_right<0x111>(x);
    x += row_shift_right<0x112>(x);
    x += row_shift_right<0x114>(x);
    x += row_shift_right<0x118>(x);
    return lane_value<15>(x);
}

// Up to four sums over the 16 peers at once: the wavefront's four rows of 16 lanes hold the
// same per-peer data, so row q reduces quantity q (one set of DPP steps for all four).
__device__ __forceinline__ void row_sum16x4(int q, double a0, double a1, double a2, double a3,
                                            double &s0, double &s1, double &s2, double &s3)
{
    double x = (q == 0) ? a0 : (q == 1) ? a1 : (q == 2) ? a2 : a3;
    x += row_shift_right<0x111>(x);
    x += row_shift_right<0x112>(x);
    x += row_shift_right<0x114>(x);
    x += row_shift_right<0x118>(x);
    s0 = lane_value<15>(x);
    s1 = lane_value<31>(x);
    s2 = lane_value<47>(x);
    s3 = lane_value<63>(x);
}

__device__ __forceinline__ void row_sum16x2(int q, double a0, double a1, double &s0, double &s1)
{
    double x = (q == 0) ? a0 : a1;
    x += row_shift_right<0x111>(x);
    x += row_shift_right<0x112>(x);
    x += row_shift_right<0x114>(x);
    x += row_shift_right<0x118>(x);
    s0 = lane_value<15>(x);
    s1 = lane_value<31>(x);
}

// Value of lane k for every lane, k known after unrolling.
__device__ __forceinline__ double lane_value_at(double x, int k)
{
    const uint64_t b = (uint64_t)__double_as_longlong(x);
    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)b, k);
    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(b >> 32), k);
    return __longlong_as_double((long long)(((uint64_t)hi << 32) | lo));
}

// sum_k row[k] * (x of lane k of the same row of 16 lanes): sixteen fused multiply-adds whose
// first factor is the broadcast itself (v_fmac_f64 with the DPP control row_newbcast:k, the
// one control the fp64 unit accepts), in two chains that are added at the end -- a third of
// the instructions of a broadcast by moves (two 32-bit moves per value) followed by a
// multiply-add.  The s_nop covers the wait states a DPP access needs after a vector
// instruction that wrote x (2) or the execution mask (5): the compiler cannot see into the
// block.  To be used where all 64 lanes are active.
__device__ __forceinline__ double row_dot16(const double (&row)[16], double x)
{
    double y0 = 0.0, y1 = 0.0;
#define BTARD_BC(k) " row_newbcast:" #k " row_mask:0xf bank_mask:0xf\n"
    asm("s_nop 4\n"
        "v_fmac_f64_dpp %0, %2, %3" BTARD_BC(0)
        "v_fmac_f64_dpp %1, %2, %4" BTARD_BC(1)
        "v_fmac_f64_dpp %0, %2, %5" BTARD_BC(2)
        "v_fmac_f64_dpp %1, %2, %6" BTARD_BC(3)
        "v_fmac_f64_dpp %0, %2, %7" BTARD_BC(4)
        "v_fmac_f64_dpp %1, %2, %8" BTARD_BC(5)
        "v_fmac_f64_dpp %0, %2, %9" BTARD_BC(6)
        "v_fmac_f64_dpp %1, %2, %10" BTARD_BC(7)
        "v_fmac_f64_dpp %0, %2, %11" BTARD_BC(8)
        "v_fmac_f64_dpp %1, %2, %12" BTARD_BC(9)
        "v_fmac_f64_dpp %0, %2, %13" BTARD_BC(10)
        "v_fmac_f64_dpp %1, %2, %14" BTARD_BC(11)
        "v_fmac_f64_dpp %0, %2, %15" BTARD_BC(12)
        "v_fmac_f64_dpp %1, %2, %16" BTARD_BC(13)
        "v_fmac_f64_dpp %0, %2, %17" BTARD_BC(14)
        "v_fmac_f64_dpp %1, %2, %18" BTARD_BC(15)
        : "+v"(y0), "+v"(y1)
        : "v"(x), "v"(row[0]), "v"(row[1]), "v"(row[2]), "v"(row[3]), "v"(row[4]), "v"(row[5]),
          "v"(row[6]), "v"(row[7]), "v"(row[8]), "v"(row[9]), "v"(row[10]), "v"(row[11]),
          "v"(row[12]), "v"(row[13]), "v"(row[14]), "v"(row[15]));
#undef BTARD_BC
    return y0 + y1;
}

// 1 / sqrt(x) for finite x > 0 to within a few units in the last place: the hardware
// estimate and two Newton steps (a dozen dependent instructions where a square root
// followed by a division takes several times as many; the iteration is a chain of
// dependent instructions in a single wavefront).
__device__ __forceinline__ double rsqrt_newton(double x)
{
    double r = __builtin_amdgcn_rsq(x);
#pragma unroll
    for (int s = 0; s < 2; ++s) {
        const double e = fma(-x * r, 0.5 * r, 0.5);      // (1 - x r^2) / 2
        r = fma(r, e, r);
    }
    return r;
}

// sum_k row[k] * (value of x in lane k)
template <int N>
__device__ __forceinline__ double row_dot(const double (&row)[N], double x)
{
    if constexpr (N == 16) {
        // (the peers are replicated in the four rows of 16 lanes)
        return row_dot16(row, x);
    } else {
        double y = 0.0;
#pragma unroll
        for (int k = 0; k < N; ++k) y = fma(row[k], lane_value_at(x, k), y);
        return y;
    }
}

// Sum over all 64 lanes (one peer per lane): DPP within the rows of 16, then the four row
// sums by v_readlane.
__device__ __forceinline__ double wave_sum64(double x)
{
    x += row_shift_right<0x111>(x);
    x += row_shift_right<0x112>(x);
    x += row_shift_right<0x114>(x);
    x += row_shift_right<0x118>(x);
    return (lane_value<15>(x) + lane_value<31>(x)) + (lane_value<47>(x) + lane_value<63>(x));
}

// The reductions of the iteration for either lane layout: N = 16 (peers replicated in the
// four rows of 16 lanes, row q reduces quantity q) or N = 64 (one peer per lane).
template <int N>
__device__ __forceinline__ void peers_sum2(int q, double a0, double a1, double &s0, double &s1)
{
    if constexpr (N == 16) {
        row_sum16x2(q, a0, a1, s0, s1);
    } else {
        s0 = wave_sum64(a0);
        s1 = wave_sum64(a1);
    }
}

template <int N>
__device__ __forceinline__ void peers_sum4(int q, double a0, double a1, double a2, double a3,
                                           double &s0, double &s1, double &s2, double &s3)
{
    if constexpr (N == 16) {
        row_sum16x4(q, a0, a1, a2, a3, s0, s1, s2, s3);
    } else {
        s0 = wave_sum64(a0);
        s1 = wave_sum64(a1);
        s2 = wave_sum64(a2);
        s3 = wave_sum64(a3);
    }
}

// One workgroup per partition: the whole iteration of eq. (CenteredClip) on the Gram
// matrix.  Starts from state buffer 0 (c^0 = 1/n) and leaves in state buffer 0 either the
// final state (done = 1) or the state at which the streaming passes must take over.
// After the workgroup has summed the partial matrices, one wavefront runs the iteration
// in registers: lane i (mod 16) owns peer i and row i of Gamma; the scalars every peer
// needs travel by v_readlane broadcasts and DPP row shifts, with no LDS and no barriers.
// N = 16: the layout above (peers replicated in the four rows of 16 lanes); N = 64 (n <= 64):
// lane i owns peer i and the partial matrices come in the block-pair layout of
// gram_pass_wide_kernel.
template <int N>
__global__ __launch_bounds__(kBlock) void gram_iterate_kernel(GramIterArgs a)
{
    static_assert(N == 16 || N == 64, "one 16 x 16 block or 4 x 4 of them");
    __shared__ double G[N][N + 1];
    // (the radii of a tau_l schedule, read once: a load from memory in every iteration would
    // put its latency into the chain of dependent instructions)
    __shared__ double s_tau[kMaxSchedule];
    const int j = blockIdx.x;
    const int t = threadIdx.x;
    const int n = a.n, R = a.st.R;
    if (a.st.has_sched) {                                    // uniform
        const int count = a.max_iters < kMaxSchedule ? a.max_iters : kMaxSchedule;
        for (int e = t; e < count; e += kBlock) s_tau[e] = a.st.tau_sched[e];
    }

    // Gamma = sum of the workgroups' partial matrices, in order
    if constexpr (N == 16) {
        const double *pj = a.gpart + (int64_t)j * a.blocks * kGramEntries;
        // (32 loads in flight at a time, added in order: otherwise the sum is a chain of
        // memory latencies)
        double s = 0.0;
        int b = 0;
        for (; b + 32 <= a.blocks; b += 32) {
            double x[32];
#pragma unroll
            for (int k = 0; k < 32; ++k) x[k] = pj[(int64_t)(b + k) * kGramEntries + t];
#pragma unroll
            for (int k = 0; k < 32; ++k) s += x[k];
        }
#pragma unroll 8
        for (; b < a.blocks; ++b) s += pj[(int64_t)b * kGramEntries + t];
        G[t / N][t % N] = s;
    } else {
        const double *pj = a.gpart + (int64_t)j * a.blocks * kWideEntries;
        // (four entries per thread at a time, so that 16 loads are in flight, each entry's
        // partial sums added in order)
        for (int e0 = t; e0 < N * N; e0 += 4 * kBlock) {
            int src[4];
            bool stored[4];
            double s[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = e0 + q * kBlock;
                const int I = e / N, K = e % N;
                const int bI = I >> 4, bK = K >> 4;
                stored[q] = bI < a.nb && bK < a.nb;
                // stored on and above the diagonal of blocks; below it, the transpose
                src[q] = !stored[q] ? 0
                         : (bI <= bK) ? wide_pair(bI, bK) * kGramEntries + (I & 15) * 16 + (K & 15)
                                      : wide_pair(bK, bI) * kGramEntries + (K & 15) * 16 + (I & 15);
                s[q] = 0.0;
            }
#pragma unroll 4
            for (int b = 0; b < a.blocks; ++b) {
#pragma unroll
                for (int q = 0; q < 4; ++q) s[q] += pj[(int64_t)b * kWideEntries + src[q]];
            }
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int e = e0 + q * kBlock;
                G[e / N][e % N] = stored[q] ? s[q] : 0.0;
            }
        }
    }
    __syncthreads();
    if (a.lambda > 0.0) {
        // Pre-clipping (App. E.3): the rows become alpha_i g_i with alpha_i =
        // min{1, lambda / ||g_i||} and ||g_i||^2 = Gamma_ii, so their Gram matrix is
        // D Gamma D -- no pass over the data.  The factors are left in st.scale for the
        // passes that follow.
        __shared__ double s_alpha[N];
        if (t < N) {
            const double Nn = sqrt(fmax(G[t][t], 0.0));
            const double al = (t < n && !(Nn <= a.lambda)) ? a.lambda / Nn : 1.0;
            s_alpha[t] = al;
            if (t < n) a.st.scale[(int64_t)j * R + t] = al;
        }
        __syncthreads();
        for (int e = t; e < N * N; e += kBlock) G[e / N][e % N] *= s_alpha[e / N] * s_alpha[e % N];
        __syncthreads();
    }
    if (t >= 64) return;

    const int i = (N == 16) ? (t & 15) : t;
    const bool peer = i < n;
    double row[N];
#pragma unroll
    for (int k = 0; k < N; ++k) row[k] = G[i][k];
    const double diag = G[i][i];
    const double rt = sqrt(fmax(diag, 0.0));
    const double inv_n = 1.0 / (double)n;

    const int q = t >> 4;                     // which of the four rows of 16 lanes
    double c = peer ? (a.fresh ? inv_n : a.st.coef[(int64_t)j * R + i]) : 0.0;
    double al = 0.0;
    int it = a.fresh ? 0 : a.st.iters[j];
    int dn = a.fresh ? 0 : a.st.done[j];
    // A row with an Inf or a NaN in it has a non-finite squared norm Gamma_ii (and only such
    // a row has: squares of fp32 values cannot overflow fp64), and then its residual norm
    // is not finite at any v: the partition is reported with iters = -1, as the
    // per-iteration passes do.  (The clamps at zero below would otherwise swallow a NaN:
    // fmax returns its other operand.)
    if (!dn && __any(peer && !isfinite(diag))) { it = -1; dn = 1; }
    double ev = 0.0;                          // bound on the error put into v so far

    // y = Gamma c, qv = c^T Gamma c and Sc = sum_i |c_i| ||g_i|| travel with c: after an
    // update a, y += Gamma a (the one matrix-vector product of an iteration), and the two
    // sums for the new c ride along in the reduction that gives the update's norm.
    double y = row_dot<N>(row, c);
    double qv, Sc;
    peers_sum2<N>(q, c * y, fabs(c) * rt, qv, Sc);

    // sqrt(kGramUnit), rounded up: error bar of a norm whose square is within its own error
    constexpr double kGramUnitRoot = 1.1920929e-7;
    while (!dn) {                             // wavefront-uniform
        // (tau_l of eq. (5) if the caller gave a schedule)
        const double tau = (a.st.has_sched && it < kMaxSchedule) ? s_tau[it] : a.tau;
        // norms, weights and how wrong the weights may be.  (Everything stays finite from
        // here on: Gamma is finite, the coefficients stay within the unit simplex's hull.)
        const double N2 = fmax(diag - 2.0 * y + qv, 0.0);
        const double eN2 = kGramUnit * (rt + Sc) * (rt + Sc);
        // ||g_i - v|| = N2 / sqrt(N2) and tau / ||g_i - v|| from one reciprocal square root
        const double rs = rsqrt_newton(N2);
        const double Nn = (N2 > 0.0) ? N2 * rs : 0.0;
        double w = 0.0, err_w = 0.0;
        if (peer) {
            w = (Nn <= tau) ? 1.0 : tau * rs;
            // a weight that is (or may be) tau/N inherits half the relative error of N^2;
            // its contribution to v is w * N <= tau
            if (N2 + eN2 > tau * tau) {
                // (error bars are bounds, rounded up by 1 %; 1 / N2 = rs^2)
                const double rel = (N2 > eN2) ? 0.505 * eN2 * (rs * rs) : 1.0;
                err_w = rel * fmin(Nn, tau) * inv_n;
            }
        }
        double W, E;
        peers_sum2<N>(q, w, err_w, W, E);
        const double ev_new = ev + E;
        // the update this would apply, and its squared norm a^T Gamma a
        const double an = peer ? (w - W * c) * inv_n : 0.0;
        const double u = row_dot<N>(row, an);
        const double cn = c + an;
        double yn = y + u;
        double Tn2, Sa, Scn, qvn;
        peers_sum4<N>(q, an * u, fabs(an) * rt, fabs(cn) * rt, cn * yn, Tn2, Sa, Scn, qvn);
        Tn2 = fmax(Tn2, 0.0);
        // error budget: the (generously bounded, never discounted) error put into v must
        // stay below 0.99e-8 ||v|| and below 1e-3 of the step itself (whose norm is compared
        // with eps below); compared in squares, which needs no square root
        if (ev_new * ev_new > fmin(0.98e-16 * fmax(qv, 0.0), 1e-6 * Tn2)) break;   // hand over before this update
        ev = ev_new;
        al = an;
        c = cn;
        it = it + 1;
        if ((it & 7) == 0) {
            // (y by running sums drifts by a rounding per update: recomputed now and then,
            // the drift stays a small fraction of the assumed accuracy kGramUnit)
            yn = row_dot<N>(row, c);
            peers_sum2<N>(q, c * yn, fabs(c) * rt, qvn, Scn);
        }
        y = yn;
        qv = qvn;
        Sc = Scn;
        if (it >= a.max_iters) dn = 1;
        // stopping rule on the update just applied, T = sqrt(Tn2) against eps, with its error
        // bar: eT bounds the error of T (from that of Tn2, eT2: eT2 / T where that is smaller
        // than sqrt(eT2); 1 / T from the hardware's estimate, rounded up by 1 %), and the plain
        // iteration's step may differ from this one by the error in v as well.  The comparisons
        // themselves are made in squares, on the exact Tn2.
        if (a.eps > 0.0) {
            const double eT2 = kGramUnit * Sa * Sa;
            const double eT = (Tn2 > eT2) ? 1.011 * eT2 * __builtin_amdgcn_rsq(Tn2)
                                          : 1.01 * kGramUnitRoot * Sa;
            const double band = eT + 2.0 * ev;
            const double below = a.eps - band, above = a.eps + band;
            if (below > 0.0 && Tn2 < below * below) dn = 1;          // certainly converged
            else if (!(Tn2 >= above * above)) break;                  // cannot tell: hand over
        }
    }
    // A partition that finished here: the norms at the final v and the norm of the last
    // update are in Gamma as well.  They are handed to the last pass (which then need not
    // form a single residual) only if their error bars are far inside the tolerances of
    // the verification quantities; otherwise the last pass measures them on the data.
    int ok = 0;
    double N2f = 0.0, T2f = 0.0;
    if (dn && it > 0) {
        const double yf = row_dot<N>(row, c);            // afresh, not the running sums
        const double uf = row_dot<N>(row, al);
        double qf, Sf, Tf, Sa;
        peers_sum4<N>(q, c * yf, fabs(c) * rt, al * uf, fabs(al) * rt, qf, Sf, Tf, Sa);
        N2f = fmax(diag - 2.0 * yf + qf, 0.0);
        const double eN2 = kGramUnit * (rt + Sf) * (rt + Sf);
        T2f = fmax(Tf, 0.0);
        const double eT2 = kGramUnit * Sa * Sa;
        bool bad = peer && !(eN2 <= kGramVouch * N2f);
        // These norms are those at the unrounded v = sum_i c_i g_i; what goes out, and what
        // the verification is of, is v rounded to fp32.  The rounding moves a norm by at
        // most 2^-24 ||v|| in absolute terms, which no tolerance here notices unless the
        // norm is tiny beside ||v||: ||g_i - v - er||^2 = ||g_i - v||^2 - 2 <g_i - v, er> +
        // ||er||^2, where the middle term has a standard deviation of 3.4e-8 ||g_i - v|| ||v||
        // / sqrt(d_j) if the rounding errors er are taken as independent of each other and of
        // the residual (uniform within half a unit in the last place), and the last one is
        // at most 2^-48 ||v||^2.  A partition is vouched for only if ten such deviations and
        // the last term are each below 1e-6 of every squared norm's root, i.e.
        // ||g_i - v|| >= 0.34 ||v|| / sqrt(d_j) and >= 6e-5 ||v||; otherwise the last pass
        // measures its norms against the rounded v.  (qf = ||v||^2.)
        const double dj = (double)(a.st.off[j + 1] - a.st.off[j]);
        bad = bad || (peer && !(N2f * dj >= kGramRoundSpread * qf && N2f >= kGramRoundFloor * qf));
        ok = !__any(bad) && (eT2 <= kGramVouch * T2f || Sa == 0.0);
    }
    if (t < n) {                                  // (N = 16: lanes 0..15 hold peers 0..15)
        a.st.coef[(int64_t)j * R + t] = c;
        a.st.delta[(int64_t)j * R + t] = al;
        a.st.gram_n2[(int64_t)j * R + t] = N2f;
    }
    if (a.fresh) {
        // what cc_begin_kernel would have set and nothing above writes
        if (t < n && !(a.lambda > 0.0)) a.st.scale[(int64_t)j * R + t] = 1.0;
        if (t == 0) {
            a.st.scale[(int64_t)j * R + n] = 1.0;
            a.st.report_buf[j] = 0;
        }
    }
    if (t == 0) {
        a.st.coef[(int64_t)j * R + n] = 0.0;      // the start vector's slot
        a.st.delta[(int64_t)j * R + n] = 0.0;
        a.st.gram_n2[(int64_t)j * R + n] = 0.0;
        a.st.iters[j] = it;
        a.st.done[j] = dn;
        a.st.final_buf[j] = 0;
        a.st.remaining[j] = dn ? 0 : (a.max_iters > it ? a.max_iters - it : 0);
        a.st.gram_ok[j] = ok;
        a.st.gram_t2[j] = T2f;
    }
}

// Test hook: the reduced Gram matrix of partition j as the iteration kernel sees it.
__global__ void gram_debug_kernel(const double *gpart, int32_t blocks, double *out)
{
    const int j = blockIdx.x, t = threadIdx.x;
    const double *pj = gpart + (int64_t)j * blocks * kGramEntries;
    double s = 0.0;
    for (int b = 0; b < blocks; ++b) s += pj[(int64_t)b * kGramEntries + t];
    out[(int64_t)j * kGramEntries + t] = s;
}

// The same for the block-pair layout: the full symmetric 64 x 64 matrix of partition j.
__global__ void gram_debug_wide_kernel(const double *gpart, int32_t blocks, int32_t nb, double *out)
{
    constexpr int N = 16 * kWideBlocks;
    const int j = blockIdx.x;
    const double *pj = gpart + (int64_t)j * blocks * kWideEntries;
    for (int e = threadIdx.x; e < N * N; e += blockDim.x) {
        const int I = e / N, K = e % N;
        const int bI = I >> 4, bK = K >> 4;
        double s = 0.0;
        if (bI < nb && bK < nb) {
            const int src = (bI <= bK) ? wide_pair(bI, bK) * kGramEntries + (I & 15) * 16 + (K & 15)
                                       : wide_pair(bK, bI) * kGramEntries + (K & 15) * 16 + (I & 15);
            for (int b = 0; b < blocks; ++b) s += pj[(int64_t)b * kWideEntries + src];
        }
        out[(int64_t)j * N * N + e] = s;
    }
}

}  // namespace btard
