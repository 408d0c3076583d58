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
};

// Gamma entry held by register r of lane `lane` in the 16x16x4 fp64 MFMA accumulator: row
// lane/16 + 4 r, column lane % 16 (checked against a plain matrix product by the tests; the
// matrix is symmetric, so which of the two is "row" is immaterial).
__device__ __forceinline__ int gram_entry(int lane, int r) { return ((lane >> 4) + 4 * r) * kGramPeers + (lane & 15); }

// Lane (p = lane % 16, q = lane / 16) reads peer p's row.  A tile is 256 coordinates = 16
// groups of 16; in group s the lane loads coordinates 16 s + 4 q .. + 3 (one 128-bit load)
// and feeds them, one at a time, to v_mfma_f64_16x16x4_f64 as BOTH operands: in MFMA k-slot
// q the 16 lanes that share q hold the 16 peers' values of one coordinate, which is what
// A (16 x 4) and B (4 x 16) of Gamma += X_tile X_tile^T look like.
__global__ __launch_bounds__(kBlock) void gram_pass_kernel(GramArgs a)
{
    constexpr int kW = 256;
    const int j = blockIdx.y;
    const int n = a.n;
    const int64_t lo = a.off[j], hi = a.off[j + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int p = lane & 15, q = lane >> 4;
    const bool have = p < n;
    global_f32 row = (global_f32)a.g + (int64_t)(have ? p : n - 1) * a.ld;

    f64x4 acc = {0.0, 0.0, 0.0, 0.0};
    const TileRange tr = tile_range<kW>(lo, hi);
    for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
        const int64_t xu = tr.xa + u * kW;
        const bool interior = (xu >= lo) && (xu + kW <= hi);     // wavefront-uniform
        float val[16][4];
        if (interior) {
            global_f32 p0 = row + xu + 4 * q;
#pragma unroll
            for (int s = 0; s < 16; ++s) {
                const f32x4_u t = *(global_f32x4)(p0 + 16 * s);
                val[s][0] = t.x; val[s][1] = t.y; val[s][2] = t.z; val[s][3] = t.w;
            }
        } else {
#pragma unroll
            for (int s = 0; s < 16; ++s) {
#pragma unroll
                for (int e = 0; e < 4; ++e) {
                    const int64_t x = xu + 16 * s + 4 * q + e;
                    val[s][e] = (x >= lo && x < hi) ? row[x] : 0.0f;
                }
            }
        }
#pragma unroll
        for (int s = 0; s < 16; ++s) {
#pragma unroll
            for (int e = 0; e < 4; ++e) {
                const double d = have ? (double)val[s][e] : 0.0;
                acc = __builtin_amdgcn_mfma_f64_16x16x4f64(d, d, acc, 0, 0, 0);
            }
        }
    }

    // workgroup partial: the 4 wavefronts' matrices added in order
    __shared__ double sh[kWaves][kGramEntries];
#pragma unroll
    for (int r = 0; r < 4; ++r) sh[wave][gram_entry(lane, r)] = acc[r];
    __syncthreads();
    const int t = threadIdx.x;
    double s = 0.0;
#pragma unroll
    for (int w = 0; w < kWaves; ++w) s += sh[w][t];
    a.gpart[((int64_t)j * gridDim.x + blockIdx.x) * kGramEntries + t] = s;
}

struct GramIterArgs {
    CcState st;
    const double *gpart;
    int32_t blocks;          // workgroups per partition of gram_pass_kernel
    int32_t n;
    double tau, eps;
    int32_t max_iters;
};

// Relative accuracy assumed for a Gram entry and for a quadratic form in it, in units of
// sum |x_k x_l|: 2^-46 (about 130 roundings; the accumulation per lane is a chain of a few
// hundred fused multiply-adds of exact products, the rest are short fixed-order sums).
constexpr double kGramUnit = 1.4210854715202004e-14;

// Sum over the 16 lanes of a row of the wavefront (every lane gets the total, in a
// fixed order).
__device__ __forceinline__ double row_sum16(double x)
{
#pragma unroll
    for (int m = 8; m >= 1; m >>= 1) x += __shfl_xor(x, m, 16);
    return x;
}

// One workgroup per partition: the whole iteration of eq. (CenteredClip) on the Gram
// matrix.  Starts from state buffer 0 (c^0 = 1/n) and leaves in state buffer 0 either the
// final state (done = 1) or the state at which the streaming passes must take over.
// After the workgroup has summed the partial matrices, one wavefront runs the iteration
// in registers: lane i (mod 16) owns peer i and row i of Gamma; the scalars every peer
// needs travel by lane broadcasts and 16-lane butterflies, with no LDS and no barriers.
__global__ __launch_bounds__(kBlock) void gram_iterate_kernel(GramIterArgs a)
{
    constexpr int N = kGramPeers;
    __shared__ double G[N][N + 1];
    const int j = blockIdx.x;
    const int t = threadIdx.x;
    const int n = a.n, R = a.st.R;

    {   // Gamma = sum of the workgroups' partial matrices, in order
        const double *pj = a.gpart + (int64_t)j * a.blocks * kGramEntries;
        double s = 0.0;
#pragma unroll 8
        for (int b = 0; b < a.blocks; ++b) s += pj[(int64_t)b * kGramEntries + t];
        G[t / N][t % N] = s;
    }
    __syncthreads();
    if (t >= 64) return;

    const int i = t & 15;
    const bool peer = i < n;
    double row[N];
#pragma unroll
    for (int k = 0; k < N; ++k) row[k] = G[i][k];
    const double diag = G[i][i];
    const double rt = sqrt(fmax(diag, 0.0));
    const double inv_n = 1.0 / (double)n;     // only used as a factor of error bounds

    double c = peer ? a.st.coef[(int64_t)j * R + i] : 0.0;
    double al = 0.0;
    int it = a.st.iters[j];
    int dn = a.st.done[j];
    double ev = 0.0;                          // bound on the error put into v so far

    while (!dn) {                             // wavefront-uniform
        double y = 0.0;
#pragma unroll
        for (int k = 0; k < N; ++k) y = fma(row[k], __shfl(c, k, 16), y);
        const double qv = row_sum16(c * y);
        const double Sc = row_sum16(fabs(c) * rt);
        // norms, weights and how wrong the weights may be
        const double N2 = fmax(diag - 2.0 * y + qv, 0.0);
        const double eN2 = kGramUnit * (rt + Sc) * (rt + Sc);
        const double Nn = sqrt(N2);
        if (__any(peer && !isfinite(Nn))) { it = -1; dn = 1; break; }
        double w = 0.0, err_w = 0.0;
        if (peer) {
            w = (Nn <= a.tau) ? 1.0 : a.tau / Nn;
            // a weight that is (or may be) tau/N inherits half the relative error of N^2;
            // its contribution to v is w * N <= tau
            if (N2 + eN2 > a.tau * a.tau) {
                const double rel = (N2 > eN2) ? 0.5 * eN2 / N2 : 1.0;
                err_w = rel * fmin(Nn, a.tau) * inv_n;
            }
        }
        const double W = row_sum16(w);
        const double ev_new = ev + row_sum16(err_w);
        // the update this would apply, and its norm sqrt(a^T Gamma a)
        const double an = peer ? (w - W * c) / (double)n : 0.0;
        double u = 0.0;
#pragma unroll
        for (int k = 0; k < N; ++k) u = fma(row[k], __shfl(an, k, 16), u);
        const double Tn2 = row_sum16(an * u);
        const double Sa = row_sum16(fabs(an) * rt);
        const double T = sqrt(fmax(Tn2, 0.0));
        // error budget: the (generously bounded, never discounted) error put into v must
        // stay a small fraction of ||v|| and of the step itself (whose norm is compared
        // with eps below; the norm that is reported is recomputed from the data at the end)
        const double budget = fmin(1e-8 * sqrt(fmax(qv, 0.0)), 1e-3 * T);
        if (ev_new > budget) break;                               // hand over before this update
        ev = ev_new;
        al = an;
        c = c + an;
        it = it + 1;
        if (it >= a.max_iters) dn = 1;
        // stopping rule on the update just applied, with its error bar
        if (a.eps > 0.0) {
            const double eT2 = kGramUnit * Sa * Sa;
            const double eT = (T * T > eT2) ? eT2 / T : sqrt(eT2);
            // the plain iteration's step may differ from this one by the error in v as well
            const double band = eT + 2.0 * ev;
            if (T + band < a.eps) dn = 1;                         // certainly converged
            else if (!(T - band >= a.eps)) break;                 // cannot tell: hand over
        }
    }
    if (t < R) {
        a.st.coef[(int64_t)j * R + t] = (t < n) ? c : 0.0;
        a.st.delta[(int64_t)j * R + t] = (t < n) ? al : 0.0;
    }
    if (t == 0) {
        a.st.iters[j] = it;
        a.st.done[j] = dn;
        a.st.final_buf[j] = 0;
        a.st.remaining[j] = dn ? 0 : (a.max_iters > it ? a.max_iters - it : 0);
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

}  // namespace btard
