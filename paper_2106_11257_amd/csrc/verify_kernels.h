// Verification kernels: norms, clip weights, projections onto the random unit
// direction z and (optionally) the clipped residuals Delta (Alg. 6 lines 6-12,
// eq. (2)).  z is generated in registers from the seed (Philox4x32-10 + Box-
// Muller) and never touches memory.
#pragma once

#include "kernels_common.h"

namespace btard {

// Philox4x32 with 10 rounds (Salmon et al., SC'11): counter (c0..c3), key (k0,k1).
__device__ __forceinline__ void philox4x32_10(uint32_t c0, uint32_t c1, uint32_t c2, uint32_t c3,
                                              uint32_t k0, uint32_t k1, uint32_t (&out)[4])
{
    constexpr uint32_t kMulA = 0xD2511F53u, kMulB = 0xCD9E8D57u;
    constexpr uint32_t kWeylA = 0x9E3779B9u, kWeylB = 0xBB67AE85u;
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        const uint32_t hiA = __umulhi(kMulA, c0), loA = kMulA * c0;
        const uint32_t hiB = __umulhi(kMulB, c2), loB = kMulB * c2;
        c0 = hiB ^ c1 ^ k0;
        c1 = loB;
        c2 = hiA ^ c3 ^ k1;
        c3 = loA;
        k0 += kWeylA;
        k1 += kWeylB;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

// The four un-normalised Gaussian coordinates 4q .. 4q+3 of zhat.
__device__ __forceinline__ void zhat_block(uint64_t seed, int64_t q, float (&z)[4])
{
    uint32_t u[4];
    philox4x32_10((uint32_t)((uint64_t)q & 0xFFFFFFFFull), (uint32_t)((uint64_t)q >> 32), 0u, 0u,
                  (uint32_t)(seed & 0xFFFFFFFFull), (uint32_t)(seed >> 32), u);
    constexpr float kScale = 1.0f / 8388608.0f;   // 2^-23
#pragma unroll
    for (int h = 0; h < 2; ++h) {
        // (u >> 9) + 1/2 has at most 24 significant bits: exact in fp32
        const float a = ((float)(u[2 * h] >> 9) + 0.5f) * kScale;
        const float b = ((float)(u[2 * h + 1] >> 9) + 0.5f) * kScale;
        const float rho = sqrtf(-2.0f * logf(a));
        float s, c;
        sincospif(2.0f * b, &s, &c);
        z[2 * h] = rho * c;
        z[2 * h + 1] = rho * s;
    }
}

static __global__ void zhat_debug_kernel(uint64_t seed, int64_t x_begin, int64_t count, float *out)
{
    const int64_t q0 = x_begin / 4;
    const int64_t nq = (x_begin + count + 3) / 4 - q0;
    for (int64_t t = (int64_t)blockIdx.x * blockDim.x + threadIdx.x; t < nq;
         t += (int64_t)gridDim.x * blockDim.x) {
        float z[4];
        zhat_block(seed, q0 + t, z);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            const int64_t x = 4 * (q0 + t) + e;
            if (x >= x_begin && x < x_begin + count) out[x - x_begin] = z[e];
        }
    }
}

struct VerifyArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    const float *v;
    uint64_t seed;
    const int64_t *off;      // [P+1] device copy
    double *partial;         // [P][B][S], S = 2n + 1: n norms^2, n <zhat, r_i>, |zhat|^2
    int32_t S;
    // SCALED kernels only: pre-clipping factors alpha_ij at scale[j * R + i] (BTARD-Clipped-SGD,
    // App. E.3): the residuals are those of the rows alpha_ij g_i[j]
    const double *scale;
    int32_t R;
};

// One tile of the verification pass; INTERIOR as in fused_tile: a straight-line body for
// tiles wholly inside the partition, a guarded one for its first and last tile.
template <int NP, int LG, bool RAGGED, bool INTERIOR, bool SCALED>
__device__ __forceinline__ void verify_tile(const float *__restrict__ g, int64_t ld, int n,
                                            const float *__restrict__ v, uint64_t seed, int lg,
                                            int sub, int64_t xu, int64_t lo, int64_t hi,
                                            const double (&al)[NP],
                                            double (&accN)[NP], double (&accR)[NP], double &z2)
{
    const int64_t x0 = xu + (int64_t)sub * kVec;               // a multiple of 4
    float val[NP][4];
    load_tile<NP, LG, RAGGED>(g, ld, n, lg, sub, xu, lo, hi, INTERIOR, val);
    float vf[4];
    if (INTERIOR) load_row4_vec(v + x0, vf);
    else load_row4_guarded(v, x0, lo, hi, vf);

    float zf[4];
    zhat_block(seed, x0 >> 2, zf);
    double z[4], vv[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const int64_t x = x0 + e;
        z[e] = (INTERIOR || (x >= lo && x < hi)) ? (double)zf[e] : 0.0;
        vv[e] = (double)vf[e];
    }
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            double r;
            if constexpr (SCALED) r = fma(al[k], (double)val[k][e], -vv[e]);
            else r = (double)val[k][e] - vv[e];
            accN[k] = fma(r, r, accN[k]);
            accR[k] = fma(z[e], r, accR[k]);
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) z2 = fma(z[e], z[e], z2);
    }
}

// The arithmetic of an interior tile whose rows (val) and slice of v (vf) are already in
// registers.
template <int NP, int LG, bool SCALED>
__device__ __forceinline__ void verify_rows(uint64_t seed, int lg, int sub, int64_t xu,
                                            float (&val)[NP][4], float (&vf)[4],
                                            const double (&al)[NP],
                                            double (&accN)[NP], double (&accR)[NP], double &z2)
{
    const int64_t x0 = xu + (int64_t)sub * kVec;               // a multiple of 4
    float zf[4];
    zhat_block(seed, x0 >> 2, zf);
    double z[4], vv[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        z[e] = (double)zf[e];
        forget(vf[e]);           // no use of the tile moves ahead of the next tile's loads
        vv[e] = (double)vf[e];
    }
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            forget(val[k][e]);   // converted here, row by row; also keeps this after the loads
            double r;
            if constexpr (SCALED) r = fma(al[k], (double)val[k][e], -vv[e]);
            else r = (double)val[k][e] - vv[e];
            accN[k] = fma(r, r, accN[k]);
            accR[k] = fma(z[e], r, accR[k]);
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) z2 = fma(z[e], z[e], z2);
    }
}

// SCALED: on pre-clipped rows (the factors cost registers the plain variant does not pay for).
template <int NP, int LG, bool RAGGED, bool SCALED>
__global__ __launch_bounds__(kBlock, 2) void verify_pass_kernel(VerifyArgs a)
{
    using G = Geo<NP, LG>;
    __shared__ double sh[kWaves][2 * G::kPeers + 1];
    const int j = blockIdx.y;
    const int n = a.n, S = a.S;
    const int64_t lo = a.off[j], hi = a.off[j + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    double accN[NP], accR[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) { accN[k] = 0.0; accR[k] = 0.0; }
    double z2 = 0.0;
    double al[NP];
    if constexpr (SCALED) fetch_scale_factors<NP, LG, RAGGED>(a.scale + (int64_t)j * a.R, n, lg, al);

    // interior tiles first ...
    const TileRange tr = tile_range<G::kW>(lo, hi);
    // Two register sets take turns: the loads of the wavefront's next tile are issued
    // before the arithmetic of the current one, so that memory requests are in flight all
    // the time and not only while the wavefront waits.
    const InteriorWalk iw = interior_walk<G::kW>(tr, lo, hi);
    if constexpr (SCALED && LG > 1) {
        // (the factors live in vector registers here and a second register set does not fit)
        for (int64_t u = iw.begin; u < iw.end; u += tr.stride)
            verify_tile<NP, LG, RAGGED, true, SCALED>(a.g, a.ld, n, a.v, a.seed, lg, sub,
                                                      tr.xa + u * G::kW, lo, hi, al, accN, accR, z2);
    } else if (iw.begin < iw.end) {
        float va[NP][4], vb[NP][4], fa[4], fb[4];
        int64_t u = iw.begin;
        load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, tr.xa + u * G::kW, lo, hi, true, va);
        load_row4_vec(a.v + tr.xa + u * G::kW + sub * kVec, fa);
        // In the loop every tile's arithmetic follows the next tile's loads on a straight
        // path (no join in between), so the wait before it is for the current tile only.
        for (;;) {
            const int64_t u1 = u + tr.stride;
            if (u1 >= iw.end) break;                 // the last tile is in (va, fa)
            load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, tr.xa + u1 * G::kW, lo, hi, true, vb);
            load_row4_vec(a.v + tr.xa + u1 * G::kW + sub * kVec, fb);
            verify_rows<NP, LG, SCALED>(a.seed, lg, sub, tr.xa + u * G::kW, va, fa, al, accN, accR, z2);
            const int64_t u2 = u1 + tr.stride;
            if (u2 >= iw.end) {                      // the last tile is in (vb, fb): move it
#pragma unroll
                for (int k = 0; k < NP; ++k) {
#pragma unroll
                    for (int e = 0; e < kVec; ++e) va[k][e] = vb[k][e];
                }
#pragma unroll
                for (int e = 0; e < kVec; ++e) fa[e] = fb[e];
                u = u1;
                break;
            }
            load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, tr.xa + u2 * G::kW, lo, hi, true, va);
            load_row4_vec(a.v + tr.xa + u2 * G::kW + sub * kVec, fa);
            verify_rows<NP, LG, SCALED>(a.seed, lg, sub, tr.xa + u1 * G::kW, vb, fb, al, accN, accR, z2);
            u = u2;
        }
        verify_rows<NP, LG, SCALED>(a.seed, lg, sub, tr.xa + u * G::kW, va, fa, al, accN, accR, z2);
    }
    sum_within_group_all<G::kLanes, NP>(accN);
    sum_within_group_all<G::kLanes, NP>(accR);
    z2 = sum_within_group<G::kLanes>(z2);
    if (sub == 0) {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            sh[wave][lg * NP + k] = accN[k];
            sh[wave][G::kPeers + lg * NP + k] = accR[k];
        }
    }
    if (lane == 0) sh[wave][2 * G::kPeers] = z2;
    // ... then the partition's first and last tile where they are not interior, by the
    // wavefronts that own them, with accumulators of their own (see cc_finish_verify_kernel)
    {
        double eN[NP], eR[NP], ez2 = 0.0;
#pragma unroll
        for (int k = 0; k < NP; ++k) { eN[k] = 0.0; eR[k] = 0.0; }
        bool any = false;   // wavefront-uniform
#pragma unroll 1
        for (int t = 0; t < 2; ++t) {
            const int64_t u = (t == 0) ? 0 : tr.units - 1;
            if ((t == 1 && tr.units < 2) || !owns_tile(tr, u)) continue;
            const int64_t xu = tr.xa + u * G::kW;
            if (tile_is_interior<G::kW>(xu, lo, hi)) continue;
            verify_tile<NP, LG, RAGGED, false, SCALED>(a.g, a.ld, n, a.v, a.seed, lg, sub, xu, lo,
                                                       hi, al, eN, eR, ez2);
            any = true;
        }
        if (any) {
            sum_within_group_all<G::kLanes, NP>(eN);
            sum_within_group_all<G::kLanes, NP>(eR);
            ez2 = sum_within_group<G::kLanes>(ez2);
            if (sub == 0) {
#pragma unroll
                for (int k = 0; k < NP; ++k) {
                    sh[wave][lg * NP + k] += eN[k];
                    sh[wave][G::kPeers + lg * NP + k] += eR[k];
                }
            }
            if (lane == 0) sh[wave][2 * G::kPeers] += ez2;
        }
    }
    __syncthreads();
    const int B = gridDim.x;
    double *__restrict__ pb = a.partial + ((int64_t)j * B + blockIdx.x) * S;
    for (int q = threadIdx.x; q < S; q += kBlock) {
        int src;
        if (q < n) src = q;
        else if (q < 2 * n) src = G::kPeers + (q - n);
        else src = 2 * G::kPeers;
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w][src];
        pb[q] = s;
    }
}

struct VerifyFinishArgs {
    const double *partial;
    int32_t n, P, B, S;
    double tau;
    double *norms, *weights, *proj, *colsum;   // colsum may be null
    // after the fused last pass (S = 2n + 2) also: iters and ||last applied update||
    int32_t report;
    const int32_t *state_iters;                // [2][P]
    const int32_t *report_buf;                 // [P]
    int32_t *iters_out;
    double *step_norm_out;                     // may be null
};

// One workgroup per partition.  |zhat|^2 is summed over every partition's
// partial sums in a fixed order (each workgroup repeats that small sum).
constexpr int kFinishThreads = 1024;

static __global__ __launch_bounds__(kFinishThreads) void verify_finish_kernel(VerifyFinishArgs a)
{
    const int j = blockIdx.x;
    const int n = a.n, P = a.P, B = a.B, S = a.S;
    const int t = threadIdx.x;
    __shared__ double s_red[kFinishThreads];
    __shared__ double s_proj[256];
    // quantity q < n: norm^2 of peer q; n <= q < 2n: <zhat, r> of peer q - n
    // (with report: all S = 2n + 2 quantities, the last being ||last applied update||^2)
    // (this partition's loads are issued first and travel while |zhat|^2 is summed)
    const int Q = a.report ? S : 2 * n;
    const double mine = reduce_partials_load<kFinishThreads>(a.partial + (int64_t)j * B * S, B, S, Q);
    double zz = 0.0;
    for (int64_t e = t; e < (int64_t)P * B; e += kFinishThreads) zz += a.partial[e * S + 2 * n];
    s_red[t] = zz;
    __syncthreads();
    for (int h = kFinishThreads / 2; h > 0; h >>= 1) {
        if (t < h) s_red[t] += s_red[t + h];
        __syncthreads();
    }
    const double Z = sqrt(s_red[0]);

    const double tot = reduce_partials_combine<kFinishThreads>(mine, Q, s_red);
    __syncthreads();
    if (t < Q) s_red[t] = tot;
    __syncthreads();
    if (a.report && t == 0) {
        const int it = a.state_iters[a.report_buf[j] * P + j];
        a.iters_out[j] = it;
        if (a.step_norm_out) a.step_norm_out[j] = (it > 0) ? sqrt(s_red[2 * n + 1]) : 0.0;
    }
    if (t < n) {
        const double N = sqrt(s_red[t]);
        const double Rr = s_red[n + t];
        const double w = (N <= a.tau) ? 1.0 : a.tau / N;
        const double s = (Z > 0.0) ? w * Rr / Z : 0.0;
        a.norms[(int64_t)t * P + j] = N;
        a.weights[(int64_t)t * P + j] = w;
        a.proj[(int64_t)t * P + j] = s;
        s_proj[t] = s;
    }
    __syncthreads();
    if (t == 0 && a.colsum) {
        double cs = 0.0;
        for (int i = 0; i < n; ++i) cs += s_proj[i];
        a.colsum[j] = cs;
    }
}

struct DeltaArgs {
    const float *g;
    int64_t ld;
    int32_t n, P;
    const float *v;
    const int64_t *off;
    const double *weights;   // [n][P]
    float *delta;
    int64_t ldd;
    const double *scale;     // pre-clipping factors at scale[j * R + i], or null: the rows as given
    int32_t R;
};

// Delta_i^j = w_ij (g_i[j] - v[j]) (of the rows alpha_ij g_i[j] if factors are given), one
// pass: read n + 1 rows, write n rows.
static __global__ __launch_bounds__(kBlock) void delta_kernel(DeltaArgs a)
{
    const int j = blockIdx.y;
    const int64_t lo = a.off[j], hi = a.off[j + 1];
    const int64_t xa = tile_origin<kVec>(lo);
    const int64_t units = (hi > lo) ? (hi - xa + kVec - 1) / kVec : 0;
    for (int64_t u = (int64_t)blockIdx.x * kBlock + threadIdx.x; u < units;
         u += (int64_t)gridDim.x * kBlock) {
        const int64_t x0 = xa + u * kVec;
        const bool full = (x0 >= lo) && (x0 + kVec <= hi);
        float vf[4];
        if (full) load_row4_vec(a.v + x0, vf);
        else load_row4_guarded(a.v, x0, lo, hi, vf);
        for (int i = 0; i < a.n; ++i) {
            const double w = a.weights[(int64_t)i * a.P + j];
            const double al = a.scale ? a.scale[(int64_t)j * a.R + i] : 1.0;
            float gv[4];
            if (full) load_row4_vec(a.g + (int64_t)i * a.ld + x0, gv);
            else load_row4_guarded(a.g + (int64_t)i * a.ld, x0, lo, hi, gv);
            float o[4];
#pragma unroll
            for (int e = 0; e < kVec; ++e) o[e] = (float)(w * fma(al, (double)gv[e], -(double)vf[e]));
            float *dst = a.delta + (int64_t)i * a.ldd;
            if (full) {
                f32x4_u t;
                t.x = o[0]; t.y = o[1]; t.z = o[2]; t.w = o[3];
                *reinterpret_cast<f32x4_u *>(dst + x0) = t;
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const int64_t x = x0 + e;
                    if (x >= lo && x < hi) dst[x] = o[e];
                }
            }
        }
    }
}

}  // namespace btard
