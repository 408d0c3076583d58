// The last pass of CenteredClip and the verification pass in one: the aggregate
// v = sum_i c_i g_i is rounded to fp32 and written, and in the same sweep the residuals
// against that rounded v give the norms, the projections onto zhat and |zhat|^2 (Alg. 6
// lines 6-12) -- what btard_cc_finish followed by btard_verify_projections compute with
// two reads of the slab, here with one.
#pragma once

#include "cc_kernels.h"
#include "verify_kernels.h"

namespace btard {

struct FusedArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    float *v;
    double tau, eps;
    int32_t max_iters;
    int32_t pass;            // number of passes that were enqueued
    int32_t prev_blocks;
    uint64_t seed;
    int32_t S;               // 2n + 2: n norms^2, n <zhat, r_i>, |zhat|^2, |last update|^2
    CcState st;
};

template <int NP, int LG, bool RAGGED>
__global__ __launch_bounds__(kBlock, 2) void cc_finish_verify_kernel(FusedArgs a)
{
    using G = Geo<NP, LG>;
    __shared__ double s_c[kBlock], s_a[kBlock], s_red[kBlock];
    __shared__ int s_flags[2];
    __shared__ double sh[kWaves][2 * G::kPeers + 2];

    const int j = blockIdx.y;
    const int n = a.n, S = a.S;
    int iters_now;
    if (a.st.done[j]) {
        const int buf = a.st.final_buf[j];
        if ((int)threadIdx.x < a.st.R) {
            s_c[threadIdx.x] = a.st.coef[((int64_t)buf * a.st.P + j) * a.st.R + threadIdx.x];
            s_a[threadIdx.x] = a.st.delta[((int64_t)buf * a.st.P + j) * a.st.R + threadIdx.x];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) a.st.report_buf[j] = buf;
        __syncthreads();
    } else {
        control_step(a.st, j, n, a.tau, a.eps, a.max_iters, a.pass, a.prev_blocks, false, s_c, s_a,
                     s_red, s_flags, &iters_now);
        if (blockIdx.x == 0 && threadIdx.x == 0) a.st.report_buf[j] = a.pass & 1;
    }

    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    double c[NP], dl[NP], cb, db;
    fetch_coefficients<NP, LG, RAGGED>(s_c, s_a, n, lg, c, dl, cb, db);
    double accN[NP], accR[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) { accN[k] = 0.0; accR[k] = 0.0; }
    double t2 = 0.0, z2 = 0.0;

    const TileRange tr = tile_range<G::kW>(lo, hi);
    for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
        const int64_t xu = tr.xa + u * G::kW;
        const bool interior = (xu >= lo) && (xu + G::kW <= hi);
        const int64_t x0 = xu + (int64_t)sub * kVec;
        float val[NP][4];
        load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, interior, val);
        const float base[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        double vv[4], ss[4];
        combine_rows<NP, LG, false>(val, base, c, dl, cb, db, vv, ss);

        // the aggregate as the caller will see it: rounded to fp32
        float vf[4];
#pragma unroll
        for (int e = 0; e < kVec; ++e) vf[e] = (float)vv[e];
        if (lg == 0) {
            if (interior) {
                f32x4_u o;
                o.x = vf[0]; o.y = vf[1]; o.z = vf[2]; o.w = vf[3];
                *reinterpret_cast<f32x4_u *>(a.v + x0) = o;
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const int64_t x = x0 + e;
                    if (x >= lo && x < hi) a.v[x] = vf[e];
                }
            }
#pragma unroll
            for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
        }

        float zf[4];
        zhat_block(a.seed, x0 >> 2, zf);
        double z[4], vd[4];
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            const int64_t x = x0 + e;
            z[e] = (interior || (x >= lo && x < hi)) ? (double)zf[e] : 0.0;
            vd[e] = (double)vf[e];
        }
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                forget(val[k][e]);
                const double r = (double)val[k][e] - vd[e];
                accN[k] = fma(r, r, accN[k]);
                accR[k] = fma(z[e], r, accR[k]);
            }
        }
        if (lg == 0) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) z2 = fma(z[e], z[e], z2);
        }
    }

    sum_within_group_all<G::kLanes, NP>(accN);
    sum_within_group_all<G::kLanes, NP>(accR);
    z2 = sum_within_group<G::kLanes>(z2);
    t2 = sum_within_group<G::kLanes>(t2);
    if (sub == 0) {
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            sh[wave][lg * NP + k] = accN[k];
            sh[wave][G::kPeers + lg * NP + k] = accR[k];
        }
    }
    if (lane == 0) {
        sh[wave][2 * G::kPeers] = z2;
        sh[wave][2 * G::kPeers + 1] = t2;
    }
    __syncthreads();
    const int B = gridDim.x;
    // buffer (pass & 1) is free: what the earlier passes stored there has been consumed
    double *__restrict__ pb =
        a.st.partial + (a.pass & 1) * a.st.partial_stride + ((int64_t)j * B + blockIdx.x) * S;
    for (int q = threadIdx.x; q < S; q += kBlock) {
        int src;
        if (q < n) src = q;
        else if (q < 2 * n) src = G::kPeers + (q - n);
        else src = 2 * G::kPeers + (q - 2 * n);
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w][src];
        pb[q] = s;
    }
}

// iters and ||last applied update|| after cc_finish_verify_kernel
struct FusedReportArgs {
    CcState st;
    const double *partial;   // [P][blocks][S]
    int32_t blocks, S, index;
    int32_t *iters_out;
    double *step_norm_out;   // may be null
};

__global__ __launch_bounds__(kBlock) void fused_report_kernel(FusedReportArgs a)
{
    __shared__ double s_red[kBlock];
    const int j = blockIdx.x;
    const double *pj = a.partial + (int64_t)j * a.blocks * a.S + a.index;
    const double tot = reduce_partials<kBlock>(pj, a.blocks, a.S, 1, s_red);
    if (threadIdx.x == 0) {
        const int it = a.st.iters[a.st.report_buf[j] * a.st.P + j];
        a.iters_out[j] = it;
        if (a.step_norm_out) a.step_norm_out[j] = (it > 0) ? sqrt(tot) : 0.0;
    }
}

}  // namespace btard
