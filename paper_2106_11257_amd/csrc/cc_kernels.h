// CenteredClip kernels (App. D.2, eq. (CenteredClip)), coefficient form.
//
// The iterate is never stored between iterations.  Every update of
// eq. (CenteredClip) adds a linear combination of the residuals g_i - v^l to
// v^l, so v^l = c_0 v0 + sum_i c_i g_i for coefficients c^l that obey
//
//     a_i = (w_i - W c_i) / n,  a_0 = -W c_0 / n,  c^{l+1} = c^l + a,
//     w_i = min{1, tau/||g_i - v^l||},  W = sum_i w_i,
//
// (c^0 = 1/n without v0, else c_0 = 1 and the rest 0).  One iteration is then
// ONE pass over the n x d_j slab: recompute v^l[x] from the n values of
// coordinate x that are in registers anyway, accumulate ||g_i - v^l||^2 for
// every peer, and ||sum_i a_i g_i||^2 = ||v^l - v^{l-1}||^2 for the stopping
// rule.  The last workgroup of a partition to finish reduces the partial sums
// in a fixed order and advances the coefficients, so the host never
// synchronises inside the iteration.
#pragma once

#include "kernels_common.h"

namespace btard {

struct CcState {
    const int64_t *off;      // [P+1] partition offsets (device copy)
    double *coef;            // [P][R]  c_i, i < n; entry n = coefficient of v0
    double *delta;           // [P][R]  a_i of the last applied update
    double *partial;         // [P][B][R] per-workgroup partial sums (n norms^2, step^2)
    unsigned int *counter;   // [P] workgroups finished in the current pass
    int32_t *iters;          // [P] updates applied so far (-1: non-finite norm)
    int32_t *done;           // [P] partition stopped
    int32_t R;               // n + 1
};

struct CcArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    const float *v0;         // may be null
    double tau, eps;
    int32_t max_iters;
    CcState st;
};

// ---------------------------------------------------------------------------
// begin: upload offsets (through the kernel arguments), set c^0, clear state
// ---------------------------------------------------------------------------
constexpr int kOffChunk = 256;
struct OffChunk {
    int64_t v[kOffChunk];
};

__global__ void upload_offsets_kernel(int64_t *off, int32_t first, int32_t count, OffChunk chunk)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) off[first + t] = chunk.v[t];
}

__global__ void cc_init_kernel(CcState st, int32_t n, int32_t P, int32_t has_v0, int32_t max_iters)
{
    const int j = blockIdx.x;
    if (j >= P) return;
    for (int q = threadIdx.x; q < st.R; q += blockDim.x) {
        double c;
        if (has_v0) c = (q == n) ? 1.0 : 0.0;
        else        c = (q == n) ? 0.0 : 1.0 / (double)n;
        st.coef[(int64_t)j * st.R + q] = c;
        st.delta[(int64_t)j * st.R + q] = 0.0;
    }
    if (threadIdx.x == 0) {
        st.counter[j] = 0u;
        st.iters[j] = 0;
        st.done[j] = (max_iters <= 0) ? 1 : 0;
    }
}

// ---------------------------------------------------------------------------
// one iteration: S2 (norms) + S3 (weights) + S4 (update, in coefficients) + S5
// ---------------------------------------------------------------------------
template <int NP, int LG>
__global__ __launch_bounds__(kBlock) void cc_pass_kernel(CcArgs a)
{
    using G = Geo<NP, LG>;
    const int j = blockIdx.y;
    if (a.st.done[j]) return;                       // uniform: whole partition skipped

    const int n = a.n, R = a.st.R;
    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    const double *__restrict__ cj = a.st.coef + (int64_t)j * R;
    const double *__restrict__ dj = a.st.delta + (int64_t)j * R;
    double c[NP], dl[NP];
    const float *rp[NP];
    bool have[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = lg * NP + k;
        have[k] = i < n;
        c[k] = have[k] ? cj[i] : 0.0;
        dl[k] = have[k] ? dj[i] : 0.0;
        rp[k] = a.g + (int64_t)(have[k] ? i : 0) * a.ld;
    }
    const bool has_v0 = a.v0 != nullptr;
    const double cb = cj[n], db = dj[n];

    double acc[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) acc[k] = 0.0;
    double t2 = 0.0;

    const int64_t xa = tile_origin(lo);
    const int64_t units = (hi > lo) ? (hi - xa + G::kW - 1) / G::kW : 0;
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    for (int64_t u = (int64_t)blockIdx.x * kWaves + wave; u < units; u += stride) {
        const int64_t x0 = xa + u * G::kW + (int64_t)sub * kVec;
        const bool full = (x0 >= lo) && (x0 + kVec <= hi);
        float val[NP][4];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            if (have[k]) load_row4(rp[k], x0, lo, hi, full, val[k]);
            else { val[k][0] = val[k][1] = val[k][2] = val[k][3] = 0.0f; }
        }
        float base[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (has_v0) load_row4(a.v0, x0, lo, hi, full, base);

        // v^l[x] and (v^l - v^{l-1})[x] from this lane group's peers ...
        double vv[4] = {0.0, 0.0, 0.0, 0.0}, ss[4] = {0.0, 0.0, 0.0, 0.0};
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const double gd = (double)val[k][e];
                vv[e] = fma(c[k], gd, vv[e]);
                ss[e] = fma(dl[k], gd, ss[e]);
            }
        }
        // ... then over all peers, and the v0 term
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            vv[e] = sum_across_groups<G::kLanes>(vv[e]);
            ss[e] = sum_across_groups<G::kLanes>(ss[e]);
            vv[e] = fma(cb, (double)base[e], vv[e]);
            ss[e] = fma(db, (double)base[e], ss[e]);
        }
        // residual norms ||g_i - v^l||^2 (masked coordinates hold zeros everywhere)
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const double r = (double)val[k][e] - vv[e];
                acc[k] = fma(r, r, acc[k]);
            }
        }
        if (lg == 0) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
        }
    }

    // workgroup partial sums: lanes -> wavefront -> LDS -> one value per quantity
    __shared__ double sh[kWaves][G::kPeers + 1];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const double s = sum_within_group<G::kLanes>(acc[k]);
        if (sub == 0) sh[wave][lg * NP + k] = s;
    }
    {
        const double s = sum_within_group<G::kLanes>(t2);
        if (lane == 0) sh[wave][G::kPeers] = s;
    }
    __syncthreads();
    const int B = gridDim.x;
    double *__restrict__ pj = a.st.partial + (int64_t)j * B * R;
    if ((int)threadIdx.x < R) {
        const int q = threadIdx.x;
        const int src = (q == n) ? G::kPeers : q;
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w][src];
        pj[(int64_t)blockIdx.x * R + q] = s;
    }

    if (!last_block_of_partition(&a.st.counter[j], (unsigned)B)) return;

    // ---- control: fixed-order reduction, weights, coefficient update, stopping rule
    __shared__ double s_w[kBlock];
    __shared__ int s_bad;
    __shared__ int s_stop;
    const int q = threadIdx.x;
    if (q == 0) { s_bad = 0; s_stop = 0; }
    double tot = 0.0;
    if (q < R)
        for (int b = 0; b < B; ++b) tot += pj[(int64_t)b * R + q];
    __syncthreads();
    const int it = a.st.iters[j];
    if (q == n) {
        // tot = ||v^it - v^{it-1}||^2: did update number `it` already converge?
        if (it >= 1 && sqrt(tot) < a.eps) s_stop = 1;
    }
    double w = 0.0;
    if (q < n) {
        const double N = sqrt(tot);
        if (!isfinite(N)) s_bad = 1;
        w = (N <= a.tau) ? 1.0 : a.tau / N;
        s_w[q] = w;
    }
    __syncthreads();
    if (s_stop) {
        if (q == 0) { a.st.done[j] = 1; a.st.counter[j] = 0u; }
        return;
    }
    if (s_bad) {
        if (q == 0) { a.st.iters[j] = -1; a.st.done[j] = 1; a.st.counter[j] = 0u; }
        return;
    }
    double W = 0.0;
    for (int i = 0; i < n; ++i) W += s_w[i];
    if (q < R) {
        double *cw = a.st.coef + (int64_t)j * R;
        double *dw = a.st.delta + (int64_t)j * R;
        const double cq = cw[q];
        const double aq = ((q < n ? w : 0.0) - W * cq) / (double)n;
        dw[q] = aq;
        cw[q] = cq + aq;
    }
    if (q == 0) {
        a.st.iters[j] = it + 1;
        if (it + 1 >= a.max_iters) a.st.done[j] = 1;
        a.st.counter[j] = 0u;
    }
}

// ---------------------------------------------------------------------------
// finish: v = c_0 v0 + sum_i c_i g_i rounded to fp32, ||last update||, iters
// ---------------------------------------------------------------------------
struct CcFinishArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    const float *v0;
    float *v;
    int32_t *iters_out;
    double *step_norm_out;   // may be null
    CcState st;
};

template <int NP, int LG>
__global__ __launch_bounds__(kBlock) void cc_finish_kernel(CcFinishArgs a)
{
    using G = Geo<NP, LG>;
    const int j = blockIdx.y;
    const int n = a.n, R = a.st.R;
    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    const double *__restrict__ cj = a.st.coef + (int64_t)j * R;
    const double *__restrict__ dj = a.st.delta + (int64_t)j * R;
    double c[NP], dl[NP];
    const float *rp[NP];
    bool have[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = lg * NP + k;
        have[k] = i < n;
        c[k] = have[k] ? cj[i] : 0.0;
        dl[k] = have[k] ? dj[i] : 0.0;
        rp[k] = a.g + (int64_t)(have[k] ? i : 0) * a.ld;
    }
    const bool has_v0 = a.v0 != nullptr;
    const double cb = cj[n], db = dj[n];
    double t2 = 0.0;

    const int64_t xa = tile_origin(lo);
    const int64_t units = (hi > lo) ? (hi - xa + G::kW - 1) / G::kW : 0;
    const int64_t stride = (int64_t)gridDim.x * kWaves;
    for (int64_t u = (int64_t)blockIdx.x * kWaves + wave; u < units; u += stride) {
        const int64_t x0 = xa + u * G::kW + (int64_t)sub * kVec;
        const bool full = (x0 >= lo) && (x0 + kVec <= hi);
        double vv[4] = {0.0, 0.0, 0.0, 0.0}, ss[4] = {0.0, 0.0, 0.0, 0.0};
        float val[NP][4];
#pragma unroll
        for (int k = 0; k < NP; ++k) {
            if (have[k]) load_row4(rp[k], x0, lo, hi, full, val[k]);
            else { val[k][0] = val[k][1] = val[k][2] = val[k][3] = 0.0f; }
        }
        float base[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (has_v0) load_row4(a.v0, x0, lo, hi, full, base);
#pragma unroll
        for (int k = 0; k < NP; ++k) {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const double gd = (double)val[k][e];
                vv[e] = fma(c[k], gd, vv[e]);
                ss[e] = fma(dl[k], gd, ss[e]);
            }
        }
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            vv[e] = sum_across_groups<G::kLanes>(vv[e]);
            ss[e] = sum_across_groups<G::kLanes>(ss[e]);
            vv[e] = fma(cb, (double)base[e], vv[e]);
            ss[e] = fma(db, (double)base[e], ss[e]);
        }
        if (lg == 0) {
            if (full) {
                f32x4_u o;
                o.x = (float)vv[0]; o.y = (float)vv[1]; o.z = (float)vv[2]; o.w = (float)vv[3];
                *reinterpret_cast<f32x4_u *>(a.v + x0) = o;
            } else {
#pragma unroll
                for (int e = 0; e < kVec; ++e) {
                    const int64_t x = x0 + e;
                    if (x >= lo && x < hi) a.v[x] = (float)vv[e];
                }
            }
#pragma unroll
            for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
        }
    }

    __shared__ double sh[kWaves];
    {
        const double s = sum_within_group<G::kLanes>(t2);
        if (lane == 0) sh[wave] = s;
    }
    __syncthreads();
    const int B = gridDim.x;
    double *__restrict__ pj = a.st.partial + (int64_t)j * B * R;
    if (threadIdx.x == 0) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w];
        pj[blockIdx.x] = s;
    }
    if (!last_block_of_partition(&a.st.counter[j], (unsigned)B)) return;
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int b = 0; b < B; ++b) tot += pj[b];
        const int it = a.st.iters[j];
        a.iters_out[j] = it;
        if (a.step_norm_out) a.step_norm_out[j] = (it > 0) ? sqrt(tot) : 0.0;
        a.st.counter[j] = 0u;
    }
}

}  // namespace btard
