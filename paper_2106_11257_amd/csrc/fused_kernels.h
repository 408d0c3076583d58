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
    int32_t use_gram_norms;  // partitions with gram_ok set take the light body (project_partition)
    int32_t scaled;          // rows are taken times st.scale (pre-clipping)
    uint32_t epoch_mult;     // write bursts of v: 2^32 / ticks per epoch (0: the default)
    CcState st;
};

// The arithmetic of one tile whose rows are in registers (val).  INTERIOR (the whole tile
// lies inside the partition, a wavefront-uniform fact) selects a body with a vector store
// and no masks; the other body guards every coordinate.
template <int NP, int LG, bool INTERIOR, bool SCALED>
__device__ __forceinline__ void fused_rows(float *__restrict__ v, uint64_t seed, int lg, int sub,
                                           int64_t xu, int64_t lo, int64_t hi, float (&val)[NP][4],
                                           const double (&c)[NP], const double (&dl)[NP],
                                           const double (&al)[NP],
                                           double (&accN)[NP], double (&accR)[NP], double &t2,
                                           double &z2, TileStage *stage = nullptr, int64_t u_tile = 0)
{
    const int64_t x0 = xu + (int64_t)sub * kVec;
    // nothing below moves ahead of loads issued before this call (the next tile's)
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) forget(val[k][e]);
    }
    const float base[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    double vv[4], ss[4];
    combine_rows<NP, LG, false>(val, base, c, dl, 0.0, 0.0, vv, ss);

    // the aggregate as the caller will see it: rounded to fp32
    float vf[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) vf[e] = (float)vv[e];
    if (lg == 0) {
        if (INTERIOR) {
            f32x4_u o;
            o.x = vf[0]; o.y = vf[1]; o.z = vf[2]; o.w = vf[3];
            if (stage) stage->template put<64>(u_tile, sub, o);   // (one lane group when staged)
            else stream_store(v + x0, o);
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const int64_t x = x0 + e;
                if (x >= lo && x < hi) v[x] = vf[e];
            }
        }
#pragma unroll
        for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
    }

    float zf[4];
    zhat_block(seed, x0 >> 2, zf);
    double z[4], vd[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const int64_t x = x0 + e;
        z[e] = (INTERIOR || (x >= lo && x < hi)) ? (double)zf[e] : 0.0;
        vd[e] = (double)vf[e];
    }
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            forget(val[k][e]);   // converted again here instead of kept as 2x the registers
            double r;
            if constexpr (SCALED) r = fma(al[k], (double)val[k][e], -vd[e]);
            else r = (double)val[k][e] - vd[e];
            accN[k] = fma(r, r, accN[k]);
            accR[k] = fma(z[e], r, accR[k]);
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) z2 = fma(z[e], z[e], z2);
    }
}

// ---------------------------------------------------------------------------
// The last pass for partitions the Gram iteration finished and vouches for (gram_ok): the
// norms ||g_i - v|| and the last step norm are already known from the Gram matrix, so one
// sweep over the tile gives everything else: v = sum_i c_i g_i (rounded to fp32, written)
// and, with the same converted values, <zhat, g_i>; <zhat, v> is taken on the rounded v.
// The workgroup's partial sums go out in the layout of the general body of
// cc_finish_verify_kernel (<zhat, r_i> = <zhat, g_i> - <zhat, v>; workgroup 0 supplies the
// known norms), so the kernel that follows does not care which of the two ran.
// ---------------------------------------------------------------------------
template <int NP, int LG, bool INTERIOR>
__device__ __forceinline__ void project_rows(float *__restrict__ v, uint64_t seed, int lg, int sub,
                                             int64_t xu, int64_t lo, int64_t hi,
                                             float (&val)[NP][4], const double (&c)[NP],
                                             double (&accR)[NP], double &zv, double &z2,
                                             TileStage *stage = nullptr, int64_t u_tile = 0)
{
    const int64_t x0 = xu + (int64_t)sub * kVec;
    float zf[4];
    zhat_block(seed, x0 >> 2, zf);          // needs no data: runs while the loads travel
    double z[4], vv[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        const int64_t x = x0 + e;
        z[e] = (INTERIOR || (x >= lo && x < hi)) ? (double)zf[e] : 0.0;
        vv[e] = 0.0;
    }
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            forget(val[k][e]);              // nothing here moves ahead of the next tile's loads
            const double gd = (double)val[k][e];
            vv[e] = fma(c[k], gd, vv[e]);
            accR[k] = fma(z[e], gd, accR[k]);
        }
    }
    float vf[4];
#pragma unroll
    for (int e = 0; e < kVec; ++e) {
        vv[e] = sum_across_groups<Geo<NP, LG>::kLanes>(vv[e]);   // (nothing to do with one group)
        vf[e] = (float)vv[e];
    }
    if (INTERIOR && stage) {
        // (every lane holds the sums; those of lane group 0 keep them for the burst)
        f32x4_u o;
        o.x = vf[0]; o.y = vf[1]; o.z = vf[2]; o.w = vf[3];
        stage->template put<Geo<NP, LG>::kLanes>(u_tile, sub, o, lg == 0);
    }
    if (lg == 0) {
        if (INTERIOR) {
            if (!stage) {
                f32x4_u o;
                o.x = vf[0]; o.y = vf[1]; o.z = vf[2]; o.w = vf[3];
                stream_store(v + x0, o);
            }
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const int64_t x = x0 + e;
                if (x >= lo && x < hi) v[x] = vf[e];
            }
        }
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            zv = fma(z[e], (double)vf[e], zv);
            z2 = fma(z[e], z[e], z2);
        }
    }
}

template <int NP, int LG, bool RAGGED>
__device__ __forceinline__ void project_partition(const FusedArgs &a, int j, double *s_c,
                                                  double *s_a,
                                                  double (&sh)[kWaves][2 * NP * LG + 2],
                                                  f32x4_u *stage_area)
{
    using G = Geo<NP, LG>;
    const int n = a.n, S = a.S, R = a.st.R;
    if ((int)threadIdx.x < R) {                      // final state: buffer 0
        // With pre-clipping v = sum_i c_i (alpha_i g_i): the factor joins the coefficient,
        // and <zhat, alpha_i g_i> = alpha_i <zhat, g_i> is applied to the sums at the end
        // (exact products here; the Gram iteration worked on the exactly scaled matrix).
        const double al = a.scaled ? a.st.scale[(int64_t)j * R + threadIdx.x] : 1.0;
        s_c[threadIdx.x] = a.st.coef[(int64_t)j * R + threadIdx.x] * al;
        s_a[threadIdx.x] = al;
    }
    if (blockIdx.x == 0 && threadIdx.x == 0) a.st.report_buf[j] = 0;
    __syncthreads();

    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    double c[NP], dl[NP], cb, db;
    fetch_coefficients<NP, LG, RAGGED>(s_c, s_a, n, lg, c, dl, cb, db);
    double accR[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) accR[k] = 0.0;
    double zv = 0.0, z2 = 0.0;

    // interior tiles, two register sets taking turns (see cc_finish_verify_kernel; one set
    // with several lane groups, whose coefficients take vector registers) ...
    const TileRange tr = tile_range<G::kW>(lo, hi);
    const InteriorWalk iw = interior_walk<G::kW>(tr, lo, hi);
    TileStage stage;
    stage.begin(stage_area, wave, a.v, tr.xa, tr.stride, a.epoch_mult);
    if constexpr (LG > 1) {
        for (int64_t u = iw.begin; u < iw.end; u += tr.stride) {
            stage.template flush_if_due<G::kLanes>(sub, 1, lg == 0);
            const int64_t xu = tr.xa + u * G::kW;
            float val[NP][4];
            load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, true, val);
            project_rows<NP, LG, true>(a.v, a.seed, lg, sub, xu, lo, hi, val, c, accR, zv, z2, &stage, u);
        }
    } else if (iw.begin < iw.end) {
        float va[NP][4], vb[NP][4];
        int64_t u = iw.begin;
        bool last_in_b = false;
        uint32_t lane_off = (uint32_t)sub * (uint32_t)(kVec * sizeof(float));
        load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u * G::kW, lane_off, va);
        for (;;) {
            stage.template flush_if_due<64>(lane, 2);        // (one tile until the next check, one after the loop)
            const int64_t u1 = u + tr.stride;
            if (u1 >= iw.end) break;                 // the last tile is in va
            load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u1 * G::kW, lane_off, vb);
            project_rows<NP, LG, true>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, va, c, accR, zv, z2, &stage, u);
            const int64_t u2 = u1 + tr.stride;
            if (u2 >= iw.end) {                      // the last tile is in vb
                u = u1;
                last_in_b = true;
                break;
            }
            stage.template flush_if_due<64>(lane, 2);
            load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u2 * G::kW, lane_off, va);
            project_rows<NP, LG, true>(a.v, a.seed, lg, sub, tr.xa + u1 * G::kW, lo, hi, vb, c, accR, zv, z2, &stage, u1);
            u = u2;
        }
        if (last_in_b)
            project_rows<NP, LG, true>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, vb, c, accR, zv, z2, &stage, u);
        else
            project_rows<NP, LG, true>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, va, c, accR, zv, z2, &stage, u);
    }
    stage.template flush<G::kLanes>(sub, lg == 0);
    // ... then the partition's first and last tile where they are not interior
#pragma unroll 1
    for (int t = 0; t < 2; ++t) {
        const int64_t u = (t == 0) ? 0 : tr.units - 1;
        if ((t == 1 && tr.units < 2) || !owns_tile(tr, u)) continue;
        const int64_t xu = tr.xa + u * G::kW;
        if (tile_is_interior<G::kW>(xu, lo, hi)) continue;
        float val[NP][4];
        load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, false, val);
        project_rows<NP, LG, false>(a.v, a.seed, lg, sub, xu, lo, hi, val, c, accR, zv, z2);
    }

    sum_within_group_all<G::kLanes, NP>(accR);
    zv = sum_within_group<G::kLanes>(zv);
    z2 = sum_within_group<G::kLanes>(z2);
    if (sub == 0) {
#pragma unroll
        for (int k = 0; k < NP; ++k) sh[wave][lg * NP + k] = accR[k];
    }
    if (lane == 0) {
        sh[wave][G::kPeers] = zv;
        sh[wave][G::kPeers + 1] = z2;
    }
    __syncthreads();
    const int B = gridDim.x;
    double *__restrict__ pb =
        a.st.partial + (a.pass & 1) * a.st.partial_stride + ((int64_t)j * B + blockIdx.x) * S;
    const bool first = blockIdx.x == 0;
    for (int q = threadIdx.x; q < S; q += kBlock) {
        double s = 0.0;
        if (q < n) {
            s = first ? a.st.gram_n2[(int64_t)j * R + q] : 0.0;
        } else if (q < 2 * n) {
            const double al = s_a[q - n];
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += al * sh[w][q - n] - sh[w][G::kPeers];
        } else if (q == 2 * n) {
#pragma unroll
            for (int w = 0; w < kWaves; ++w) s += sh[w][G::kPeers + 1];
        } else {
            s = first ? a.st.gram_t2[j] : 0.0;
        }
        pb[q] = s;
    }
}

// SCALED: with pre-clipping factors (general body; the light body folds them for free).
template <int NP, int LG, bool RAGGED, bool SCALED>
__global__ __launch_bounds__(kBlock, 2) void cc_finish_verify_kernel(FusedArgs a)
{
    using G = Geo<NP, LG>;
    __shared__ double s_c[kBlock], s_a[kBlock], s_red[kBlock];
    __shared__ int s_flags[2];
    __shared__ double sh[kWaves][2 * G::kPeers + 2];
    // (tiles of v parked before they are written in bursts)
    __shared__ f32x4_u s_stage[LG <= 4 ? kStageSlots : 1];

    const int j = blockIdx.y;
    const int n = a.n, S = a.S;
    if constexpr (LG <= 4) {
        // (the Gram formulation serves n <= 64: up to four lane groups)
        if (a.use_gram_norms && a.st.gram_ok[j]) {   // uniform
            project_partition<NP, LG, RAGGED>(a, j, s_c, s_a, sh, s_stage);
            return;
        }
    }
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
    double al[NP];
    if constexpr (SCALED) fold_scales<NP, LG, RAGGED>(a.st, j, n, lg, true, c, dl, al);
    double accN[NP], accR[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) { accN[k] = 0.0; accR[k] = 0.0; }
    double t2 = 0.0, z2 = 0.0;

    // Interior tiles first.  Two register sets take turns: the loads of the wavefront's
    // next tile are issued before the arithmetic of the current one, so that memory requests
    // are in flight all the time and not only while the wavefront waits; every tile's
    // arithmetic follows the next tile's loads on a straight path (no join in between), so
    // the wait before it is for the current tile only.
    // (With several lane groups the coefficients live in vector registers, with pre-clipping
    // the factors do, and a second register set does not fit: one set then.)
    const TileRange tr = tile_range<G::kW>(lo, hi);
    const InteriorWalk iw = interior_walk<G::kW>(tr, lo, hi);
    // (v is staged where the registers allow it: with 16 peers per lane this body has none
    // to spare for it)
    constexpr bool kStaged = LG == 1 && NP <= 8;
    TileStage stage;
    TileStage *const staged = kStaged ? &stage : nullptr;
    stage.begin(s_stage, wave, a.v, tr.xa, tr.stride, a.epoch_mult);
    if constexpr (LG > 1 || SCALED) {
        for (int64_t u = iw.begin; u < iw.end; u += tr.stride) {
            if constexpr (kStaged) stage.template flush_if_due<64>(lane, 1);
            const int64_t xu = tr.xa + u * G::kW;
            float val[NP][4];
            load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, true, val);
            fused_rows<NP, LG, true, SCALED>(a.v, a.seed, lg, sub, xu, lo, hi, val, c, dl, al, accN, accR, t2,
                                     z2, staged, u);
        }
    } else if (iw.begin < iw.end) {
        float va[NP][4], vb[NP][4];
        int64_t u = iw.begin;
        bool last_in_b = false;
        uint32_t lane_off = (uint32_t)sub * (uint32_t)(kVec * sizeof(float));
        load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u * G::kW, lane_off, va);
        for (;;) {
            if constexpr (kStaged) stage.template flush_if_due<64>(lane, 3);   // (two tiles per round, one after)
            const int64_t u1 = u + tr.stride;
            if (u1 >= iw.end) break;                 // the last tile is in va
            load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u1 * G::kW, lane_off, vb);
            fused_rows<NP, LG, true, SCALED>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, va, c, dl, al,
                                     accN, accR, t2, z2, staged, u);
            const int64_t u2 = u1 + tr.stride;
            if (u2 >= iw.end) {                      // the last tile is in vb
                u = u1;
                last_in_b = true;
                break;
            }
            load_tile_interior<NP, RAGGED>(a.g, a.ld, n, tr.xa + u2 * G::kW, lane_off, va);
            fused_rows<NP, LG, true, SCALED>(a.v, a.seed, lg, sub, tr.xa + u1 * G::kW, lo, hi, vb, c, dl, al,
                                     accN, accR, t2, z2, staged, u1);
            u = u2;
        }
        if (last_in_b)
            fused_rows<NP, LG, true, SCALED>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, vb, c, dl, al,
                                     accN, accR, t2, z2, staged, u);
        else
            fused_rows<NP, LG, true, SCALED>(a.v, a.seed, lg, sub, tr.xa + u * G::kW, lo, hi, va, c, dl, al,
                                     accN, accR, t2, z2, staged, u);
    }
    if constexpr (kStaged) stage.template flush<64>(lane);
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
    // ... then the at most two edge tiles of the partition (its first and its last), by the
    // wavefronts that own them, with the guarded body and accumulators of their own: the
    // main loop's are dead by now, so the guarded body costs the main loop no registers.
    {
        double eN[NP], eR[NP], et2 = 0.0, ez2 = 0.0;
#pragma unroll
        for (int k = 0; k < NP; ++k) { eN[k] = 0.0; eR[k] = 0.0; }
        bool any = false;   // wavefront-uniform
#pragma unroll 1
        for (int t = 0; t < 2; ++t) {
            const int64_t u = (t == 0) ? 0 : tr.units - 1;
            if ((t == 1 && tr.units < 2) || !owns_tile(tr, u)) continue;
            const int64_t xu = tr.xa + u * G::kW;
            if (tile_is_interior<G::kW>(xu, lo, hi)) continue;
            float val[NP][4];
            load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, false, val);
            fused_rows<NP, LG, false, SCALED>(a.v, a.seed, lg, sub, xu, lo, hi, val, c, dl, al, eN, eR, et2,
                                      ez2);
            any = true;
        }
        if (any) {
            sum_within_group_all<G::kLanes, NP>(eN);
            sum_within_group_all<G::kLanes, NP>(eR);
            ez2 = sum_within_group<G::kLanes>(ez2);
            et2 = sum_within_group<G::kLanes>(et2);
            if (sub == 0) {
#pragma unroll
                for (int k = 0; k < NP; ++k) {
                    sh[wave][lg * NP + k] += eN[k];
                    sh[wave][G::kPeers + lg * NP + k] += eR[k];
                }
            }
            if (lane == 0) {
                sh[wave][2 * G::kPeers] += ez2;
                sh[wave][2 * G::kPeers + 1] += et2;
            }
        }
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

}  // namespace btard
