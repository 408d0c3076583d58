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
// rule; each workgroup stores its partial sums.
//
// The scalar work between two passes (fixed-order reduction of the partial
// sums, weights, coefficient update, stopping rule: "the control step") is done
// at the START of the next kernel by every workgroup of the partition, each for
// itself, from the previous pass's partial sums: all of them execute the same
// instructions on the same data and so reach the same coefficients and the same
// decision.  That needs no atomics, no device-wide fences and no extra launch;
// the kernel boundary makes the partial sums visible.  State and partial sums
// are double-buffered by pass parity, so a workgroup that is still reading
// pass l-1's results is never overtaken by one that already stores pass l's.
#pragma once

#include "kernels_common.h"

namespace btard {

struct CcState {
    const int64_t *off;      // [P+1] partition offsets (device copy)
    double *coef;            // [2][P][R]  c_i, i < n; entry n = coefficient of v0
    double *delta;           // [2][P][R]  a_i of the last applied update
    double *partial;         // [2][P*B*R] per-workgroup partial sums (n norms^2, step^2)
    int32_t *iters;          // [2][P] updates applied so far (-1: non-finite norm)
    int32_t *done;           // [P] partition stopped (set once, by workgroup 0 of the pass
                             //     that decides; later kernels skip the partition)
    int32_t *final_buf;      // [P] state buffer that holds a stopped partition's final state
    int32_t *report_buf;     // [P] state buffer the finish kernel left the reported state in
    int32_t *remaining;      // [P] iterations still to run after the Gram iteration
    int32_t *gram_ok;        // [P] the Gram iteration finished the partition AND vouches for
                             //     the final norms and the last step norm it left below
    double *gram_n2;         // [P][R] ||g_i - v||^2 at the final v, from the Gram matrix
    double *gram_t2;         // [P]    ||last applied update||^2, from the Gram matrix
    double *scale;           // [P][R] pre-clipping factors alpha_ij (1 unless pre-clipping)
    const double *tau_sched; // [kMaxSchedule] clipping radius of update l (only if has_sched)
    int32_t has_sched;
    int64_t partial_stride;  // doubles between the two partial-sum buffers
    int32_t R;               // n + 1
    int32_t P;
};

struct CcArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    const float *v0;         // may be null
    double tau, eps;
    int32_t max_iters;
    int32_t pass;            // index l of this pass (0-based)
    int32_t prev_blocks;     // workgroups per partition of the previous pass
    int32_t scaled;          // rows are taken times st.scale (pre-clipping)
    int32_t rule;            // kRuleCenteredClip or kRuleGeometricMedian
    CcState st;
};

// What the control step does with the norms (the passes are the same for both):
//   CenteredClip      w_i = min{1, tau / N_i},  c += (w - W c) / n       (eq. (CenteredClip))
//   geometric median  w_i = 1 / max(N_i, tau),  c  = w / W               (Weiszfeld's iteration
//                     for the minimiser of sum_i ||g_i - v||, the tau -> 0 end of CenteredClip
//                     and one of the baselines of Sec. 4.1; tau is the floor under the norms)
constexpr int kRuleCenteredClip = 0;
constexpr int kRuleGeometricMedian = 1;

// ---------------------------------------------------------------------------
// begin: upload offsets (through the kernel arguments), set c^0, clear state
// ---------------------------------------------------------------------------
constexpr int kMaxSchedule = 1024;   // longest per-iteration schedule of clipping radii
constexpr int kOffChunk = 256;
struct OffChunk {
    int64_t v[kOffChunk];
};

struct DblChunk {
    double v[kOffChunk];
};

static __global__ void upload_doubles_kernel(double *dst, int32_t first, int32_t count, DblChunk chunk)
{
    const int t = threadIdx.x;
    if (t < count) dst[first + t] = chunk.v[t];
}

static __global__ void upload_offsets_kernel(int64_t *off, int32_t first, int32_t count, OffChunk chunk)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < count) off[first + t] = chunk.v[t];
}

// One launch per chunk of offsets: workgroup b sets up partition first + b (if there is
// one: the last chunk entry may be the end offset only), workgroup 0 also stores the chunk.
// zero_start: all coefficients 0 (v^0 = 0), for the pass that measures the rows' own norms.
static __global__ __launch_bounds__(kOffChunk) void cc_begin_kernel(CcState st, int32_t n, int32_t has_v0,
                                                             int32_t max_iters, int32_t first,
                                                             int32_t count, int32_t zero_start,
                                                             OffChunk chunk)
{
    const int t = threadIdx.x;
    if (blockIdx.x == 0 && t < count) const_cast<int64_t *>(st.off)[first + t] = chunk.v[t];
    const int j = first + blockIdx.x;
    if (j >= st.P) return;
    for (int q = t; q < st.R; q += blockDim.x) {
        double c;
        if (has_v0) c = (q == n) ? 1.0 : 0.0;
        else        c = (q == n) ? 0.0 : 1.0 / (double)n;
        st.coef[(int64_t)j * st.R + q] = zero_start ? 0.0 : c;
        st.delta[(int64_t)j * st.R + q] = 0.0;
        st.scale[(int64_t)j * st.R + q] = 1.0;
    }
    if (t == 0) {
        st.iters[j] = 0;
        st.done[j] = (max_iters <= 0) ? 1 : 0;
        st.final_buf[j] = 0;
        st.report_buf[j] = 0;
        st.remaining[j] = max_iters > 0 ? max_iters : 0;
        st.gram_ok[j] = 0;
    }
}

// ---------------------------------------------------------------------------
// control step: weights, update in coefficients, stopping rule
// ---------------------------------------------------------------------------
// Brings partition j's state from "after pass-1" to "ready for pass `pass`": every thread
// of the workgroup takes part.  The partition must have been running when pass-1 ended (the
// callers skip stopped partitions before they get here).  On return s_c / s_a hold
// c^pass / a^pass (R entries), *iters_out the updates applied, and the function value is
// true if the partition stops now.  Workgroup 0 of the partition records the new state in
// buffer (pass & 1) and, with mark_done, publishes a stop in done / final_buf.  Other
// workgroups may see that flag while they are still starting the same pass; all they do
// with it is leave, which is what they would decide themselves.
__device__ __forceinline__ bool control_step(const CcState &st, int j, int n, double tau,
                                             double eps, int max_iters, int pass, int prev_blocks,
                                             bool mark_done, double *s_c, double *s_a,
                                             double *s_red, int *s_flags, int *iters_out,
                                             int rule = kRuleCenteredClip)
{
    const int R = st.R, P = st.P;
    const int t = threadIdx.x;
    if (pass == 0) {
        // state buffer 0 as set by cc_begin_kernel (or left by the Gram iteration)
        if (t < R) {
            s_c[t] = st.coef[(int64_t)j * R + t];
            s_a[t] = st.delta[(int64_t)j * R + t];
        }
        __syncthreads();
        *iters_out = st.iters[j];
        return false;
    }
    const int prev = (pass - 1) & 1, cur = pass & 1;
    const double *cp = st.coef + ((int64_t)prev * P + j) * R;
    const double *ap = st.delta + ((int64_t)prev * P + j) * R;
    double cq = 0.0, aq = 0.0;
    if (t < R) { cq = cp[t]; aq = ap[t]; }
    int it = st.iters[prev * P + j];
    int dn = 0;
    // update number `it` (0-based) is the one prepared here: tau_l of eq. (5) if scheduled
    if (st.has_sched && it >= 0 && it < kMaxSchedule) tau = st.tau_sched[it];

    const double *pj = st.partial + prev * st.partial_stride + (int64_t)j * prev_blocks * R;
    const double tot = reduce_partials<kBlock>(pj, prev_blocks, R, R, s_red);
    if (t == 0) { s_flags[0] = 0; s_flags[1] = 0; }
    __syncthreads();
    // quantity n is ||v^it - v^{it-1}||^2: did update number `it` already converge?
    if (t == n && it >= 1 && sqrt(tot) < eps) s_flags[0] = 1;
    double w = 0.0;
    if (t < n) {
        const double N = sqrt(tot);
        if (!isfinite(N)) s_flags[1] = 1;
        if (rule == kRuleGeometricMedian) w = 1.0 / fmax(N, tau);
        else w = (N <= tau) ? 1.0 : tau / N;
    }
    __syncthreads();
    s_red[t] = w;
    __syncthreads();
    if (s_flags[0]) {
        dn = 1;                                              // v^it is final; c, a unchanged
    } else if (s_flags[1]) {
        dn = 1; it = -1;
    } else {
        double W = 0.0;
        for (int i = 0; i < n; ++i) W += s_red[i];
        if (t < R) {
            if (rule == kRuleGeometricMedian) {
                const double cn = (t < n) ? w / W : 0.0;
                aq = cn - cq;
                cq = cn;
            } else {
                aq = ((t < n ? w : 0.0) - W * cq) / (double)n;
                cq = cq + aq;
            }
        }
        it = it + 1;
        if (it >= max_iters) dn = 1;
    }
    if (t < R) { s_c[t] = cq; s_a[t] = aq; }
    if (blockIdx.x == 0) {
        if (t < R) {
            st.coef[((int64_t)cur * P + j) * R + t] = cq;
            st.delta[((int64_t)cur * P + j) * R + t] = aq;
        }
        if (t == 0) {
            st.iters[cur * P + j] = it;
            if (dn && mark_done) { st.final_buf[j] = cur; st.done[j] = 1; }
        }
    }
    __syncthreads();
    *iters_out = it;
    return dn != 0;
}

// This lane group's coefficients out of LDS.
template <int NP, int LG, bool RAGGED>
__device__ __forceinline__ void fetch_coefficients(const double *s_c, const double *s_a, int n, int lg,
                                                   double (&c)[NP], double (&dl)[NP], double &cb,
                                                   double &db)
{
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = lg * NP + k;
        const bool have = !RAGGED || i < n;
        double ck = have ? s_c[have ? i : 0] : 0.0;
        double ak = have ? s_a[have ? i : 0] : 0.0;
        if (LG == 1) { ck = uniform_double(ck); ak = uniform_double(ak); }
        c[k] = ck;
        dl[k] = ak;
    }
    cb = uniform_double(s_c[n]);
    db = uniform_double(s_a[n]);
}

// Per tile: v^l[x] = c_0 v0[x] + sum_i c_i g_i[x] and u[x] = a_0 v0[x] + sum_i a_i g_i[x]
// (= (v^l - v^{l-1})[x]) for the lane's 4 coordinates, from the peers' values held in
// registers.  With several lane groups the per-group partial sums are combined by a
// butterfly over the groups.
template <int NP, int LG, bool HAS_BASE>
__device__ __forceinline__ void combine_rows(const float (&val)[NP][4], const float (&base)[4],
                                             const double (&c)[NP], const double (&dl)[NP],
                                             double cb, double db, double (&vv)[4], double (&ss)[4])
{
    using G = Geo<NP, LG>;
#pragma unroll
    for (int e = 0; e < kVec; ++e) { vv[e] = 0.0; ss[e] = 0.0; }
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
        if (HAS_BASE) {
            vv[e] = fma(cb, (double)base[e], vv[e]);
            ss[e] = fma(db, (double)base[e], ss[e]);
        }
    }
}

// Pre-clipping (BTARD-Clipped-SGD, App. E.3): row i of partition j counts as alpha_ij g_i.
// The factor costs no instruction: in v = sum_i c_i (alpha_i g_i) it joins the coefficient,
// and a residual alpha_i g - v is one fused multiply-add where it was one subtraction
// (with alpha = 1, the case without pre-clipping, that is the same number bit for bit).
// This fetches this lane group's factors (1 if `scaled` is false) and folds them into the
// coefficients c and dl.
template <int NP, int LG, bool RAGGED>
__device__ __forceinline__ void fold_scales(const CcState &st, int j, int n, int lg, bool scaled,
                                            double (&c)[NP], double (&dl)[NP], double (&al)[NP])
{
#pragma unroll
    for (int k = 0; k < NP; ++k) {
        const int i = lg * NP + k;
        const bool have = scaled && (!RAGGED || i < n);
        const double f = have ? st.scale[(int64_t)j * st.R + (have ? i : 0)] : 1.0;
        al[k] = f;                                  // (stays in vector registers)
        c[k] = (LG == 1) ? uniform_double(c[k] * f) : c[k] * f;
        dl[k] = (LG == 1) ? uniform_double(dl[k] * f) : dl[k] * f;
    }
}

// The tile at xu (interior or not) of this lane group's rows, and of the start vector.
template <int NP, int LG, bool RAGGED, bool HAS_BASE>
__device__ __forceinline__ void pass_load_any(const CcArgs &a, int n, int lg, int sub, int64_t xu,
                                              int64_t lo, int64_t hi, float (&val)[NP][4],
                                              float (&base)[4])
{
    constexpr int kW = Geo<NP, LG>::kW;
    const bool interior = (xu >= lo) && (xu + kW <= hi);   // wavefront-uniform
    load_tile<NP, LG, RAGGED>(a.g, a.ld, n, lg, sub, xu, lo, hi, interior, val);
    if (HAS_BASE) {
        const int64_t x0 = xu + (int64_t)sub * kVec;
        if (interior) load_row4_vec(a.v0 + x0, base);
        else load_row4_guarded(a.v0, x0, lo, hi, base);
    }
}

// The same for an interior tile with one lane group.
template <int NP, bool RAGGED, bool HAS_BASE>
__device__ __forceinline__ void pass_load_interior(const CcArgs &a, int n, int sub, int64_t xu,
                                                   uint32_t &lane_off, float (&val)[NP][4],
                                                   float (&base)[4])
{
    load_tile_interior<NP, RAGGED>(a.g, a.ld, n, xu, lane_off, val);
    if (HAS_BASE) load_row4_vec(a.v0 + xu + (int64_t)sub * kVec, base);
}

// One tile of a pass: v^l and the step direction on its 4 coordinates per lane, then the
// residual norms ||g_i - v^l||^2 (masked coordinates hold zeros in every row).
template <int NP, int LG, bool HAS_BASE, bool SCALED>
__device__ __forceinline__ void pass_tile_sums(float (&val)[NP][4], const float (&base)[4],
                                               const double (&c)[NP], const double (&dl)[NP],
                                               double cb, double db, const double (&al)[NP], int lg,
                                               double (&acc)[NP], double &t2)
{
    double vv[4], ss[4];
    combine_rows<NP, LG, HAS_BASE>(val, base, c, dl, cb, db, vv, ss);
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) {
            forget(val[k][e]);
            double r;
            if constexpr (SCALED) r = fma(al[k], (double)val[k][e], -vv[e]);
            else r = (double)val[k][e] - vv[e];
            acc[k] = fma(r, r, acc[k]);
        }
    }
    if (lg == 0) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
    }
}

// ---------------------------------------------------------------------------
// one iteration: control step for the previous pass, then norms at v^l
// ---------------------------------------------------------------------------
// SCALED: with pre-clipping factors (a variant of its own: the factors cost 32 registers that
// the plain pass does not pay for).
template <int NP, int LG, bool RAGGED, bool HAS_BASE, bool SCALED>
__global__ __launch_bounds__(kBlock, (LG == 1 && !SCALED && NP <= 8 ? 4 : 2)) void cc_pass_kernel(CcArgs a)
{
    using G = Geo<NP, LG>;
    // (one lane group, no factors: the registers allow a second set of tile values)
    constexpr bool kTwoSets = LG == 1 && !SCALED;
    __shared__ double s_c[kBlock], s_a[kBlock], s_red[kBlock];
    __shared__ int s_flags[2];
    __shared__ double sh[kWaves][G::kPeers + 1];

    const int j = blockIdx.y;
    const int stopped = a.st.done[j];               // the three loads travel together
    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    if (stopped) return;                            // stopped in an earlier kernel (uniform)
    const int n = a.n, R = a.st.R;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;
    const TileRange tr = tile_range<G::kW>(lo, hi);

    // (interior tiles, one lane group: scalar row base + the lane's byte offset)
    uint32_t lane_off = (uint32_t)sub * (uint32_t)(kVec * sizeof(float));
    const InteriorWalk iw = interior_walk<G::kW>(tr, lo, hi);

    // The first tile's loads do not depend on the coefficients: they are issued before the
    // control step and travel while it runs.
    float va[NP][4];
    float base_a[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if constexpr (kTwoSets) {
        if (iw.begin < iw.end) pass_load_interior<NP, RAGGED, HAS_BASE>(a, n, sub, tr.xa + iw.begin * G::kW, lane_off, va, base_a);
    } else {
        if (tr.first < tr.units) pass_load_any<NP, LG, RAGGED, HAS_BASE>(a, n, lg, sub, tr.xa + tr.first * G::kW, lo, hi, va, base_a);
    }

    int iters_now;
    if (control_step(a.st, j, n, a.tau, a.eps, a.max_iters, a.pass, a.prev_blocks, true, s_c, s_a,
                     s_red, s_flags, &iters_now, a.rule))
        return;                                     // uniform: this partition stops now

    double c[NP], dl[NP], cb, db;
    fetch_coefficients<NP, LG, RAGGED>(s_c, s_a, n, lg, c, dl, cb, db);

    double al[NP];
    if constexpr (SCALED) fold_scales<NP, LG, RAGGED>(a.st, j, n, lg, true, c, dl, al);

    double acc[NP];
#pragma unroll
    for (int k = 0; k < NP; ++k) acc[k] = 0.0;
    double t2 = 0.0;

    if constexpr (kTwoSets) {
        // Interior tiles with two register sets taking turns: the loads of the wavefront's
        // next tile are issued before the arithmetic of the current one.  On a small slab,
        // where a wavefront has the compute unit almost to itself, its tiles then cost one
        // memory latency together instead of one each.
        if (iw.begin < iw.end) {
            float vb[NP][4];
            float base_b[4] = {0.0f, 0.0f, 0.0f, 0.0f};
            int64_t u = iw.begin;
            bool last_in_b = false;
            for (;;) {
                const int64_t u1 = u + tr.stride;
                if (u1 >= iw.end) break;                 // the last tile is in va
                pass_load_interior<NP, RAGGED, HAS_BASE>(a, n, sub, tr.xa + u1 * G::kW, lane_off, vb, base_b);
                pass_tile_sums<NP, LG, HAS_BASE, SCALED>(va, base_a, c, dl, cb, db, al, lg, acc, t2);
                const int64_t u2 = u1 + tr.stride;
                if (u2 >= iw.end) {                      // the last tile is in vb
                    last_in_b = true;
                    break;
                }
                pass_load_interior<NP, RAGGED, HAS_BASE>(a, n, sub, tr.xa + u2 * G::kW, lane_off, va, base_a);
                pass_tile_sums<NP, LG, HAS_BASE, SCALED>(vb, base_b, c, dl, cb, db, al, lg, acc, t2);
                u = u2;
            }
            if (last_in_b) pass_tile_sums<NP, LG, HAS_BASE, SCALED>(vb, base_b, c, dl, cb, db, al, lg, acc, t2);
            else pass_tile_sums<NP, LG, HAS_BASE, SCALED>(va, base_a, c, dl, cb, db, al, lg, acc, t2);
        }
        // ... then the partition's first and last tile where they are not interior
#pragma unroll 1
        for (int t = 0; t < 2; ++t) {
            const int64_t u = (t == 0) ? 0 : tr.units - 1;
            if ((t == 1 && tr.units < 2) || tr.units < 1 || !owns_tile(tr, u)) continue;
            if (tile_is_interior<G::kW>(tr.xa + u * G::kW, lo, hi)) continue;
            pass_load_any<NP, LG, RAGGED, HAS_BASE>(a, n, lg, sub, tr.xa + u * G::kW, lo, hi, va, base_a);
            pass_tile_sums<NP, LG, HAS_BASE, SCALED>(va, base_a, c, dl, cb, db, al, lg, acc, t2);
        }
    } else {
        for (int64_t u = tr.first; u < tr.units; u += tr.stride) {
            if (u != tr.first) pass_load_any<NP, LG, RAGGED, HAS_BASE>(a, n, lg, sub, tr.xa + u * G::kW, lo, hi, va, base_a);
            pass_tile_sums<NP, LG, HAS_BASE, SCALED>(va, base_a, c, dl, cb, db, al, lg, acc, t2);
        }
    }

    // workgroup partial sums: lanes -> wavefront -> LDS -> one value per quantity
    sum_within_group_all<G::kLanes, NP>(acc);
    t2 = sum_within_group<G::kLanes>(t2);
    if (sub == 0) {
#pragma unroll
        for (int k = 0; k < NP; ++k) sh[wave][lg * NP + k] = acc[k];
    }
    if (lane == 0) sh[wave][G::kPeers] = t2;
    __syncthreads();
    const int B = gridDim.x;
    double *__restrict__ pj =
        a.st.partial + (a.pass & 1) * a.st.partial_stride + (int64_t)j * B * R;
    if ((int)threadIdx.x < R) {
        const int q = threadIdx.x;
        const int src = (q == n) ? G::kPeers : q;
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w][src];
        pj[(int64_t)blockIdx.x * R + q] = s;
    }
}

// ---------------------------------------------------------------------------
// finish: last control step, v = c_0 v0 + sum_i c_i g_i rounded to fp32,
// partial sums of ||last update||^2
// ---------------------------------------------------------------------------
struct CcFinishArgs {
    const float *g;
    int64_t ld;
    int32_t n;
    const float *v0;
    float *v;
    double tau, eps;
    int32_t max_iters;
    int32_t pass;            // number of passes that were enqueued
    int32_t prev_blocks;
    int32_t scaled;          // rows are taken times st.scale (pre-clipping)
    int32_t rule;            // as in CcArgs
    uint32_t epoch_mult;     // write bursts of v: 2^32 / ticks per epoch (0: the default)
    CcState st;
};

// One tile of the last pass: v = c_0 v0 + sum_i c_i g_i rounded to fp32 and written, and
// the squared norm of the last applied update.  INTERIOR: the whole tile lies inside the
// partition (wavefront-uniform): vector loads and store, no masks.
template <int NP, int LG, bool RAGGED, bool HAS_BASE, bool INTERIOR>
__device__ __forceinline__ void finish_tile(const float *__restrict__ g, int64_t ld, int n,
                                            const float *__restrict__ v0, float *__restrict__ v,
                                            int lg, int sub, int64_t xu, int64_t lo, int64_t hi,
                                            const double (&c)[NP], const double (&dl)[NP],
                                            double cb, double db, double &t2,
                                            TileStage *stage = nullptr, int64_t u_tile = 0)
{
    const int64_t x0 = xu + (int64_t)sub * kVec;
    float val[NP][4];
    load_tile<NP, LG, RAGGED>(g, ld, n, lg, sub, xu, lo, hi, INTERIOR, val);
    float base[4] = {0.0f, 0.0f, 0.0f, 0.0f};
    if (HAS_BASE) {
        if (INTERIOR) load_row4_vec(v0 + x0, base);
        else load_row4_guarded(v0, x0, lo, hi, base);
    }
    // (converted one by one where they are used: few registers, many wavefronts)
#pragma unroll
    for (int k = 0; k < NP; ++k) {
#pragma unroll
        for (int e = 0; e < kVec; ++e) forget(val[k][e]);
    }
    double vv[4], ss[4];
    combine_rows<NP, LG, HAS_BASE>(val, base, c, dl, cb, db, vv, ss);
    if (INTERIOR && stage) {
        // (every lane holds the sums; those of lane group 0 keep them for the burst)
        f32x4_u o;
        o.x = (float)vv[0]; o.y = (float)vv[1]; o.z = (float)vv[2]; o.w = (float)vv[3];
        stage->template put<Geo<NP, LG>::kLanes>(u_tile, sub, o, lg == 0);
    }
    if (lg == 0) {
        if (INTERIOR) {
            if (!stage) {
                f32x4_u o;
                o.x = (float)vv[0]; o.y = (float)vv[1]; o.z = (float)vv[2]; o.w = (float)vv[3];
                stream_store(v + x0, o);
            }
        } else {
#pragma unroll
            for (int e = 0; e < kVec; ++e) {
                const int64_t x = x0 + e;
                if (x >= lo && x < hi) v[x] = (float)vv[e];
            }
        }
#pragma unroll
        for (int e = 0; e < kVec; ++e) t2 = fma(ss[e], ss[e], t2);
    }
}

template <int NP, int LG, bool RAGGED, bool HAS_BASE>
__global__ __launch_bounds__(kBlock, 3) void cc_finish_kernel(CcFinishArgs a)
{
    using G = Geo<NP, LG>;
    __shared__ double s_c[kBlock], s_a[kBlock], s_red[kBlock];
    __shared__ int s_flags[2];
    __shared__ double sh[kWaves];
    // (tiles of v parked before they are written in bursts; up to four lane groups)
    __shared__ f32x4_u s_stage[LG <= 4 ? kStageSlots : 1];

    const int j = blockIdx.y;
    const int n = a.n;
    int iters_now;
    if (a.st.done[j]) {
        // stopped earlier: its final state is where the deciding kernel left it
        const int buf = a.st.final_buf[j];
        if ((int)threadIdx.x < a.st.R) {
            s_c[threadIdx.x] = a.st.coef[((int64_t)buf * a.st.P + j) * a.st.R + threadIdx.x];
            s_a[threadIdx.x] = a.st.delta[((int64_t)buf * a.st.P + j) * a.st.R + threadIdx.x];
        }
        if (blockIdx.x == 0 && threadIdx.x == 0) a.st.report_buf[j] = buf;
        __syncthreads();
    } else {
        // still running: apply the update the last pass prepared (this kernel does not
        // publish a stop: nothing runs after it that would need to skip the partition)
        control_step(a.st, j, n, a.tau, a.eps, a.max_iters, a.pass, a.prev_blocks, false, s_c, s_a,
                     s_red, s_flags, &iters_now, a.rule);
        if (blockIdx.x == 0 && threadIdx.x == 0) a.st.report_buf[j] = a.pass & 1;
    }

    const int64_t lo = a.st.off[j], hi = a.st.off[j + 1];
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int lg = lane / G::kLanes, sub = lane % G::kLanes;

    double c[NP], dl[NP], cb, db;
    fetch_coefficients<NP, LG, RAGGED>(s_c, s_a, n, lg, c, dl, cb, db);
    if (a.scaled) {                                 // uniform
        double al[NP];                              // (only the folded coefficients are used)
        fold_scales<NP, LG, RAGGED>(a.st, j, n, lg, true, c, dl, al);
    }
    double t2 = 0.0;

    // interior tiles, then the partition's first and last tile where they are not interior
    // (by the wavefronts that own them): two bodies, so that the guarded one costs the
    // common one no registers
    const TileRange tr = tile_range<G::kW>(lo, hi);
    const InteriorWalk iw = interior_walk<G::kW>(tr, lo, hi);
    constexpr bool kStaged = LG <= 4;
    TileStage stage;
    TileStage *const staged = kStaged ? &stage : nullptr;
    stage.begin(s_stage, wave, a.v, tr.xa, tr.stride, a.epoch_mult);
    for (int64_t u = iw.begin; u < iw.end; u += tr.stride) {
        if constexpr (kStaged) stage.template flush_if_due<G::kLanes>(sub, 1, lg == 0);
        finish_tile<NP, LG, RAGGED, HAS_BASE, true>(a.g, a.ld, n, a.v0, a.v, lg, sub,
                                                    tr.xa + u * G::kW, lo, hi, c, dl, cb, db, t2,
                                                    staged, u);
    }
    if constexpr (kStaged) stage.template flush<G::kLanes>(sub, lg == 0);
#pragma unroll 1
    for (int t = 0; t < 2; ++t) {
        const int64_t u = (t == 0) ? 0 : tr.units - 1;
        if ((t == 1 && tr.units < 2) || !owns_tile(tr, u)) continue;
        const int64_t xu = tr.xa + u * G::kW;
        if (tile_is_interior<G::kW>(xu, lo, hi)) continue;
        finish_tile<NP, LG, RAGGED, HAS_BASE, false>(a.g, a.ld, n, a.v0, a.v, lg, sub, xu, lo, hi, c,
                                                     dl, cb, db, t2);
    }

    t2 = sum_within_group<G::kLanes>(t2);
    if (lane == 0) sh[wave] = t2;
    __syncthreads();
    if (threadIdx.x == 0) {
        double s = 0.0;
#pragma unroll
        for (int w = 0; w < kWaves; ++w) s += sh[w];
        // buffer (pass & 1) is free: what the earlier passes stored there has been consumed
        a.st.partial[(a.pass & 1) * a.st.partial_stride + (int64_t)j * gridDim.x + blockIdx.x] = s;
    }
}

// iters and ||last applied update|| for the caller, one workgroup per partition
struct CcReportArgs {
    CcState st;
    int32_t pass;            // as in cc_finish_kernel
    int32_t blocks;          // workgroups per partition of cc_finish_kernel
    int32_t *iters_out;
    double *step_norm_out;   // may be null
};

static __global__ __launch_bounds__(kBlock) void cc_report_kernel(CcReportArgs a)
{
    __shared__ double s_red[kBlock];
    const int j = blockIdx.x;
    const double *pj = a.st.partial + (a.pass & 1) * a.st.partial_stride + (int64_t)j * a.blocks;
    const double tot = reduce_partials<kBlock>(pj, a.blocks, 1, 1, s_red);
    if (threadIdx.x == 0) {
        const int it = a.st.iters[a.st.report_buf[j] * a.st.P + j];
        a.iters_out[j] = it;
        if (a.step_norm_out) a.step_norm_out[j] = (it > 0) ? sqrt(tot) : 0.0;
    }
}

// ---------------------------------------------------------------------------
// pre-clipping factors (BTARD-Clipped-SGD, App. E.3, Alg. 9 line 3 and the text after the
// algorithm): alpha_ij = min{1, lambda / ||g_i[j]||}.  The norms come from one ordinary pass
// started at v^0 = 0 (cc_begin_kernel with zero_start), whose partial sums this kernel
// reduces; it then sets the coefficients to the real start (the caller's vector, else the
// mean of the clipped rows).
// One workgroup per partition.
// ---------------------------------------------------------------------------
static __global__ __launch_bounds__(kBlock) void preclip_scales_kernel(CcState st, int32_t n,
                                                                       int32_t blocks, double lambda,
                                                                       int32_t max_iters,
                                                                       int32_t has_v0)
{
    __shared__ double s_red[kBlock];
    const int j = blockIdx.x, R = st.R, t = threadIdx.x;
    const double *pj = st.partial + (int64_t)j * blocks * R;
    const double tot = reduce_partials<kBlock>(pj, blocks, R, R, s_red);
    if (t < R) {
        double al = 1.0;
        if (t < n) {
            const double N = sqrt(tot);
            al = (N <= lambda) ? 1.0 : lambda / N;      // (a non-finite norm gives a NaN factor,
        }                                               //  which the first real pass reports)
        st.scale[(int64_t)j * R + t] = al;
        // the real start: the caller's vector, else the mean of the clipped rows
        st.coef[(int64_t)j * R + t] = has_v0 ? ((t == n) ? 1.0 : 0.0) : ((t < n) ? 1.0 / (double)n : 0.0);
    }
    if (t == 0) {                                   // (the norm pass ran with a cap of >= 1)
        st.done[j] = (max_iters <= 0) ? 1 : 0;
        st.remaining[j] = max_iters > 0 ? max_iters : 0;
    }
}

// the factors for the caller: out[i * P + j] = alpha_ij
static __global__ void preclip_export_kernel(CcState st, int32_t n, double *out)
{
    const int j = blockIdx.x;
    for (int i = threadIdx.x; i < n; i += blockDim.x) out[(int64_t)i * st.P + j] = st.scale[(int64_t)j * st.R + i];
}

// the caller's factors into the workspace: scale[j * R + i] = in[i * P + j]
static __global__ void preclip_import_kernel(CcState st, int32_t n, const double *in)
{
    const int j = blockIdx.x;
    for (int i = threadIdx.x; i < n; i += blockDim.x) st.scale[(int64_t)j * st.R + i] = in[(int64_t)i * st.P + j];
}

// Verification 3 of Alg. 6: check_ij = [norm_ij > Delta_max], votes per partition and the
// strict-majority trigger of CheckAveraging.  One thread per partition.
static __global__ void verification3_kernel(const double *norms, int32_t n, int32_t P, double delta_max,
                                     uint8_t *check, int32_t *votes, uint8_t *trigger)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= P) return;
    int cnt = 0;
    for (int i = 0; i < n; ++i) {
        const uint8_t c = norms[(int64_t)i * P + j] > delta_max ? 1 : 0;
        check[(int64_t)i * P + j] = c;
        cnt += c;
    }
    votes[j] = cnt;
    trigger[j] = (2 * cnt > n) ? 1 : 0;
}

// Verifications 1 and 2 of Alg. 6 as comparisons of what peers broadcast with what was
// recomputed: a value "does not match" when it differs by more than atol + rtol |recomputed|
// (or is NaN); the broadcast projections of a partition "do not sum to zero" when
// |sum_i s_ij| > atol + rtol sum_i |s_ij| (summed over i = 0 .. n-1 in order).  One thread per
// partition.
static __global__ void verification12_kernel(const double *claimed_norms, const double *claimed_proj,
                                      const double *norms, const double *proj, int32_t n,
                                      int32_t P, double rtol, double atol, uint8_t *bad_norm,
                                      uint8_t *bad_proj, uint8_t *bad_sum)
{
    const int j = blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= P) return;
    double sum = 0.0, mag = 0.0;
    for (int i = 0; i < n; ++i) {
        const int64_t q = (int64_t)i * P + j;
        bad_norm[q] = (fabs(claimed_norms[q] - norms[q]) <= atol + rtol * fabs(norms[q])) ? 0 : 1;
        bad_proj[q] = (fabs(claimed_proj[q] - proj[q]) <= atol + rtol * fabs(proj[q])) ? 0 : 1;
        sum += claimed_proj[q];
        mag += fabs(claimed_proj[q]);
    }
    bad_sum[j] = (fabs(sum) <= atol + rtol * mag) ? 0 : 1;
}

}  // namespace btard
