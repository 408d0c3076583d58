/*
 * fp64 CPU oracle for the robust-aggregation hot path of Byzantine-tolerant
 * all-reduce ("Secure Distributed Training at Scale", arXiv 2106.11257).
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * step-by-step transcription of what the paper defines, used only by the
 * tests, the smoke check and the CPU-baseline leg of the benchmark.  It shares
 * no code, table or constant generator with the HIP library and neither side
 * includes the other.
 *
 * What is computed, and where the paper defines it:
 *   - Split:            App. D.1 ("Basic building blocks"), item Split(v, n)
 *   - CenteredClip:     App. D.2, eq. (CenteredClip), run per partition as in
 *                       Alg. 2 (ButterflyClip) line 5; stopping rule from
 *                       Sec. 4.1 ("to convergence with eps = 1e-6") and the
 *                       iteration cap M of App. I.1
 *   - Delta, norm, w, s: Alg. 1 lines 8-9; Alg. 6 (BTARD) lines 8-12; eq. (2)
 *   - column check:     Alg. 1 line 16; Alg. 6 Verification 2
 *   - tau_l schedule:   App. D.2, eq. (5)
 *   - baselines:        Sec. 4.1 names them (coordinate-wise and geometric
 *                       medians); their textbook definitions are used
 *   - Verification 3:   Alg. 6 (BTARD), the block of that name
 *   - pre-clipping:     App. E.3, Alg. 9 (BTARD-Clipped-SGD) line 3 and the
 *                       paragraph after the algorithm (per-partition clipping)
 *   - GetRandomVector:  Alg. 6 line 6 and the paragraph after it (a unit vector,
 *                       uniform on the sphere, derived from the scalar seed r by
 *                       "any standard" generator) -- the concrete generator is
 *                       this build's z-spec: Philox4x32-10 (Salmon et al., SC'11)
 *                       feeding Box-Muller; a normalised Gaussian vector is
 *                       uniform on the sphere.
 *
 * Arithmetic: inputs are fp32 (the gradients), widened to fp64 on load; every
 * state variable, reduction and output is fp64.  The paper does not state a
 * precision.
 *
 * Loops over coordinates carry "#pragma omp parallel for" so that the large
 * workloads finish; this changes only the order of fp64 additions.
 *
 * Pins (tests/test_oracle_*.py): Split closed form; tau=inf => mean; identical
 * peers; n=1; collinear inputs => scalar clamp recursion; hand-worked n=3,d=8
 * case (tests/golden); fixed point == minimiser of the summed Huber potential
 * found by an independent optimiser; monotone decrease of that potential;
 * |step| <= tau; translation/rotation/permutation equivariance; partition
 * independence; column-sum identity n<z,next step>; Philox known-answer
 * vectors; |z| = 1, normality (KS) and Box-Muller inversion of z-hat.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

int oracle_num_threads(void)
{
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Threads the coordinate loops use from now on (k >= 1); the arithmetic is    */
/* untouched, only the order of the fp64 additions in the reductions changes. */
void oracle_set_num_threads(int k)
{
#ifdef _OPENMP
    if (k >= 1) omp_set_num_threads(k);
#else
    (void)k;
#endif
}

/* ------------------------------------------------------------------------ */
/* Split(v, n): App. D.1.  The first (d mod parts) parts have ceil(d/parts)   */
/* entries, the others floor(d/parts).  off has parts+1 entries.             */
/* ------------------------------------------------------------------------ */
int oracle_split(int64_t d, int32_t parts, int64_t *off)
{
    if (d < 0 || parts <= 0 || !off) return -1;
    int64_t q = d / parts, r = d % parts;
    off[0] = 0;
    for (int32_t j = 0; j < parts; ++j)
        off[j + 1] = off[j] + q + (j < r ? 1 : 0);
    return 0;
}

/* ------------------------------------------------------------------------ */
/* CenteredClip on ONE partition: columns [lo, hi) of the n x ld row-major   */
/* fp32 matrix G (row i = peer i's gradient g_i).                             */
/*                                                                          */
/*   v^{l+1} = v^l + (1/n) sum_i (g_i - v^l) min{1, tau/||g_i - v^l||_2}      */
/*                                                  (eq. CenteredClip)      */
/*                                                                          */
/* Readings where the paper is silent:                                       */
/*   v^0     = caller's vector, else the coordinate-wise mean of the n rows   */
/*   stop    = after applying update number it, if ||v^{it} - v^{it-1}||_2   */
/*             < eps (strict), or when it == M                                */
/*   weight  = 1 whenever the norm is <= tau (covers norm == 0)              */
/*   n       = the number of rows passed in                                   */
/* A partition whose residual norm is not finite gets iters = -1.            */
/* trace (optional) receives ||step|| of every applied update, M per part.   */
/* ------------------------------------------------------------------------ */
/* srow (optional): n factors; row i of this partition is srow[i] * G[i][.]  */
/* (the pre-clipped gradients of BTARD-Clipped-SGD), else the rows as given. */
/* tau_l (optional): M clipping radii, update number l (0-based) uses        */
/* tau_l[l] as eq. (CenteredClip) is written (tau_l of eq. (5)), else tau.    */
static void centered_clip_partition(const float *G, int64_t ld, int32_t n,
                                    int64_t lo, int64_t hi, double tau,
                                    double eps, int32_t M, const double *v0,
                                    const double *srow, const double *tau_l,
                                    double *v, int32_t *iters,
                                    double *step_norm, double *trace)
{
    const int64_t dj = hi - lo;
    double *step = (double *)malloc(sizeof(double) * (size_t)(dj > 0 ? dj : 1));
    double *w = (double *)malloc(sizeof(double) * (size_t)n);
    double *sc = (double *)malloc(sizeof(double) * (size_t)n);
    for (int32_t i = 0; i < n; ++i) sc[i] = srow ? srow[i] : 1.0;

    /* v^0 */
    if (v0) {
        for (int64_t x = lo; x < hi; ++x) v[x] = v0[x];
    } else {
#pragma omp parallel for schedule(static)
        for (int64_t x = lo; x < hi; ++x) {
            double sum = 0.0;
            for (int32_t i = 0; i < n; ++i) sum += sc[i] * (double)G[i * ld + x];
            v[x] = sum / (double)n;
        }
    }

    int32_t it = 0;
    double T = 0.0;
    int bad = 0;
    while (it < M) {
        const double tau_now = tau_l ? tau_l[it] : tau;
        /* norms ||g_i - v^l|| and clip weights min{1, tau/norm} */
        for (int32_t i = 0; i < n; ++i) {
            const float *gi = G + i * ld;
            const double si = sc[i];
            double N2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : N2)
            for (int64_t x = lo; x < hi; ++x) {
                double r = si * (double)gi[x] - v[x];
                N2 += r * r;
            }
            double N = sqrt(N2);
            if (!isfinite(N)) bad = 1;
            w[i] = (N <= tau_now) ? 1.0 : tau_now / N;
        }
        if (bad) break;

        /* step = (1/n) sum_i w_i (g_i - v^l) ;  v^{l+1} = v^l + step */
        double T2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : T2)
        for (int64_t x = lo; x < hi; ++x) {
            double sum = 0.0;
            for (int32_t i = 0; i < n; ++i)
                sum += w[i] * (sc[i] * (double)G[i * ld + x] - v[x]);
            step[x - lo] = sum / (double)n;
            T2 += step[x - lo] * step[x - lo];
        }
#pragma omp parallel for schedule(static)
        for (int64_t x = lo; x < hi; ++x) v[x] += step[x - lo];

        T = sqrt(T2);
        if (trace) trace[it] = T;
        ++it;
        if (T < eps) break;
    }
    *iters = bad ? -1 : it;
    if (step_norm) *step_norm = T;
    free(step);
    free(w);
    free(sc);
}

/* All partitions, independently (Alg. 2: each aggregator runs its own
 * CenteredClip on its own partition).  off[0..P] ascending, off[0] >= 0,
 * off[P] <= ld.  v0 (fp64, indexed like v) may be NULL.  trace may be NULL or
 * P*M doubles (row j = partition j).  Returns 0, or -1 on bad arguments. */
/* scale (optional): n x P row-major factors alpha_ij: CenteredClip then runs on
 * the rows alpha_ij * g_i[j] (App. E.3, Alg. 9: BTARD-Clipped-SGD hands the
 * pre-clipped gradients to BTARD). */
int oracle_centered_clip_general(const float *G, int64_t ld, int32_t n,
                                 const int64_t *off, int32_t P, double tau, double eps,
                                 int32_t M, const double *v0, const double *scale,
                                 const double *tau_l, double *v, int32_t *iters,
                                 double *step_norm, double *trace)
{
    if (!G || n <= 0 || !off || P <= 0 || !v || !iters || M < 0 || !(tau > 0.0) ||
        !(eps >= 0.0))
        return -1;
    if (tau_l)
        for (int32_t l = 0; l < M; ++l)
            if (!(tau_l[l] > 0.0)) return -1;
    for (int32_t j = 0; j < P; ++j)
        if (off[j] > off[j + 1] || off[j] < 0 || off[j + 1] > ld) return -1;
    double *srow = (double *)malloc(sizeof(double) * (size_t)n);
    for (int32_t j = 0; j < P; ++j) {
        if (trace)
            for (int32_t l = 0; l < M; ++l) trace[(int64_t)j * M + l] = -1.0;
        if (scale)
            for (int32_t i = 0; i < n; ++i) srow[i] = scale[(int64_t)i * P + j];
        centered_clip_partition(G, ld, n, off[j], off[j + 1], tau, eps, M, v0,
                                scale ? srow : NULL, tau_l, v, &iters[j],
                                step_norm ? &step_norm[j] : NULL,
                                trace ? trace + (int64_t)j * M : NULL);
    }
    free(srow);
    return 0;
}

int oracle_centered_clip_scaled(const float *G, int64_t ld, int32_t n,
                                const int64_t *off, int32_t P, double tau, double eps,
                                int32_t M, const double *v0, const double *scale,
                                double *v, int32_t *iters, double *step_norm,
                                double *trace)
{
    return oracle_centered_clip_general(G, ld, n, off, P, tau, eps, M, v0, scale, NULL, v,
                                        iters, step_norm, trace);
}

int oracle_centered_clip(const float *G, int64_t ld, int32_t n,
                         const int64_t *off, int32_t P, double tau, double eps,
                         int32_t M, const double *v0, double *v,
                         int32_t *iters, double *step_norm, double *trace)
{
    return oracle_centered_clip_general(G, ld, n, off, P, tau, eps, M, v0, NULL, NULL, v,
                                        iters, step_norm, trace);
}

/* ------------------------------------------------------------------------ */
/* Baseline aggregators of Sec. 4.1 (the comparison set: "the coordinate-wise */
/* and geometric medians"), per partition like CenteredClip.                  */
/*                                                                            */
/* Geometric median: the minimiser of sum_i ||g_i - v||_2, by Weiszfeld's     */
/* iteration  v <- sum_i w_i g_i / sum_i w_i,  w_i = 1 / max(||g_i - v||, nu) */
/* (nu > 0 guards the division when v reaches an input), from v0 (mean if     */
/* NULL), stopped like CenteredClip: ||v_new - v|| < eps after the update, or */
/* M updates.  App. D.2 describes it as the tau -> 0 end of CenteredClip.     */
/* ------------------------------------------------------------------------ */
int oracle_geometric_median(const float *G, int64_t ld, int32_t n, const int64_t *off,
                            int32_t P, double nu, double eps, int32_t M, const double *v0,
                            double *v, int32_t *iters, double *step_norm)
{
    if (!G || n <= 0 || !off || P <= 0 || !v || !iters || M < 0 || !(nu > 0.0) || !(eps >= 0.0))
        return -1;
    double *w = (double *)malloc(sizeof(double) * (size_t)n);
    for (int32_t j = 0; j < P; ++j) {
        const int64_t lo = off[j], hi = off[j + 1];
        if (lo > hi || lo < 0 || hi > ld) { free(w); return -1; }
        if (v0) {
            for (int64_t x = lo; x < hi; ++x) v[x] = v0[x];
        } else {
#pragma omp parallel for schedule(static)
            for (int64_t x = lo; x < hi; ++x) {
                double sum = 0.0;
                for (int32_t i = 0; i < n; ++i) sum += (double)G[i * ld + x];
                v[x] = sum / (double)n;
            }
        }
        int32_t it = 0;
        double T = 0.0;
        int bad = 0;
        while (it < M) {
            double W = 0.0;
            for (int32_t i = 0; i < n; ++i) {
                const float *gi = G + i * ld;
                double N2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : N2)
                for (int64_t x = lo; x < hi; ++x) {
                    double r = (double)gi[x] - v[x];
                    N2 += r * r;
                }
                const double N = sqrt(N2);
                if (!isfinite(N)) bad = 1;
                w[i] = 1.0 / (N > nu ? N : nu);
                W += w[i];
            }
            if (bad) break;
            double T2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : T2)
            for (int64_t x = lo; x < hi; ++x) {
                double sum = 0.0;
                for (int32_t i = 0; i < n; ++i) sum += w[i] * (double)G[i * ld + x];
                const double vn = sum / W;
                T2 += (vn - v[x]) * (vn - v[x]);
                v[x] = vn;
            }
            T = sqrt(T2);
            ++it;
            if (T < eps) break;
        }
        iters[j] = bad ? -1 : it;
        if (step_norm) step_norm[j] = T;
    }
    free(w);
    return 0;
}

static int cmp_double(const void *a, const void *b)
{
    const double x = *(const double *)a, y = *(const double *)b;
    return (x > y) - (x < y);
}

/* Coordinate-wise median: v[x] = median of G[0][x] .. G[n-1][x]; for even n   */
/* the mean of the two middle values.  x in [0, d).                            */
int oracle_coordinate_median(const float *G, int64_t ld, int32_t n, int64_t d, double *v)
{
    if (!G || n <= 0 || d < 0 || ld < d || !v) return -1;
#pragma omp parallel
    {
        double *col = (double *)malloc(sizeof(double) * (size_t)n);
#pragma omp for schedule(static)
        for (int64_t x = 0; x < d; ++x) {
            for (int32_t i = 0; i < n; ++i) col[i] = (double)G[i * ld + x];
            qsort(col, (size_t)n, sizeof(double), cmp_double);
            v[x] = (n & 1) ? col[n / 2] : 0.5 * (col[n / 2 - 1] + col[n / 2]);
        }
        free(col);
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* The clipping radii of eq. (5) (App. D.2):                                 */
/*   tau_l = 4 sqrt( (1 - delta)(B_l^2/3 + sigma^2) / (sqrt(3) delta) ),      */
/*   B_{l+1}^2 = 6.45 delta B_l^2 + 5 sigma^2,                               */
/* delta = fraction of Byzantine inputs, sigma^2 = bound on the honest       */
/* inputs' pairwise variance, B_0^2 = bound on E||v^0 - mean||^2.            */
/* tau[count], B2[count] (optional) = B_l^2.                                 */
/* ------------------------------------------------------------------------ */
int oracle_tau_schedule(double delta, double sigma, double B0, int32_t count,
                        double *tau, double *B2)
{
    if (!(delta > 0.0) || !(delta < 1.0) || !(sigma >= 0.0) || !(B0 >= 0.0) || count < 0 ||
        !tau)
        return -1;
    double b2 = B0 * B0;
    for (int32_t l = 0; l < count; ++l) {
        tau[l] = 4.0 * sqrt((1.0 - delta) * (b2 / 3.0 + sigma * sigma) / (sqrt(3.0) * delta));
        if (B2) B2[l] = b2;
        b2 = 6.45 * delta * b2 + 5.0 * sigma * sigma;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Verification 3 of Alg. 6 (BTARD): check_ij = [ ||g_i(j) - g^(j)|| >       */
/* Delta_max ], votes_j = sum_i check_ij, and CheckAveraging(j) is triggered */
/* when votes_j > n/2.  norms is n x P row-major (as oracle_verify returns). */
/* ------------------------------------------------------------------------ */
int oracle_verification3(const double *norms, int32_t n, int32_t P, double delta_max,
                         uint8_t *check, int32_t *votes, uint8_t *trigger)
{
    if (!norms || n <= 0 || P <= 0 || !check || !votes || !trigger) return -1;
    for (int32_t j = 0; j < P; ++j) {
        int32_t cnt = 0;
        for (int32_t i = 0; i < n; ++i) {
            const uint8_t c = norms[(int64_t)i * P + j] > delta_max ? 1 : 0;
            check[(int64_t)i * P + j] = c;
            cnt += c;
        }
        votes[j] = cnt;
        trigger[j] = (2 * cnt > n) ? 1 : 0;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Verifications 1 and 2 of Alg. 6 as comparisons.  The algorithm tests       */
/* "norm_ji != ||g_j(i) - g^(i)||", "s_j^i != <z[j], Delta_j^i>" and          */
/* "sum_i s_i^j != 0" in exact arithmetic; in floating point a broadcast      */
/* value matches the recomputed one b when |a - b| <= atol + rtol |b| (NaN    */
/* never matches), and the broadcast projections of partition j sum to zero   */
/* when |sum_i s_ij| <= atol + rtol sum_i |s_ij|.  All arrays n x P row-major. */
/* ------------------------------------------------------------------------ */
int oracle_verification12(const double *claimed_norms, const double *claimed_proj,
                          const double *norms, const double *proj, int32_t n, int32_t P,
                          double rtol, double atol, uint8_t *bad_norm, uint8_t *bad_proj,
                          uint8_t *bad_sum)
{
    if (!claimed_norms || !claimed_proj || !norms || !proj || n <= 0 || P <= 0 ||
        !(rtol >= 0.0) || !(atol >= 0.0) || !bad_norm || !bad_proj || !bad_sum)
        return -1;
    for (int32_t j = 0; j < P; ++j) {
        double sum = 0.0, mag = 0.0;
        for (int32_t i = 0; i < n; ++i) {
            const int64_t q = (int64_t)i * P + j;
            const double dn = fabs(claimed_norms[q] - norms[q]);
            const double dp = fabs(claimed_proj[q] - proj[q]);
            bad_norm[q] = (dn <= atol + rtol * fabs(norms[q])) ? 0 : 1;
            bad_proj[q] = (dp <= atol + rtol * fabs(proj[q])) ? 0 : 1;
            sum += claimed_proj[q];
            mag += fabs(claimed_proj[q]);
        }
        bad_sum[j] = (fabs(sum) <= atol + rtol * mag) ? 0 : 1;
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Pre-clipping of BTARD-Clipped-SGD (App. E.3, Alg. 9 line 3 and the text   */
/* after it): every peer clips each PARTITION of its gradient to radius      */
/* lambda:  g~_i(l) = min{1, lambda / ||g_i(l)||_2} g_i(l).  This returns the */
/* factors alpha_il (n x P row-major; 1 where the norm is <= lambda, also at  */
/* norm 0) and, optionally, the norms ||g_i(l)||.                            */
/* ------------------------------------------------------------------------ */
int oracle_preclip_scales(const float *G, int64_t ld, int32_t n, const int64_t *off,
                          int32_t P, double lambda, double *alpha, double *norms)
{
    if (!G || n <= 0 || !off || P <= 0 || !alpha || !(lambda > 0.0)) return -1;
    for (int32_t j = 0; j < P; ++j) {
        const int64_t lo = off[j], hi = off[j + 1];
        if (lo > hi || lo < 0 || hi > ld) return -1;
        for (int32_t i = 0; i < n; ++i) {
            const float *gi = G + i * ld;
            double N2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : N2)
            for (int64_t x = lo; x < hi; ++x) N2 += (double)gi[x] * (double)gi[x];
            const double N = sqrt(N2);
            alpha[(int64_t)i * P + j] = (N <= lambda) ? 1.0 : lambda / N;
            if (norms) norms[(int64_t)i * P + j] = N;
        }
    }
    return 0;
}

/* ------------------------------------------------------------------------ */
/* Philox4x32-10 (Salmon, Moraes, Dror, Shaw: "Parallel random numbers: as    */
/* easy as 1, 2, 3", SC'11).  Counter 4 x 32 bit, key 2 x 32 bit, 10 rounds. */
/* ------------------------------------------------------------------------ */
void oracle_philox4x32_10(const uint32_t ctr[4], const uint32_t key[2],
                          uint32_t out[4])
{
    const uint64_t M0 = 0xD2511F53u, M1 = 0xCD9E8D57u; /* round multipliers */
    const uint32_t W0 = 0x9E3779B9u, W1 = 0xBB67AE85u; /* key increments    */
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t p0 = M0 * (uint64_t)c0;
        uint64_t p1 = M1 * (uint64_t)c2;
        uint32_t hi0 = (uint32_t)(p0 >> 32), lo0 = (uint32_t)p0;
        uint32_t hi1 = (uint32_t)(p1 >> 32), lo1 = (uint32_t)p1;
        c0 = hi1 ^ c1 ^ k0;
        c1 = lo1;
        c2 = hi0 ^ c3 ^ k1;
        c3 = lo0;
        k0 += W0;
        k1 += W1;
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* ------------------------------------------------------------------------ */
/* z-spec (this build's concrete GetRandomVector).  For global coordinate x, */
/* q = floor(x/4): Philox counter (q lo, q hi, 0, 0), key (seed lo, seed hi) */
/* gives words u0..u3.  a = ((u0>>9)+0.5)/2^23, b = ((u1>>9)+0.5)/2^23 (a     */
/* grid whose points are exact in fp32 as well as fp64),                      */
/* rho = sqrt(-2 ln a): zhat[4q] = rho cos(2 pi b), zhat[4q+1] = rho sin(2 pi */
/* b); the same with (u2,u3) for 4q+2, 4q+3.  z = zhat/||zhat||_2, the norm  */
/* over ALL d coordinates of the gradient.                                   */
/* ------------------------------------------------------------------------ */
static const double TWO_PI = 6.283185307179586476925286766559;

static void z_hat_block(uint64_t seed, int64_t q, double z4[4])
{
    uint32_t ctr[4] = {(uint32_t)((uint64_t)q & 0xFFFFFFFFu),
                       (uint32_t)((uint64_t)q >> 32), 0u, 0u};
    uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
    uint32_t u[4];
    oracle_philox4x32_10(ctr, key, u);
    for (int h = 0; h < 2; ++h) {
        double a = ((double)(u[2 * h] >> 9) + 0.5) / 8388608.0;
        double b = ((double)(u[2 * h + 1] >> 9) + 0.5) / 8388608.0;
        double rho = sqrt(-2.0 * log(a));
        z4[2 * h] = rho * cos(TWO_PI * b);
        z4[2 * h + 1] = rho * sin(TWO_PI * b);
    }
}

/* raw uniforms (a, b) on the 2^-23 grid, for the tests of the z-spec */
void oracle_z_uniforms(uint64_t seed, int64_t x_begin, int64_t count, double *ab)
{
    for (int64_t t = 0; t < count; ++t) {
        int64_t x = x_begin + t, q = x / 4;
        uint32_t ctr[4] = {(uint32_t)((uint64_t)q & 0xFFFFFFFFu),
                           (uint32_t)((uint64_t)q >> 32), 0u, 0u};
        uint32_t key[2] = {(uint32_t)(seed & 0xFFFFFFFFu), (uint32_t)(seed >> 32)};
        uint32_t u[4];
        oracle_philox4x32_10(ctr, key, u);
        ab[t] = ((double)(u[x % 4] >> 9) + 0.5) / 8388608.0;
    }
}

/* un-normalised Gaussian coordinates zhat[x_begin .. x_begin+count) */
void oracle_z_hat(uint64_t seed, int64_t x_begin, int64_t count, double *zhat)
{
#pragma omp parallel for schedule(static)
    for (int64_t t = 0; t < count; ++t) {
        int64_t x = x_begin + t;
        double z4[4];
        z_hat_block(seed, x / 4, z4);
        zhat[t] = z4[x % 4];
    }
}

/* ||zhat||_2 over coordinates 0 .. d-1 */
double oracle_z_norm(uint64_t seed, int64_t d)
{
    double Z2 = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : Z2)
    for (int64_t q = 0; q < (d + 3) / 4; ++q) {
        double z4[4];
        z_hat_block(seed, q, z4);
        for (int e = 0; e < 4; ++e)
            if (4 * q + e < d) Z2 += z4[e] * z4[e];
    }
    return sqrt(Z2);
}

/* ------------------------------------------------------------------------ */
/* Verification quantities for the aggregate v (Alg. 6 lines 6-12):          */
/*   norm_ij = ||g_i[j] - v[j]||_2                                            */
/*   w_ij    = min{1, tau/norm_ij}   (1 when norm_ij <= tau)                  */
/*   Delta_i^j = w_ij (g_i[j] - v[j])                                         */
/*   s_i^j   = <z[j], Delta_i^j>                       (eq. 2)               */
/*   colsum_j = sum_i s_i^j          (the quantity Verification 2 tests)     */
/* Column x of G / v here is global coordinate x_base + x of the gradient    */
/* (so that one partition can be checked on its own); z = zhat/znorm with    */
/* znorm = oracle_z_norm(seed, d_total).  Outputs are row-major n x P;       */
/* delta (optional) is n x ldd fp64.                                          */
/* ------------------------------------------------------------------------ */
int oracle_verify_scaled(const float *G, int64_t ld, int32_t n, const int64_t *off,
                         int32_t P, const double *v, double tau, uint64_t seed,
                         int64_t x_base, double znorm, const double *scale,
                         double *norms, double *weights, double *proj, double *colsum,
                         double *delta, int64_t ldd);

int oracle_verify(const float *G, int64_t ld, int32_t n, const int64_t *off,
                  int32_t P, const double *v, double tau, uint64_t seed,
                  int64_t x_base, double znorm, double *norms, double *weights,
                  double *proj, double *colsum, double *delta, int64_t ldd)
{
    return oracle_verify_scaled(G, ld, n, off, P, v, tau, seed, x_base, znorm, NULL, norms,
                                weights, proj, colsum, delta, ldd);
}

/* scale (optional) as in oracle_centered_clip_scaled: the quantities of the
 * rows alpha_ij * g_i[j]. */
int oracle_verify_scaled(const float *G, int64_t ld, int32_t n, const int64_t *off,
                         int32_t P, const double *v, double tau, uint64_t seed,
                         int64_t x_base, double znorm, const double *scale,
                         double *norms, double *weights, double *proj, double *colsum,
                         double *delta, int64_t ldd)
{
    if (!G || n <= 0 || !off || P <= 0 || !v || !(tau > 0.0) || !(znorm > 0.0) ||
        !norms || !weights || !proj)
        return -1;
    for (int32_t j = 0; j < P; ++j) {
        const int64_t lo = off[j], hi = off[j + 1];
        if (lo > hi || lo < 0 || hi > ld) return -1;
        /* zhat for this partition's coordinates, generated once */
        double *zj = (double *)malloc(sizeof(double) * (size_t)(hi > lo ? hi - lo : 1));
        oracle_z_hat(seed, x_base + lo, hi - lo, zj);
        double cs = 0.0;
        for (int32_t i = 0; i < n; ++i) {
            const float *gi = G + i * ld;
            const double si = scale ? scale[(int64_t)i * P + j] : 1.0;
            double N2 = 0.0, R = 0.0;
#pragma omp parallel for schedule(static) reduction(+ : N2, R)
            for (int64_t x = lo; x < hi; ++x) {
                double r = si * (double)gi[x] - v[x];
                N2 += r * r;
                R += zj[x - lo] * r;
            }
            double N = sqrt(N2);
            double w = (N <= tau) ? 1.0 : tau / N;
            norms[(int64_t)i * P + j] = N;
            weights[(int64_t)i * P + j] = w;
            proj[(int64_t)i * P + j] = w * R / znorm;
            cs += proj[(int64_t)i * P + j];
            if (delta) {
                double *di = delta + i * ldd;
#pragma omp parallel for schedule(static)
                for (int64_t x = lo; x < hi; ++x)
                    di[x] = w * (si * (double)gi[x] - v[x]);
            }
        }
        free(zj);
        if (colsum) colsum[j] = cs;
    }
    return 0;
}
