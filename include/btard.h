/*
 * btard.h -- C ABI of the MI355X (gfx950) library for the robust-aggregation
 * hot path of Byzantine-tolerant all-reduce ("Secure Distributed Training at
 * Scale", arXiv 2106.11257).
 *
 * One process on one GPU plays all n aggregators of ButterflyClip (Alg. 2):
 * the n peers' gradients are the rows of one matrix, the partitions are column
 * ranges of it, and every partition is aggregated independently.
 *
 * Conventions for every entry point
 *   - "DEVICE" pointers are HIP device memory, "HOST" pointers ordinary host
 *     memory.  Every buffer is owned by the caller; the library allocates no
 *     device memory and never frees or keeps a pointer after the call returns.
 *   - g is fp32, row-major, n rows of leading dimension ldg >= d; row i is peer
 *     i's whole gradient g_i.  Partition j is columns
 *     [offsets_host[j], offsets_host[j+1]).  g is never written.
 *   - Work is enqueued on `stream` (a hipStream_t; NULL = the default stream)
 *     and the call returns without synchronising.  Outputs are valid once the
 *     caller has synchronised the stream.  offsets_host is consumed before the
 *     call returns.
 *   - Return value: BTARD_OK or a negative btard_status.  Argument errors are
 *     detected on the host before anything is enqueued.  A partition whose
 *     residual norms are not finite is reported through iters[j] = -1.
 *   - Calls that share a workspace must be ordered on one stream.  Results are
 *     bit-reproducible from run to run on the same device (no atomics; every
 *     reduction in a fixed order).
 *   - Every entry point that neither takes BTARD_FLAG_HOST_SYNC nor reads a
 *     result back (btard_cc_remaining) only launches kernels -- state is cleared
 *     by kernels, never by memset operations -- so a sequence of calls may be
 *     captured into a HIP graph on `stream` and replayed.
 *   - Limits: 1 <= n <= 255, 1 <= parts <= 65535, 0 <= d <= ldg.
 */
#ifndef BTARD_H_
#define BTARD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum btard_status {
    BTARD_OK = 0,
    BTARD_ERR_INVALID_ARG = -1, /* null pointer, bad size, bad offsets, tau <= 0 ... */
    BTARD_ERR_WORKSPACE = -2,   /* workspace missing, misaligned (256 B) or too small */
    BTARD_ERR_DEVICE = -3       /* a HIP runtime call or kernel launch failed        */
} btard_status;

#define BTARD_FLAG_NONE 0u
/* btard_centered_clip / btard_cc_*: run the iteration on the n x n Gram matrix of each
 * partition (one pass over the data for all iterations) wherever that is accurate enough
 * to reproduce the plain iteration, and fall back to one pass per iteration elsewhere.
 * Takes effect for n <= 64 and v0 == NULL; ignored otherwise.  Same results contract. */
#define BTARD_FLAG_GRAM 1u
/* btard_centered_clip with BTARD_FLAG_GRAM: allow ONE synchronisation of the stream inside
 * the call (after the Gram iteration), so that the per-iteration passes are only enqueued
 * if some partition still needs them.  Without it the call stays asynchronous and enqueues
 * max_iters passes that return at once for stopped partitions (about 2 us each). */
#define BTARD_FLAG_HOST_SYNC 2u
/* btard_cc_* (btard_cc_begin, btard_cc_iterate, btard_cc_finish): Weiszfeld's iteration for
 * the GEOMETRIC MEDIAN of each partition's rows instead of CenteredClip -- the same passes
 * with the weights 1 / max(||g_i - v||, tau), normalised (v <- sum w_i g_i / sum w_i): the
 * tau -> 0 end of CenteredClip (App. D.2) and one of the baselines of Sec. 4.1.  `tau` is
 * then the floor under the norms; stopping rule, v0, iters, last_step_norm as for
 * CenteredClip.  Not with BTARD_FLAG_GRAM (ignored), tau_schedule or
 * btard_cc_finish_verify (there are no clipped residuals to verify). */
#define BTARD_FLAG_GEOMETRIC_MEDIAN 4u
/* Phased interface with BTARD_FLAG_GRAM: the caller leaves out btard_cc_begin, and
 * btard_cc_gram_matrix / btard_cc_gram_iterate do its work (the partition offsets travel as a
 * kernel argument, the Gram iteration starts from the mean by itself): one kernel launch
 * less.  Where that is not possible (no Gram formulation for this problem, more than 255
 * partitions, a tau_schedule) btard_cc_gram_matrix calls btard_cc_begin itself.  The one-call
 * entry points do this on their own. */
#define BTARD_FLAG_GRAM_BEGINS 8u

/* Human-readable name of a status code (static storage). */
const char *btard_status_string(int status);

/*
 * Split(v, parts) of App. D.1: the first (d mod parts) partitions get
 * ceil(d/parts) coordinates, the others floor(d/parts).
 * offsets_host: HOST, parts + 1 entries, written.  Pure host function.
 */
int btard_split_offsets(int64_t d, int32_t parts, int64_t *offsets_host);

/*
 * Bytes of DEVICE workspace (256-byte aligned) that btard_centered_clip,
 * the btard_cc_* calls and btard_verify_projections need for n peers and
 * `parts` partitions.  Pure host arithmetic; 0 if the arguments are out of
 * range.  Independent of d.
 */
size_t btard_workspace_bytes(int32_t n, int32_t parts);

/*
 * CenteredClip (App. D.2, eq. (CenteredClip)) on every partition, as in
 * Alg. 2 line 5:
 *
 *     v^{l+1}[j] = v^l[j] + (1/n) sum_i (g_i[j] - v^l[j]) min{1, tau / ||g_i[j] - v^l[j]||_2}
 *
 * started from v0 (or, if v0 is NULL, from the coordinate-wise mean of the n
 * rows) and stopped, per partition, after the first update whose L2 norm is
 * < eps (Sec. 4.1: "to convergence with eps = 1e-6") or after max_iters
 * updates (App. I.1).  The weight is 1 whenever the norm is <= tau.
 *
 *   g, ldg, n, d        DEVICE matrix as described above
 *   offsets_host, parts HOST, parts + 1 ascending entries, first 0, last d
 *   tau                 > 0; +INF allowed (every weight 1: one step to the mean)
 *   eps                 >= 0; 0 disables the convergence test
 *   max_iters           >= 0; 0 returns v = v0 (or the mean)
 *   v0                  DEVICE [d] fp32 or NULL; must not overlap v
 *   v                   DEVICE [d] fp32, written: the aggregate g-hat
 *   iters               DEVICE [parts] int32, written: updates applied to
 *                       partition j, or -1 if a residual norm was not finite
 *   last_step_norm      DEVICE [parts] fp64 or NULL, written: L2 norm of the
 *                       last applied update (0 if none was applied)
 *   workspace(_bytes)   DEVICE scratch of >= btard_workspace_bytes(n, parts)
 *   flags               BTARD_FLAG_NONE, or BTARD_FLAG_GRAM [| BTARD_FLAG_HOST_SYNC]
 *
 * Arithmetic: fp32 inputs are widened to fp64; the iterate is carried as fp64
 * coefficients of the rows (v^l = c_0 v0 + sum_i c_i g_i), every reduction is
 * fp64 in a fixed order; v is rounded to fp32 once, when it is written.
 */
int btard_centered_clip(const float *g, int64_t ldg, int32_t n, int64_t d,
                        const int64_t *offsets_host, int32_t parts,
                        float tau, float eps, int32_t max_iters,
                        const float *v0, float *v, int32_t *iters,
                        double *last_step_norm, void *workspace,
                        size_t workspace_bytes, void *stream, uint32_t flags);

/*
 * The same computation in three phases, for callers that drive the iteration
 * themselves (timing one pass, interleaving other work, stopping earlier):
 *
 *   btard_cc_begin    validates, uploads the offsets, sets v^0 (the state lives
 *                     in the workspace)
 *   btard_cc_gram     (optional, right after begin; does something only with
 *                     BTARD_FLAG_GRAM) one pass that forms each partition's Gram
 *                     matrix and runs the iteration on it as far as its accuracy
 *                     is guaranteed; partitions it could not finish are left
 *                     in the state at which btard_cc_iterate must take over
 *   btard_cc_remaining (optional) synchronises the stream and returns an upper
 *                     bound on the iterations the partitions that have not
 *                     stopped still need (0: btard_cc_iterate can be skipped).
 *                     It may also be asked AFTER a finish call that was enqueued
 *                     right behind btard_cc_gram with iterations = 0: if it
 *                     returns 0 that finish was complete; otherwise
 *                     btard_cc_iterate(0, remaining) and a second finish call
 *                     complete the run (the state is kept).  That way nothing
 *                     waits for the device inside the run.
 *   btard_cc_iterate  enqueues iterations first_iteration .. first_iteration +
 *                     count - 1 of eq. (CenteredClip) (one pass over the n x d
 *                     matrix each) on every partition that has not stopped;
 *                     stopped partitions are skipped on the device, without
 *                     host involvement.  Iterations must be enqueued in order,
 *                     starting at 0, without gaps: the caller keeps the count.
 *   btard_cc_finish   `iterations` = how many were enqueued in total; applies
 *                     the last update and writes v, iters and last_step_norm
 *                     (one more pass)
 *
 * btard_centered_clip == begin; gram; iterate(0, max_iters); finish(max_iters).
 * The problem description must be identical in all calls of one run.
 */
typedef struct btard_cc_problem {
    const float *g;              /* DEVICE */
    int64_t ldg;
    int32_t n;
    int64_t d;
    const int64_t *offsets_host; /* HOST */
    int32_t parts;
    float tau;
    float eps;
    int32_t max_iters;
    const float *v0;             /* DEVICE or NULL */
    void *workspace;             /* DEVICE */
    size_t workspace_bytes;
    void *stream;
    uint32_t flags;
    float preclip;               /* pre-clipping radius lambda, see below; 0 or +INF: none */
    const float *tau_schedule;   /* HOST, max_iters radii tau_l (eq. (5)), or NULL: constant tau */
} btard_cc_problem;

/*
 * Pre-clipping (BTARD-Clipped-SGD, App. E.3, Alg. 9 line 3 and the paragraph after the
 * algorithm): with 0 < preclip < +INF every peer's partition is first clipped to radius
 * lambda = preclip,
 *     g~_i[j] = min{1, lambda / ||g_i[j]||_2} g_i[j],
 * and everything the calls below compute (v, iters, last_step_norm, norms, weights, proj,
 * colsum) is that of the clipped rows.  g itself is not modified: the factors are applied
 * as the data is read.  They come from the diagonal of the Gram matrix with
 * BTARD_FLAG_GRAM (no extra pass), else from one extra pass over g in btard_cc_begin.
 * The factors are fp64 and g~ is the exact product alpha * g (fp32 value widened to fp64,
 * one fused multiply-add per residual): nothing is rounded to fp32 on the way.  With
 * v0 == NULL the iteration starts at the mean of the clipped rows; a start vector is taken
 * as given (it is not clipped).
 */
/*
 * Clipping radii per iteration: eq. (CenteredClip) is written with tau_l, which App. D.2,
 * eq. (5) derives from the Byzantine fraction delta, the honest inputs' variance bound
 * sigma^2 and a bound B_0^2 on E||v^0 - mean||^2 (btard_tau_schedule below computes it).
 * With tau_schedule != NULL update number l (0-based) of every partition uses
 * tau_schedule[l]; max_iters must not exceed BTARD_MAX_SCHEDULE.  The weights of the
 * verification quantities use `tau` (Alg. 6 has one tau).
 */
#define BTARD_MAX_SCHEDULE 1024
int btard_cc_begin(const btard_cc_problem *p);
int btard_cc_gram(const btard_cc_problem *p);          /* = gram_matrix; gram_iterate */
int btard_cc_gram_matrix(const btard_cc_problem *p);   /* the pass that forms the Gram matrices */
int btard_cc_gram_iterate(const btard_cc_problem *p);  /* the iteration on them */
int btard_cc_remaining(const btard_cc_problem *p, int32_t *remaining_host);
int btard_cc_iterate(const btard_cc_problem *p, int32_t first_iteration, int32_t count);
int btard_cc_finish(const btard_cc_problem *p, int32_t iterations, float *v, int32_t *iters,
                    double *last_step_norm);

/*
 * Verification quantities of BTARD (Alg. 6 lines 6-12; Alg. 1 lines 5-9;
 * eq. (2)) for an aggregate v:
 *
 *     norm_ij  = ||g_i[j] - v[j]||_2
 *     w_ij     = min{1, tau / norm_ij}                  (1 when norm_ij <= tau)
 *     Delta_i^j = w_ij (g_i[j] - v[j])
 *     s_i^j    = <z[j], Delta_i^j>
 *     colsum_j = sum_i s_i^j        (the sum Verification 2 compares with 0)
 *
 * z = GetRandomVector(seed): a unit vector of R^d, uniform on the sphere,
 * generated inside the kernel and never stored.  Its definition: for
 * coordinate x, the Philox4x32-10 block with counter (floor(x/4), 0) and key
 * (seed low word, seed high word) yields u0..u3; a = ((u0 >> 9) + 1/2) 2^-23,
 * b = ((u1 >> 9) + 1/2) 2^-23, rho = sqrt(-2 ln a), zhat[4q] = rho cos(2 pi b),
 * zhat[4q+1] = rho sin(2 pi b), and (u2, u3) give zhat[4q+2], zhat[4q+3] the
 * same way; z = zhat / ||zhat||_2 with the norm taken over all d coordinates.
 *
 *   v         DEVICE [d] fp32: the aggregate being verified (read only)
 *   seed      the MPRNG output r of Alg. 6 line 5
 *   norms, weights, proj   DEVICE [n * parts] fp64, written, entry (i, j) at
 *             index i * parts + j
 *   colsum    DEVICE [parts] fp64 or NULL, written
 *   delta, ldd  DEVICE n x ldd fp32 (ldd >= d) or NULL: if given, Delta_i^j is
 *             written to row i, columns of partition j (one more pass); must
 *             not overlap g or v
 *
 * Arithmetic: residuals and reductions in fp64; zhat in fp32.
 */
int btard_verify_projections(const float *g, int64_t ldg, int32_t n, int64_t d,
                             const int64_t *offsets_host, int32_t parts,
                             const float *v, float tau, uint64_t seed,
                             double *norms, double *weights, double *proj,
                             double *colsum, float *delta, int64_t ldd,
                             void *workspace, size_t workspace_bytes,
                             void *stream, uint32_t flags);

/*
 * The same quantities for PRE-CLIPPED rows (BTARD-Clipped-SGD, App. E.3, Alg. 9 line 3 with
 * Alg. 6 lines 6-12): a peer that receives an aggregate v of clipped gradients and verifies
 * it without having run CenteredClip itself.  Everything is that of the rows
 * g~_i[j] = alpha_ij g_i[j]; g is not modified.  The factors are either the caller's
 * (factors_in: DEVICE, n * parts doubles, entry (i, j) at i * parts + j; lambda is then
 * ignored) or, with factors_in == NULL, alpha_ij = min{1, lambda / ||g_i[j]||_2} from the
 * radius 0 < lambda < +INF, which costs one more pass over g for the norms.  factors_out
 * (DEVICE, n * parts doubles, or NULL) receives the factors that were used.  Other
 * arguments, outputs, workspace and errors as btard_verify_projections.
 */
int btard_verify_projections_preclipped(const float *g, int64_t ldg, int32_t n, int64_t d,
                                        const int64_t *offsets_host, int32_t parts,
                                        const float *v, float lambda, const double *factors_in,
                                        float tau, uint64_t seed, double *norms,
                                        double *weights, double *proj, double *colsum,
                                        float *delta, int64_t ldd, double *factors_out,
                                        void *workspace, size_t workspace_bytes, void *stream,
                                        uint32_t flags);

/*
 * CenteredClip and the verification quantities of its own result in one call:
 * what btard_centered_clip followed by btard_verify_projections(v = that result,
 * delta = NULL) return, with the last pass of the one and the pass of the other
 * merged into a single read of g (the projections are taken against v as it is
 * written, rounded to fp32).  Arguments as in those two calls.
 * With BTARD_FLAG_GRAM, for partitions the Gram iteration finished, norms and
 * last_step_norm are those it derives from the Gram matrix whenever their error
 * bars are below 1e-8 relative (they then differ from norms measured against the
 * rounded v by less than that); otherwise they are measured on the data.
 */
int btard_centered_clip_verify(const float *g, int64_t ldg, int32_t n, int64_t d,
                               const int64_t *offsets_host, int32_t parts,
                               float tau, float eps, int32_t max_iters,
                               const float *v0, float *v, int32_t *iters,
                               double *last_step_norm, uint64_t seed,
                               double *norms, double *weights, double *proj,
                               double *colsum, void *workspace,
                               size_t workspace_bytes, void *stream, uint32_t flags);

/*
 * btard_centered_clip_verify for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc.  The workspace is an array of BTARD_NOALLOC_SCRATCH_BYTES inside the library
 * (one copy per device, held until the process ends); inputs and outputs are still the
 * caller's.  The call allocates nothing and does not synchronise.
 *   - Limit: btard_workspace_bytes(n, parts) <= BTARD_NOALLOC_SCRATCH_BYTES (n <= 16 peers and
 *     up to about 2000 partitions; any d); beyond it the call returns BTARD_ERR_WORKSPACE
 *     before anything is enqueued.
 *   - flags: BTARD_FLAG_NONE or BTARD_FLAG_GRAM (BTARD_FLAG_HOST_SYNC is refused: nothing in
 *     here waits for the device).
 *   - All calls on one device share that device's array, whatever their stream: calls that
 *     overlap in time on one device race.  Order them on one stream (or by events).  The
 *     array keeps the previous call's contents; every call sets up the state it reads.
 * Results are those of btard_centered_clip_verify with a workspace of the caller's, bit for
 * bit.
 */
#define BTARD_NOALLOC_SCRATCH_BYTES (12u << 20)
int btard_centered_clip_verify_noalloc(const float *g, int64_t ldg, int32_t n, int64_t d,
                                       const int64_t *offsets_host, int32_t parts, float tau,
                                       float eps, int32_t max_iters, const float *v0, float *v,
                                       int32_t *iters, double *last_step_norm, uint64_t seed,
                                       double *norms, double *weights, double *proj,
                                       double *colsum, void *stream, uint32_t flags);

/* The same for the phased interface: btard_cc_finish + btard_verify_projections. */
int btard_cc_finish_verify(const btard_cc_problem *p, int32_t iterations, float *v,
                           int32_t *iters, double *last_step_norm, uint64_t seed,
                           double *norms, double *weights, double *proj, double *colsum);

/*
 * Baseline aggregators of Sec. 4.1 on the same layout.
 * btard_geometric_median: per partition, the minimiser of sum_i ||g_i - v||_2 by Weiszfeld's
 * iteration (BTARD_FLAG_GEOMETRIC_MEDIAN above) from v0 (NULL: the mean); nu > 0 is the floor
 * under the norms; arguments otherwise as btard_centered_clip.
 * btard_coordinate_median: v[x] = median of g[0][x] .. g[n-1][x] (mean of the two middle
 * values for even n), x in [0, d); inputs must not be NaN.  No workspace.
 */
int btard_geometric_median(const float *g, int64_t ldg, int32_t n, int64_t d,
                           const int64_t *offsets_host, int32_t parts, float nu, float eps,
                           int32_t max_iters, const float *v0, float *v, int32_t *iters,
                           double *last_step_norm, void *workspace, size_t workspace_bytes,
                           void *stream);
int btard_coordinate_median(const float *g, int64_t ldg, int32_t n, int64_t d, float *v,
                            void *stream);

/*
 * The commitments of Alg. 2 (lines 2 and 6): digests[(i * parts + j) * 32 .. + 31] (DEVICE,
 * 4-byte aligned) = hash(g_i[j]), the hash of the bytes of row i's columns
 * [offsets_host[j], offsets_host[j+1]) as they lie in memory (fp32, little-endian).  With
 * n = 1 and g = the aggregate this is hash(g^[j]).  The paper names no hash function; this one
 * is SHA-256 (FIPS 180-4) arranged as a tree: the bytes are cut into chunks of 1024 (an empty
 * partition is one empty chunk), each chunk's SHA-256 is a node; while a partition has more
 * than one node, every run of 32 consecutive node digests (the last may be shorter) is
 * replaced by the SHA-256 of their concatenation; the remaining node is the hash.  A
 * partition of at most 1024 bytes is hashed by plain SHA-256.
 * workspace: DEVICE, 256-byte aligned, btard_hash_workspace_bytes(n, offsets_host, parts)
 * bytes (0 for bad arguments).  Enqueued on `stream`.
 */
size_t btard_hash_workspace_bytes(int32_t n, const int64_t *offsets_host, int32_t parts);
int btard_partition_hashes(const float *g, int64_t ldg, int32_t n, int64_t d,
                           const int64_t *offsets_host, int32_t parts, uint8_t *digests,
                           void *workspace, size_t workspace_bytes, void *stream);

/*
 * tau_l of App. D.2, eq. (5), for l = 0 .. count - 1 (HOST out):
 *   tau_l = 4 sqrt((1 - delta)(B_l^2 / 3 + sigma^2) / (sqrt(3) delta)),
 *   B_{l+1}^2 = 6.45 delta B_l^2 + 5 sigma^2,  B_0 = b0.
 * 0 < delta < 1, sigma >= 0, b0 >= 0.  Pure host function.
 */
int btard_tau_schedule(double delta, double sigma, double b0, int32_t count, float *tau_host);

/*
 * Verification 3 of Alg. 6 on the norms btard_verify_projections returned (DEVICE,
 * norms[i * parts + j]): check[i * parts + j] = [norm_ij > delta_max] (DEVICE uint8),
 * votes[j] = sum_i check_ij (DEVICE int32), trigger[j] = [votes_j > n / 2] (DEVICE uint8: the
 * partitions for which CheckAveraging must run).  Enqueued on `stream`.
 */
int btard_verification3(const double *norms, int32_t n, int32_t parts, double delta_max,
                        uint8_t *check, int32_t *votes, uint8_t *trigger, void *stream);

/*
 * Verifications 1 and 2 of Alg. 6 as comparisons (all arrays DEVICE, [i * parts + j]):
 * claimed_norms / claimed_proj are what the peers broadcast (norm_ij, s_i^j), norms / proj
 * what btard_verify_projections recomputed.  bad_norm_ij = 1 when the broadcast norm does not
 * match (Verification 1), bad_proj_ij = 1 when the broadcast projection does not match
 * (Verification 2, first test), bad_sum_j = 1 when the broadcast projections of partition j
 * do not sum to zero (Verification 2, second test).  The algorithm states the tests in exact
 * arithmetic; here "a matches b" means |a - b| <= atol + rtol |b| (b recomputed; NaN never
 * matches) and "sums to zero" means |sum_i s_ij| <= atol + rtol sum_i |s_ij|, rtol, atol >= 0.
 * What follows a failed test (Accuse) is the caller's.  Enqueued on `stream`.
 */
int btard_verification12(const double *claimed_norms, const double *claimed_proj,
                         const double *norms, const double *proj, int32_t n, int32_t parts,
                         double rtol, double atol, uint8_t *bad_norm, uint8_t *bad_proj,
                         uint8_t *bad_sum, void *stream);

/*
 * The pre-clipping factors of a run: factors[i * parts + j] = alpha_ij (DEVICE, n * parts
 * doubles; all 1 without pre-clipping).  Valid after btard_cc_begin, with BTARD_FLAG_GRAM
 * after btard_cc_gram.  Enqueued on the problem's stream.
 */
int btard_cc_preclip_factors(const btard_cc_problem *p, double *factors);

/*
 * btard_centered_clip_verify on pre-clipped rows (see btard_cc_problem.preclip): lambda > 0
 * is the radius; factors (DEVICE, n * parts doubles) may be NULL.
 */
int btard_centered_clip_verify_preclipped(const float *g, int64_t ldg, int32_t n, int64_t d,
                                          const int64_t *offsets_host, int32_t parts,
                                          float lambda, float tau, float eps,
                                          int32_t max_iters, float *v, int32_t *iters,
                                          double *last_step_norm, uint64_t seed,
                                          double *norms, double *weights, double *proj,
                                          double *colsum, double *factors, void *workspace,
                                          size_t workspace_bytes, void *stream,
                                          uint32_t flags);

/*
 * Test hook for the z-spec: writes zhat[x_begin .. x_begin + count) (fp32,
 * not normalised) to DEVICE out, with the same device code the verification
 * kernel uses.
 */
int btard_debug_zhat(uint64_t seed, int64_t x_begin, int64_t count, float *out,
                     void *stream);

/*
 * Test hook for the Gram formulation: writes the n x n Gram matrix G G^T of every
 * partition (fp64, row-major, zero-padded to 16 x 16 for n <= 16 and to 64 x 64 for
 * 16 < n <= 64: parts * 256 or parts * 4096 entries) to DEVICE gram_out.  Uses the
 * workspace of `p`.
 */
int btard_debug_gram(const btard_cc_problem *p, double *gram_out);

/*
 * Measurement hook: launches only the first of the two kernels of btard_cc_finish_verify,
 * the fused last pass over g (v is written; the verification quantities stay behind as
 * per-workgroup partial sums in the workspace), so that this kernel can be timed by
 * itself.  Same preconditions as btard_cc_finish_verify, and v0 must be NULL; calling it
 * again, or btard_cc_finish_verify after it, repeats the same work on the same state.
 */
int btard_debug_last_pass(const btard_cc_problem *p, int32_t iterations, float *v,
                          uint64_t seed);

/*
 * Measurement hook, not part of the method: a plain grid-stride kernel with the memory
 * traffic of one CenteredClip pass (v == NULL: the n rows of DEVICE g are read, nothing is
 * written) or of the last pass (v != NULL: DEVICE v[0..d) receives the fp32 sum of the
 * rows, added in the order of the peers), launched with `blocks` workgroups of 256 threads
 * on `stream`.  It is the yardstick beside which bench.py reports the kernels of the method:
 * what a straightforward kernel reaches on the same slab.  ldg >= d >= 0, 1 <= n <= 255,
 * 1 <= blocks <= 2^20 (BTARD_ERR_INVALID_ARG otherwise); rows need only be 4-byte aligned.
 */
int btard_debug_plain_stream(const float *g, int64_t ldg, int32_t n, int64_t d, float *v,
                             int32_t blocks, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* BTARD_H_ */
