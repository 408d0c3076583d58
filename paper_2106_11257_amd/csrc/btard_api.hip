// Host side of the C ABI declared in include/btard.h: argument validation,
// workspace carving, grid sizing and kernel launches.  Nothing here allocates
// device memory or synchronises the stream.
#include "../../include/btard.h"

#include <hip/hip_runtime.h>

#include <cmath>
#include <cstdint>
#include <map>
#include <mutex>
#include <utility>
#include <vector>

#include "dispatch.h"
#include "gram_kernels.h"
#include "hash_kernels.h"
#include "plain_kernels.h"

namespace btard {
namespace {

constexpr int kMaxPeers = 255;
constexpr int kMaxParts = 65535;
constexpr int kMaxBlocks = 4096;      // workgroups per launch the partial-sum area is sized for
constexpr size_t kAlign = 256;
constexpr int kMinTilesPerWave = 4;

size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct WsLayout {
    size_t off, coef, delta, iters, done, aux, gram_n2, scale, sched, partial, partial_stride_doubles, gram, total;
};

// State and partial sums exist twice (double-buffered by pass parity).
WsLayout ws_layout(int32_t n, int32_t P)
{
    WsLayout L{};
    const size_t R = (size_t)n + 1, S = 2 * (size_t)n + 2;
    size_t p = kAlign;                                    // 256-byte header, reserved
    L.off = p;      p = align_up(p + sizeof(int64_t) * ((size_t)P + 1));
    L.coef = p;     p = align_up(p + 2 * sizeof(double) * P * R);
    L.delta = p;    p = align_up(p + 2 * sizeof(double) * P * R);
    L.iters = p;    p = align_up(p + 2 * sizeof(int32_t) * P);
    L.done = p;     p = align_up(p + 2 * sizeof(int32_t) * P);      // done | final_buf
    L.aux = p;      p = align_up(p + 3 * sizeof(int32_t) * P);      // report_buf | remaining | gram_ok
    L.gram_n2 = p;  p = align_up(p + sizeof(double) * P * (R + 1));  // gram_n2 [P][R] | gram_t2 [P]
    L.scale = p;    p = align_up(p + sizeof(double) * P * R);        // pre-clipping factors
    L.sched = p;    p = align_up(p + sizeof(double) * kMaxSchedule); // clipping radii per iteration
    const size_t blocks = (size_t)(P > kMaxBlocks ? P : kMaxBlocks);
    L.partial_stride_doubles = align_up(sizeof(double) * blocks * S) / sizeof(double);
    L.partial = p;  p = align_up(p + 2 * sizeof(double) * L.partial_stride_doubles);
    // partial Gram matrices: one 16 x 16 block per workgroup, or the 10 block pairs of n <= 64
    const size_t gram_entries = n <= kGramPeers ? kGramEntries : (n <= 16 * kWideBlocks ? kWideEntries : 0);
    L.gram = p;     p = align_up(p + sizeof(double) * blocks * gram_entries);
    L.total = p;
    return L;
}

bool basic_args_ok(const float *g, int64_t ldg, int32_t n, int64_t d, const int64_t *off,
                   int32_t P)
{
    if (!g || !off) return false;
    if (n < 1 || n > kMaxPeers || P < 1 || P > kMaxParts) return false;
    if (d < 0 || ldg < d) return false;
    if (off[0] != 0 || off[P] != d) return false;
    for (int32_t j = 0; j < P; ++j)
        if (off[j] > off[j + 1]) return false;
    return true;
}

int check_workspace(const void *ws, size_t bytes, int32_t n, int32_t P)
{
    if (!ws || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return BTARD_ERR_WORKSPACE;
    if (bytes < ws_layout(n, P).total) return BTARD_ERR_WORKSPACE;
    return BTARD_OK;
}

CcState carve_cc(void *ws, int32_t n, int32_t P)
{
    const WsLayout L = ws_layout(n, P);
    char *b = static_cast<char *>(ws);
    CcState st;
    st.off = reinterpret_cast<const int64_t *>(b + L.off);
    st.coef = reinterpret_cast<double *>(b + L.coef);
    st.delta = reinterpret_cast<double *>(b + L.delta);
    st.partial = reinterpret_cast<double *>(b + L.partial);
    st.iters = reinterpret_cast<int32_t *>(b + L.iters);
    st.done = reinterpret_cast<int32_t *>(b + L.done);
    st.final_buf = st.done + P;
    st.report_buf = reinterpret_cast<int32_t *>(b + L.aux);
    st.remaining = st.report_buf + P;
    st.gram_ok = st.report_buf + 2 * (size_t)P;
    st.gram_n2 = reinterpret_cast<double *>(b + L.gram_n2);
    st.gram_t2 = st.gram_n2 + (size_t)P * ((size_t)n + 1);
    st.scale = reinterpret_cast<double *>(b + L.scale);
    st.tau_sched = reinterpret_cast<const double *>(b + L.sched);
    st.has_sched = 0;
    st.partial_stride = (int64_t)L.partial_stride_doubles;
    st.R = n + 1;
    st.P = P;
    return st;
}

// ---- kernel variants: peers per lane group (NP) x lane groups per wavefront (LG)
Variant pick_variant(int32_t n)
{
    if (n <= 4) return V4x1;
    if (n <= 8) return V8x1;
    if (n <= 16) return V16x1;
    if (n <= 32) return V16x2;
    if (n <= 64) return V16x4;
    if (n <= 128) return V16x8;
    return V16x16;
}

int variant_tile_width(Variant v)
{
    switch (v) {
        case V16x2: return Geo<16, 2>::kW;
        case V16x4: return Geo<16, 4>::kW;
        case V16x8: return Geo<16, 8>::kW;
        case V16x16: return Geo<16, 16>::kW;
        default: return Geo<16, 1>::kW;
    }
}

int variant_peers(Variant v)
{
    static const int peers[kVariants] = {4, 8, 16, 32, 64, 128, 256};
    return peers[v];
}

// Workgroups that are resident at once for a kernel on the current device
// (compute units x occupancy), cached per (device, kernel); .second = the compute units.
struct ResidentCache {
    std::mutex mu;
    std::map<std::pair<int, const void *>, std::pair<int, int>> value;
};
ResidentCache g_resident;

struct Resident {
    int blocks;   // 0: the query failed
    int cus;
};

Resident resident_blocks(const void *fn)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess) return Resident{0, 0};
    std::lock_guard<std::mutex> lock(g_resident.mu);
    std::pair<int, int> &slot = g_resident.value[std::make_pair(dev, fn)];
    if (slot.first == 0) {
        int cus = 0, occ = 0;
        if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess)
            return Resident{0, 0};
        if (hipOccupancyMaxActiveBlocksPerMultiprocessor(&occ, fn, kBlock, 0) != hipSuccess)
            return Resident{0, 0};
        if (occ < 1) occ = 1;
        if (cus < 1) cus = 1;
        slot = std::make_pair(cus * occ, cus);
    }
    return Resident{slot.first, slot.second};
}

// Epoch of the write bursts of v (TileStage): half the time in which a wavefront fills its
// staging area (measured: 0.35 and 0.75 of it are both slower on the large slabs), when `waves` wavefronts share ~6.5 TB/s and each tile
// costs tile_bytes of traffic; between 10 and 80 us.  Returned as 2^32 / ticks (100 MHz).
uint32_t stage_epoch_multiplier(int64_t waves, double tile_bytes, int capacity_tiles)
{
    const double tile_us = (double)waves * tile_bytes / 6.5e6;            // bytes / (6.5e12 B/s) in us
    double us = 0.5 * (double)capacity_tiles * tile_us;
    if (us < 10.0) us = 10.0;
    if (us > 80.0) us = 80.0;
    return epoch_multiplier((uint32_t)(us * 100.0));
}

// Workgroups per partition.  The device is filled once (no tail wave); what is chosen is how
// many partitions stream side by side.
//   - By default all of them: B = resident / P.
//   - On slabs far beyond the caches that is many concurrent row streams (P x n rows, each
//     read through a narrow window), which costs bandwidth: measured on an 84 GB slab with
//     n = P = 16, B = 256 workgroups per partition (2 or 4 partitions at a time instead of
//     16) takes 12.27 against 12.79 ms for the Gram pass, 13.72 against 14.21 ms for the last
//     pass and 12.08 against 12.19 ms for an iteration's pass, while one partition at a time
//     is slower again (12.8, 14.6, 12.85 ms); with n = 8 rows per partition on an 8.6 GB slab
//     the best figures are those of 64 (passes) to 16-32 (last pass) concurrent rows as well.
//     So where every wavefront still gets kStreamTiles tiles, as many partitions run at a
//     time as make 16 rows per resident workgroup of a compute unit: B = 16 n.
//   - Never more than the partial-sum area holds, nor so many that a wavefront gets fewer
//     than kMinTilesPerWave tiles: on small slabs fewer, longer-lived workgroups cost less
//     than the start-up of many (dispatch, the control step's sums over all workgroups'
//     partial results, the first loads' latency; 64 MiB slab with 16 partitions: 25.0 us per
//     pass with 1 tile per wavefront, 17.8 with 2, 17.4 with 4, 18.6 with 6).
constexpr int kStreamTiles = 32;
int blocks_per_partition(Resident r, int32_t n, int32_t P, const int64_t *off, int tile_w)
{
    int64_t max_units = 1;
    for (int32_t j = 0; j < P; ++j) {
        const int64_t lo = off[j], hi = off[j + 1];
        const int64_t units = hi > lo ? (hi - tile_origin_for(lo, tile_w) + tile_w - 1) / tile_w : 0;
        if (units > max_units) max_units = units;
    }
    int64_t B = r.blocks / P;
    {
        const int64_t occ = r.blocks / r.cus > 0 ? r.blocks / r.cus : 1;
        int64_t at_once = 16 * occ / n;
        if (at_once < 1) at_once = 1;
        if (at_once > P) at_once = P;
        const int64_t Bs = r.blocks / at_once;
        if (Bs > B && max_units / (kWaves * Bs) >= kStreamTiles) B = Bs;
    }
    const int64_t cap_ws = kMaxBlocks / P;
    if (B > cap_ws) B = cap_ws;
    const int64_t cap_work = (max_units + kWaves * kMinTilesPerWave - 1) / (kWaves * kMinTilesPerWave);
    if (B > cap_work) B = cap_work;
    if (B < 1) B = 1;
    return (int)B;
}

int upload_offsets(const int64_t *off_host, int32_t P, const int64_t *off_dev, hipStream_t s)
{
    int64_t *dst = const_cast<int64_t *>(off_dev);
    for (int32_t first = 0; first < P + 1; first += kOffChunk) {
        OffChunk chunk;
        const int32_t count = (P + 1 - first < kOffChunk) ? (P + 1 - first) : kOffChunk;
        for (int32_t t = 0; t < kOffChunk; ++t) chunk.v[t] = (t < count) ? off_host[first + t] : 0;
        hipLaunchKernelGGL(upload_offsets_kernel, dim3(1), dim3(kOffChunk), 0, s, dst, first, count,
                           chunk);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

bool overlaps(const void *a, const void *b, int64_t elems)
{
    if (!a || !b || elems <= 0) return false;
    const uintptr_t pa = reinterpret_cast<uintptr_t>(a), pb = reinterpret_cast<uintptr_t>(b);
    const uintptr_t len = (uintptr_t)elems * sizeof(float);
    return pa < pb + len && pb < pa + len;
}

// the state of a problem's run (carve_cc + what depends on the problem description)
CcState carve_problem(const btard_cc_problem *p)
{
    CcState st = carve_cc(p->workspace, p->n, p->parts);
    st.has_sched = p->tau_schedule ? 1 : 0;
    return st;
}

int rule_of(const btard_cc_problem *p)
{
    return (p->flags & BTARD_FLAG_GEOMETRIC_MEDIAN) != 0 ? kRuleGeometricMedian : kRuleCenteredClip;
}

// pre-clipping of the rows (BTARD-Clipped-SGD) asked for: a positive, finite radius
bool preclip_on(const btard_cc_problem *p) { return p->preclip > 0.0f && std::isfinite(p->preclip); }

int check_problem(const btard_cc_problem *p)
{
    if (!p) return BTARD_ERR_INVALID_ARG;
    if (!basic_args_ok(p->g, p->ldg, p->n, p->d, p->offsets_host, p->parts))
        return BTARD_ERR_INVALID_ARG;
    if (!(p->tau > 0.0f) || !(p->eps >= 0.0f) || p->max_iters < 0) return BTARD_ERR_INVALID_ARG;
    if ((p->flags & ~(uint32_t)(BTARD_FLAG_GRAM | BTARD_FLAG_HOST_SYNC |
                                BTARD_FLAG_GEOMETRIC_MEDIAN | BTARD_FLAG_GRAM_BEGINS)) != 0)
        return BTARD_ERR_INVALID_ARG;
    if ((p->flags & BTARD_FLAG_GEOMETRIC_MEDIAN) != 0 && p->tau_schedule) return BTARD_ERR_INVALID_ARG;
    if (p->tau_schedule) {
        if (p->max_iters > kMaxSchedule) return BTARD_ERR_INVALID_ARG;
        for (int32_t l = 0; l < p->max_iters; ++l)
            if (!(p->tau_schedule[l] > 0.0f)) return BTARD_ERR_INVALID_ARG;
    }
    if (!(p->preclip >= 0.0f)) return BTARD_ERR_INVALID_ARG;             // NaN or negative
    return check_workspace(p->workspace, p->workspace_bytes, p->n, p->parts);
}

}  // namespace
}  // namespace btard

using namespace btard;

extern "C" {

const char *btard_status_string(int status)
{
    switch (status) {
        case BTARD_OK: return "BTARD_OK";
        case BTARD_ERR_INVALID_ARG: return "BTARD_ERR_INVALID_ARG";
        case BTARD_ERR_WORKSPACE: return "BTARD_ERR_WORKSPACE";
        case BTARD_ERR_DEVICE: return "BTARD_ERR_DEVICE";
        default: return "BTARD_ERR_UNKNOWN";
    }
}

int btard_split_offsets(int64_t d, int32_t parts, int64_t *offsets_host)
{
    if (d < 0 || parts < 1 || !offsets_host) return BTARD_ERR_INVALID_ARG;
    const int64_t small = d / parts, big_count = d % parts;
    int64_t at = 0;
    for (int32_t j = 0; j < parts; ++j) {
        offsets_host[j] = at;
        at += small + (j < big_count ? 1 : 0);
    }
    offsets_host[parts] = at;
    return BTARD_OK;
}

size_t btard_workspace_bytes(int32_t n, int32_t parts)
{
    if (n < 1 || n > kMaxPeers || parts < 1 || parts > kMaxParts) return 0;
    return ws_layout(n, parts).total;
}

static bool gram_applies(const btard_cc_problem *p);
static int pass_blocks(const btard_cc_problem *p, Variant var, int ragged, int based);
static int launch_verification(const float *g, int64_t ldg, int32_t n, const int64_t *offsets_host,
                               int32_t parts, const float *v, float tau, uint64_t seed,
                               double *norms, double *weights, double *proj, double *colsum,
                               float *delta, int64_t ldd, const CcState &st, bool scaled,
                               hipStream_t s);

int btard_cc_begin(const btard_cc_problem *p)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    CcState st = carve_problem(p);
    const int32_t P = p->parts;
    // With pre-clipping the factors need the rows' norms: the Gram formulation reads them
    // off its diagonal (btard_cc_gram_iterate), otherwise a pass of its own does it here.
    const bool norm_pass = preclip_on(p) && !gram_applies(p);
    for (int32_t first = 0; first < P + 1; first += kOffChunk) {
        OffChunk chunk;
        const int32_t count = (P + 1 - first < kOffChunk) ? (P + 1 - first) : kOffChunk;
        for (int32_t t = 0; t < kOffChunk; ++t)
            chunk.v[t] = (t < count) ? p->offsets_host[first + t] : 0;
        hipLaunchKernelGGL(cc_begin_kernel, dim3(count), dim3(kOffChunk), 0, s, st, p->n,
                           p->v0 ? 1 : 0, (norm_pass && p->max_iters < 1) ? 1 : p->max_iters, first,
                           count, norm_pass ? 1 : 0, chunk);
    }
    if (p->tau_schedule) {
        double *dst = const_cast<double *>(st.tau_sched);
        for (int32_t first = 0; first < p->max_iters; first += kOffChunk) {
            DblChunk chunk;
            const int32_t count = (p->max_iters - first < kOffChunk) ? (p->max_iters - first) : kOffChunk;
            for (int32_t t = 0; t < kOffChunk; ++t)
                chunk.v[t] = (t < count) ? (double)p->tau_schedule[first + t] : 0.0;
            hipLaunchKernelGGL(upload_doubles_kernel, dim3(1), dim3(kOffChunk), 0, s, dst, first,
                               count, chunk);
        }
    }
    if (norm_pass) {
        // the rows' own norms: one ordinary pass from v^0 = 0, then the factors
        const Variant var = pick_variant(p->n);
        const int ragged = p->n < variant_peers(var) ? 1 : 0;
        const int B = pass_blocks(p, var, ragged, 0);
        if (B <= 0) return BTARD_ERR_DEVICE;
        CcArgs a;
        a.g = p->g; a.ld = p->ldg; a.n = p->n; a.v0 = nullptr;
        a.tau = (double)p->tau; a.eps = (double)p->eps; a.max_iters = p->max_iters;
        a.prev_blocks = B; a.pass = 0; a.scaled = 0; a.rule = kRuleCenteredClip; a.st = st;
        hipLaunchKernelGGL(cc_pass_fn(var, ragged, false, false), dim3(B, P), dim3(kBlock), 0, s, a);
        hipLaunchKernelGGL(preclip_scales_kernel, dim3(P), dim3(kBlock), 0, s, st, p->n, B,
                           (double)p->preclip, p->max_iters, p->v0 ? 1 : 0);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

// The Gram formulation is built for up to 4 x 4 MFMA blocks of 16 peers and a start at the mean.
constexpr int kGramMaxPeers = 16 * kWideBlocks;
static bool gram_applies(const btard_cc_problem *p)
{
    return (p->flags & BTARD_FLAG_GRAM) != 0 && (p->flags & BTARD_FLAG_GEOMETRIC_MEDIAN) == 0 &&
           p->n <= kGramMaxPeers && p->v0 == nullptr && p->max_iters > 0;
}

// With BTARD_FLAG_GRAM_BEGINS the two Gram kernels also do what cc_begin_kernel does (the
// offsets travel as a kernel argument): possible when the Gram formulation runs at all, the
// offsets fit one argument block and no schedule of radii has to be uploaded.
static bool gram_begins(const btard_cc_problem *p)
{
    return (p->flags & BTARD_FLAG_GRAM_BEGINS) != 0 && gram_applies(p) &&
           p->parts + 1 <= kOffChunk && p->tau_schedule == nullptr;
}

// n <= 8: two coordinates per MFMA row block (512-wide tiles); n <= 16: one block (256-wide);
// n <= 64: ceil(n / 16) blocks of peers, the block pairs on and above the diagonal (64-wide)
typedef void (*GramFn)(GramArgs);
static int gram_peer_blocks(const btard_cc_problem *p) { return (p->n + 15) / 16; }
static GramFn gram_kernel(const btard_cc_problem *p)
{
    if (p->n < 8) return gram_pass_band_kernel<8, true>;
    if (p->n == 8) return gram_pass_band_kernel<8, false>;
#ifdef BTARD_GRAM16_BAND
    if (p->n < kGramPeers) return gram_pass_band_kernel<16, true>;
    if (p->n == kGramPeers) return gram_pass_band_kernel<16, false>;
#endif
    if (p->n < kGramPeers) return gram_pass_kernel<true>;
    if (p->n == kGramPeers) return gram_pass_kernel<false>;
    switch (gram_peer_blocks(p)) {
        case 2: return p->n < 32 ? gram_pass_wide_kernel<2, true> : gram_pass_wide_kernel<2, false>;
        case 3: return p->n < 48 ? gram_pass_wide_kernel<3, true> : gram_pass_wide_kernel<3, false>;
        default: return p->n < 64 ? gram_pass_wide_kernel<4, true> : gram_pass_wide_kernel<4, false>;
    }
}

// The last pass reads the slab again right after the Gram pass.  What the Gram pass read
// last is then still in the memory-side cache (256 MB) if it was read with ordinary loads;
// the rest is read with non-temporal loads, which are faster and leave that cache alone.
static int gram_stream_permille(const btard_cc_problem *p)
{
    const double slab = 4.0 * (double)p->n * (double)p->d;
    const double keep = 192.0e6;                          // of the 256 MB, leaving room for v
    if (slab <= keep) return 0;
    return (int)(1000.0 * (1.0 - keep / slab));
}

static int gram_blocks(const btard_cc_problem *p)
{
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(gram_kernel(p)));
    if (resident.blocks <= 0) return 0;
    // n <= 8: a workgroup's wavefronts share its 256-coordinate tiles, i.e. 64 per wavefront
#ifdef BTARD_GRAM16_BAND
    const int tile = 64;
#else
    const int tile = p->n <= 8 ? 64 : (p->n <= kGramPeers ? 256 : 64);
#endif
    return blocks_per_partition(resident, p->n, p->parts, p->offsets_host, tile);
}

int btard_cc_gram_matrix(const btard_cc_problem *p)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if ((p->flags & BTARD_FLAG_GRAM_BEGINS) != 0 && !gram_begins(p)) {
        // the caller left btard_cc_begin to this call, and the kernels cannot take it over
        const int rb = btard_cc_begin(p);
        if (rb != BTARD_OK) return rb;
    }
    if (!gram_applies(p)) return BTARD_OK;               // nothing to do: streaming passes only
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const int B = gram_blocks(p);
    if (B <= 0) return BTARD_ERR_DEVICE;
    const WsLayout L = ws_layout(p->n, p->parts);
    GramArgs ga;
    ga.g = p->g; ga.ld = p->ldg; ga.n = p->n;
    ga.stream_permille = gram_stream_permille(p);
    ga.off = carve_problem(p).off;
    ga.from_args = gram_begins(p) ? 1 : 0;
    ga.parts = p->parts;
    ga.off_out = const_cast<int64_t *>(ga.off);
    for (int32_t t = 0; t < kOffChunk; ++t)
        ga.chunk.v[t] = (ga.from_args && t <= p->parts) ? p->offsets_host[t] : 0;
    ga.gpart = reinterpret_cast<double *>(static_cast<char *>(p->workspace) + L.gram);
    hipLaunchKernelGGL(gram_kernel(p), dim3(B, p->parts), dim3(kBlock), 0, s, ga);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_cc_gram_iterate(const btard_cc_problem *p)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!gram_applies(p)) return BTARD_OK;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const int B = gram_blocks(p);
    if (B <= 0) return BTARD_ERR_DEVICE;
    const WsLayout L = ws_layout(p->n, p->parts);
    GramIterArgs gi;
    gi.st = carve_problem(p);
    gi.gpart = reinterpret_cast<const double *>(static_cast<char *>(p->workspace) + L.gram);
    gi.blocks = B; gi.n = p->n;
    gi.tau = (double)p->tau; gi.eps = (double)p->eps; gi.max_iters = p->max_iters;
    gi.lambda = preclip_on(p) ? (double)p->preclip : 0.0;
    gi.nb = gram_peer_blocks(p);
    gi.fresh = gram_begins(p) ? 1 : 0;
    if (p->n <= kGramPeers)
        hipLaunchKernelGGL(gram_iterate_kernel<16>, dim3(p->parts), dim3(kBlock), 0, s, gi);
    else
        hipLaunchKernelGGL(gram_iterate_kernel<64>, dim3(p->parts), dim3(kBlock), 0, s, gi);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_cc_gram(const btard_cc_problem *p)
{
    const int rc = btard_cc_gram_matrix(p);
    if (rc != BTARD_OK) return rc;
    return btard_cc_gram_iterate(p);
}

int btard_cc_remaining(const btard_cc_problem *p, int32_t *remaining_host)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!remaining_host) return BTARD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const CcState st = carve_problem(p);
    std::vector<int32_t> host((size_t)p->parts);
    if (hipMemcpyAsync(host.data(), st.remaining, sizeof(int32_t) * (size_t)p->parts,
                       hipMemcpyDeviceToHost, s) != hipSuccess)
        return BTARD_ERR_DEVICE;
    if (hipStreamSynchronize(s) != hipSuccess) return BTARD_ERR_DEVICE;
    int32_t most = 0;
    for (int32_t r : host)
        if (r > most) most = r;
    *remaining_host = most;
    return BTARD_OK;
}

int btard_debug_gram(const btard_cc_problem *p, double *gram_out)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!gram_out || p->n > kGramMaxPeers) return BTARD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const int B = gram_blocks(p);
    if (B <= 0) return BTARD_ERR_DEVICE;
    const WsLayout L = ws_layout(p->n, p->parts);
    CcState st = carve_problem(p);
    const int up = upload_offsets(p->offsets_host, p->parts, st.off, s);
    if (up != BTARD_OK) return up;
    GramArgs ga;
    ga.g = p->g; ga.ld = p->ldg; ga.n = p->n; ga.off = st.off;
    ga.stream_permille = gram_stream_permille(p);
    ga.from_args = 0; ga.parts = p->parts; ga.off_out = nullptr;
    ga.gpart = reinterpret_cast<double *>(static_cast<char *>(p->workspace) + L.gram);
    hipLaunchKernelGGL(gram_kernel(p), dim3(B, p->parts), dim3(kBlock), 0, s, ga);
    if (p->n <= kGramPeers)
        hipLaunchKernelGGL(gram_debug_kernel, dim3(p->parts), dim3(kGramEntries), 0, s, ga.gpart, B,
                           gram_out);
    else
        hipLaunchKernelGGL(gram_debug_wide_kernel, dim3(p->parts), dim3(kBlock), 0, s, ga.gpart, B,
                           gram_peer_blocks(p), gram_out);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

// Workgroups per partition of the pass kernel for this problem (the same in every pass).
static int pass_blocks(const btard_cc_problem *p, Variant var, int ragged, int based)
{
    const CcPassFn fn = cc_pass_fn(var, ragged, based, preclip_on(p));
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(fn));
    if (resident.blocks <= 0) return 0;
    return blocks_per_partition(resident, p->n, p->parts, p->offsets_host, variant_tile_width(var));
}

int btard_cc_iterate(const btard_cc_problem *p, int32_t first_iteration, int32_t count)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (count < 0 || first_iteration < 0) return BTARD_ERR_INVALID_ARG;
    if (count == 0) return BTARD_OK;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const Variant var = pick_variant(p->n);
    const int ragged = p->n < variant_peers(var) ? 1 : 0, based = p->v0 ? 1 : 0;
    const CcPassFn fn = cc_pass_fn(var, ragged, based, preclip_on(p));
    const int B = pass_blocks(p, var, ragged, based);
    if (B <= 0) return BTARD_ERR_DEVICE;
    CcArgs a;
    a.g = p->g; a.ld = p->ldg; a.n = p->n; a.v0 = p->v0;
    a.tau = (double)p->tau; a.eps = (double)p->eps; a.max_iters = p->max_iters;
    a.prev_blocks = B; a.scaled = preclip_on(p) ? 1 : 0; a.rule = rule_of(p);
    a.st = carve_problem(p);
    for (int32_t l = 0; l < count; ++l) {
        a.pass = first_iteration + l;
        hipLaunchKernelGGL(fn, dim3(B, p->parts), dim3(kBlock), 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_cc_finish(const btard_cc_problem *p, int32_t iterations, float *v, int32_t *iters,
                    double *last_step_norm)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || iterations < 0) return BTARD_ERR_INVALID_ARG;
    if (overlaps(v, p->v0, p->d)) return BTARD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const Variant var = pick_variant(p->n);
    const int ragged = p->n < variant_peers(var) ? 1 : 0, based = p->v0 ? 1 : 0;
    const CcFinishFn fn = cc_finish_fn(var, ragged, based);
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(fn));
    if (resident.blocks <= 0) return BTARD_ERR_DEVICE;
    const int B = blocks_per_partition(resident, p->n, p->parts, p->offsets_host, variant_tile_width(var));
    const int Bpass = pass_blocks(p, var, ragged, based);
    if (Bpass <= 0) return BTARD_ERR_DEVICE;
    CcFinishArgs a;
    a.g = p->g; a.ld = p->ldg; a.n = p->n; a.v0 = p->v0; a.v = v;
    a.tau = (double)p->tau; a.eps = (double)p->eps; a.max_iters = p->max_iters;
    a.pass = iterations; a.prev_blocks = Bpass; a.scaled = preclip_on(p) ? 1 : 0;
    a.rule = rule_of(p);
    {
        // (a tile: the n rows' and v's 4 bytes per coordinate; tiles staged: see TileStage)
        const int W = variant_tile_width(var);
        // (the wavefronts that share the memory at any time: those resident at once)
        const int64_t running = (int64_t)B * p->parts < resident.blocks ? (int64_t)B * p->parts : resident.blocks;
        a.epoch_mult = stage_epoch_multiplier(running * kWaves,
                                              4.0 * (p->n + 1 + (p->v0 ? 1 : 0)) * W,
                                              kStageTiles * (256 / W));
    }
    a.st = carve_problem(p);
    hipLaunchKernelGGL(fn, dim3(B, p->parts), dim3(kBlock), 0, s, a);
    CcReportArgs r;
    r.st = a.st; r.pass = iterations; r.blocks = B; r.iters_out = iters;
    r.step_norm_out = last_step_norm;
    hipLaunchKernelGGL(cc_report_kernel, dim3(p->parts), dim3(kBlock), 0, s, r);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_centered_clip(const float *g, int64_t ldg, int32_t n, int64_t d,
                        const int64_t *offsets_host, int32_t parts, float tau, float eps,
                        int32_t max_iters, const float *v0, float *v, int32_t *iters,
                        double *last_step_norm, void *workspace, size_t workspace_bytes,
                        void *stream, uint32_t flags)
{
    btard_cc_problem p;
    p.g = g; p.ldg = ldg; p.n = n; p.d = d; p.offsets_host = offsets_host; p.parts = parts;
    p.tau = tau; p.eps = eps; p.max_iters = max_iters; p.v0 = v0;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes; p.stream = stream;
    p.flags = flags; p.preclip = 0.0f; p.tau_schedule = nullptr;
    int rc = check_problem(&p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || overlaps(v, v0, d)) return BTARD_ERR_INVALID_ARG;
    // (btard_cc_begin's work: done by the Gram kernels where they can, else by the call below)
    p.flags |= BTARD_FLAG_GRAM_BEGINS;
    rc = btard_cc_gram(&p);
    if (rc != BTARD_OK) return rc;
    int32_t passes = max_iters;
    if ((flags & BTARD_FLAG_HOST_SYNC) != 0 && gram_applies(&p)) {
        // one look at what the Gram iteration left undone saves the launches of passes
        // that would find every partition stopped
        rc = btard_cc_remaining(&p, &passes);
        if (rc != BTARD_OK) return rc;
    }
    rc = btard_cc_iterate(&p, 0, passes);
    if (rc != BTARD_OK) return rc;
    return btard_cc_finish(&p, passes, v, iters, last_step_norm);
}

// The fused last pass (cc_finish_verify_kernel) alone; *blocks = its workgroups per partition.
static int launch_fused_pass(const btard_cc_problem *p, int32_t iterations, float *v,
                             uint64_t seed, int *blocks)
{
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    const Variant var = pick_variant(p->n);
    const int ragged = p->n < variant_peers(var) ? 1 : 0;
    const FusedFn fn = fused_pass_fn(var, ragged, preclip_on(p));
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(fn));
    if (resident.blocks <= 0) return BTARD_ERR_DEVICE;
    const int B = blocks_per_partition(resident, p->n, p->parts, p->offsets_host, variant_tile_width(var));
    const int Bpass = pass_blocks(p, var, ragged, 0);
    if (Bpass <= 0) return BTARD_ERR_DEVICE;
    FusedArgs a;
    a.g = p->g; a.ld = p->ldg; a.n = p->n; a.v = v;
    a.tau = (double)p->tau; a.eps = (double)p->eps; a.max_iters = p->max_iters;
    a.pass = iterations; a.prev_blocks = Bpass; a.seed = seed; a.S = 2 * p->n + 2;
    // partitions the Gram iteration finished and vouches for take the kernel's light body
    a.use_gram_norms = gram_applies(p) ? 1 : 0;
    a.scaled = preclip_on(p) ? 1 : 0;
    {
        const int W = variant_tile_width(var);
        const int64_t running = (int64_t)B * p->parts < resident.blocks ? (int64_t)B * p->parts : resident.blocks;
        a.epoch_mult = stage_epoch_multiplier(running * kWaves, 4.0 * (p->n + 1) * W,
                                              kStageTiles * (256 / W));
    }
    a.st = carve_problem(p);
    hipLaunchKernelGGL(fn, dim3(B, p->parts), dim3(kBlock), 0, s, a);
    *blocks = B;
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_cc_finish_verify(const btard_cc_problem *p, int32_t iterations, float *v, int32_t *iters,
                           double *last_step_norm, uint64_t seed, double *norms, double *weights,
                           double *proj, double *colsum)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || iterations < 0 || !norms || !weights || !proj) return BTARD_ERR_INVALID_ARG;
    if ((p->flags & BTARD_FLAG_GEOMETRIC_MEDIAN) != 0) return BTARD_ERR_INVALID_ARG;
    if (p->v0) {
        // with a caller-supplied start vector: the two separate passes (the offsets and, with
        // pre-clipping, the factors are in the workspace already)
        const int r1 = btard_cc_finish(p, iterations, v, iters, last_step_norm);
        if (r1 != BTARD_OK) return r1;
        return launch_verification(p->g, p->ldg, p->n, p->offsets_host, p->parts, v, p->tau, seed,
                                   norms, weights, proj, colsum, nullptr, 0, carve_problem(p),
                                   preclip_on(p), static_cast<hipStream_t>(p->stream));
    }
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    int B = 0;
    const int r1 = launch_fused_pass(p, iterations, v, seed, &B);
    if (r1 != BTARD_OK) return r1;
    const CcState st = carve_problem(p);
    VerifyFinishArgs f;
    f.partial = st.partial + (iterations & 1) * st.partial_stride;
    f.n = p->n; f.P = p->parts; f.B = B; f.S = 2 * p->n + 2; f.tau = (double)p->tau;
    f.norms = norms; f.weights = weights; f.proj = proj; f.colsum = colsum;
    f.report = 1; f.state_iters = st.iters; f.report_buf = st.report_buf;
    f.iters_out = iters; f.step_norm_out = last_step_norm;
    hipLaunchKernelGGL(verify_finish_kernel, dim3(p->parts), dim3(kFinishThreads), 0, s, f);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_debug_last_pass(const btard_cc_problem *p, int32_t iterations, float *v, uint64_t seed)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!v || iterations < 0 || p->v0 || (p->flags & BTARD_FLAG_GEOMETRIC_MEDIAN) != 0)
        return BTARD_ERR_INVALID_ARG;
    int B = 0;
    return launch_fused_pass(p, iterations, v, seed, &B);
}

int btard_debug_plain_stream(const float *g, int64_t ldg, int32_t n, int64_t d, float *v,
                             int32_t blocks, void *stream)
{
    if (!g || n < 1 || n > kMaxPeers || d < 0 || ldg < d || blocks < 1 || blocks > (1 << 20))
        return BTARD_ERR_INVALID_ARG;
    if (d == 0) return BTARD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (v)
        hipLaunchKernelGGL(plain_rowsum_kernel<true>, dim3(blocks), dim3(kBlock), 0, s, g, ldg, n, d, v);
    else
        hipLaunchKernelGGL(plain_rowsum_kernel<false>, dim3(blocks), dim3(kBlock), 0, s, g, ldg, n, d,
                           static_cast<float *>(nullptr));
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_centered_clip_verify(const float *g, int64_t ldg, int32_t n, int64_t d,
                               const int64_t *offsets_host, int32_t parts, float tau, float eps,
                               int32_t max_iters, const float *v0, float *v, int32_t *iters,
                               double *last_step_norm, uint64_t seed, double *norms,
                               double *weights, double *proj, double *colsum, void *workspace,
                               size_t workspace_bytes, void *stream, uint32_t flags)
{
    btard_cc_problem p;
    p.g = g; p.ldg = ldg; p.n = n; p.d = d; p.offsets_host = offsets_host; p.parts = parts;
    p.tau = tau; p.eps = eps; p.max_iters = max_iters; p.v0 = v0;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes; p.stream = stream;
    p.flags = flags; p.preclip = 0.0f; p.tau_schedule = nullptr;
    int rc = check_problem(&p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || overlaps(v, v0, d) || !norms || !weights || !proj)
        return BTARD_ERR_INVALID_ARG;
    // (btard_cc_begin's work: done by the Gram kernels where they can, else by the call below)
    p.flags |= BTARD_FLAG_GRAM_BEGINS;
    rc = btard_cc_gram(&p);
    if (rc != BTARD_OK) return rc;
    int32_t passes = max_iters;
    if ((flags & BTARD_FLAG_HOST_SYNC) != 0 && gram_applies(&p)) {
        rc = btard_cc_remaining(&p, &passes);
        if (rc != BTARD_OK) return rc;
    }
    rc = btard_cc_iterate(&p, 0, passes);
    if (rc != BTARD_OK) return rc;
    return btard_cc_finish_verify(&p, passes, v, iters, last_step_norm, seed, norms, weights, proj,
                                  colsum);
}

// ---- the entry point that allocates nothing: its workspace is this array.  Every device the
// library runs on holds its own copy at its own address; host code uses the address that
// hipGetSymbolAddress returns for the current device, never the array's name.
static __device__ __align__(256) unsigned char scratch[BTARD_NOALLOC_SCRATCH_BYTES];

namespace {
constexpr int kMaxDevices = 64;
std::mutex g_scratch_mu;
void *g_scratch_ptr[kMaxDevices];        // per device, set on the first call there

// Address of `scratch` on the current device (nullptr on failure).
void *scratch_on_current_device()
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_scratch_mu);
    if (!g_scratch_ptr[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess) return nullptr;
        g_scratch_ptr[dev] = ptr;
    }
    return g_scratch_ptr[dev];
}
}  // namespace

int btard_centered_clip_verify_noalloc(const float *g, int64_t ldg, int32_t n, int64_t d,
                                       const int64_t *offsets_host, int32_t parts, float tau,
                                       float eps, int32_t max_iters, const float *v0, float *v,
                                       int32_t *iters, double *last_step_norm, uint64_t seed,
                                       double *norms, double *weights, double *proj,
                                       double *colsum, void *stream, uint32_t flags)
{
    // (no synchronisation and no read-back in here: the look BTARD_FLAG_HOST_SYNC permits
    // is not available)
    if ((flags & ~(uint32_t)BTARD_FLAG_GRAM) != 0) return BTARD_ERR_INVALID_ARG;
    if (n < 1 || n > kMaxPeers || parts < 1 || parts > kMaxParts) return BTARD_ERR_INVALID_ARG;
    if (ws_layout(n, parts).total > (size_t)BTARD_NOALLOC_SCRATCH_BYTES) return BTARD_ERR_WORKSPACE;
    void *ws = scratch_on_current_device();
    if (!ws) return BTARD_ERR_DEVICE;
    return btard_centered_clip_verify(g, ldg, n, d, offsets_host, parts, tau, eps, max_iters, v0, v,
                                      iters, last_step_norm, seed, norms, weights, proj, colsum, ws,
                                      (size_t)BTARD_NOALLOC_SCRATCH_BYTES, stream, flags);
}

int btard_geometric_median(const float *g, int64_t ldg, int32_t n, int64_t d,
                           const int64_t *offsets_host, int32_t parts, float nu, float eps,
                           int32_t max_iters, const float *v0, float *v, int32_t *iters,
                           double *last_step_norm, void *workspace, size_t workspace_bytes,
                           void *stream)
{
    btard_cc_problem p;
    p.g = g; p.ldg = ldg; p.n = n; p.d = d; p.offsets_host = offsets_host; p.parts = parts;
    p.tau = nu; p.eps = eps; p.max_iters = max_iters; p.v0 = v0;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes; p.stream = stream;
    p.flags = BTARD_FLAG_GEOMETRIC_MEDIAN; p.preclip = 0.0f; p.tau_schedule = nullptr;
    int rc = check_problem(&p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || overlaps(v, v0, d)) return BTARD_ERR_INVALID_ARG;
    rc = btard_cc_begin(&p);
    if (rc != BTARD_OK) return rc;
    rc = btard_cc_iterate(&p, 0, max_iters);
    if (rc != BTARD_OK) return rc;
    return btard_cc_finish(&p, max_iters, v, iters, last_step_norm);
}

int btard_coordinate_median(const float *g, int64_t ldg, int32_t n, int64_t d, float *v,
                            void *stream)
{
    if (n < 1 || n > kMaxPeers || d < 0 || ldg < d) return BTARD_ERR_INVALID_ARG;
    if (d == 0) return BTARD_OK;                       // nothing to read or write
    if (!g || !v) return BTARD_ERR_INVALID_ARG;
    const Variant var = pick_variant(n);
    const int ragged = n < variant_peers(var) ? 1 : 0;
    const MedianFn fn = median_fn(var, ragged);
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(fn));
    if (resident.blocks <= 0) return BTARD_ERR_DEVICE;
    const int64_t whole[2] = {0, d};
    const int B = blocks_per_partition(resident, n, 1, whole, variant_tile_width(var));
    MedianArgs a;
    a.g = g; a.ld = ldg; a.n = n; a.d = d; a.v = v;
    a.epoch_mult = stage_epoch_multiplier((int64_t)B * kWaves, 4.0 * (n + 1) * variant_tile_width(var),
                                          kStageTiles);
    hipLaunchKernelGGL(fn, dim3(B), dim3(kBlock), 0, static_cast<hipStream_t>(stream), a);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

// ---- partition hashes: the tree's shape, on the host
namespace {
struct HashPlan {
    std::vector<std::vector<int64_t>> node;      // per level: [P + 1] prefix sums of node counts
    size_t off_bytes = 0;                        // [P + 1] offsets
    size_t tables_bytes = 0;                     // all node tables
    size_t total = 0;                            // workspace bytes
    std::vector<size_t> table_at, digest_at;     // byte offsets per level
};

bool hash_plan(int32_t n, const int64_t *off, int32_t P, HashPlan &h)
{
    std::vector<int64_t> cnt((size_t)P);
    for (int32_t j = 0; j < P; ++j) {
        const int64_t bytes = (off[j + 1] - off[j]) * 4;
        cnt[(size_t)j] = bytes > 0 ? (bytes + kHashChunkBytes - 1) / kHashChunkBytes : 1;
    }
    for (;;) {
        std::vector<int64_t> pre((size_t)P + 1, 0);
        bool single = true;
        for (int32_t j = 0; j < P; ++j) {
            pre[(size_t)j + 1] = pre[(size_t)j] + cnt[(size_t)j];
            if (cnt[(size_t)j] > 1) single = false;
        }
        h.node.push_back(pre);
        if (single) break;
        for (int32_t j = 0; j < P; ++j)
            if (cnt[(size_t)j] > 1) cnt[(size_t)j] = (cnt[(size_t)j] + kHashFanout - 1) / kHashFanout;
    }
    size_t at = 0;
    h.off_bytes = align_up(sizeof(int64_t) * ((size_t)P + 1));
    at += h.off_bytes;
    for (size_t k = 0; k < h.node.size(); ++k) {
        h.table_at.push_back(at);
        at += align_up(sizeof(int64_t) * ((size_t)P + 1));
    }
    // the last level's digests go to the caller's array; the others live in the workspace
    for (size_t k = 0; k + 1 < h.node.size(); ++k) {
        h.digest_at.push_back(at);
        at += align_up((size_t)n * (size_t)h.node[k][(size_t)P] * kDigestBytes);
    }
    h.total = at;
    return true;
}

int upload_int64(const std::vector<int64_t> &src, int64_t *dst, hipStream_t s)
{
    const int32_t count_all = (int32_t)src.size();
    for (int32_t first = 0; first < count_all; first += kOffChunk) {
        OffChunk chunk;
        const int32_t count = (count_all - first < kOffChunk) ? (count_all - first) : kOffChunk;
        for (int32_t t = 0; t < kOffChunk; ++t) chunk.v[t] = (t < count) ? src[(size_t)(first + t)] : 0;
        hipLaunchKernelGGL(upload_offsets_kernel, dim3(1), dim3(kOffChunk), 0, s, dst, first, count,
                           chunk);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}
}  // namespace

size_t btard_hash_workspace_bytes(int32_t n, const int64_t *offsets_host, int32_t parts)
{
    if (n < 1 || n > kMaxPeers || parts < 1 || parts > kMaxParts || !offsets_host) return 0;
    for (int32_t j = 0; j < parts; ++j)
        if (offsets_host[j] > offsets_host[j + 1]) return 0;
    HashPlan h;
    hash_plan(n, offsets_host, parts, h);
    return h.total < kAlign ? kAlign : h.total;
}

int btard_partition_hashes(const float *g, int64_t ldg, int32_t n, int64_t d,
                           const int64_t *offsets_host, int32_t parts, uint8_t *digests,
                           void *workspace, size_t workspace_bytes, void *stream)
{
    // (with d = 0 there is nothing to read and g may be NULL: every digest is that of the
    // empty message)
    static const float nothing = 0.0f;
    if (!basic_args_ok((d == 0 && !g) ? &nothing : g, ldg, n, d, offsets_host, parts) || !digests)
        return BTARD_ERR_INVALID_ARG;
    if (!workspace || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0) return BTARD_ERR_WORKSPACE;
    if ((reinterpret_cast<uintptr_t>(digests) % 4) != 0) return BTARD_ERR_INVALID_ARG;
    HashPlan h;
    hash_plan(n, offsets_host, parts, h);
    if (workspace_bytes < h.total) return BTARD_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(stream);
    char *ws = static_cast<char *>(workspace);
    int64_t *off_dev = reinterpret_cast<int64_t *>(ws);
    std::vector<int64_t> off_vec(offsets_host, offsets_host + parts + 1);
    int rc = upload_int64(off_vec, off_dev, s);
    if (rc != BTARD_OK) return rc;
    const size_t levels = h.node.size();
    for (size_t k = 0; k < levels; ++k) {
        rc = upload_int64(h.node[k], reinterpret_cast<int64_t *>(ws + h.table_at[k]), s);
        if (rc != BTARD_OK) return rc;
    }
    for (size_t k = 0; k < levels; ++k) {
        HashArgs a;
        a.g = g; a.ld = ldg; a.off = off_dev;
        a.in = k > 0 ? reinterpret_cast<const uint32_t *>(ws + h.digest_at[k - 1]) : nullptr;
        a.node_in = k > 0 ? reinterpret_cast<const int64_t *>(ws + h.table_at[k - 1]) : nullptr;
        a.total_in = k > 0 ? h.node[k - 1][(size_t)parts] : 0;
        a.out = (k + 1 < levels) ? reinterpret_cast<uint32_t *>(ws + h.digest_at[k])
                                 : reinterpret_cast<uint32_t *>(digests);
        a.node_out = reinterpret_cast<const int64_t *>(ws + h.table_at[k]);
        a.total_out = h.node[k][(size_t)parts];
        a.n = n; a.P = parts; a.level = (int32_t)k;
        const int64_t lanes = (int64_t)n * a.total_out;
        const int64_t blocks = (lanes + kBlock - 1) / kBlock;
        if (blocks > 0x7fffffffLL) return BTARD_ERR_INVALID_ARG;
        hipLaunchKernelGGL(hash_level_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, a);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_tau_schedule(double delta, double sigma, double b0, int32_t count, float *tau_host)
{
    if (!(delta > 0.0) || !(delta < 1.0) || !(sigma >= 0.0) || !(b0 >= 0.0) || count < 0 ||
        (count > 0 && !tau_host))
        return BTARD_ERR_INVALID_ARG;
    double b2 = b0 * b0;
    for (int32_t l = 0; l < count; ++l) {
        tau_host[l] = (float)(4.0 * std::sqrt((1.0 - delta) * (b2 / 3.0 + sigma * sigma) /
                                              (std::sqrt(3.0) * delta)));
        b2 = 6.45 * delta * b2 + 5.0 * sigma * sigma;
    }
    return BTARD_OK;
}

int btard_verification3(const double *norms, int32_t n, int32_t parts, double delta_max,
                        uint8_t *check, int32_t *votes, uint8_t *trigger, void *stream)
{
    if (!norms || !check || !votes || !trigger || n < 1 || n > kMaxPeers || parts < 1 ||
        parts > kMaxParts || delta_max != delta_max)
        return BTARD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(verification3_kernel, dim3((parts + 63) / 64), dim3(64), 0,
                       static_cast<hipStream_t>(stream), norms, n, parts, delta_max, check, votes,
                       trigger);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_verification12(const double *claimed_norms, const double *claimed_proj,
                         const double *norms, const double *proj, int32_t n, int32_t parts,
                         double rtol, double atol, uint8_t *bad_norm, uint8_t *bad_proj,
                         uint8_t *bad_sum, void *stream)
{
    if (!claimed_norms || !claimed_proj || !norms || !proj || !bad_norm || !bad_proj || !bad_sum ||
        n < 1 || n > kMaxPeers || parts < 1 || parts > kMaxParts || !(rtol >= 0.0) ||
        !(atol >= 0.0))
        return BTARD_ERR_INVALID_ARG;
    hipLaunchKernelGGL(verification12_kernel, dim3((parts + 63) / 64), dim3(64), 0,
                       static_cast<hipStream_t>(stream), claimed_norms, claimed_proj, norms, proj,
                       n, parts, rtol, atol, bad_norm, bad_proj, bad_sum);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_cc_preclip_factors(const btard_cc_problem *p, double *factors)
{
    const int rc = check_problem(p);
    if (rc != BTARD_OK) return rc;
    if (!factors) return BTARD_ERR_INVALID_ARG;
    hipStream_t s = static_cast<hipStream_t>(p->stream);
    hipLaunchKernelGGL(preclip_export_kernel, dim3(p->parts), dim3(64), 0, s,
                       carve_problem(p), p->n, factors);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_centered_clip_verify_preclipped(const float *g, int64_t ldg, int32_t n, int64_t d,
                                          const int64_t *offsets_host, int32_t parts,
                                          float lambda, float tau, float eps,
                                          int32_t max_iters, float *v, int32_t *iters,
                                          double *last_step_norm, uint64_t seed,
                                          double *norms, double *weights, double *proj,
                                          double *colsum, double *factors, void *workspace,
                                          size_t workspace_bytes, void *stream, uint32_t flags)
{
    btard_cc_problem p;
    p.g = g; p.ldg = ldg; p.n = n; p.d = d; p.offsets_host = offsets_host; p.parts = parts;
    p.tau = tau; p.eps = eps; p.max_iters = max_iters; p.v0 = nullptr;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes; p.stream = stream;
    p.flags = flags; p.preclip = lambda; p.tau_schedule = nullptr;
    if (!(lambda > 0.0f)) return BTARD_ERR_INVALID_ARG;
    int rc = check_problem(&p);
    if (rc != BTARD_OK) return rc;
    if (!v || !iters || !norms || !weights || !proj) return BTARD_ERR_INVALID_ARG;
    // (btard_cc_begin's work: done by the Gram kernels where they can, else by the call below)
    p.flags |= BTARD_FLAG_GRAM_BEGINS;
    rc = btard_cc_gram(&p);
    if (rc != BTARD_OK) return rc;
    int32_t passes = max_iters;
    if ((flags & BTARD_FLAG_HOST_SYNC) != 0 && gram_applies(&p)) {
        rc = btard_cc_remaining(&p, &passes);
        if (rc != BTARD_OK) return rc;
    }
    rc = btard_cc_iterate(&p, 0, passes);
    if (rc != BTARD_OK) return rc;
    rc = btard_cc_finish_verify(&p, passes, v, iters, last_step_norm, seed, norms, weights, proj,
                                colsum);
    if (rc != BTARD_OK) return rc;
    return factors ? btard_cc_preclip_factors(&p, factors) : BTARD_OK;
}

// The verification pass, its finish and (optionally) the Delta pass on an aggregate v.
// scaled: the rows are taken times the factors in the workspace (st.scale), which the caller
// of this function has put there on the same stream.
static int launch_verification(const float *g, int64_t ldg, int32_t n, const int64_t *offsets_host,
                               int32_t parts, const float *v, float tau, uint64_t seed,
                               double *norms, double *weights, double *proj, double *colsum,
                               float *delta, int64_t ldd, const CcState &st, bool scaled,
                               hipStream_t s)
{
    const Variant var = pick_variant(n);
    const int ragged = n < variant_peers(var) ? 1 : 0;
    const VerifyFn vfn = verify_pass_fn(var, ragged, scaled);
    const Resident resident = resident_blocks(reinterpret_cast<const void *>(vfn));
    if (resident.blocks <= 0) return BTARD_ERR_DEVICE;
    const int B = blocks_per_partition(resident, n, parts, offsets_host, variant_tile_width(var));

    VerifyArgs a;
    a.g = g; a.ld = ldg; a.n = n; a.v = v; a.seed = seed; a.off = st.off;
    a.partial = st.partial; a.S = 2 * n + 1;
    a.scale = scaled ? st.scale : nullptr; a.R = st.R;
    hipLaunchKernelGGL(vfn, dim3(B, parts), dim3(kBlock), 0, s, a);

    VerifyFinishArgs f;
    f.partial = st.partial; f.n = n; f.P = parts; f.B = B; f.S = a.S; f.tau = (double)tau;
    f.norms = norms; f.weights = weights; f.proj = proj; f.colsum = colsum;
    f.report = 0; f.state_iters = nullptr; f.report_buf = nullptr;
    f.iters_out = nullptr; f.step_norm_out = nullptr;
    hipLaunchKernelGGL(verify_finish_kernel, dim3(parts), dim3(kFinishThreads), 0, s, f);

    if (delta) {
        DeltaArgs da;
        da.g = g; da.ld = ldg; da.n = n; da.P = parts; da.v = v; da.off = st.off;
        da.weights = weights; da.delta = delta; da.ldd = ldd;
        da.scale = scaled ? st.scale : nullptr; da.R = st.R;
        int64_t max_len = 1;
        for (int32_t j = 0; j < parts; ++j)
            if (offsets_host[j + 1] - offsets_host[j] > max_len)
                max_len = offsets_host[j + 1] - offsets_host[j];
        int64_t bx = (max_len / kVec + 2 + kBlock - 1) / kBlock;
        const int64_t cap = (kMaxBlocks * 4) / parts > 0 ? (kMaxBlocks * 4) / parts : 1;
        if (bx > cap) bx = cap;
        hipLaunchKernelGGL(delta_kernel, dim3((unsigned)bx, parts), dim3(kBlock), 0, s, da);
    }
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

int btard_verify_projections(const float *g, int64_t ldg, int32_t n, int64_t d,
                             const int64_t *offsets_host, int32_t parts, const float *v,
                             float tau, uint64_t seed, double *norms, double *weights,
                             double *proj, double *colsum, float *delta, int64_t ldd,
                             void *workspace, size_t workspace_bytes, void *stream,
                             uint32_t flags)
{
    if (!basic_args_ok(g, ldg, n, d, offsets_host, parts)) return BTARD_ERR_INVALID_ARG;
    if (!v || !norms || !weights || !proj || !(tau > 0.0f) || flags != BTARD_FLAG_NONE)
        return BTARD_ERR_INVALID_ARG;
    if (delta && (ldd < d || overlaps(delta, v, d))) return BTARD_ERR_INVALID_ARG;
    const int wrc = check_workspace(workspace, workspace_bytes, n, parts);
    if (wrc != BTARD_OK) return wrc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    CcState st = carve_cc(workspace, n, parts);
    const int up = upload_offsets(offsets_host, parts, st.off, s);
    if (up != BTARD_OK) return up;
    return launch_verification(g, ldg, n, offsets_host, parts, v, tau, seed, norms, weights, proj,
                               colsum, delta, ldd, st, false, s);
}

int btard_verify_projections_preclipped(const float *g, int64_t ldg, int32_t n, int64_t d,
                                        const int64_t *offsets_host, int32_t parts,
                                        const float *v, float lambda, const double *factors_in,
                                        float tau, uint64_t seed, double *norms, double *weights,
                                        double *proj, double *colsum, float *delta, int64_t ldd,
                                        double *factors_out, void *workspace,
                                        size_t workspace_bytes, void *stream, uint32_t flags)
{
    if (!basic_args_ok(g, ldg, n, d, offsets_host, parts)) return BTARD_ERR_INVALID_ARG;
    if (!v || !norms || !weights || !proj || !(tau > 0.0f) || flags != BTARD_FLAG_NONE)
        return BTARD_ERR_INVALID_ARG;
    if (delta && (ldd < d || overlaps(delta, v, d))) return BTARD_ERR_INVALID_ARG;
    // the factors: the caller's, or from the radius (one pass over g for the rows' norms)
    if (!factors_in && !(lambda > 0.0f && std::isfinite(lambda))) return BTARD_ERR_INVALID_ARG;
    const int wrc = check_workspace(workspace, workspace_bytes, n, parts);
    if (wrc != BTARD_OK) return wrc;

    hipStream_t s = static_cast<hipStream_t>(stream);
    btard_cc_problem p;
    p.g = g; p.ldg = ldg; p.n = n; p.d = d; p.offsets_host = offsets_host; p.parts = parts;
    p.tau = tau; p.eps = 0.0f; p.max_iters = 0; p.v0 = nullptr;
    p.workspace = workspace; p.workspace_bytes = workspace_bytes; p.stream = stream;
    p.flags = BTARD_FLAG_NONE; p.preclip = factors_in ? 0.0f : lambda; p.tau_schedule = nullptr;
    // (uploads the offsets; with a radius also measures the norms and leaves the factors in
    // the workspace)
    const int rb = btard_cc_begin(&p);
    if (rb != BTARD_OK) return rb;
    const CcState st = carve_problem(&p);
    if (factors_in)
        hipLaunchKernelGGL(preclip_import_kernel, dim3(parts), dim3(64), 0, s, st, n, factors_in);
    if (factors_out)
        hipLaunchKernelGGL(preclip_export_kernel, dim3(parts), dim3(64), 0, s, st, n, factors_out);
    return launch_verification(g, ldg, n, offsets_host, parts, v, tau, seed, norms, weights, proj,
                               colsum, delta, ldd, st, true, s);
}

int btard_debug_zhat(uint64_t seed, int64_t x_begin, int64_t count, float *out, void *stream)
{
    if (x_begin < 0 || count < 0 || (!out && count > 0)) return BTARD_ERR_INVALID_ARG;
    if (count == 0) return BTARD_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    int64_t blocks = (count / 4 + 2 + kBlock - 1) / kBlock;
    if (blocks > 2048) blocks = 2048;
    hipLaunchKernelGGL(zhat_debug_kernel, dim3((unsigned)blocks), dim3(kBlock), 0, s, seed, x_begin,
                       count, out);
    return hipGetLastError() == hipSuccess ? BTARD_OK : BTARD_ERR_DEVICE;
}

}  // extern "C"
