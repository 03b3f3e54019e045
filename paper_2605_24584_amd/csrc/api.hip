// Host side of liblaplex: argument checks (before any HIP call), workspace
// carving, and the order in which the kernels are enqueued.  No arithmetic of the
// method happens here.
#include "../../include/laplex.h"
#include "../../include/laplex_diag.h"
#include "laplex_internal.h"

#include <atomic>
#include <cmath>
#include <mutex>
#include <string>
#include <utility>
#include <vector>

using namespace laplex;

// ---------------------------------------------------------------------------
// Kernel-family timing (diagnostics for benchmarks).
// ---------------------------------------------------------------------------
namespace {
struct ProfEvent { std::string family; hipEvent_t e0, e1; };
struct ProfTotal { std::string family; double ms; int64_t launches; };
std::atomic<bool> g_prof_on{false};
std::mutex g_prof_mutex;
std::string g_prof_family;            // the family that is timed, or "*" for every family
std::vector<ProfEvent> g_prof_events;
std::vector<ProfTotal> g_prof_totals; // per family, filled by laplex_profile_end
hipEvent_t g_prof_open = nullptr;
}  // namespace

void laplex::profile_before(const char* family, hipStream_t st)
{
    if (!g_prof_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (g_prof_family != "*" && g_prof_family != family) return;
    hipEvent_t e0 = nullptr;
    if (hipEventCreate(&e0) != hipSuccess) return;
    (void)hipEventRecord(e0, st);
    g_prof_open = e0;
}

void laplex::profile_after(const char* family, hipStream_t st)
{
    if (!g_prof_on.load(std::memory_order_relaxed)) return;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if ((g_prof_family != "*" && g_prof_family != family) || !g_prof_open) return;
    hipEvent_t e1 = nullptr;
    if (hipEventCreate(&e1) != hipSuccess) { (void)hipEventDestroy(g_prof_open); g_prof_open = nullptr; return; }
    (void)hipEventRecord(e1, st);
    g_prof_events.push_back(ProfEvent{family, g_prof_open, e1});
    g_prof_open = nullptr;
}

namespace {

thread_local std::string g_hip_error;

int hip_fail(hipError_t e)
{
    g_hip_error = hipGetErrorString(e);
    return LAPLEX_ERR_HIP;
}

#define LAPLEX_HIP(expr)                                   \
    do {                                                   \
        const hipError_t e_ = (expr);                      \
        if (e_ != hipSuccess) return hip_fail(e_);         \
    } while (0)

bool misaligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

int check_sizes(int64_t k, int64_t n, int64_t batch)
{
    if (k < 0 || n < 0 || batch < 0) return LAPLEX_ERR_SIZE;
    if (k > LAPLEX_MAX_MERGED || n > LAPLEX_MAX_MERGED || k + n > LAPLEX_MAX_MERGED) return LAPLEX_ERR_SIZE;
    // a matrix must be addressable with 63-bit element offsets
    const int64_t rows = k > n ? k : n;
    if (batch > 0 && rows > (INT64_MAX / 8) / batch) return LAPLEX_ERR_SIZE;
    return LAPLEX_OK;
}

int check_matrix(const float* p, int64_t rows, int64_t ld, int64_t batch, bool required)
{
    if (rows == 0 || batch == 0) return LAPLEX_OK;     // never dereferenced
    if (!p) return required ? LAPLEX_ERR_NULL : LAPLEX_OK;
    if (misaligned(p, 4)) return LAPLEX_ERR_ALIGN;
    if (ld < batch) return LAPLEX_ERR_LD;
    if (rows > (INT64_MAX / 8) / ld) return LAPLEX_ERR_SIZE;
    return LAPLEX_OK;
}

int check_vector(const float* p, int64_t len, bool required)
{
    if (len == 0) return LAPLEX_OK;
    if (!p) return required ? LAPLEX_ERR_NULL : LAPLEX_OK;
    return misaligned(p, 4) ? LAPLEX_ERR_ALIGN : LAPLEX_OK;
}

int check_ws(const void* ws, size_t ws_bytes, const Layout& L)
{
    if (L.total == 0) return LAPLEX_OK;
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < L.total) return LAPLEX_ERR_WORKSPACE;
    return LAPLEX_OK;
}

#define LAPLEX_CHECK(expr)                       \
    do {                                         \
        const int rc_ = (expr);                  \
        if (rc_ != LAPLEX_OK) return rc_;        \
    } while (0)

struct Plan {
    uint32_t* ids; float* dh; float* pk; float* z;
    float2* pk8;    // every eighth sorted anchor with its successor (batch 1 with the sorted-order routes, else null)
    float* xs;      // saved region: the forward's injected rows in sorted order (narrow batches, else null)
    float* stage;   // scratch: the current problem's injected rows in sorted order (narrow batches, else null)
};

Plan plan_of(const Layout& L, char* ws)
{
    const bool narrow = L.batch <= kStageMaxBatch;
    return Plan{reinterpret_cast<uint32_t*>(ws + L.off_ids), reinterpret_cast<float*>(ws + L.off_dh),
                reinterpret_cast<float*>(ws + L.off_pk), reinterpret_cast<float*>(ws + L.off_z),
                L.permute ? reinterpret_cast<float2*>(ws + L.off_pk8) : nullptr,
                narrow ? reinterpret_cast<float*>(ws + L.off_xs) : nullptr,
                narrow ? reinterpret_cast<float*>(ws + L.off_stage) : nullptr};
}

// ----------------------------------------------------------------------------
// Batch 1 with many rows: x and gy reach the sorted order, and the results the caller's order, as records through
// partition passes (permute_kernels.hip) instead of by one random access per value.  Below g_permute_min merged
// positions the tables fit the device's caches and the random accesses are as fast.
// ----------------------------------------------------------------------------
std::atomic<int64_t> g_permute_min{int64_t(1) << 22};

bool use_permute(const Layout& L) { return L.permute && L.N >= g_permute_min.load(std::memory_order_relaxed); }

PermuteJob permute_job(const Layout& L, char* ws, const char* tag)
{
    PermuteJob J;
    for (int lv = 0; lv < 2; ++lv) {
        J.rec_dv[lv] = reinterpret_cast<uint2*>(ws + L.off_rec_dv[lv]);
        J.rec_v1[lv] = reinterpret_cast<float*>(ws + L.off_rec_v1[lv]);
    }
    J.cursors = reinterpret_cast<uint32_t*>(ws + L.off_pt_cursors);
    J.poison = reinterpret_cast<const uint32_t*>(ws + L.off_counters) + kPlanStatusWord;
    J.tag = tag;
    return J;
}

// dst[rank[first_id + i]] = src[i * ld] for i < count, zero at every other sorted position: rows of the caller's matrix
// (the inputs: first_id = k; the outputs: first_id = 0) into sorted order.
int rows_to_sorted(const Layout& L, char* ws, const float* src, int64_t ld, int64_t first_id, int64_t count, float* dst,
                   const char* tag, hipStream_t st)
{
    PermuteJob J = permute_job(L, ws, tag);
    J.source = PermuteJob::kValues;
    J.rank = reinterpret_cast<const uint32_t*>(ws + L.off_rank) + first_id;
    J.val0 = src; J.ld_val = ld; J.source_count = count; J.dest_count = L.N;
    J.values = 1; J.out0 = dst; J.ld0 = 1;
    LAPLEX_HIP(launch_permute(J, st));
    return LAPLEX_OK;
}

// One scan problem with everything in sorted order (`p.stage` holds the injected rows already): its results leave the
// downsweep as records on their way home, out0[(id - res_lo) * ld0] = the first output of the row (if want_first) or
// its second, out1[(id - res_lo) * ld1] = the second when both are wanted.
int scan_and_send_home(ScanProblem& p, const Layout& L, char* ws, bool want_first, bool want_second,
                       float* out0, int64_t ld0, float* out1, int64_t ld1, hipStream_t st)
{
    PermuteJob J = permute_job(L, ws, p.tag);
    J.source = PermuteJob::kRows;
    J.source_count = L.N; J.dest_count = (int64_t)p.res_hi - (int64_t)p.res_lo;
    J.values = (want_first && want_second) ? 2 : 1;
    J.out0 = out0; J.ld0 = ld0; J.out1 = out1; J.ld1 = ld1;
    PartEmit E;
    LAPLEX_HIP(permute_begin(J, &E, st));
    p.inj_sorted = p.out_sorted = true;
    p.emit = &E; p.emit_values = J.values; p.emit_first = want_first; p.emit_strict = want_second;
    LAPLEX_HIP(launch_scan(p, L, ws, st));
    LAPLEX_HIP(permute_finish(J, st));
    return LAPLEX_OK;
}

// Sort (or merge) the anchors and compute the neighbour decays, unless the plan is reused.
int build_plan(const float* a, int64_t k, const float* b, int64_t n, float tau, const Layout& L, char* ws,
               uint32_t flags, bool both_sorted, hipStream_t st)
{
    if (flags & LAPLEX_REUSE_PLAN) return LAPLEX_OK;
    const Plan P = plan_of(L, ws);
    uint2* pair0 = reinterpret_cast<uint2*>(ws + L.off_pair0);
    uint2* pair1 = reinterpret_cast<uint2*>(ws + L.off_pair1);
    uint32_t* keys0 = reinterpret_cast<uint32_t*>(pair0);      // the merge leaves its sorted keys here
    uint32_t* small = reinterpret_cast<uint32_t*>(ws + L.off_sort_small);
    uint32_t* counters = reinterpret_cast<uint32_t*>(ws + L.off_counters);
    if (both_sorted) {
        LAPLEX_HIP(launch_merge(a, k, b, n, tau, keys0, P.ids, st));
        LAPLEX_HIP(launch_decay(keys0, nullptr, P.dh, P.pk, P.pk8, counters, L.N, st));
    } else {
        LAPLEX_HIP(launch_onesweep_sort(a, k, b, n, tau, pair0, pair1, P.ids, P.pk, small,
                                        reinterpret_cast<unsigned long long*>(ws + L.off_status), st));
        LAPLEX_HIP(launch_decay(nullptr, small, P.dh, P.pk, P.pk8, counters, L.N, st));
    }
    if (use_permute(L)) {        // the inverse permutation, part of the plan: rank[ids[j]] = j
        PermuteJob J = permute_job(L, ws, "rank");
        J.source = PermuteJob::kRowIndex;
        J.ids = P.ids; J.source_count = L.N; J.dest_count = L.N;
        J.values = 1; J.out0 = reinterpret_cast<float*>(ws + L.off_rank); J.ld0 = 1;
        J.poison = nullptr;          // positions, not values: an invalid plan shows in the results
        LAPLEX_HIP(launch_permute(J, st));
    }
    return LAPLEX_OK;
}

// Arguments of the one-launch path for small problems (one operator; callers add problems and strides).
SmallArgs small_args(const float* a, int64_t k, const float* b, int64_t n, float tau, const Plan& P, const Layout& L,
                     uint32_t flags)
{
    SmallArgs S{};
    S.a = a; S.b = b; S.k = k; S.n = n; S.tau = tau;
    S.ids = P.ids; S.dh = P.dh; S.pk = P.pk;
    S.reuse_plan = (flags & LAPLEX_REUSE_PLAN) ? 1 : 0;
    S.batch = L.batch; S.cols = small_cols(L.batch);
    return S;
}

// The plan's status word (nonzero: the radix sort gave up a wait), or null for plans sorted by counting, which never wait.
const uint32_t* plan_status_word(const Layout& L, const char* ws)
{
    if (L.N <= kSmallMax) return nullptr;
    return reinterpret_cast<const uint32_t*>(ws + L.off_counters) + kPlanStatusWord;
}

ScanProblem problem(const Plan& P, const Layout& L)
{
    ScanProblem p{};
    p.ids = P.ids; p.dh = P.dh; p.pk = P.pk; p.pk8 = P.pk8; p.N = L.N; p.batch = L.batch;
    return p;
}

// Workspace of the phased entry points: the workspace of the plain apply on the doubled batch
// (so the plan stays at the front), then the cosine / sine halves of x, y, gy and gx.
struct PhasedLayout {
    size_t inner = 0, off_x2 = 0, off_y2 = 0, off_g2 = 0, off_gx2 = 0, off_state = 0, total = 0;
};

PhasedLayout phased_layout(int64_t k, int64_t n, int64_t batch)
{
    PhasedLayout P;
    P.inner = align_up(make_layout(k + n, k, 2 * batch).total);
    size_t o = P.inner;
    const size_t in_bytes = sizeof(float) * 2 * (size_t)batch * (size_t)n, out_bytes = sizeof(float) * 2 * (size_t)batch * (size_t)k;
    P.off_x2 = o;  o = align_up(o + in_bytes);
    P.off_y2 = o;  o = align_up(o + out_bytes);
    P.off_g2 = o;  o = align_up(o + out_bytes);
    P.off_gx2 = o; o = align_up(o + in_bytes);
    P.off_state = o; o = align_up(o + sizeof(uint32_t) * 64);      // word 0: the doubled copy of x holds every row
    P.total = o;
    return P;
}

// Can the phased backward leave the merge of the two halves to the streaming downsweep (PhaseFuse)?  The inner problem must
// take the wide geometry with one wavefront across a half-row, and every row the kernel touches must allow 16-byte accesses.
bool phase_fusable(int64_t k, int64_t n, int64_t batch, const float* x, int64_t ldx, const float* gx, int64_t ldgx)
{
    if (k + n <= kSmallMax || batch % 4 != 0 || batch > 256) return false;
    const ScanGeom g = scan_geom(k + n, 2 * batch, 4);
    if (!g.sub_shift || g.slabs > 2) return false;
    if (x && (misaligned(x, 16) || ldx % 4 != 0)) return false;
    if (gx && (misaligned(gx, 16) || ldgx % 4 != 0)) return false;
    return true;
}

int check_phased_sizes(int64_t k, int64_t n, int64_t batch)
{
    if (batch < 0 || batch > INT64_MAX / 4) return LAPLEX_ERR_SIZE;
    return check_sizes(k, n, 2 * batch);
}

// ----------------------------------------------------------------------------
// Weighted Gram matrix (gram_kernels.hip).  Workspace: the plain workspace for batch 1 (the plan of the
// doubled anchors at its front), then U, V, W f64[k] each and five f64 per tile of the scan.  The fp32 and
// the fp64 entry point share it.
// ----------------------------------------------------------------------------
struct Wgram64Layout {
    size_t inner = 0, off_u = 0, off_v = 0, off_w = 0, off_summ = 0, off_pb = 0, total = 0;
};

Wgram64Layout wgram64_layout(int64_t k, int64_t n)
{
    Wgram64Layout G;
    G.inner = make_layout(k + n, k, 1, false).total;
    size_t o = align_up(G.inner);
    G.off_u = o;    o = align_up(o + sizeof(double) * (size_t)k);
    G.off_v = o;    o = align_up(o + sizeof(double) * (size_t)k);
    G.off_w = o;    o = align_up(o + sizeof(double) * (size_t)k);
    G.off_summ = o; o = align_up(o + sizeof(double) * 6 * (size_t)wgram_tiles(k + n));
    G.off_pb = o;   o = align_up(o + sizeof(double) * (size_t)n);
    G.total = o;
    return G;
}

// The plan (ids, sorted anchors) of the doubled anchors: few merged positions are ranked by counting in one
// launch, more go through the radix sort (or the merge path).
int build_wgram_plan(const float* a, int64_t k, const float* b, int64_t n, const Layout& L, const Plan& P, char* w,
                     uint32_t flags, hipStream_t st)
{
    if (L.N <= kSmallMax) {
        SmallArgs S = small_args(a, k, b, n, 2.0f, P, L, flags);      // no scan problem: the sort alone
        LAPLEX_HIP(launch_small(S, 1, st));
        return LAPLEX_OK;
    }
    const bool sorted = (flags & LAPLEX_A_SORTED) && (flags & LAPLEX_B_SORTED);
    return build_plan(a, k, b, n, 2.0f, L, w, flags, sorted, st);
}

int check_wgram_sizes(int64_t k, int64_t n)
{
    LAPLEX_CHECK(check_sizes(k, n, 1));
    if (k > LAPLEX_WGRAM_MAX_ANCHORS) return LAPLEX_ERR_SIZE;
    return LAPLEX_OK;
}


// ----------------------------------------------------------------------------
// LAPLEX^(r): r plain workspaces back to back (each operator keeps its own plan and saved scans), then
// the r products L_q x (kept for the gradient of the mixing weights), the scaled upstream gradient of
// the operator at hand, its gx, and the partial sums of the inner products.
// ----------------------------------------------------------------------------
struct MixLayout {
    size_t inner = 0, off_parts = 0, off_gyq = 0, off_gxq = 0, off_gxp = 0, off_partial = 0, total = 0;
    int lanes = 1;      // operators in flight at a time on the large path (each on a stream of its own)
};

// Beyond the small path an operator is a chain of two dozen launches; while the matrices are small each of them fills a
// fraction of the device for a few microseconds, and the chains of different operators share nothing but x and gy: up to
// kMixLanes of them run side by side, each on a stream of the library's own, with its own copy of the per-operator scratch.
constexpr int kMixLanes = 4;
constexpr int64_t kMixLanesMaxElements = int64_t(1) << 24;      // (k + n) * batch up to which that pays

int mix_lanes(int64_t r, int64_t k, int64_t n, int64_t batch)
{
    if (k + n <= kSmallMax || r < 2 || (k + n) * batch > kMixLanesMaxElements) return 1;
    return r < kMixLanes ? (int)r : kMixLanes;
}

MixLayout mix_layout(int64_t r, int64_t k, int64_t n, int64_t batch)
{
    MixLayout M;
    M.lanes = mix_lanes(r, k, n, batch);
    M.inner = align_up(make_layout(k + n, k, batch).total);
    size_t o = M.inner * (size_t)r;
    M.off_parts = o;   o = align_up(o + sizeof(float) * (size_t)r * (size_t)k * (size_t)batch);
    // small problems run all operators in one launch and need these per operator; the large path per lane
    const size_t per_op = (k + n <= kSmallMax) ? (size_t)r : (size_t)M.lanes;
    M.off_gyq = o;     o = align_up(o + sizeof(float) * per_op * (size_t)k * (size_t)batch);
    M.off_gxq = o;     o = align_up(o + sizeof(float) * per_op * (size_t)n * (size_t)batch);
    M.off_gxp = o;     if (M.lanes > 1) o = align_up(o + sizeof(float) * (size_t)M.lanes * (size_t)n * (size_t)batch);   // the lanes' sums of gx
    const size_t dots = (size_t)M.lanes * kTauPartials > (size_t)r * kDotGroups ? (size_t)M.lanes * kTauPartials : (size_t)r * kDotGroups;
    M.off_partial = o; o = align_up(o + sizeof(float) * dots);
    M.total = o;
    return M;
}

constexpr int kMaxDevices = 64;

// The lanes' streams (default priority, not synchronising with the null stream) and the events that fork them from the
// caller's stream and join them back: created on a device's first use, kept until the process ends.
struct MixStreams {
    hipStream_t lane[kMixLanes];
    hipEvent_t fork, join[kMixLanes];
};
std::mutex g_mix_mutex;             // held while a call enqueues on the lanes: the events are shared
MixStreams* g_mix_streams[kMaxDevices] = {};

// The current device's lanes, or null when the work has to stay on the caller's stream: a stream that is being captured
// (the lanes are not part of the caller's graph), or streams that could not be created.  Call with g_mix_mutex held.
MixStreams* mix_streams(hipStream_t caller)
{
    hipStreamCaptureStatus capture = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(caller, &capture) != hipSuccess) { (void)hipGetLastError(); return nullptr; }
    if (capture != hipStreamCaptureStatusNone) return nullptr;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) { (void)hipGetLastError(); return nullptr; }
    if (!g_mix_streams[dev]) {
        MixStreams* m = new MixStreams();
        bool ok = hipEventCreateWithFlags(&m->fork, hipEventDisableTiming) == hipSuccess;
        for (int l = 0; ok && l < kMixLanes; ++l)
            ok = hipStreamCreateWithFlags(&m->lane[l], hipStreamNonBlocking) == hipSuccess &&
                 hipEventCreateWithFlags(&m->join[l], hipEventDisableTiming) == hipSuccess;
        if (!ok) { (void)hipGetLastError(); delete m; return nullptr; }      // (what was created stays: a handful of handles, once)
        g_mix_streams[dev] = m;
    }
    return g_mix_streams[dev];
}

// The lanes start after everything the caller's stream holds so far ...
hipError_t mix_fork(MixStreams* m, int lanes, hipStream_t caller)
{
    hipError_t e = hipEventRecord(m->fork, caller);
    for (int l = 0; e == hipSuccess && l < lanes; ++l) e = hipStreamWaitEvent(m->lane[l], m->fork, 0);
    return e;
}
// ... and the caller's stream goes on after everything the lanes hold.
hipError_t mix_join(MixStreams* m, int lanes, hipStream_t caller)
{
    hipError_t e = hipSuccess;
    for (int l = 0; e == hipSuccess && l < lanes; ++l) {
        e = hipEventRecord(m->join[l], m->lane[l]);
        if (e == hipSuccess) e = hipStreamWaitEvent(caller, m->join[l], 0);
    }
    return e;
}

int check_mix_sizes(int64_t r, int64_t k, int64_t n, int64_t batch)
{
    if (r < 0 || r > LAPLEX_MIX_MAX_OPERATORS) return LAPLEX_ERR_SIZE;
    return check_sizes(k, n, batch);
}

}  // namespace

extern "C" {

int laplex_workspace_bytes(int64_t k, int64_t n, int64_t batch, size_t* out)
{
    if (!out) return LAPLEX_ERR_NULL;
    LAPLEX_CHECK(check_sizes(k, n, batch));
    // k == 0 is the Gram form: its saved-scan region has one row per anchor
    *out = make_layout(k + n, k == 0 ? n : k, batch).total;
    return LAPLEX_OK;
}

// Host checks of the forward apply's arguments (everything but the workspace).
static int apply_check(const float* a, int64_t k, const float* b, int64_t n,
                       const float* x, int64_t ldx, int64_t batch, const float* y, int64_t ldy, uint32_t flags)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_sizes(k, n, batch));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, true));
    LAPLEX_CHECK(check_matrix(y, k, ldy, batch, true));
    return LAPLEX_OK;
}

static int apply_impl(const float* a, int64_t k, const float* b, int64_t n,
                 const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                 void* ws, size_t ws_bytes, uint32_t flags, float tau, laplex_stream_t stream,
                 const PhaseIn* pin = nullptr)
{
    LAPLEX_CHECK(apply_check(a, k, b, n, x, ldx, batch, y, ldy, flags));
    if (k == 0 || batch == 0) return LAPLEX_OK;
    const Layout L = make_layout(k + n, k, batch);
    LAPLEX_CHECK(check_ws(ws, ws_bytes, L));
    char* w = static_cast<char*>(ws);
    const Plan P = plan_of(L, w);
    hipStream_t st = stream;
    if (n == 0) {
        LAPLEX_HIP(launch_fill(y, k, batch, ldy, 0.0f, st));
        if (flags & LAPLEX_SAVE_SCANS) LAPLEX_HIP(launch_fill(P.z, k, batch, batch, 0.0f, st));
        return LAPLEX_OK;
    }
    if (L.N <= kSmallMax) {        // sort, decays, both scans and the scatter in one launch
        SmallArgs S = small_args(a, k, b, n, tau, P, L, flags);
        S.nprob = 1;
        SmallProblem& q = S.prob[0];
        q.inj = x; q.ld_inj = ldx; q.inj_lo = (uint32_t)k; q.inj_hi = (uint32_t)(k + n);
        q.res_lo = 0; q.res_hi = (uint32_t)k;
        q.out_p = y; q.ld_p = ldy;
        q.out_z = (flags & LAPLEX_SAVE_SCANS) ? P.z : nullptr;
        LAPLEX_HIP(launch_small(S, 1, st));
        return LAPLEX_OK;
    }
    const bool sorted = (flags & LAPLEX_A_SORTED) && (flags & LAPLEX_B_SORTED);
    LAPLEX_CHECK(build_plan(a, k, b, n, tau, L, w, flags, sorted, st));
    ScanProblem p = problem(P, L);
    p.inj = x; p.ld_inj = ldx; p.inj_lo = (uint32_t)k; p.inj_hi = (uint32_t)(k + n);
    p.res_lo = 0; p.res_hi = (uint32_t)k;
    p.out_p = y; p.ld_p = ldy;
    p.out_z = (flags & LAPLEX_SAVE_SCANS) ? P.z : nullptr;
    p.stage = (flags & LAPLEX_SAVE_SCANS) ? P.xs : P.stage;   // kept for the backward's weights when saving
    p.tag = "fwd";
    p.phase_in = pin;             // phased: x is modulated on the way into the reduce (see phase_fusable)
    if (use_permute(L)) {          // x into sorted order, the scans there, y (and the saved scans) home
        LAPLEX_CHECK(rows_to_sorted(L, w, x, ldx, k, n, p.stage, "fwd", st));
        const bool save = p.out_z != nullptr;
        p.out_p = nullptr; p.out_z = nullptr;
        return scan_and_send_home(p, L, w, true, save, y, ldy, save ? P.z : nullptr, 1, st);
    }
    float* const pairs = reinterpret_cast<float*>(w + L.off_pair);
    const bool paired = batch == 1 && p.out_z != nullptr;      // y and the saved scan of a row as one 8-byte slot
    if (paired) { p.out_p = pairs; p.ld_p = 2; p.out_z = pairs + 1; p.ld_z = 2; }
    LAPLEX_HIP(launch_scan(p, L, w, st));
    if (paired) LAPLEX_HIP(launch_unpair(pairs, k, y, ldy, P.z, st));
    return LAPLEX_OK;
}

static int apply_backward_impl(const float* a, int64_t k, const float* b, int64_t n,
                          const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                          float* gx, int64_t ldgx, float* ga, float* gb,
                          void* ws, size_t ws_bytes, uint32_t flags, float tau, float* gtau, laplex_stream_t stream,
                          const PhaseFuse* fuse = nullptr, const PhaseIn* pin_fwd = nullptr, const PhaseIn* pin_bwd = nullptr)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_sizes(k, n, batch));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, ga || gb));
    LAPLEX_CHECK(check_matrix(gy, k, ldgy, batch, true));
    LAPLEX_CHECK(check_matrix(gx, n, ldgx, batch, false));
    LAPLEX_CHECK(check_vector(ga, k, false));
    LAPLEX_CHECK(check_vector(gb, n, false));
    LAPLEX_CHECK(check_vector(gtau, 1, false));
    if (gtau && ((!ga && k > 0) || (!gb && n > 0))) return LAPLEX_ERR_NULL;   // the temperature gradient is formed from ga and gb
    const Layout L = make_layout(k + n, k, batch);
    const bool degenerate = k == 0 || n == 0 || batch == 0;
    if (!degenerate) LAPLEX_CHECK(check_ws(ws, ws_bytes, L));
    hipStream_t st = stream;
    if (degenerate) {   // one side is empty: every wanted gradient is zero
        if (gx) LAPLEX_HIP(launch_fill(gx, n, batch, ldgx, 0.0f, st));
        if (ga) LAPLEX_HIP(launch_fill(ga, k, 1, 1, 0.0f, st));
        if (gb) LAPLEX_HIP(launch_fill(gb, n, 1, 1, 0.0f, st));
        if (gtau) LAPLEX_HIP(launch_fill(gtau, 1, 1, 1, 0.0f, st));
        return LAPLEX_OK;
    }
    char* w = static_cast<char*>(ws);
    const Plan P = plan_of(L, w);
    if (L.N <= kSmallMax) {        // one launch for the sort and both scan problems, then the two row reductions
        SmallArgs S = small_args(a, k, b, n, tau, P, L, flags);
        float* zg = reinterpret_cast<float*>(w + L.off_small);
        if (ga && !(flags & LAPLEX_SAVE_SCANS)) {     // strict scans of x at the outputs, not kept by the forward
            SmallProblem& q = S.prob[S.nprob++];
            q.inj = x; q.ld_inj = ldx; q.inj_lo = (uint32_t)k; q.inj_hi = (uint32_t)(k + n);
            q.res_lo = 0; q.res_hi = (uint32_t)k;
            q.out_z = P.z;
        }
        if (gx || gb) {
            SmallProblem& q = S.prob[S.nprob++];
            q.inj = gy; q.ld_inj = ldgy; q.inj_lo = 0; q.inj_hi = (uint32_t)k;
            q.res_lo = (uint32_t)k; q.res_hi = (uint32_t)(k + n);
            q.out_p = gx; q.ld_p = ldgx;
            q.out_z = gb ? zg : nullptr;
        }
        if (S.nprob > 0) LAPLEX_HIP(launch_small(S, 1, st));
        if (ga) LAPLEX_HIP(launch_rowdot(gy, ldgy, P.z, batch, k, batch, ga, st));
        if (gb) LAPLEX_HIP(launch_rowdot(x, ldx, zg, batch, n, batch, gb, st));
        if (gtau) LAPLEX_HIP(launch_tau_grad(a, ga, k, b, gb, n, reinterpret_cast<float*>(w + L.off_scratch), gtau, st));
        if (tau != 1.0f) {
            if (ga) LAPLEX_HIP(launch_scale(ga, k, tau, st));
            if (gb) LAPLEX_HIP(launch_scale(gb, n, tau, st));
        }
        return LAPLEX_OK;
    }
    const bool sorted = (flags & LAPLEX_A_SORTED) && (flags & LAPLEX_B_SORTED);
    LAPLEX_CHECK(build_plan(a, k, b, n, tau, L, w, flags, sorted, st));
    const bool routed = use_permute(L);        // batch 1, many rows: no random accesses (see rows_to_sorted)
    if (ga) {
        if (!(flags & LAPLEX_SAVE_SCANS)) {   // strict scans of x at the outputs, not kept by the forward
            ScanProblem p = problem(P, L);
            p.inj = x; p.ld_inj = ldx; p.inj_lo = (uint32_t)k; p.inj_hi = (uint32_t)(k + n);
            p.res_lo = 0; p.res_hi = (uint32_t)k;
            p.out_z = P.z;
            p.stage = P.xs;
            p.tag = "rescan";
            p.phase_in = pin_fwd;
            if (routed) {
                LAPLEX_CHECK(rows_to_sorted(L, w, x, ldx, k, n, P.xs, "rescan", st));
                p.out_z = nullptr;
                LAPLEX_CHECK(scan_and_send_home(p, L, w, false, true, P.z, 1, nullptr, 1, st));
            } else {
                LAPLEX_HIP(launch_scan(p, L, w, st));
            }
        }
        LAPLEX_HIP(launch_rowdot(gy, ldgy, P.z, batch, k, batch, ga, st));
    }
    // sorted-order x is in the saved region if the forward kept it or the re-scan above just wrote it
    const bool have_xs = (flags & LAPLEX_SAVE_SCANS) || ga;
    if (routed && (gx || gb)) {
        if (gb && !have_xs) LAPLEX_CHECK(rows_to_sorted(L, w, x, ldx, k, n, P.xs, "bwd_x", st));    // the weights of gb
        LAPLEX_CHECK(rows_to_sorted(L, w, gy, ldgy, 0, k, P.stage, "bwd", st));
        ScanProblem p = problem(P, L);
        p.inj = gy; p.ld_inj = ldgy; p.inj_lo = 0; p.inj_hi = (uint32_t)k;
        p.res_lo = (uint32_t)k; p.res_hi = (uint32_t)(k + n);
        p.stage = P.stage;
        if (gb) { p.w = x; p.ld_w = ldx; p.wstage = P.xs; }      // the second output of an input row: x * Z = its gb
        p.tag = "bwd";
        if (gx) LAPLEX_CHECK(scan_and_send_home(p, L, w, true, gb != nullptr, gx, ldgx, gb, 1, st));
        else LAPLEX_CHECK(scan_and_send_home(p, L, w, false, true, gb, 1, nullptr, 1, st));
    } else if (gx || gb) {
        ScanProblem p = problem(P, L);
        p.inj = gy; p.ld_inj = ldgy; p.inj_lo = 0; p.inj_hi = (uint32_t)k;
        p.res_lo = (uint32_t)k; p.res_hi = (uint32_t)(k + n);
        p.out_p = gx; p.ld_p = ldgx;
        p.out_red = gb; p.w = x; p.ld_w = ldx;
        float* const pairs = reinterpret_cast<float*>(w + L.off_pair);
        const bool paired = batch == 1 && gx && gb;        // gx and gb of a row as one 8-byte slot
        if (paired) { p.out_p = pairs; p.ld_p = 2; p.out_red = pairs + 1; p.ld_red = 2; }
        p.stage = P.stage;
        p.wstage = (gb && have_xs) ? P.xs : nullptr;
        p.tag = "bwd";
        p.phase = fuse;           // phased backward: the streaming downsweep merges the two halves (see phase_fusable)
        p.phase_in = pin_bwd;     // ... and the other downsweeps' blocks get their doubled weight rows
        LAPLEX_HIP(launch_scan(p, L, w, st));
        if (paired) LAPLEX_HIP(launch_unpair(pairs, n, gx, ldgx, gb, st));
    }
    // the scans gave the gradients with respect to the scaled anchors
    if (gtau) LAPLEX_HIP(launch_tau_grad(a, ga, k, b, gb, n, reinterpret_cast<float*>(w + L.off_scratch), gtau, st));
    if (tau != 1.0f) {
        if (ga) LAPLEX_HIP(launch_scale(ga, k, tau, st));
        if (gb) LAPLEX_HIP(launch_scale(gb, n, tau, st));
    }
    return LAPLEX_OK;
}

static int gram_impl(const float* a, int64_t n, const float* x, int64_t ldx, int64_t batch,
                float* y, int64_t ldy, void* ws, size_t ws_bytes, uint32_t flags, float tau, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_sizes(0, n, batch));
    LAPLEX_CHECK(check_vector(a, n, true));
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, true));
    LAPLEX_CHECK(check_matrix(y, n, ldy, batch, true));
    if (n == 0 || batch == 0) return LAPLEX_OK;
    const Layout L = make_layout(n, n, batch);
    LAPLEX_CHECK(check_ws(ws, ws_bytes, L));
    char* w = static_cast<char*>(ws);
    const Plan P = plan_of(L, w);
    hipStream_t st = stream;
    if (L.N <= kSmallMax) {        // the two-launch path for small problems
        SmallArgs S = small_args(a, n, nullptr, 0, tau, P, L, flags);
        S.nprob = 1;
        SmallProblem& q = S.prob[0];
        q.inj = x; q.ld_inj = ldx; q.inj_lo = 0; q.inj_hi = (uint32_t)n;
        q.res_lo = 0; q.res_hi = (uint32_t)n;
        q.out_p = y; q.ld_p = ldy;
        q.out_z = (flags & LAPLEX_SAVE_SCANS) ? P.z : nullptr;
        LAPLEX_HIP(launch_small(S, 1, st));
        return LAPLEX_OK;
    }
    LAPLEX_CHECK(build_plan(a, n, nullptr, 0, tau, L, w, flags, (flags & LAPLEX_A_SORTED) != 0, st));
    ScanProblem p = problem(P, L);
    p.inj = x; p.ld_inj = ldx; p.inj_lo = 0; p.inj_hi = (uint32_t)n;
    p.res_lo = 0; p.res_hi = (uint32_t)n;
    p.out_p = y; p.ld_p = ldy;
    p.out_z = (flags & LAPLEX_SAVE_SCANS) ? P.z : nullptr;
    float* const pairs = reinterpret_cast<float*>(w + L.off_pair);
    const bool paired = batch == 1 && p.out_z != nullptr;
    if (paired) { p.out_p = pairs; p.ld_p = 2; p.out_z = pairs + 1; p.ld_z = 2; }
    p.stage = (flags & LAPLEX_SAVE_SCANS) ? P.xs : P.stage;
    p.tag = "fwd";
    if (use_permute(L)) {          // batch 1, many rows: x into sorted order, the scans there, y (and the saved scans) home
        const bool save = (flags & LAPLEX_SAVE_SCANS) != 0;
        LAPLEX_CHECK(rows_to_sorted(L, w, x, ldx, 0, n, p.stage, "fwd", st));
        p.out_p = nullptr; p.out_z = nullptr; p.ld_p = 0; p.ld_z = 0;
        return scan_and_send_home(p, L, w, true, save, y, ldy, save ? P.z : nullptr, 1, st);
    }
    LAPLEX_HIP(launch_scan(p, L, w, st));
    if (paired) LAPLEX_HIP(launch_unpair(pairs, n, y, ldy, P.z, st));
    return LAPLEX_OK;
}

static int gram_backward_impl(const float* a, int64_t n, const float* x, int64_t ldx,
                         const float* gy, int64_t ldgy, int64_t batch, float* gx, int64_t ldgx, float* ga,
                         void* ws, size_t ws_bytes, uint32_t flags, float tau, float* gtau, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_sizes(0, n, batch));
    LAPLEX_CHECK(check_vector(a, n, true));
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, ga != nullptr));
    LAPLEX_CHECK(check_matrix(gy, n, ldgy, batch, true));
    LAPLEX_CHECK(check_matrix(gx, n, ldgx, batch, false));
    LAPLEX_CHECK(check_vector(ga, n, false));
    LAPLEX_CHECK(check_vector(gtau, 1, false));
    if (gtau && !ga && n > 0) return LAPLEX_ERR_NULL;      // the temperature gradient is formed from ga
    hipStream_t st = stream;
    if (n == 0) {
        if (gtau) LAPLEX_HIP(launch_fill(gtau, 1, 1, 1, 0.0f, st));
        return LAPLEX_OK;
    }
    if (batch == 0) {
        if (ga) LAPLEX_HIP(launch_fill(ga, n, 1, 1, 0.0f, st));
        if (gtau) LAPLEX_HIP(launch_fill(gtau, 1, 1, 1, 0.0f, st));
        return LAPLEX_OK;
    }
    const Layout L = make_layout(n, n, batch);
    LAPLEX_CHECK(check_ws(ws, ws_bytes, L));
    char* w = static_cast<char*>(ws);
    const Plan P = plan_of(L, w);
    if (L.N <= kSmallMax) {        // the two-launch path for small problems, then one row reduction
        SmallArgs S = small_args(a, n, nullptr, 0, tau, P, L, flags);
        float* zg = reinterpret_cast<float*>(w + L.off_small);
        if (ga && !(flags & LAPLEX_SAVE_SCANS)) {
            SmallProblem& q = S.prob[S.nprob++];
            q.inj = x; q.ld_inj = ldx; q.inj_lo = 0; q.inj_hi = (uint32_t)n;
            q.res_lo = 0; q.res_hi = (uint32_t)n;
            q.out_z = P.z;
        }
        if (gx || ga) {
            SmallProblem& q = S.prob[S.nprob++];
            q.inj = gy; q.ld_inj = ldgy; q.inj_lo = 0; q.inj_hi = (uint32_t)n;
            q.res_lo = 0; q.res_hi = (uint32_t)n;
            q.out_p = gx; q.ld_p = ldgx;
            q.out_z = ga ? zg : nullptr;
        }
        if (S.nprob > 0) LAPLEX_HIP(launch_small(S, 1, st));
        if (ga) LAPLEX_HIP(launch_rowdot2(gy, ldgy, P.z, batch, x, ldx, zg, batch, n, batch, ga, st));
        if (gtau) LAPLEX_HIP(launch_tau_grad(a, ga, n, nullptr, nullptr, 0, reinterpret_cast<float*>(w + L.off_scratch), gtau, st));
        if (tau != 1.0f && ga) LAPLEX_HIP(launch_scale(ga, n, tau, st));
        return LAPLEX_OK;
    }
    LAPLEX_CHECK(build_plan(a, n, nullptr, 0, tau, L, w, flags, (flags & LAPLEX_A_SORTED) != 0, st));
    const bool routed = use_permute(L);        // batch 1, many rows: no random accesses (see rows_to_sorted)
    if (ga && !(flags & LAPLEX_SAVE_SCANS)) {
        ScanProblem p = problem(P, L);
        p.inj = x; p.ld_inj = ldx; p.inj_lo = 0; p.inj_hi = (uint32_t)n;
        p.res_lo = 0; p.res_hi = (uint32_t)n;
        p.out_z = P.z;
        p.stage = P.xs;
        p.tag = "rescan";
        if (routed) {
            LAPLEX_CHECK(rows_to_sorted(L, w, x, ldx, 0, n, P.xs, "rescan", st));
            p.out_z = nullptr;
            LAPLEX_CHECK(scan_and_send_home(p, L, w, false, true, P.z, 1, nullptr, 1, st));
        } else {
            LAPLEX_HIP(launch_scan(p, L, w, st));
        }
    }
    if (routed && (gx || ga)) {
        // gx and x * Z^g leave the downsweep together (the second as the row's second output, into ga); the saved scans of x
        // are in the caller's order already, so  ga = x Z^g + gy Z^x  is completed by one pointwise pass
        LAPLEX_CHECK(rows_to_sorted(L, w, gy, ldgy, 0, n, P.stage, "bwd", st));
        ScanProblem p = problem(P, L);
        p.inj = gy; p.ld_inj = ldgy; p.inj_lo = 0; p.inj_hi = (uint32_t)n;
        p.res_lo = 0; p.res_hi = (uint32_t)n;
        p.stage = P.stage;
        if (ga) { p.w = x; p.ld_w = ldx; p.wstage = P.xs; }     // (sorted-order x: kept by the forward or just written by the re-scan)
        p.tag = "bwd";
        if (gx) LAPLEX_CHECK(scan_and_send_home(p, L, w, true, ga != nullptr, gx, ldgx, ga, 1, st));
        else LAPLEX_CHECK(scan_and_send_home(p, L, w, false, true, ga, 1, nullptr, 1, st));
        if (ga) LAPLEX_HIP(launch_add_rowdot(gy, ldgy, P.z, batch, n, batch, ga, st));
    } else if (gx || ga) {
        ScanProblem p = problem(P, L);
        p.inj = gy; p.ld_inj = ldgy; p.inj_lo = 0; p.inj_hi = (uint32_t)n;
        p.res_lo = 0; p.res_hi = (uint32_t)n;
        p.out_p = gx; p.ld_p = ldgx;
        p.out_red = ga; p.w = x; p.ld_w = ldx; p.zs = ga ? P.z : nullptr;
        float* const pairs = reinterpret_cast<float*>(w + L.off_pair);
        const bool paired = batch == 1 && gx && ga;
        if (paired) { p.out_p = pairs; p.ld_p = 2; p.out_red = pairs + 1; p.ld_red = 2; }
        p.stage = P.stage;
        p.wstage = ga ? P.xs : nullptr;     // kept by the forward (SAVE_SCANS) or just written by the re-scan
        p.tag = "bwd";
        LAPLEX_HIP(launch_scan(p, L, w, st));
        if (paired) LAPLEX_HIP(launch_unpair(pairs, n, gx, ldgx, ga, st));
    }
    if (gtau) LAPLEX_HIP(launch_tau_grad(a, ga, n, nullptr, nullptr, 0, reinterpret_cast<float*>(w + L.off_scratch), gtau, st));
    if (tau != 1.0f && ga) LAPLEX_HIP(launch_scale(ga, n, tau, st));
    return LAPLEX_OK;
}

// Inverse temperature must be a positive finite number.
static int check_tau(float tau) { return (tau > 0.0f && tau < INFINITY) ? LAPLEX_OK : LAPLEX_ERR_VALUE; }

int laplex_apply(const float* a, int64_t k, const float* b, int64_t n,
                 const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                 void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    return apply_impl(a, k, b, n, x, ldx, batch, y, ldy, ws, ws_bytes, flags, 1.0f, stream);
}

// The workspace of laplex_apply_static: one copy per device, held from the moment the library is loaded on it.
// In host code the array's name is only a handle; its device address is looked up once per device.
static __device__ __align__(256) unsigned char scratch[LAPLEX_STATIC_WORKSPACE_BYTES];

namespace {
std::mutex g_scratch_mutex;
void* g_scratch_ptr[kMaxDevices] = {};

// Address of the current device's copy of `scratch` (looked up on the first call on that device).
int static_scratch(void** out)
{
    int dev = -1;
    LAPLEX_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= kMaxDevices) return hip_fail(hipErrorInvalidDevice);
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        LAPLEX_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p) return hip_fail(hipErrorInvalidSymbol);
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return LAPLEX_OK;
}
}  // namespace

int laplex_apply_static(const float* a, int64_t k, const float* b, int64_t n,
                        const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                        uint32_t flags, laplex_stream_t stream)
{
    if (flags & ~(uint32_t)(LAPLEX_A_SORTED | LAPLEX_B_SORTED)) return LAPLEX_ERR_FLAGS;
    // every argument error, and a problem that does not fit the array, is reported before any HIP call
    LAPLEX_CHECK(apply_check(a, k, b, n, x, ldx, batch, y, ldy, flags));
    if (k == 0 || batch == 0) return LAPLEX_OK;
    if (make_layout(k + n, k, batch).total > LAPLEX_STATIC_WORKSPACE_BYTES) return LAPLEX_ERR_WORKSPACE;
    void* ws = nullptr;
    LAPLEX_CHECK(static_scratch(&ws));
    // every kernel takes the looked-up address, as it takes the caller's workspace in laplex_apply
    return apply_impl(a, k, b, n, x, ldx, batch, y, ldy, ws, LAPLEX_STATIC_WORKSPACE_BYTES, flags, 1.0f, stream);
}

int laplex_apply_backward(const float* a, int64_t k, const float* b, int64_t n,
                          const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                          float* gx, int64_t ldgx, float* ga, float* gb,
                          void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    return apply_backward_impl(a, k, b, n, x, ldx, gy, ldgy, batch, gx, ldgx, ga, gb, ws, ws_bytes, flags, 1.0f, nullptr, stream);
}

int laplex_gram(const float* a, int64_t n, const float* x, int64_t ldx, int64_t batch,
                float* y, int64_t ldy, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    return gram_impl(a, n, x, ldx, batch, y, ldy, ws, ws_bytes, flags, 1.0f, stream);
}

int laplex_gram_backward(const float* a, int64_t n, const float* x, int64_t ldx,
                         const float* gy, int64_t ldgy, int64_t batch, float* gx, int64_t ldgx, float* ga,
                         void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    return gram_backward_impl(a, n, x, ldx, gy, ldgy, batch, gx, ldgx, ga, ws, ws_bytes, flags, 1.0f, nullptr, stream);
}

int laplex_apply_tau(const float* a, int64_t k, const float* b, int64_t n, float tau,
                     const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                     void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    LAPLEX_CHECK(check_tau(tau));
    return apply_impl(a, k, b, n, x, ldx, batch, y, ldy, ws, ws_bytes, flags, tau, stream);
}

int laplex_apply_backward_tau(const float* a, int64_t k, const float* b, int64_t n, float tau,
                              const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                              float* gx, int64_t ldgx, float* ga, float* gb, float* gtau,
                              void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    LAPLEX_CHECK(check_tau(tau));
    return apply_backward_impl(a, k, b, n, x, ldx, gy, ldgy, batch, gx, ldgx, ga, gb, ws, ws_bytes, flags, tau, gtau, stream);
}

int laplex_gram_tau(const float* a, int64_t n, float tau, const float* x, int64_t ldx, int64_t batch,
                    float* y, int64_t ldy, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    LAPLEX_CHECK(check_tau(tau));
    return gram_impl(a, n, x, ldx, batch, y, ldy, ws, ws_bytes, flags, tau, stream);
}

int laplex_gram_backward_tau(const float* a, int64_t n, float tau, const float* x, int64_t ldx,
                             const float* gy, int64_t ldgy, int64_t batch, float* gx, int64_t ldgx, float* ga, float* gtau,
                             void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    LAPLEX_CHECK(check_tau(tau));
    return gram_backward_impl(a, n, x, ldx, gy, ldgy, batch, gx, ldgx, ga, ws, ws_bytes, flags, tau, gtau, stream);
}

int laplex_phased_workspace_bytes(int64_t k, int64_t n, int64_t batch, size_t* out)
{
    if (!out) return LAPLEX_ERR_NULL;
    LAPLEX_CHECK(check_phased_sizes(k, n, batch));
    *out = phased_layout(k, n, batch).total;
    return LAPLEX_OK;
}

int laplex_phased_apply(const float* a, const float* phi, int64_t k, const float* b, const float* psi, int64_t n,
                        const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                        void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_phased_sizes(k, n, batch));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(phi, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    LAPLEX_CHECK(check_vector(psi, n, true));
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, true));
    LAPLEX_CHECK(check_matrix(y, k, ldy, batch, true));
    if (k == 0 || batch == 0) return LAPLEX_OK;
    hipStream_t st = stream;
    if (n == 0) {
        LAPLEX_HIP(launch_fill(y, k, batch, ldy, 0.0f, st));
        return LAPLEX_OK;
    }
    const PhasedLayout P = phased_layout(k, n, batch);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < P.total) return LAPLEX_ERR_WORKSPACE;
    char* w = static_cast<char*>(ws);
    float* x2 = reinterpret_cast<float*>(w + P.off_x2);
    float* y2 = reinterpret_cast<float*>(w + P.off_y2);
    // With a wide batch the reduce reads x itself and modulates it on the way in; only the rows of blocks that hold outputs
    // are written in doubled form (the other kernels read those).  Otherwise: one pass that writes both halves of x.
    const bool fus_in = phase_fusable(k, n, batch, x, ldx, nullptr, 0);
    uint32_t* const whole = reinterpret_cast<uint32_t*>(w + P.off_state);
    const PhaseIn pin{psi, x, ldx, x2, whole, batch, 1, true};
    if (!fus_in) LAPLEX_HIP(launch_phase_split(x, ldx, psi, n, batch, x2, st, whole));
    LAPLEX_CHECK(apply_impl(a, k, b, n, x2, 2 * batch, 2 * batch, y2, 2 * batch, ws, P.inner, flags, 1.0f, stream,
                            fus_in ? &pin : nullptr));
    LAPLEX_HIP(launch_phase_merge(y2, phi, k, batch, y, ldy, nullptr, 0, nullptr, st));
    return LAPLEX_OK;
}

int laplex_phased_apply_backward(const float* a, const float* phi, int64_t k, const float* b, const float* psi, int64_t n,
                                 const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                                 float* gx, int64_t ldgx, float* ga, float* gb, float* gphi, float* gpsi,
                                 void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_phased_sizes(k, n, batch));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(phi, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    LAPLEX_CHECK(check_vector(psi, n, true));
    const bool need_x = ga || gb || gphi || gpsi;
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, need_x));
    LAPLEX_CHECK(check_matrix(gy, k, ldgy, batch, true));
    LAPLEX_CHECK(check_matrix(gx, n, ldgx, batch, false));
    LAPLEX_CHECK(check_vector(ga, k, false));
    LAPLEX_CHECK(check_vector(gb, n, false));
    LAPLEX_CHECK(check_vector(gphi, k, false));
    LAPLEX_CHECK(check_vector(gpsi, n, false));
    hipStream_t st = stream;
    if (k == 0 || n == 0 || batch == 0) {      // one side is empty: every wanted gradient is zero
        if (gx) LAPLEX_HIP(launch_fill(gx, n, batch, ldgx, 0.0f, st));
        if (ga) LAPLEX_HIP(launch_fill(ga, k, 1, 1, 0.0f, st));
        if (gb) LAPLEX_HIP(launch_fill(gb, n, 1, 1, 0.0f, st));
        if (gphi) LAPLEX_HIP(launch_fill(gphi, k, 1, 1, 0.0f, st));
        if (gpsi) LAPLEX_HIP(launch_fill(gpsi, n, 1, 1, 0.0f, st));
        return LAPLEX_OK;
    }
    const PhasedLayout P = phased_layout(k, n, batch);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < P.total) return LAPLEX_ERR_WORKSPACE;
    char* w = static_cast<char*>(ws);
    float* x2 = reinterpret_cast<float*>(w + P.off_x2);
    float* y2 = reinterpret_cast<float*>(w + P.off_y2);
    float* g2 = reinterpret_cast<float*>(w + P.off_g2);
    float* gx2 = reinterpret_cast<float*>(w + P.off_gx2);
    const bool saved = (flags & LAPLEX_SAVE_SCANS) != 0;      // the forward left x's halves (see below), its product and its scans
    const bool want_gx2 = gx || gpsi;
    // With a wide batch (phase_fusable) nothing reads the doubled copy of x as a whole: the reduce of a forward problem
    // modulates x on the way in (fus_in), and the streaming downsweep of the backward problem forms gx and gpsi itself and
    // takes gb's weights from x (fused); the doubled rows and the doubled result matrix exist only for the blocks the other
    // downsweeps own.  One consumer is left that needs all of it: the row reduction for gb when neither gx nor gpsi is asked for.
    const bool fus_in = x != nullptr && phase_fusable(k, n, batch, x, ldx, nullptr, 0);
    const bool fused = want_gx2 && phase_fusable(k, n, batch, x, ldx, gx, ldgx);
    const bool full_split = x != nullptr && (fus_in ? (gb != nullptr && !fused) : !saved);
    uint32_t* const whole = reinterpret_cast<uint32_t*>(w + P.off_state);
    if (full_split) {
        LAPLEX_HIP(launch_phase_split(x, ldx, psi, n, batch, x2, st, whole));
    } else if (x != nullptr && !fus_in) {
        // The forward left its doubled copy of x -- all of it, unless it was given rows that allowed it to read x itself
        // (another pointer or leading dimension than this call's): the copy's own word says which, and the pass runs if needed.
        LAPLEX_HIP(launch_phase_split(x, ldx, psi, n, batch, x2, st, whole, true));
        LAPLEX_HIP(launch_set_word(whole, 1u, st));
    }
    LAPLEX_HIP(launch_phase_split(gy, ldgy, phi, k, batch, g2, st));
    const PhaseIn pin_fwd{psi, x, ldx, x2, whole, batch, 1, true};
    const PhaseIn pin_bwd{psi, x, ldx, x2, nullptr, batch, 2, false};
    uint32_t inner = flags;
    if (gphi && !saved) {       // the phase gradient of the outputs needs the two halves of the product
        LAPLEX_CHECK(apply_impl(a, k, b, n, x2, 2 * batch, 2 * batch, y2, 2 * batch, ws, P.inner,
                                flags | LAPLEX_SAVE_SCANS, 1.0f, stream, fus_in ? &pin_fwd : nullptr));
        inner = flags | LAPLEX_SAVE_SCANS | LAPLEX_REUSE_PLAN;
    }
    const PhaseFuse fuse{psi, (gb || gpsi) ? x : nullptr, ldx, gx, ldgx, gpsi, batch};
    LAPLEX_CHECK(apply_backward_impl(a, k, b, n, x ? x2 : nullptr, 2 * batch, g2, 2 * batch, 2 * batch,
                                     want_gx2 ? gx2 : nullptr, 2 * batch, ga, gb, ws, P.inner, inner, 1.0f, nullptr, stream,
                                     fused ? &fuse : nullptr, fus_in ? &pin_fwd : nullptr,
                                     (fused && gb && x && !full_split) ? &pin_bwd : nullptr));
    if (want_gx2 && !fused) LAPLEX_HIP(launch_phase_merge(gx2, psi, n, batch, gx, ldgx, x, ldx, gpsi, st));
    if (gphi) LAPLEX_HIP(launch_phase_merge(y2, phi, k, batch, nullptr, 0, gy, ldgy, gphi, st));
    return LAPLEX_OK;
}

int laplex_wgram_workspace_bytes(int64_t k, int64_t n, size_t* out)
{
    if (!out) return LAPLEX_ERR_NULL;
    LAPLEX_CHECK(check_wgram_sizes(k, n));
    *out = wgram64_layout(k, n).total;
    return LAPLEX_OK;
}

int laplex_wgram(const float* a, int64_t k, const float* b, int64_t n, const float* d,
                 float* m, int64_t ldm, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_wgram_sizes(k, n));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    LAPLEX_CHECK(check_vector(d, k > 0 ? n : 0, true));
    LAPLEX_CHECK(check_matrix(m, k, ldm, k, true));
    if (k == 0) return LAPLEX_OK;
    hipStream_t st = stream;
    if (n == 0) {
        LAPLEX_HIP(launch_fill(m, k, k, ldm, 0.0f, st));
        return LAPLEX_OK;
    }
    const Wgram64Layout G = wgram64_layout(k, n);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < G.total) return LAPLEX_ERR_WORKSPACE;
    char* w = static_cast<char*>(ws);
    const Layout L = make_layout(k + n, k, 1, false);
    const Plan P = plan_of(L, w);
    // the plan of the doubled anchors: its decays are exp(-2 gap), the kernel K = L(2a) of the theorem
    LAPLEX_CHECK(build_wgram_plan(a, k, b, n, L, P, w, flags, st));
    LAPLEX_HIP(launch_wgram_f32(P.ids, P.pk, a, d, k, k + n, reinterpret_cast<double*>(w + G.off_summ),
                                reinterpret_cast<double*>(w + G.off_u), reinterpret_cast<double*>(w + G.off_v),
                                reinterpret_cast<double*>(w + G.off_w), reinterpret_cast<double*>(w + G.off_pb), m, ldm,
                                plan_status_word(L, w), st));
    return LAPLEX_OK;
}

int laplex_wgram_f64_workspace_bytes(int64_t k, int64_t n, size_t* out)
{
    if (!out) return LAPLEX_ERR_NULL;
    LAPLEX_CHECK(check_wgram_sizes(k, n));
    *out = wgram64_layout(k, n).total;
    return LAPLEX_OK;
}

int laplex_wgram_f64(const float* a, int64_t k, const float* b, int64_t n, const double* d,
                     double* m, int64_t ldm, void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_wgram_sizes(k, n));
    LAPLEX_CHECK(check_vector(a, k, true));
    LAPLEX_CHECK(check_vector(b, n, true));
    if (n > 0 && k > 0) {
        if (!d) return LAPLEX_ERR_NULL;
        if (misaligned(d, 8)) return LAPLEX_ERR_ALIGN;
    }
    if (k > 0) {
        if (!m) return LAPLEX_ERR_NULL;
        if (misaligned(m, 8)) return LAPLEX_ERR_ALIGN;
        if (ldm < k) return LAPLEX_ERR_LD;
    }
    if (k == 0) return LAPLEX_OK;
    hipStream_t st = stream;
    if (n == 0) {        // nothing is summed: a zero matrix (as fp32 pairs of zeros)
        LAPLEX_HIP(launch_fill(reinterpret_cast<float*>(m), k, 2 * k, 2 * ldm, 0.0f, st));
        return LAPLEX_OK;
    }
    const Wgram64Layout G = wgram64_layout(k, n);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < G.total) return LAPLEX_ERR_WORKSPACE;
    char* w = static_cast<char*>(ws);
    const Layout L = make_layout(k + n, k, 1, false);
    const Plan P = plan_of(L, w);
    LAPLEX_CHECK(build_wgram_plan(a, k, b, n, L, P, w, flags, st));
    LAPLEX_HIP(launch_wgram_f64(P.ids, P.pk, a, d, k, k + n, reinterpret_cast<double*>(w + G.off_summ),
                                reinterpret_cast<double*>(w + G.off_u), reinterpret_cast<double*>(w + G.off_v),
                                reinterpret_cast<double*>(w + G.off_w), reinterpret_cast<double*>(w + G.off_pb), m, ldm,
                                plan_status_word(L, w), st));
    return LAPLEX_OK;
}

int laplex_mix_workspace_bytes(int64_t r, int64_t k, int64_t n, int64_t batch, size_t* out)
{
    if (!out) return LAPLEX_ERR_NULL;
    LAPLEX_CHECK(check_mix_sizes(r, k, n, batch));
    *out = mix_layout(r, k, n, batch).total;
    return LAPLEX_OK;
}

int laplex_mix_apply(const float* a, const float* b, const float* w, int64_t r, int64_t k, int64_t n,
                     const float* x, int64_t ldx, int64_t batch, float* y, int64_t ldy,
                     void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_mix_sizes(r, k, n, batch));
    if (r > 0) {
        LAPLEX_CHECK(check_vector(a, k, true));
        LAPLEX_CHECK(check_vector(b, n, true));
        LAPLEX_CHECK(check_vector(w, r, true));
    }
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, r > 0));
    LAPLEX_CHECK(check_matrix(y, k, ldy, batch, true));
    if (k == 0 || batch == 0) return LAPLEX_OK;
    hipStream_t st = stream;
    if (n == 0 || r == 0) {
        LAPLEX_HIP(launch_fill(y, k, batch, ldy, 0.0f, st));
        return LAPLEX_OK;
    }
    const MixLayout M = mix_layout(r, k, n, batch);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < M.total) return LAPLEX_ERR_WORKSPACE;
    char* base = static_cast<char*>(ws);
    float* parts = reinterpret_cast<float*>(base + M.off_parts);
    if (k + n <= kSmallMax) {      // every operator in the same two launches
        const Layout L = make_layout(k + n, k, batch);
        const Plan P = plan_of(L, base);
        SmallArgs S = small_args(a, k, b, n, 1.0f, P, L, flags);
        S.op_a = k; S.op_b = n; S.op_ws = (int64_t)M.inner;
        S.nprob = 1;
        SmallProblem& q = S.prob[0];
        q.inj = x; q.ld_inj = ldx; q.inj_lo = (uint32_t)k; q.inj_hi = (uint32_t)(k + n);
        q.res_lo = 0; q.res_hi = (uint32_t)k;
        q.out_p = parts; q.ld_p = batch; q.op_p = k * batch;
        q.out_z = (flags & LAPLEX_SAVE_SCANS) ? P.z : nullptr; q.op_z = (int64_t)(M.inner / sizeof(float));
        LAPLEX_HIP(launch_small(S, r, st));
    } else {
        std::unique_lock<std::mutex> lock(g_mix_mutex, std::defer_lock);
        MixStreams* lanes = nullptr;
        if (M.lanes > 1) { lock.lock(); lanes = mix_streams(st); }
        if (lanes) LAPLEX_HIP(mix_fork(lanes, M.lanes, st));
        for (int64_t q = 0; q < r; ++q)
            LAPLEX_CHECK(laplex_apply(a + q * k, k, b + q * n, n, x, ldx, batch, parts + q * k * batch, batch,
                                      base + (size_t)q * M.inner, M.inner, flags, lanes ? lanes->lane[q % M.lanes] : stream));
        if (lanes) LAPLEX_HIP(mix_join(lanes, M.lanes, st));
    }
    LAPLEX_HIP(launch_mix_combine(parts, w, r, k, batch, y, ldy, st));
    return LAPLEX_OK;
}

int laplex_mix_apply_backward(const float* a, const float* b, const float* w, int64_t r, int64_t k, int64_t n,
                              const float* x, int64_t ldx, const float* gy, int64_t ldgy, int64_t batch,
                              float* gx, int64_t ldgx, float* ga, float* gb, float* gw,
                              void* ws, size_t ws_bytes, uint32_t flags, laplex_stream_t stream)
{
    const uint32_t known = LAPLEX_A_SORTED | LAPLEX_B_SORTED | LAPLEX_REUSE_PLAN | LAPLEX_SAVE_SCANS;
    if (flags & ~known) return LAPLEX_ERR_FLAGS;
    LAPLEX_CHECK(check_mix_sizes(r, k, n, batch));
    if (r > 0) {
        LAPLEX_CHECK(check_vector(a, k, true));
        LAPLEX_CHECK(check_vector(b, n, true));
        LAPLEX_CHECK(check_vector(w, r, true));
    }
    const bool need_x = r > 0 && (ga || gb || gw);
    LAPLEX_CHECK(check_matrix(x, n, ldx, batch, need_x));
    LAPLEX_CHECK(check_matrix(gy, k, ldgy, batch, r > 0));
    LAPLEX_CHECK(check_matrix(gx, n, ldgx, batch, false));
    LAPLEX_CHECK(check_vector(ga, r > 0 ? k : 0, false));
    LAPLEX_CHECK(check_vector(gb, r > 0 ? n : 0, false));
    LAPLEX_CHECK(check_vector(gw, r, false));
    hipStream_t st = stream;
    if (r == 0 || k == 0 || n == 0 || batch == 0) {      // nothing is summed: every wanted gradient is zero
        if (gx) LAPLEX_HIP(launch_fill(gx, n, batch, ldgx, 0.0f, st));
        if (ga) LAPLEX_HIP(launch_fill(ga, r * k, 1, 1, 0.0f, st));
        if (gb) LAPLEX_HIP(launch_fill(gb, r * n, 1, 1, 0.0f, st));
        if (gw) LAPLEX_HIP(launch_fill(gw, r, 1, 1, 0.0f, st));
        return LAPLEX_OK;
    }
    const MixLayout M = mix_layout(r, k, n, batch);
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < M.total) return LAPLEX_ERR_WORKSPACE;
    char* base = static_cast<char*>(ws);
    float* parts = reinterpret_cast<float*>(base + M.off_parts);
    float* gyq = reinterpret_cast<float*>(base + M.off_gyq);
    float* gxq = reinterpret_cast<float*>(base + M.off_gxq);
    float* partial = reinterpret_cast<float*>(base + M.off_partial);
    const bool saved = (flags & LAPLEX_SAVE_SCANS) != 0;      // the forward left every operator's product and scans
    if (k + n <= kSmallMax) {      // every operator in the same launches
        const Layout L = make_layout(k + n, k, batch);
        const Plan P = plan_of(L, base);
        const int64_t op_f = (int64_t)(M.inner / sizeof(float));
        float* zg = reinterpret_cast<float*>(base + L.off_small);
        bool have_plan = (flags & LAPLEX_REUSE_PLAN) != 0;
        bool have_z = saved;
        if (gw && !saved) {        // the weights' gradients need the operators' own products (and leave the strict scans)
            SmallArgs S = small_args(a, k, b, n, 1.0f, P, L, flags);
            S.op_a = k; S.op_b = n; S.op_ws = (int64_t)M.inner;
            S.nprob = 1;
            SmallProblem& q = S.prob[0];
            q.inj = x; q.ld_inj = ldx; q.inj_lo = (uint32_t)k; q.inj_hi = (uint32_t)(k + n);
            q.res_lo = 0; q.res_hi = (uint32_t)k;
            q.out_p = parts; q.ld_p = batch; q.op_p = k * batch;
            q.out_z = P.z; q.op_z = op_f;
            LAPLEX_HIP(launch_small(S, r, st));
            have_plan = true; have_z = true;
        }
        if (gx || ga || gb) {
            LAPLEX_HIP(launch_scale_ops(gy, ldgy, w, r, k, batch, gyq, st));      // gyq[q] = w_q gy
            SmallArgs S = small_args(a, k, b, n, 1.0f, P, L, have_plan ? (flags | LAPLEX_REUSE_PLAN) : flags);
            S.op_a = k; S.op_b = n; S.op_ws = (int64_t)M.inner;
            if (ga && !have_z) {
                SmallProblem& q = S.prob[S.nprob++];
                q.inj = x; q.ld_inj = ldx; q.inj_lo = (uint32_t)k; q.inj_hi = (uint32_t)(k + n);
                q.res_lo = 0; q.res_hi = (uint32_t)k;
                q.out_z = P.z; q.op_z = op_f;
            }
            if (gx || gb) {
                SmallProblem& q = S.prob[S.nprob++];
                q.inj = gyq; q.ld_inj = batch; q.op_inj = k * batch; q.inj_lo = 0; q.inj_hi = (uint32_t)k;
                q.res_lo = (uint32_t)k; q.res_hi = (uint32_t)(k + n);
                q.out_p = gx ? gxq : nullptr; q.ld_p = batch; q.op_p = n * batch;
                q.out_z = gb ? zg : nullptr; q.op_z = op_f;
            }
            if (S.nprob > 0) LAPLEX_HIP(launch_small(S, r, st));
            if (ga) LAPLEX_HIP(launch_rowdot_ops(gyq, batch, k * batch, P.z, batch, op_f, k, batch, ga, k, r, st));
            if (gb) LAPLEX_HIP(launch_rowdot_ops(x, ldx, 0, zg, batch, op_f, n, batch, gb, n, r, st));
            if (gx) LAPLEX_HIP(launch_mix_combine(gxq, nullptr, r, n, batch, gx, ldgx, st));
        }
        if (gw) LAPLEX_HIP(launch_dot_ops(gy, ldgy, parts, r, k, batch, partial, gw, st));
        return LAPLEX_OK;
    }
    std::unique_lock<std::mutex> lock(g_mix_mutex, std::defer_lock);
    MixStreams* lanes = nullptr;
    if (M.lanes > 1) { lock.lock(); lanes = mix_streams(st); }
    if (lanes) LAPLEX_HIP(mix_fork(lanes, M.lanes, st));
    // The arithmetic follows the lanes whether or not their streams are used (a captured stream keeps everything to
    // itself): each lane sums the gx of its operators, the lanes' sums are added at the end.
    const bool split = M.lanes > 1;
    float* gxp = reinterpret_cast<float*>(base + M.off_gxp);
    for (int64_t q = 0; q < r; ++q) {
        const int l = split ? (int)(q % M.lanes) : 0;
        hipStream_t sq = lanes ? lanes->lane[l] : st;
        char* wq = base + (size_t)q * M.inner;
        float* part = parts + q * k * batch;
        float* gy_l = gyq + (size_t)l * k * batch;
        float* gx_l = gxq + (size_t)l * n * batch;
        float* sum_l = gxp + (size_t)l * n * batch;
        uint32_t inner = flags;
        if (gw && !saved) {        // the weight's gradient needs the operator's own product
            LAPLEX_CHECK(laplex_apply(a + q * k, k, b + q * n, n, x, ldx, batch, part, batch, wq, M.inner,
                                      flags | LAPLEX_SAVE_SCANS, sq));
            inner = flags | LAPLEX_SAVE_SCANS | LAPLEX_REUSE_PLAN;
        }
        if (gx || ga || gb) {      // the operator's gradients are linear in the upstream gradient: scale it by w_q
            LAPLEX_HIP(launch_scale_by_device_scalar(gy, ldgy, w + q, k, batch, gy_l, sq));
            // a lane's first operator writes the lane's sum itself, the later ones are added to it
            float* gx_out = !gx ? nullptr : (split && q < M.lanes) ? sum_l : gx_l;
            LAPLEX_CHECK(laplex_apply_backward(a + q * k, k, b + q * n, n, x, ldx, gy_l, batch, batch,
                                               gx_out, batch, ga ? ga + q * k : nullptr,
                                               gb ? gb + q * n : nullptr, wq, M.inner, inner, sq));
            if (gx && !split) LAPLEX_HIP(launch_accumulate(gx_l, n, batch, gx, ldgx, q == 0, sq));
            else if (gx && q >= M.lanes) LAPLEX_HIP(launch_accumulate(gx_l, n, batch, sum_l, batch, false, sq));
        }
        if (gw) LAPLEX_HIP(launch_dot(gy, ldgy, part, k, batch, partial + (size_t)l * kTauPartials, gw + q, sq));
    }
    if (lanes) LAPLEX_HIP(mix_join(lanes, M.lanes, st));
    if (split && gx) LAPLEX_HIP(launch_mix_combine(gxp, nullptr, M.lanes, n, batch, gx, ldgx, st));
    return LAPLEX_OK;
}

int laplex_get_perm(const void* ws, size_t ws_bytes, int64_t count, uint32_t* perm_out, laplex_stream_t stream)
{
    if (count < 0 || count > LAPLEX_MAX_MERGED) return LAPLEX_ERR_SIZE;
    if (count == 0) return LAPLEX_OK;
    if (!ws || !perm_out) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256) || misaligned(perm_out, 4)) return LAPLEX_ERR_ALIGN;
    if (ws_bytes < sizeof(uint32_t) * (size_t)count) return LAPLEX_ERR_WORKSPACE;
    LAPLEX_HIP(launch_copy_u32(static_cast<const uint32_t*>(ws), perm_out, count, stream));
    return LAPLEX_OK;
}

int laplex_get_plan_status(const void* ws, size_t ws_bytes, int64_t count, uint32_t* status_out, laplex_stream_t stream)
{
    if (count < 0 || count > LAPLEX_MAX_MERGED) return LAPLEX_ERR_SIZE;
    if (!status_out) return LAPLEX_ERR_NULL;
    if (misaligned(status_out, 4)) return LAPLEX_ERR_ALIGN;
    if (count <= kSmallMax) {       // sorted by counting ranks: nothing ever waits
        LAPLEX_HIP(launch_fill(reinterpret_cast<float*>(status_out), 1, 1, 1, 0.0f, stream));
        return LAPLEX_OK;
    }
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    const Layout L = make_layout(count, 0, 1);          // the plan's offsets depend on the merged length only
    if (ws_bytes < L.off_counters + sizeof(uint32_t) * 64) return LAPLEX_ERR_WORKSPACE;
    const uint32_t* word = reinterpret_cast<const uint32_t*>(static_cast<const char*>(ws) + L.off_counters) + kPlanStatusWord;
    LAPLEX_HIP(launch_copy_u32(word, status_out, 1, stream));
    return LAPLEX_OK;
}

int laplex_diag_set_plan_status(void* ws, size_t ws_bytes, int64_t count, uint32_t value, laplex_stream_t stream)
{
    if (count <= kSmallMax || count > LAPLEX_MAX_MERGED) return LAPLEX_ERR_SIZE;
    if (!ws) return LAPLEX_ERR_NULL;
    if (misaligned(ws, 256)) return LAPLEX_ERR_ALIGN;
    const Layout L = make_layout(count, 0, 1);          // the plan's offsets depend on the merged length only
    if (ws_bytes < L.off_counters + sizeof(uint32_t) * 64) return LAPLEX_ERR_WORKSPACE;
    float* word = reinterpret_cast<float*>(static_cast<char*>(ws) + L.off_counters) + kPlanStatusWord;
    float bits;
    static_assert(sizeof(bits) == sizeof(value), "the word is written as the bit pattern of a float");
    __builtin_memcpy(&bits, &value, sizeof(bits));
    LAPLEX_HIP(launch_fill(word, 1, 1, 1, bits, stream));
    return LAPLEX_OK;
}

int laplex_diag_set_route_min(int64_t merged_positions)
{
    if (merged_positions < 0) return LAPLEX_ERR_SIZE;
    g_permute_min.store(merged_positions);
    return LAPLEX_OK;
}

const char* laplex_status_string(int status)
{
    switch (status) {
        case LAPLEX_OK: return "ok";
        case LAPLEX_ERR_NULL: return "a required pointer is NULL";
        case LAPLEX_ERR_SIZE: return "a size is negative or too large";
        case LAPLEX_ERR_LD: return "a leading dimension is smaller than batch";
        case LAPLEX_ERR_WORKSPACE: return "workspace too small";
        case LAPLEX_ERR_FLAGS: return "unknown or inapplicable flag";
        case LAPLEX_ERR_HIP: return "a HIP call failed";
        case LAPLEX_ERR_ALIGN: return "a pointer is misaligned";
        case LAPLEX_ERR_VALUE: return "a scalar argument is out of range";
        default: return "unknown status";
    }
}

const char* laplex_last_hip_error(void) { return g_hip_error.c_str(); }

int laplex_scan_tile_rows(int64_t batch, int wide, int64_t* rows)
{
    if (!rows) return LAPLEX_ERR_NULL;
    if (batch < 1 || (wide && batch % 4 != 0)) return LAPLEX_ERR_SIZE;
    *rows = scan_geom(1, batch, wide ? 4 : 1).tile_rows;
    return LAPLEX_OK;
}

int laplex_diag_move_rows(const float* src, float* dst, const uint32_t* row_ids, int64_t rows, int64_t cols,
                          laplex_stream_t stream)
{
    if (rows < 0 || cols < 0 || cols % 4 != 0) return LAPLEX_ERR_SIZE;
    if (rows == 0 || cols == 0) return LAPLEX_OK;
    if (!src || !row_ids) return LAPLEX_ERR_NULL;
    if (misaligned(src, 16) || (dst && misaligned(dst, 16)) || misaligned(row_ids, 4)) return LAPLEX_ERR_ALIGN;
    LAPLEX_HIP(launch_diag_move_rows(src, dst, row_ids, rows, cols, stream));
    return LAPLEX_OK;
}

int laplex_profile_begin(const char* family)
{
    if (!family) return LAPLEX_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    for (auto& ev : g_prof_events) { (void)hipEventDestroy(ev.e0); (void)hipEventDestroy(ev.e1); }
    g_prof_events.clear();
    g_prof_totals.clear();
    g_prof_family = family;
    g_prof_on.store(true);
    return LAPLEX_OK;
}

int laplex_profile_end(double* total_ms, int64_t* launches)
{
    if (!total_ms || !launches) return LAPLEX_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    g_prof_on.store(false);
    g_prof_totals.clear();
    double sum = 0.0;
    int64_t count = 0;
    int rc = LAPLEX_OK;
    for (auto& ev : g_prof_events) {
        float ms = 0.0f;
        hipError_t e = hipEventSynchronize(ev.e1);
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev.e0, ev.e1);
        if (e == hipSuccess) {
            sum += ms; ++count;
            size_t f = 0;
            while (f < g_prof_totals.size() && g_prof_totals[f].family != ev.family) ++f;
            if (f == g_prof_totals.size()) g_prof_totals.push_back(ProfTotal{ev.family, 0.0, 0});
            g_prof_totals[f].ms += ms; ++g_prof_totals[f].launches;
        } else {
            rc = hip_fail(e);
        }
        (void)hipEventDestroy(ev.e0); (void)hipEventDestroy(ev.e1);
    }
    g_prof_events.clear();
    *total_ms = sum; *launches = count;
    return rc;
}

int laplex_profile_family(int64_t index, char* name, size_t name_bytes, double* total_ms, int64_t* launches)
{
    if (!name || !total_ms || !launches) return LAPLEX_ERR_NULL;
    std::lock_guard<std::mutex> lock(g_prof_mutex);
    if (index < 0 || (size_t)index >= g_prof_totals.size() || name_bytes == 0) return LAPLEX_ERR_SIZE;
    const ProfTotal& t = g_prof_totals[(size_t)index];
    const size_t len = t.family.size() < name_bytes - 1 ? t.family.size() : name_bytes - 1;
    __builtin_memcpy(name, t.family.data(), len);
    name[len] = '\0';
    *total_ms = t.ms; *launches = t.launches;
    return LAPLEX_OK;
}

}  // extern "C"
