// C ABI of liblookm: argument validation (host-only, before any launch), workspace carving and the
// launch sequence of the compression path.  See include/lookm.h for the contract.
#include "common.h"

#include <algorithm>
#include <cmath>
#include <mutex>
#include <vector>

namespace {

constexpr size_t kAlign = 256;

inline size_t align_up(size_t x) { return (x + kAlign - 1) / kAlign * kAlign; }

struct Layout {
    size_t lse, scores, evicted, assign, sim, rnorm, plan, member_pos, member_w, lists, partials, total;
};

// Hq query heads, H key / value heads (Hq = H without grouped query heads): only the row log-sum-exp and the score
// partials are per query head
Layout make_layout(int Hq, int H, int L, int d, int dt, int budget)
{
    const size_t HL = (size_t)H * L, HE = (size_t)H * (size_t)(L - budget);
    Layout w;
    size_t o = 0;
    w.lse = o;     o += align_up((size_t)Hq * L * sizeof(float));
    w.scores = o;  o += align_up(HL * sizeof(float));
    w.evicted = o; o += align_up(HE * sizeof(int32_t));
    w.assign = o;  o += align_up(HE * sizeof(int32_t));
    w.sim = o;     o += align_up(HE * sizeof(float));
    w.rnorm = o;   o += align_up(HL * sizeof(float));
    w.plan = o;    o += align_up((size_t)H * budget * 4 * sizeof(int32_t));   // merge plan, one int4 per slot
    w.member_pos = o; o += align_up(HE * sizeof(int32_t));
    w.member_w = o;   o += align_up(HE * sizeof(float));
    w.lists = o;      o += align_up(lookm_host::score_list_ints(L) * sizeof(int32_t));   // competing / protected keys
    // the score partials and the matching partials are never live at the same time: one slice serves both
    w.partials = o;
    o += align_up(std::max(lookm_host::scores_scratch_floats(Hq, L, d, (lookm_dtype)dt) * sizeof(float),
                           lookm_host::nearest_scratch_bytes(H, L, d, (lookm_dtype)dt, budget)));
    w.total = o;
    return w;
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

int check_shape(int H, int L, int d, int dt)
{
    if (H <= 0 || L <= 0 || d <= 0) return LOOKM_ERR_INVALID_ARG;
    if (dt != LOOKM_F32 && dt != LOOKM_BF16) return LOOKM_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > 256 || L > LOOKM_MAX_L) return LOOKM_ERR_UNSUPPORTED;
    if ((double)H * (double)L * (double)d >= 1099511627776.0) return LOOKM_ERR_UNSUPPORTED;
    return LOOKM_OK;
}

int check_budget(int L, int budget, int M)
{
    if (M < 0 || budget < 0) return LOOKM_ERR_INVALID_ARG;
    if (M > L || budget > L || budget < M) return LOOKM_ERR_BUDGET_RANGE;
    return LOOKM_OK;
}

int check_workspace(const void* ws, size_t bytes, int Hq, int H, int L, int d, int dt, int budget)
{
    if (ws == nullptr || (reinterpret_cast<uintptr_t>(ws) % kAlign) != 0) return LOOKM_ERR_WORKSPACE;
    if (bytes < make_layout(Hq, H, L, d, dt, budget).total) return LOOKM_ERR_WORKSPACE;
    return LOOKM_OK;
}

template <typename T> T* at(void* base, size_t off) { return reinterpret_cast<T*>(static_cast<char*>(base) + off); }

// ---- two lanes for independent jobs of a batch -----------------------------------------------------------
// Jobs that touch disjoint memory do not have to wait for each other: alternating them between the caller's
// stream and a second stream of the caller lets the short, latency-bound kernels of one job (selection, set sort,
// folds) and the tail of its long kernels run under the long kernels of the next.  Everything stays ordered
// after the work already on the caller's stream and before the work the caller enqueues next (fork / join with
// events); jobs that share a workspace or an output keep their order.

struct ByteRange {
    uintptr_t lo, hi;   // [lo, hi)
};
struct JobFootprint {
    ByteRange w[6], r[5];   // what the job writes / only reads
    int nw, nr;
};

inline void add_range(ByteRange* list, int& n, const void* p, size_t bytes)
{
    if (p == nullptr || bytes == 0) return;
    list[n].lo = reinterpret_cast<uintptr_t>(p);
    list[n].hi = list[n].lo + bytes;
    ++n;
}

JobFootprint footprint(const lookm_job& j)
{
    const size_t Hq = (size_t)j.H, H = (size_t)(j.kv_heads ? j.kv_heads : j.H), L = (size_t)j.L, d = (size_t)j.d,
                 B = (size_t)j.budget, es = (j.dt == LOOKM_BF16) ? 2 : 4;
    JobFootprint f;
    f.nw = f.nr = 0;
    add_range(f.w, f.nw, j.workspace, j.workspace_bytes);
    add_range(f.w, f.nw, j.k_out, H * B * d * es);
    add_range(f.w, f.nw, j.v_out, H * B * d * es);
    add_range(f.w, f.nw, j.kept_idx, H * B * sizeof(int32_t));
    add_range(f.w, f.nw, j.scores_out, H * L * sizeof(float));
    add_range(f.w, f.nw, j.status_out, sizeof(int32_t));
    add_range(f.r, f.nr, j.q, Hq * L * d * es);
    add_range(f.r, f.nr, j.k, H * L * d * es);
    add_range(f.r, f.nr, j.v, H * L * d * es);
    add_range(f.r, f.nr, j.modality_mask, L);
    add_range(f.r, f.nr, j.row_lse, Hq * L * sizeof(float));
    return f;
}

inline bool overlap(const ByteRange& a, const ByteRange& b) { return a.lo < b.hi && b.lo < a.hi; }

// true if the two jobs may not run at the same time: one writes what the other reads or writes
bool conflict(const JobFootprint& a, const JobFootprint& b)
{
    for (int i = 0; i < a.nw; ++i) {
        for (int k = 0; k < b.nw; ++k) if (overlap(a.w[i], b.w[k])) return true;
        for (int k = 0; k < b.nr; ++k) if (overlap(a.w[i], b.r[k])) return true;
    }
    for (int i = 0; i < a.nr; ++i)
        for (int k = 0; k < b.nw; ++k) if (overlap(a.r[i], b.w[k])) return true;
    return false;
}

// `later` waits for everything enqueued on `earlier` so far.  The event lives until the end of the call that made
// it (destroying a recorded event only releases it once it has completed).
bool order_after(std::vector<hipEvent_t>& events, hipStream_t earlier, hipStream_t later)
{
    hipEvent_t e = nullptr;
    if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return false;
    events.push_back(e);
    return hipEventRecord(e, earlier) == hipSuccess && hipStreamWaitEvent(later, e, 0) == hipSuccess;
}

int enqueue_job(const lookm_job& j, hipStream_t st);

int enqueue_batch(const lookm_job* jobs, int n_jobs, int* bad_job, hipStream_t main, hipStream_t aux, bool two_lanes)
{
    auto serial = [&](int from) {
        for (int i = from; i < n_jobs; ++i) {
            const int rc = enqueue_job(jobs[i], main);
            if (rc != LOOKM_OK) {                 // only a failing HIP runtime call can end up here
                if (bad_job) *bad_job = i;
                return rc;
            }
        }
        return (int)LOOKM_OK;
    };
    // one job, no second stream, or a stream under graph capture (no event is created while a capture is open):
    // the plain loop
    if (n_jobs < 2 || !two_lanes) return serial(0);
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone, cap2 = hipStreamCaptureStatusNone;
    if (hipStreamIsCapturing(main, &cap) != hipSuccess || cap != hipStreamCaptureStatusNone ||
        hipStreamIsCapturing(aux, &cap2) != hipSuccess || cap2 != hipStreamCaptureStatusNone)
        return serial(0);

    std::vector<hipEvent_t> events;
    hipStream_t lane[2] = {main, aux};
    // jobs of a lane that the other lane has not been ordered after yet; before the fork only the caller's lane
    // exists, and the fork itself orders the second lane after all of it
    std::vector<JobFootprint> open[2];
    bool forked = false;
    int rc = LOOKM_OK, bad = 0;
    for (int i = 0; i < n_jobs && rc == LOOKM_OK; ++i) {
        bad = i;
        const JobFootprint f = footprint(jobs[i]);
        bool hit[2] = {false, false};
        for (int l = 0; l < 2; ++l)
            for (const JobFootprint& o : open[l])
                if (conflict(f, o)) { hit[l] = true; break; }
        // alternate; a job that depends on one lane only follows it there (stream order, no event needed)
        int want = i & 1;
        if (hit[0] != hit[1]) want = hit[0] ? 0 : 1;
        const int other = 1 - want;
        if (want == 1 && !forked) {           // the second lane starts after the work already on the first
            if (!order_after(events, main, aux)) { rc = LOOKM_ERR_DEVICE; break; }
            forked = true;
            open[0].clear();
        }
        if (hit[other]) {                     // depends on both lanes: wait for the other one here
            if (!order_after(events, lane[other], lane[want])) { rc = LOOKM_ERR_DEVICE; break; }
            open[other].clear();
        }
        rc = enqueue_job(jobs[i], lane[want]);
        open[want].push_back(f);
        if (open[want].size() >= 64) {        // keep the lists short: let the other lane catch up with this one
            if (forked) {
                if (!order_after(events, lane[want], lane[other])) { rc = LOOKM_ERR_DEVICE; break; }
                open[want].clear();
            } else {
                open[want].erase(open[want].begin());
            }
        }
    }
    // join: whatever the caller enqueues next on hip_stream comes after both lanes
    if (forked && !order_after(events, aux, main) && rc == LOOKM_OK) rc = LOOKM_ERR_DEVICE;
    for (hipEvent_t e : events) (void)hipEventDestroy(e);
    if (rc != LOOKM_OK && bad_job) *bad_job = bad;
    return rc;
}

// kernel attributes, once per device (see common.h)
constexpr int kMaxDevices = 64;
std::mutex g_ready_mutex;
bool g_ready[kMaxDevices];

}  // namespace

namespace lookm_host {
int ensure_device_ready()
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return LOOKM_ERR_DEVICE;
    std::lock_guard<std::mutex> lock(g_ready_mutex);
    if (g_ready[dev]) return LOOKM_OK;
    if (set_attributes_score_generic() != LOOKM_OK || set_attributes_nearest_generic() != LOOKM_OK ||
        set_attributes_merge() != LOOKM_OK || decode_static_scratch_setup() != LOOKM_OK)
        return LOOKM_ERR_DEVICE;
    g_ready[dev] = true;
    return LOOKM_OK;
}
}  // namespace lookm_host

extern "C" {

const char* lookm_version(void) { return "lookm 0.2 (gfx950)"; }

int lookm_init(void) { return lookm_host::ensure_device_ready(); }

const char* lookm_status_string(int status)
{
    switch (status) {
        case LOOKM_OK: return "ok";
        case LOOKM_ERR_INVALID_ARG: return "invalid argument";
        case LOOKM_ERR_UNSUPPORTED: return "unsupported dtype, head_dim or length";
        case LOOKM_ERR_BUDGET_RANGE: return "budget or recent_window out of range";
        case LOOKM_ERR_BUDGET_BELOW_PROTECTED: return "budget smaller than text plus recent window";
        case LOOKM_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case LOOKM_ERR_DEVICE: return "HIP runtime error";
        default: return "unknown status";
    }
}

int lookm_protected_count(const uint8_t* mask_host, int L, int recent_window)
{
    if (mask_host == nullptr || L <= 0 || recent_window < 0) return LOOKM_ERR_INVALID_ARG;
    if (recent_window > L) return LOOKM_ERR_BUDGET_RANGE;
    int n = 0;
    for (int j = 0; j < L; ++j) n += (mask_host[j] == 0 || j >= L - recent_window) ? 1 : 0;
    return n;
}

size_t lookm_workspace_bytes(int H, int L, int d, int budget, lookm_dtype dt)
{
    if (check_shape(H, L, d, (int)dt) != LOOKM_OK || budget < 0 || budget > L) return 0;
    return make_layout(H, H, L, d, (int)dt, budget).total;
}

size_t lookm_workspace_offset(int H, int kv_heads, int L, int d, int budget, lookm_dtype dt, lookm_workspace_item item)
{
    if (check_shape(H, L, d, (int)dt) != LOOKM_OK || budget < 0 || budget > L || kv_heads <= 0 || H % kv_heads != 0)
        return (size_t)-1;
    const Layout w = make_layout(H, kv_heads, L, d, (int)dt, budget);
    switch (item) {
        case LOOKM_WS_EVICTED: return w.evicted;
        case LOOKM_WS_ASSIGN: return w.assign;
        case LOOKM_WS_SIM: return w.sim;
        default: return (size_t)-1;
    }
}

static int scores_impl(const void* q, const void* k, const float* row_lse, int H, int kv_heads, int L, int d,
                       lookm_dtype dt, int window, float* scores_out, void* workspace, size_t workspace_bytes,
                       void* hip_stream)
{
    if (!q || !k || !scores_out) return LOOKM_ERR_INVALID_ARG;
    int rc = check_shape(H, L, d, (int)dt);
    if (rc != LOOKM_OK) return rc;
    if (kv_heads <= 0 || H % kv_heads != 0) return LOOKM_ERR_INVALID_ARG;
    if (window < 0 || window > L) return LOOKM_ERR_INVALID_ARG;
    if (!aligned16(q) || !aligned16(k) || !aligned16(scores_out)) return LOOKM_ERR_INVALID_ARG;
    rc = check_workspace(workspace, workspace_bytes, H, kv_heads, L, d, (int)dt, 0);
    if (rc != LOOKM_OK) return rc;
    const Layout w = make_layout(H, kv_heads, L, d, (int)dt, 0);
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    return lookm_host::launch_scores(q, k, H, kv_heads, L, d, dt, window ? L - window : 0, at<float>(workspace, w.lse),
                                     row_lse, scores_out, nullptr, at<float>(workspace, w.partials), nullptr, 0, nullptr,
                                     (hipStream_t)hip_stream);
}

int lookm_scores(const void* q, const void* k, int H, int L, int d, lookm_dtype dt, float* scores_out,
                 void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return scores_impl(q, k, nullptr, H, H, L, d, dt, 0, scores_out, workspace, workspace_bytes, hip_stream);
}

int lookm_scores_lse(const void* q, const void* k, const float* row_lse, int H, int L, int d, lookm_dtype dt,
                     float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!row_lse) return LOOKM_ERR_INVALID_ARG;
    return scores_impl(q, k, row_lse, H, H, L, d, dt, 0, scores_out, workspace, workspace_bytes, hip_stream);
}

int lookm_scores_window(const void* q, const void* k, int H, int L, int d, lookm_dtype dt, int window,
                        float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (window <= 0) return LOOKM_ERR_INVALID_ARG;
    return scores_impl(q, k, nullptr, H, H, L, d, dt, window, scores_out, workspace, workspace_bytes, hip_stream);
}

int lookm_scores_grouped(const void* q, const void* k, int H, int kv_heads, int L, int d, lookm_dtype dt,
                         float* scores_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return scores_impl(q, k, nullptr, H, kv_heads, L, d, dt, 0, scores_out, workspace, workspace_bytes, hip_stream);
}

int lookm_select_rule_(const float* scores, const uint8_t* modality_mask, int H, int L, int budget,
                       int recent_window, lookm_select_rule rule, int32_t* kept_idx, int32_t* evicted_idx,
                       int32_t* status_out, void* hip_stream)
{
    if (!scores || !modality_mask || !status_out) return LOOKM_ERR_INVALID_ARG;
    if (H <= 0 || L <= 0) return LOOKM_ERR_INVALID_ARG;
    if ((int)rule < LOOKM_SELECT_PROTECT_TEXT || (int)rule > LOOKM_SELECT_LITERAL) return LOOKM_ERR_INVALID_ARG;
    if (L > LOOKM_MAX_L) return LOOKM_ERR_UNSUPPORTED;
    int rc = check_budget(L, budget, recent_window);
    if (rc != LOOKM_OK) return rc;
    // an empty list (budget 0, or budget L) may be passed as NULL
    if ((budget > 0 && !kept_idx) || (budget < L && !evicted_idx)) return LOOKM_ERR_INVALID_ARG;
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    return lookm_host::launch_select(scores, modality_mask, H, L, budget, recent_window, (int)rule, kept_idx,
                                     evicted_idx, status_out, (hipStream_t)hip_stream);
}

int lookm_select(const float* scores, const uint8_t* modality_mask, int H, int L, int budget, int recent_window,
                 int32_t* kept_idx, int32_t* evicted_idx, int32_t* status_out, void* hip_stream)
{
    return lookm_select_rule_(scores, modality_mask, H, L, budget, recent_window, LOOKM_SELECT_PROTECT_TEXT, kept_idx,
                              evicted_idx, status_out, hip_stream);
}

int lookm_budget_from_ratios(int L, double alpha_recent, double alpha_important, int* recent_window, int* budget)
{
    if (L <= 0 || !recent_window || !budget) return LOOKM_ERR_INVALID_ARG;
    if (!(alpha_recent >= 0.0 && alpha_recent <= 1.0) || !(alpha_important >= 0.0 && alpha_important <= 1.0))
        return LOOKM_ERR_INVALID_ARG;
    const long M = (long)std::floor(alpha_recent * (double)L + 0.5), N = (long)std::floor(alpha_important * (double)L + 0.5);
    if (M + N > (long)L) return LOOKM_ERR_BUDGET_RANGE;
    *recent_window = (int)M;
    *budget = (int)(M + N);
    return LOOKM_OK;
}

int lookm_nearest(const void* k, const int32_t* kept_idx, const int32_t* evicted_idx, int H, int L, int d,
                  lookm_dtype dt, int budget, int32_t* assign, float* sim, void* workspace, size_t workspace_bytes,
                  void* hip_stream)
{
    if (!k || !kept_idx) return LOOKM_ERR_INVALID_ARG;
    int rc = check_shape(H, L, d, (int)dt);
    if (rc != LOOKM_OK) return rc;
    if (budget < 1 || budget > L) return LOOKM_ERR_BUDGET_RANGE;
    if (budget < L && (!evicted_idx || !assign || !sim)) return LOOKM_ERR_INVALID_ARG;   // empty lists may be NULL
    if (!aligned16(k)) return LOOKM_ERR_INVALID_ARG;
    rc = check_workspace(workspace, workspace_bytes, H, H, L, d, (int)dt, budget);
    if (rc != LOOKM_OK) return rc;
    const Layout w = make_layout(H, H, L, d, (int)dt, budget);
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    return lookm_host::launch_nearest(k, kept_idx, evicted_idx, H, L, d, dt, budget, at<float>(workspace, w.rnorm),
                                      false, assign, sim, at<void>(workspace, w.partials), (hipStream_t)hip_stream);
}

int lookm_merge(const void* k, const void* v, const int32_t* kept_idx, const int32_t* evicted_idx,
                const int32_t* assign, const float* sim, int H, int L, int d, lookm_dtype dt, int budget,
                lookm_merge_mode merge_mode, void* k_out, void* v_out, void* workspace, size_t workspace_bytes,
                void* hip_stream)
{
    if (!k || !v) return LOOKM_ERR_INVALID_ARG;
    if (budget > 0 && (!kept_idx || !k_out || !v_out)) return LOOKM_ERR_INVALID_ARG;   // empty outputs may be NULL
    if ((int)merge_mode < LOOKM_MERGE_NONE || (int)merge_mode > LOOKM_MERGE_WEIGHTED) return LOOKM_ERR_INVALID_ARG;
    int rc = check_shape(H, L, d, (int)dt);
    if (rc != LOOKM_OK) return rc;
    if (budget < 0 || budget > L) return LOOKM_ERR_BUDGET_RANGE;
    if (merge_mode != LOOKM_MERGE_NONE && budget < L && (!evicted_idx || !assign || !sim)) return LOOKM_ERR_INVALID_ARG;
    if (!aligned16(k) || !aligned16(v) || !aligned16(k_out) || !aligned16(v_out)) return LOOKM_ERR_INVALID_ARG;
    rc = check_workspace(workspace, workspace_bytes, H, H, L, d, (int)dt, budget);
    if (rc != LOOKM_OK) return rc;
    const Layout w = make_layout(H, H, L, d, (int)dt, budget);
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    return lookm_host::launch_merge(k, v, kept_idx, evicted_idx, assign, sim, H, L, d, dt, budget, (int)merge_mode,
                                    at<int32_t>(workspace, w.plan), at<int32_t>(workspace, w.member_pos),
                                    at<float>(workspace, w.member_w), k_out, v_out, (hipStream_t)hip_stream);
}

// everything the host can check about one job, without touching the device
static int validate_job(const lookm_job& j)
{
    if (!j.q || !j.k || !j.v || !j.modality_mask || !j.status_out) return LOOKM_ERR_INVALID_ARG;
    if (j.budget > 0 && (!j.k_out || !j.v_out || !j.kept_idx)) return LOOKM_ERR_INVALID_ARG;   // empty outputs may be NULL
    if ((int)j.merge_mode < LOOKM_MERGE_NONE || (int)j.merge_mode > LOOKM_MERGE_WEIGHTED) return LOOKM_ERR_INVALID_ARG;
    if ((int)j.rule < LOOKM_SELECT_PROTECT_TEXT || (int)j.rule > LOOKM_SELECT_LITERAL) return LOOKM_ERR_INVALID_ARG;
    if (j.score_window < 0 || j.score_window > j.L) return LOOKM_ERR_INVALID_ARG;
    if (j.kv_heads < 0 || (j.kv_heads > 0 && (j.H <= 0 || j.H % j.kv_heads != 0))) return LOOKM_ERR_INVALID_ARG;
    int rc = check_shape(j.H, j.L, j.d, (int)j.dt);
    if (rc != LOOKM_OK) return rc;
    rc = check_budget(j.L, j.budget, j.recent_window);
    if (rc != LOOKM_OK) return rc;
    if (!aligned16(j.q) || !aligned16(j.k) || !aligned16(j.v) || !aligned16(j.k_out) || !aligned16(j.v_out) ||
        (j.scores_out && !aligned16(j.scores_out)) || (j.row_lse && !aligned16(j.row_lse)))
        return LOOKM_ERR_INVALID_ARG;
    return check_workspace(j.workspace, j.workspace_bytes, j.H, j.kv_heads ? j.kv_heads : j.H, j.L, j.d, (int)j.dt,
                           j.budget);
}

// the launch sequence of one validated job
}  // extern "C"

namespace {
int enqueue_job(const lookm_job& j, hipStream_t st)
{
    // Hq query heads; everything after the scores runs per key / value head
    const int Hq = j.H, H = j.kv_heads ? j.kv_heads : j.H, L = j.L, d = j.d, budget = j.budget;
    const lookm_dtype dt = j.dt;
    void* workspace = j.workspace;
    const Layout w = make_layout(Hq, H, L, d, (int)dt, budget);
    float* scores = j.scores_out ? j.scores_out : at<float>(workspace, w.scores);
    int32_t* evicted = at<int32_t>(workspace, w.evicted);
    int32_t* assign = at<int32_t>(workspace, w.assign);
    float* sim = at<float>(workspace, w.sim);

    // the matching needs the inverse key norms; the matrix-core score pass writes them from the key rows it holds
    const bool match = j.merge_mode != LOOKM_MERGE_NONE && budget < L && budget > 0;
    float* rnorm = at<float>(workspace, w.rnorm);
    // Only the image tokens before the window compete for places (Eq. 5-8): when the caller does not ask for the
    // scores themselves and every text token is protected, the other keys' scores are never looked at
    const bool competing_only = j.scores_out == nullptr && j.rule == LOOKM_SELECT_PROTECT_TEXT;
    int rc = lookm_host::launch_scores(j.q, j.k, Hq, H, L, d, dt, j.score_window ? L - j.score_window : 0,
                                       at<float>(workspace, w.lse), j.row_lse, scores,
                                       match ? rnorm : nullptr, at<float>(workspace, w.partials),
                                       competing_only ? j.modality_mask : nullptr, j.recent_window,
                                       competing_only ? at<int32_t>(workspace, w.lists) : nullptr, st);
    if (rc != LOOKM_OK) return rc;
    rc = lookm_host::launch_select(scores, j.modality_mask, H, L, budget, j.recent_window, (int)j.rule, j.kept_idx,
                                   evicted, j.status_out, st);
    if (rc != LOOKM_OK) return rc;
    if (j.merge_mode != LOOKM_MERGE_NONE && budget < L) {
        if (budget == 0) return LOOKM_OK;   // nothing conserved: nothing to merge into
        rc = lookm_host::launch_nearest(j.k, j.kept_idx, evicted, H, L, d, dt, budget, rnorm,
                                        lookm_host::scores_write_rnorm(d, dt), assign, sim,
                                        at<void>(workspace, w.partials), st);
        if (rc != LOOKM_OK) return rc;
    }
    return lookm_host::launch_merge(j.k, j.v, j.kept_idx, evicted, assign, sim, H, L, d, dt, budget, (int)j.merge_mode,
                                    at<int32_t>(workspace, w.plan), at<int32_t>(workspace, w.member_pos),
                                    at<float>(workspace, w.member_w), j.k_out, j.v_out, st);
}
}  // namespace

extern "C" {

static int compress_impl(const void* q, const void* k, const void* v, const uint8_t* modality_mask,
                         const float* row_lse, int H, int L, int d, lookm_dtype dt, int budget, int recent_window,
                         lookm_merge_mode merge_mode, void* k_out, void* v_out, int32_t* kept_idx, float* scores_out,
                         int32_t* status_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    lookm_job j;
    j.q = q; j.k = k; j.v = v; j.modality_mask = modality_mask; j.row_lse = row_lse;
    j.H = H; j.L = L; j.d = d; j.dt = dt;
    j.budget = budget; j.recent_window = recent_window; j.merge_mode = merge_mode; j.rule = LOOKM_SELECT_PROTECT_TEXT;
    j.score_window = 0; j.kv_heads = 0;
    j.k_out = k_out; j.v_out = v_out; j.kept_idx = kept_idx; j.scores_out = scores_out; j.status_out = status_out;
    j.workspace = workspace; j.workspace_bytes = workspace_bytes;
    int rc = validate_job(j);
    if (rc != LOOKM_OK) return rc;
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    return enqueue_job(j, (hipStream_t)hip_stream);
}

int lookm_compress(const void* q, const void* k, const void* v, const uint8_t* modality_mask, int H, int L, int d,
                   lookm_dtype dt, int budget, int recent_window, lookm_merge_mode merge_mode, void* k_out,
                   void* v_out, int32_t* kept_idx, float* scores_out, int32_t* status_out, void* workspace,
                   size_t workspace_bytes, void* hip_stream)
{
    return compress_impl(q, k, v, modality_mask, nullptr, H, L, d, dt, budget, recent_window, merge_mode, k_out, v_out,
                         kept_idx, scores_out, status_out, workspace, workspace_bytes, hip_stream);
}

int lookm_compress_lse(const void* q, const void* k, const void* v, const uint8_t* modality_mask,
                       const float* row_lse, int H, int L, int d, lookm_dtype dt, int budget, int recent_window,
                       lookm_merge_mode merge_mode, void* k_out, void* v_out, int32_t* kept_idx, float* scores_out,
                       int32_t* status_out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!row_lse) return LOOKM_ERR_INVALID_ARG;
    return compress_impl(q, k, v, modality_mask, row_lse, H, L, d, dt, budget, recent_window, merge_mode, k_out, v_out,
                         kept_idx, scores_out, status_out, workspace, workspace_bytes, hip_stream);
}

static int batch_impl(const lookm_job* jobs, int n_jobs, int* bad_job, hipStream_t main, hipStream_t aux, bool two_lanes)
{
    if (n_jobs < 0 || (n_jobs > 0 && !jobs)) return LOOKM_ERR_INVALID_ARG;
    for (int i = 0; i < n_jobs; ++i) {
        const int rc = validate_job(jobs[i]);
        if (rc != LOOKM_OK) {
            if (bad_job) *bad_job = i;
            return rc;
        }
    }
    if (n_jobs == 0) return LOOKM_OK;
    const int rc = lookm_host::ensure_device_ready();
    if (rc != LOOKM_OK) return rc;
    return enqueue_batch(jobs, n_jobs, bad_job, main, aux, two_lanes);
}

int lookm_compress_batch(const lookm_job* jobs, int n_jobs, int* bad_job, void* hip_stream)
{
    return batch_impl(jobs, n_jobs, bad_job, (hipStream_t)hip_stream, nullptr, false);
}

int lookm_compress_batch_two_streams(const lookm_job* jobs, int n_jobs, int* bad_job, void* hip_stream,
                                     void* hip_stream_aux)
{
    if (hip_stream_aux == hip_stream) return LOOKM_ERR_INVALID_ARG;
    return batch_impl(jobs, n_jobs, bad_job, (hipStream_t)hip_stream, (hipStream_t)hip_stream_aux, true);
}

size_t lookm_decode_workspace_bytes(int H, int d)
{
    if (H <= 0 || d <= 0 || d % 8 != 0 || d > 256) return 0;
    return lookm_host::decode_scratch_bytes(H, d);
}

int lookm_decode_attention(const void* q, const void* k_cache, const void* v_cache, int H, int rows, int S, int d,
                           lookm_dtype dt, void* out, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!q || !k_cache || !v_cache || !out) return LOOKM_ERR_INVALID_ARG;
    if (H <= 0 || rows <= 0 || S <= 0 || S > rows || d <= 0) return LOOKM_ERR_INVALID_ARG;
    if (dt != LOOKM_F32 && dt != LOOKM_BF16) return LOOKM_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > 256) return LOOKM_ERR_UNSUPPORTED;
    if ((double)H * (double)rows * (double)d >= 1099511627776.0) return LOOKM_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return LOOKM_ERR_INVALID_ARG;
    if (workspace == nullptr || (reinterpret_cast<uintptr_t>(workspace) % kAlign) != 0 ||
        workspace_bytes < lookm_host::decode_scratch_bytes(H, d))
        return LOOKM_ERR_WORKSPACE;
    const int rdy = lookm_host::ensure_device_ready();
    if (rdy != LOOKM_OK) return rdy;
    return lookm_host::launch_decode(q, k_cache, v_cache, H, rows, S, d, dt, out, static_cast<float*>(workspace),
                                     (hipStream_t)hip_stream);
}

int lookm_decode_attention_noalloc(const void* q, const void* k_cache, const void* v_cache, int H, int rows, int S, int d,
                                   lookm_dtype dt, void* out, void* hip_stream)
{
    if (!q || !k_cache || !v_cache || !out) return LOOKM_ERR_INVALID_ARG;
    if (H <= 0 || rows <= 0 || S <= 0 || S > rows || d <= 0) return LOOKM_ERR_INVALID_ARG;
    if (dt != LOOKM_F32 && dt != LOOKM_BF16) return LOOKM_ERR_INVALID_ARG;
    if (d % 8 != 0 || d > 256) return LOOKM_ERR_UNSUPPORTED;
    if ((double)H * (double)rows * (double)d >= 1099511627776.0) return LOOKM_ERR_UNSUPPORTED;
    if (!aligned16(q) || !aligned16(k_cache) || !aligned16(v_cache) || !aligned16(out)) return LOOKM_ERR_INVALID_ARG;
    // sizes whose partial results do not fit the static array are refused, before anything is launched
    if (lookm_host::decode_partial_bytes(H, S, d) > (size_t)LOOKM_DECODE_NOALLOC_SCRATCH_BYTES) return LOOKM_ERR_WORKSPACE;
    const int rdy = lookm_host::ensure_device_ready();      // first call on a device: resolves the array's address
    if (rdy != LOOKM_OK) return rdy;
    float* part = lookm_host::decode_static_scratch();
    if (part == nullptr) return LOOKM_ERR_DEVICE;
    return lookm_host::launch_decode(q, k_cache, v_cache, H, rows, S, d, dt, out, part, (hipStream_t)hip_stream);
}

int lookm_job_profile(const lookm_job* job, int reps, float* kernel_ms_host, void* hip_stream)
{
    if (!job || reps <= 0 || kernel_ms_host == nullptr) return LOOKM_ERR_INVALID_ARG;
    int rc = validate_job(*job);
    if (rc != LOOKM_OK) return rc;
    if ((rc = lookm_host::ensure_device_ready()) != LOOKM_OK) return rc;
    lookm_host::KernelTimer timer;
    timer.st = (hipStream_t)hip_stream;
    for (int i = 0; i <= LOOKM_N_KERNELS; ++i)
        if (hipEventCreate(&timer.ev[i]) != hipSuccess) {
            while (--i >= 0) (void)hipEventDestroy(timer.ev[i]);
            return LOOKM_ERR_DEVICE;
        }
    double sum[LOOKM_N_KERNELS] = {0};
    for (int r = 0; r < reps && rc == LOOKM_OK; ++r) {
        // a kernel that is skipped for these sizes leaves its event at this early time (handled below); the
        // start event goes last, so that the first kernel's interval does not contain the other records
        for (int i = LOOKM_N_KERNELS; i >= 0; --i) (void)hipEventRecord(timer.ev[i], timer.st);
        lookm_host::g_timer = &timer;
        rc = enqueue_job(*job, timer.st);
        lookm_host::g_timer = nullptr;
        if (hipStreamSynchronize(timer.st) != hipSuccess) rc = LOOKM_ERR_DEVICE;
        float prev = 0.f;   // time since ev[0] of the latest kernel that actually ran
        for (int i = 0; i < LOOKM_N_KERNELS && rc == LOOKM_OK; ++i) {
            float t = 0.f;
            if (hipEventElapsedTime(&t, timer.ev[0], timer.ev[i + 1]) != hipSuccess) rc = LOOKM_ERR_DEVICE;
            if (t > prev) { sum[i] += t - prev; prev = t; }
        }
    }
    for (int i = 0; i <= LOOKM_N_KERNELS; ++i) (void)hipEventDestroy(timer.ev[i]);
    for (int i = 0; i < LOOKM_N_KERNELS; ++i) kernel_ms_host[i] = (float)(sum[i] / reps);
    return rc;
}

int lookm_compress_profile(const void* q, const void* k, const void* v, const uint8_t* modality_mask, int H, int L,
                           int d, lookm_dtype dt, int budget, int recent_window, lookm_merge_mode merge_mode,
                           void* k_out, void* v_out, int32_t* kept_idx, float* scores_out, int32_t* status_out,
                           void* workspace, size_t workspace_bytes, void* hip_stream, int reps, float* kernel_ms_host)
{
    lookm_job j;
    j.q = q; j.k = k; j.v = v; j.modality_mask = modality_mask; j.row_lse = nullptr;
    j.H = H; j.L = L; j.d = d; j.dt = dt;
    j.budget = budget; j.recent_window = recent_window; j.merge_mode = merge_mode; j.rule = LOOKM_SELECT_PROTECT_TEXT;
    j.score_window = 0; j.kv_heads = 0;
    j.k_out = k_out; j.v_out = v_out; j.kept_idx = kept_idx; j.scores_out = scores_out; j.status_out = status_out;
    j.workspace = workspace; j.workspace_bytes = workspace_bytes;
    return lookm_job_profile(&j, reps, kernel_ms_host, hip_stream);
}

}  // extern "C"

namespace lookm_host {
thread_local KernelTimer* g_timer = nullptr;
}
