// C ABI of libslipstream: argument validation on the host, then launches.
#include <math.h>
#include <stdarg.h>
#include <stdio.h>
#include <string.h>

#include <mutex>
#include <vector>

#include "ss_common.h"

namespace ss {

static thread_local char g_err[512] = "";

int32_t fail(int32_t code, const char *fmt, ...)
{
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return code;
}

int32_t check_tables(const ss_tables *tb, const char *who)
{
    if (!tb) return fail(SS_ERR_INVALID_ARG, "%s: tables is NULL", who);
    if (tb->num_tables < 1 || tb->num_tables > 65535)
        return fail(SS_ERR_INVALID_ARG, "%s: num_tables = %d (need 1..65535)", who,
                    tb->num_tables);
    if (tb->dim < 4 || tb->dim % 4 != 0 || tb->dim > 1024)
        return fail(SS_ERR_INVALID_ARG,
                    "%s: dim = %d (need a multiple of 4 in [4, 1024])", who, tb->dim);
    if (tb->rows < 1 || tb->rows >= (1LL << 31))
        return fail(SS_ERR_INVALID_ARG, "%s: rows = %lld (need 1 <= rows < 2^31)",
                    who, (long long)tb->rows);
    if (!tb->weights)
        return fail(SS_ERR_INVALID_ARG, "%s: tables->weights is NULL", who);
    return SS_OK;
}

int32_t check_launch(const char *who)
{
    const hipError_t e = hipGetLastError();
    if (e != hipSuccess)
        return fail(SS_ERR_HIP, "%s: %s", who, hipGetErrorString(e));
    return SS_OK;
}

// ---- optional per-kernel timing ---------------------------------------
namespace {
struct ProfRec {
    const char *kernel;
    hipEvent_t start, stop;
};
std::mutex g_prof_mu;
bool g_prof_on = false;
std::vector<ProfRec> g_prof;
constexpr size_t kProfMax = 1u << 20;
}  // namespace

static thread_local int t_prof_slot = -1;
static thread_local int t_prof_mute = 0;
static thread_local const char *t_prof_kernel = nullptr;   // name of the innermost live ProfScope

// ---- trace mode ---------------------------------------------------------
namespace {
bool g_trace_on = false;
unsigned long long *g_trace_buf = nullptr;                 // [2][kTraceMax][kTraceLanes]
std::vector<const char *> g_trace_names;                   // kernel of each used slot
}  // namespace

TraceSlot next_trace_slot()
{
    if (!g_trace_on || t_prof_mute > 0 || !t_prof_kernel) return TraceSlot{nullptr};
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (!g_trace_buf || g_trace_names.size() >= kTraceMax) return TraceSlot{nullptr};
    g_trace_names.push_back(t_prof_kernel);
    return TraceSlot{g_trace_buf + (g_trace_names.size() - 1) * kTraceLanes};
}

ProfMute::ProfMute() { ++t_prof_mute; }
ProfMute::~ProfMute() { --t_prof_mute; }

ProfScope::ProfScope(const char *kernel, hipStream_t)
{
    t_prof_slot = -1;
    t_prof_kernel = kernel;
    if (!g_prof_on || t_prof_mute > 0) return;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (g_prof.size() >= kProfMax) return;
    ProfRec r{kernel, nullptr, nullptr};
    if (hipEventCreate(&r.start) != hipSuccess) return;
    if (hipEventCreate(&r.stop) != hipSuccess) {
        (void)hipEventDestroy(r.start);
        return;
    }
    g_prof.push_back(r);
    t_prof_slot = (int)g_prof.size() - 1;
}

ProfScope::~ProfScope()
{
    t_prof_slot = -1;
    t_prof_kernel = nullptr;
}

static thread_local hipEvent_t t_stop_event = nullptr;
void stop_event_for_next_launch(hipEvent_t ev) { t_stop_event = ev; }
hipEvent_t take_stop_event()
{
    const hipEvent_t ev = t_stop_event;
    t_stop_event = nullptr;
    return ev;
}

bool prof_events(hipEvent_t *start, hipEvent_t *stop)
{
    if (t_prof_slot < 0) return false;
    std::lock_guard<std::mutex> lk(g_prof_mu);
    if (t_prof_slot >= (int)g_prof.size()) return false;
    *start = g_prof[t_prof_slot].start;
    *stop = g_prof[t_prof_slot].stop;
    t_prof_slot = -1;          // one launch per scope
    return true;
}

__global__ void wait_marker_kernel() {}

void after_stream_wait(hipStream_t s)
{
    if (!g_prof_on) return;
    hipLaunchKernelGGL(wait_marker_kernel, dim3(1), dim3(64), 0, s);
}

static int32_t check_batch(const char *who, const void *idx, int64_t B, int64_t L,
                           int64_t T)
{
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    if (B < 1) return fail(SS_ERR_INVALID_ARG, "%s: batch = %lld", who, (long long)B);
    if (L < 1) return fail(SS_ERR_INVALID_ARG, "%s: L = %lld", who, (long long)L);
    if (B * L >= (1LL << 31) || T * L >= (1LL << 31))
        return fail(SS_ERR_UNSUPPORTED, "%s: B*L or T*L does not fit in int32", who);
    return SS_OK;
}

static int32_t check_hot_tables(const char *who, int32_t T, int64_t rows)
{
    if (T < 1 || T > 65535)
        return fail(SS_ERR_INVALID_ARG, "%s: num_tables = %d (need 1..65535)", who, T);
    if (rows < 1 || rows >= (1LL << 31))
        return fail(SS_ERR_INVALID_ARG, "%s: rows = %lld (need 1 <= rows < 2^31)", who,
                    (long long)rows);
    return SS_OK;
}

static int32_t check_ws(const char *who, const void *ws, size_t have, size_t need)
{
    if (!ws) return fail(SS_ERR_WORKSPACE, "%s: workspace is NULL", who);
    if (reinterpret_cast<uintptr_t>(ws) % 256 != 0)
        return fail(SS_ERR_WORKSPACE, "%s: workspace is not 256-byte aligned", who);
    if (have < need)
        return fail(SS_ERR_WORKSPACE, "%s: workspace has %zu bytes, needs %zu", who,
                    have, need);
    return SS_OK;
}

int32_t check_filter(const char *who, const ss_tables *tables, const int32_t *idx,
                     int32_t B, int32_t L, const uint8_t *skip_mask,
                     const int32_t *kept_ids, const int32_t *n_kept,
                     const int32_t *idx_c, const void *ws, size_t ws_bytes)
{
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    rc = check_batch(who, idx, B, L, tables->num_tables);
    if (rc) return rc;
    if (!skip_mask || !kept_ids || !n_kept || !idx_c)
        return fail(SS_ERR_INVALID_ARG, "%s: an output pointer is NULL", who);
    if (idx_c == idx)
        return fail(SS_ERR_INVALID_ARG, "%s: idx_c must not alias idx", who);
    return check_ws(who, ws, ws_bytes, filter_ws_bytes(tables->num_tables, B, L));
}

int32_t check_backward(const char *who, const ss_tables *tables, int32_t Bcap,
                       int32_t L, const void *ws, size_t ws_bytes)
{
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    if (Bcap < 1) return fail(SS_ERR_INVALID_ARG, "%s: batch = %d", who, Bcap);
    if (L < 1) return fail(SS_ERR_INVALID_ARG, "%s: L = %d", who, L);
    if ((int64_t)Bcap * L >= (1LL << 31) - 4096)
        return fail(SS_ERR_UNSUPPORTED, "%s: Bcap*L too large", who);
    return check_ws(who, ws, ws_bytes,
                    backward_ws_bytes(tables->num_tables, Bcap, L, tables->dim));
}

}  // namespace ss

using namespace ss;

extern "C" {

const char *ss_last_error(void) { return g_err; }

void ss_profile_enable(int32_t on)
{
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_prof_on = on == 1;
    g_trace_on = false;
    if (on == 2) {
        // trace mode: a device buffer of one slot per launch, start stamps at the
        // largest value, end stamps at zero (a measurement aid may allocate)
        const size_t words = kTraceMax * 2 * kTraceLanes;
        if (!g_trace_buf &&
            hipMalloc(reinterpret_cast<void **>(&g_trace_buf), words * 8) != hipSuccess) {
            g_trace_buf = nullptr;
            return;
        }
        (void)hipMemset(g_trace_buf, 0xFF, words / 2 * 8);
        (void)hipMemset(g_trace_buf + words / 2, 0, words / 2 * 8);
        (void)hipDeviceSynchronize();
        g_trace_names.clear();
        g_trace_on = true;
    }
}

int32_t ss_profile_trace(char *buf, size_t buf_bytes)
{
    if (!buf || buf_bytes < 2)
        return fail(SS_ERR_INVALID_ARG, "ss_profile_trace: buffer missing");
    std::lock_guard<std::mutex> lk(g_prof_mu);
    g_trace_on = false;
    buf[0] = 0;
    const size_t n = g_trace_names.size();
    if (!g_trace_buf || n == 0) return SS_OK;
    if (hipDeviceSynchronize() != hipSuccess)
        return fail(SS_ERR_HIP, "ss_profile_trace: device synchronisation failed");
    std::vector<unsigned long long> starts(n * kTraceLanes), ends(n * kTraceLanes);
    if (hipMemcpy(starts.data(), g_trace_buf, starts.size() * 8, hipMemcpyDeviceToHost) !=
            hipSuccess ||
        hipMemcpy(ends.data(), g_trace_buf + kTraceMax * kTraceLanes, ends.size() * 8,
                  hipMemcpyDeviceToHost) != hipSuccess)
        return fail(SS_ERR_HIP, "ss_profile_trace: copy failed");
    unsigned long long origin = ~0ull;
    std::vector<unsigned long long> t0(n, ~0ull), t1(n, 0ull);
    for (size_t i = 0; i < n; ++i) {
        for (int l = 0; l < kTraceLanes; ++l) {
            const unsigned long long a = starts[i * kTraceLanes + l], b = ends[i * kTraceLanes + l];
            if (a < t0[i]) t0[i] = a;
            if (b > t1[i]) t1[i] = b;
        }
        if (t0[i] < origin) origin = t0[i];
    }
    size_t off = 0;
    for (size_t i = 0; i < n; ++i) {
        if (t0[i] == ~0ull || t1[i] == 0ull) continue;          // the launch did not run
        // the clock ticks at 100 MHz: 10 ns per tick
        const int w = snprintf(buf + off, buf_bytes - off, "%s %llu %llu\n", g_trace_names[i],
                               (t0[i] - origin) * 10ull, (t1[i] - origin) * 10ull);
        if (w < 0 || (size_t)w >= buf_bytes - off) {
            buf[off] = 0;
            return fail(SS_ERR_INVALID_ARG, "ss_profile_trace: buffer too small");
        }
        off += (size_t)w;
    }
    g_trace_names.clear();
    return SS_OK;
}

int32_t ss_profile_report(char *buf, size_t buf_bytes)
{
    if (!buf || buf_bytes < 2)
        return fail(SS_ERR_INVALID_ARG, "ss_profile_report: buffer missing");
    std::lock_guard<std::mutex> lk(g_prof_mu);
    struct Acc { const char *k; long n; double ms; };
    std::vector<Acc> acc;
    int32_t rc = SS_OK;
    for (const ProfRec &r : g_prof) {
        float ms = 0.f;
        if (hipEventSynchronize(r.stop) != hipSuccess ||
            hipEventElapsedTime(&ms, r.start, r.stop) != hipSuccess)
            rc = fail(SS_ERR_HIP, "ss_profile_report: event query failed");
        (void)hipEventDestroy(r.start);
        (void)hipEventDestroy(r.stop);
        size_t i = 0;
        while (i < acc.size() && strcmp(acc[i].k, r.kernel) != 0) ++i;
        if (i == acc.size()) acc.push_back(Acc{r.kernel, 0, 0.0});
        acc[i].n += 1;
        acc[i].ms += ms;
    }
    g_prof.clear();
    size_t off = 0;
    buf[0] = 0;
    for (const Acc &a : acc) {
        const int w = snprintf(buf + off, buf_bytes - off, "%s %ld %.6f\n", a.k,
                               a.n, a.ms);
        if (w < 0 || (size_t)w >= buf_bytes - off) {
            buf[off] = 0;
            return fail(SS_ERR_INVALID_ARG, "ss_profile_report: buffer too small");
        }
        off += (size_t)w;
    }
    return rc;
}

size_t ss_filter_batch_workspace_bytes(int32_t T, int32_t B, int32_t L)
{
    if (T < 1 || B < 1 || L < 1) return 0;
    return filter_ws_bytes(T, B, L);
}

size_t ss_backward_workspace_bytes(int32_t T, int32_t Bcap, int32_t L, int32_t dim)
{
    if (T < 1 || Bcap < 1 || L < 1 || dim < 4 || dim % 4 != 0) return 0;
    if ((int64_t)Bcap * L >= (1LL << 31) - 4096) return 0;
    return backward_ws_bytes(T, Bcap, L, dim);
}

int32_t ss_filter_batch(const ss_tables *tables, const int32_t *idx, int32_t B,
                        int32_t L, int32_t alpha, uint8_t *skip_mask,
                        int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c,
                        void *ws, size_t ws_bytes, void *stream)
{
    const int32_t rc = check_filter("ss_filter_batch", tables, idx, B, L, skip_mask,
                                    kept_ids, n_kept, idx_c, ws, ws_bytes);
    if (rc) return rc;
    if (int32_t bad = checked_indices("ss_filter_batch", tables->num_tables, tables->rows, idx,
                                      B, L, nullptr, static_cast<hipStream_t>(stream)))
        return bad;
    return launch_filter(tables, idx, B, L, alpha, skip_mask, kept_ids, n_kept,
                         idx_c, ws, static_cast<hipStream_t>(stream));
}

int32_t ss_filter_batch_split(const ss_tables *tables, uint32_t *const *hot_bits,
                              const int32_t *idx, int32_t B, int32_t L, int32_t alpha,
                              uint8_t *skip_mask, uint8_t *hot_mask, int32_t *kept_ids,
                              int32_t *n_kept, int32_t *idx_c, void *ws, size_t ws_bytes,
                              void *stream)
{
    const char *who = "ss_filter_batch_split";
    const int32_t rc = check_filter(who, tables, idx, B, L, skip_mask, kept_ids, n_kept, idx_c,
                                    ws, ws_bytes);
    if (rc) return rc;
    if (!hot_mask) return fail(SS_ERR_INVALID_ARG, "%s: hot_mask is NULL", who);
    if (int32_t bad = checked_indices(who, tables->num_tables, tables->rows, idx, B, L, nullptr,
                                      static_cast<hipStream_t>(stream)))
        return bad;
    return launch_filter_split(tables, hot_bits, idx, B, L, alpha, skip_mask, hot_mask, kept_ids,
                               n_kept, idx_c, ws, static_cast<hipStream_t>(stream));
}

int32_t ss_embbag_forward(const ss_tables *tables, const int32_t *idx,
                          int32_t Bcap, int32_t L, const int32_t *n_valid,
                          float *out, void *stream)
{
    const char *who = "ss_embbag_forward";
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    rc = check_batch(who, idx, Bcap, L, tables->num_tables);
    if (rc) return rc;
    if (!out) return fail(SS_ERR_INVALID_ARG, "%s: out is NULL", who);
    if (reinterpret_cast<uintptr_t>(out) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: out is not 16-byte aligned", who);
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_forward(tables, idx, Bcap, L, n_valid, out,
                          static_cast<hipStream_t>(stream));
}

static int32_t check_grad(const char *who, const float *grad)
{
    if (!grad) return fail(SS_ERR_INVALID_ARG, "%s: grad is NULL", who);
    if (reinterpret_cast<uintptr_t>(grad) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: grad is not 16-byte aligned", who);
    return SS_OK;
}

int32_t ss_embbag_backward_prepare(const ss_tables *tables, const int32_t *idx,
                                   int32_t Bcap, int32_t L, const int32_t *n_valid,
                                   void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ss_embbag_backward_prepare";
    int32_t rc = check_backward(who, tables, Bcap, L, ws, ws_bytes);
    if (rc) return rc;
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_backward_prepare(tables, idx, Bcap, L, n_valid, ws,
                                   static_cast<hipStream_t>(stream));
}

int32_t ss_embbag_forward_grouped(const ss_tables *tables, const int32_t *idx,
                                  int32_t Bcap, int32_t L, const int32_t *n_valid,
                                  float *out, void *bwd_ws, size_t bwd_ws_bytes,
                                  void *stream)
{
    const char *who = "ss_embbag_forward_grouped";
    int32_t rc = check_backward(who, tables, Bcap, L, bwd_ws, bwd_ws_bytes);
    if (rc) return rc;
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    if (!out) return fail(SS_ERR_INVALID_ARG, "%s: out is NULL", who);
    if (reinterpret_cast<uintptr_t>(out) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: out is not 16-byte aligned", who);
    hipStream_t s = static_cast<hipStream_t>(stream);
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid, s);
    if (rc) return rc;
    if (can_fuse_forward_group(tables, Bcap, L)) {
        uint2 *ent;
        int NP;
        backward_first_buffers(tables->num_tables, Bcap, L, tables->dim, bwd_ws, &ent, &NP);
        return launch_forward_group(tables, idx, Bcap, n_valid, out, ent, NP, s);
    }
    rc = launch_forward(tables, idx, Bcap, L, n_valid, out, s);
    if (rc) return rc;
    return launch_backward_prepare(tables, idx, Bcap, L, n_valid, bwd_ws, s);
}

int32_t ss_embbag_backward_apply(const ss_tables *tables, int32_t Bcap, int32_t L,
                                 const float *grad, float lr, void *ws,
                                 size_t ws_bytes, void *stream)
{
    const char *who = "ss_embbag_backward_apply";
    int32_t rc = check_backward(who, tables, Bcap, L, ws, ws_bytes);
    if (rc) return rc;
    rc = check_grad(who, grad);
    if (rc) return rc;
    return launch_backward_apply(tables, Bcap, L, grad, lr, ws,
                                 static_cast<hipStream_t>(stream));
}

int32_t ss_embbag_backward_update(const ss_tables *tables, const int32_t *idx,
                                  int32_t Bcap, int32_t L,
                                  const int32_t *n_valid, const float *grad,
                                  float lr, void *ws, size_t ws_bytes,
                                  void *stream)
{
    const char *who = "ss_embbag_backward_update";
    int32_t rc = check_backward(who, tables, Bcap, L, ws, ws_bytes);
    if (rc) return rc;
    if (!idx) return fail(SS_ERR_INVALID_ARG, "%s: idx is NULL", who);
    rc = check_grad(who, grad);
    if (rc) return rc;
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    rc = launch_backward_prepare(tables, idx, Bcap, L, n_valid, ws,
                                 static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_backward_apply(tables, Bcap, L, grad, lr, ws,
                                 static_cast<hipStream_t>(stream));
}

int32_t ss_detect_stale(const ss_tables *tables, int32_t *const *hot_ids,
                        int32_t H, float **snapshot, float threshold,
                        int32_t refresh_snapshot, uint8_t **stale_hot,
                        double **drift, uint32_t *stale_count, void *stream)
{
    const char *who = "ss_detect_stale";
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    if (!tables->stale_bits)
        return fail(SS_ERR_INVALID_ARG, "%s: tables->stale_bits is NULL", who);
    if (!hot_ids || !snapshot)
        return fail(SS_ERR_INVALID_ARG, "%s: hot_ids or snapshot is NULL", who);
    if (H < 1) return fail(SS_ERR_INVALID_ARG, "%s: H = %d", who, H);
    if (threshold != threshold)
        return fail(SS_ERR_INVALID_ARG, "%s: threshold is NaN", who);
    rc = checked_hot_ids(who, tables->num_tables, tables->rows, hot_ids, H,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_detect(tables, hot_ids, H, snapshot, threshold,
                         refresh_snapshot != 0, stale_hot, drift, stale_count,
                         static_cast<hipStream_t>(stream));
}

int32_t ss_sample_drop(int32_t num_tables, int32_t *const *hot_ids, int32_t H,
                       double *const *drift, const int32_t *sidx, int32_t S,
                       int32_t L, int32_t alpha, const float *thresholds,
                       int32_t n_thr, uint32_t *counts, void *stream)
{
    const char *who = "ss_sample_drop";
    if (num_tables < 1 || num_tables > 65535)
        return fail(SS_ERR_INVALID_ARG, "%s: num_tables = %d (need 1..65535)", who,
                    num_tables);
    if (!hot_ids || !drift)
        return fail(SS_ERR_INVALID_ARG, "%s: hot_ids or drift is NULL", who);
    if (H < 0) return fail(SS_ERR_INVALID_ARG, "%s: H = %d", who, H);
    if (S < 0) return fail(SS_ERR_INVALID_ARG, "%s: S = %d", who, S);
    if (L < 1) return fail(SS_ERR_INVALID_ARG, "%s: L = %d", who, L);
    if (S > 0 && !sidx) return fail(SS_ERR_INVALID_ARG, "%s: sidx is NULL", who);
    if ((int64_t)S * L >= (1LL << 31) || (int64_t)num_tables * L >= (1LL << 31))
        return fail(SS_ERR_UNSUPPORTED, "%s: S*L or T*L does not fit in int32", who);
    if (alpha < 0) return fail(SS_ERR_INVALID_ARG, "%s: alpha = %d", who, alpha);
    if (n_thr < 1 || n_thr > SS_MAX_THRESHOLDS)
        return fail(SS_ERR_INVALID_ARG, "%s: n_thr = %d (need 1..%d)", who, n_thr,
                    SS_MAX_THRESHOLDS);
    if (!thresholds || !counts)
        return fail(SS_ERR_INVALID_ARG, "%s: thresholds or counts is NULL", who);
    for (int k = 0; k < n_thr; ++k)
        if (thresholds[k] != thresholds[k])
            return fail(SS_ERR_INVALID_ARG, "%s: thresholds[%d] is NaN", who, k);
    return launch_sample_drop(num_tables, hot_ids, H, drift, sidx, S, L, alpha,
                              thresholds, n_thr, counts,
                              static_cast<hipStream_t>(stream));
}

int32_t ss_drop_stats(uint32_t count, int64_t n_samples, int64_t population,
                      int64_t n_hot_inputs, double t_crit, double *out)
{
    const char *who = "ss_drop_stats";
    if (!out) return fail(SS_ERR_INVALID_ARG, "%s: out is NULL", who);
    if (n_samples < 1 || population < n_samples)
        return fail(SS_ERR_INVALID_ARG, "%s: n_samples = %lld, population = %lld", who,
                    (long long)n_samples, (long long)population);
    if ((int64_t)count > n_samples)
        return fail(SS_ERR_INVALID_ARG, "%s: count = %u exceeds n_samples = %lld", who,
                    count, (long long)n_samples);
    if (n_hot_inputs < 0 || !(t_crit >= 0.0))
        return fail(SS_ERR_INVALID_ARG, "%s: n_hot_inputs = %lld, t_crit = %g", who,
                    (long long)n_hot_inputs, t_crit);
    // The indicator is 0 or 1, so its mean square deviation from D is D (1 - D).
    const double share = (double)count / (double)n_samples;
    const double var = share * (1.0 - share);
    const double unsampled = (double)(population - n_samples) / (double)population;
    const double half = t_crit * sqrt(unsampled * var / (double)n_samples);
    const double scale = (double)n_hot_inputs;
    out[0] = share;
    out[1] = sqrt(var);
    out[2] = half;
    out[3] = share - half;
    out[4] = share + half;
    out[5] = share * scale;
    out[6] = (share - half) * scale;
    out[7] = (share + half) * scale;
    return SS_OK;
}

int32_t ss_count_accesses(int32_t num_tables, int64_t rows, const int32_t *idx, int32_t B,
                          int32_t L, const int32_t *n_valid, uint32_t *const *counts,
                          void *stream)
{
    const char *who = "ss_count_accesses";
    int32_t rc = check_hot_tables(who, num_tables, rows);
    if (rc) return rc;
    rc = check_batch(who, idx, B, L, num_tables);
    if (rc) return rc;
    if (!counts) return fail(SS_ERR_INVALID_ARG, "%s: counts is NULL", who);
    rc = checked_indices(who, num_tables, rows, idx, B, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_count_accesses(num_tables, idx, B, L, n_valid, counts,
                                 static_cast<hipStream_t>(stream));
}

size_t ss_select_hot_workspace_bytes(int32_t num_tables, int64_t rows)
{
    if (num_tables < 1 || num_tables > 65535 || rows < 1 || rows >= (1LL << 31)) return 0;
    return select_hot_ws_bytes(num_tables, rows);
}

int32_t ss_select_hot_ratio(int32_t num_tables, int64_t rows, uint32_t *const *counts,
                            double lambda, int64_t total, int32_t cap,
                            int32_t *const *hot_ids, uint32_t *const *hot_bits,
                            uint32_t *n_hot, void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ss_select_hot_ratio";
    int32_t rc = check_hot_tables(who, num_tables, rows);
    if (rc) return rc;
    if (!counts) return fail(SS_ERR_INVALID_ARG, "%s: counts is NULL", who);
    if (lambda != lambda) return fail(SS_ERR_INVALID_ARG, "%s: lambda is NaN", who);
    if (total < 1) return fail(SS_ERR_INVALID_ARG, "%s: total = %lld", who, (long long)total);
    if (cap < 0 || (cap > 0 && !hot_ids))
        return fail(SS_ERR_INVALID_ARG, "%s: cap = %d, hot_ids %s", who, cap,
                    hot_ids ? "given" : "NULL");
    rc = check_ws(who, ws, ws_bytes, select_hot_ws_bytes(num_tables, rows));
    if (rc) return rc;
    // Smallest count whose share reaches lambda, with the share taken exactly as
    // the definition has it: an fp64 quotient.  The quotient grows with the
    // count, so a product gives the neighbourhood and two short loops the answer.
    const double tot = (double)total, x = lambda * tot;
    const uint64_t limit = 1ull << 32;               // "no 32-bit count is enough"
    uint64_t need = !(x > 0.0) ? 0 : (x >= 4294967296.0 ? limit : (uint64_t)ceil(x));
    while (need > 0 && (double)(need - 1) / tot >= lambda) --need;
    while (need < limit && (double)need / tot < lambda) ++need;
    const uint32_t c = need == 0 ? 0u : (uint32_t)(need - 1);
    const uint32_t e = need == 0 ? 0xFFFFFFFFu : 0u;
    return launch_select_hot(num_tables, rows, counts, false, c, e, cap > 0 ? hot_ids : nullptr,
                             cap, hot_bits, n_hot, ws, static_cast<hipStream_t>(stream));
}

int32_t ss_select_hot_top(int32_t num_tables, int64_t rows, uint32_t *const *counts,
                          int32_t H, int32_t *const *hot_ids, uint32_t *const *hot_bits,
                          void *ws, size_t ws_bytes, void *stream)
{
    const char *who = "ss_select_hot_top";
    int32_t rc = check_hot_tables(who, num_tables, rows);
    if (rc) return rc;
    if (!counts) return fail(SS_ERR_INVALID_ARG, "%s: counts is NULL", who);
    if (H < 0 || H > rows)
        return fail(SS_ERR_INVALID_ARG, "%s: H = %d (need 0 <= H <= rows)", who, H);
    if (H > 0 && !hot_ids) return fail(SS_ERR_INVALID_ARG, "%s: hot_ids is NULL", who);
    rc = check_ws(who, ws, ws_bytes, select_hot_ws_bytes(num_tables, rows));
    if (rc) return rc;
    // H = 0: no count is above the largest one, and no equal row is taken
    return launch_select_hot(num_tables, rows, counts, H > 0, H > 0 ? 0u : 0xFFFFFFFFu,
                             (uint32_t)H, H > 0 ? hot_ids : nullptr, H, hot_bits, nullptr, ws,
                             static_cast<hipStream_t>(stream));
}

// Vectors are read and written 16 bytes at a time.
static int32_t check_f4(const char *who, const void *p, const char *name)
{
    if (reinterpret_cast<uintptr_t>(p) % 16 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: %s is not 16-byte aligned", who, name);
    return SS_OK;
}

static int32_t check_f4_all(const char *who, const void *const *ptrs, const char *const *names,
                            int n)
{
    for (int i = 0; i < n; ++i) {
        const int32_t rc = check_f4(who, ptrs[i], names[i]);      // NULL passes
        if (rc) return rc;
    }
    return SS_OK;
}

static int32_t check_ln(const char *who, int32_t T, int32_t dim, int32_t Bcap)
{
    if (T < 1 || T > 65535)
        return fail(SS_ERR_INVALID_ARG, "%s: num_tables = %d (need 1..65535)", who, T);
    if (dim < 4 || dim % 4 != 0 || dim > 1024)
        return fail(SS_ERR_INVALID_ARG, "%s: dim = %d (need a multiple of 4 in [4, 1024])",
                    who, dim);
    if (Bcap < 1) return fail(SS_ERR_INVALID_ARG, "%s: Bcap = %d", who, Bcap);
    return SS_OK;
}

int32_t ss_layernorm_forward(int32_t num_tables, int32_t dim, const float *x, int32_t Bcap,
                             const int32_t *n_valid, const float *gamma, const float *beta,
                             float eps, float *y, float *mean, float *rstd, void *stream)
{
    const char *who = "ss_layernorm_forward";
    int32_t rc = check_ln(who, num_tables, dim, Bcap);
    if (rc) return rc;
    if (!x || !y || !mean || !rstd)
        return fail(SS_ERR_INVALID_ARG, "%s: x, y, mean or rstd is NULL", who);
    if (!(eps >= 0.0f)) return fail(SS_ERR_INVALID_ARG, "%s: eps = %g", who, (double)eps);
    {
        const void *const ptrs[] = {x, y, gamma, beta};
        const char *const names[] = {"x", "y", "gamma", "beta"};
        rc = check_f4_all(who, ptrs, names, 4);
        if (rc) return rc;
    }
    return launch_layernorm_forward(num_tables, dim, x, nullptr, nullptr, 1, Bcap, n_valid,
                                    gamma, beta, eps, y, mean, rstd,
                                    static_cast<hipStream_t>(stream));
}

int32_t ss_embbag_forward_ln(const ss_tables *tables, const int32_t *idx, int32_t Bcap,
                             int32_t L, const int32_t *n_valid, const float *gamma,
                             const float *beta, float eps, float *y, float *mean,
                             float *rstd, void *stream)
{
    const char *who = "ss_embbag_forward_ln";
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    rc = check_batch(who, idx, Bcap, L, tables->num_tables);
    if (rc) return rc;
    if (!y || !mean || !rstd)
        return fail(SS_ERR_INVALID_ARG, "%s: y, mean or rstd is NULL", who);
    if (!(eps >= 0.0f)) return fail(SS_ERR_INVALID_ARG, "%s: eps = %g", who, (double)eps);
    {
        const void *const ptrs[] = {y, gamma, beta};
        const char *const names[] = {"y", "gamma", "beta"};
        rc = check_f4_all(who, ptrs, names, 3);
        if (rc) return rc;
    }
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_layernorm_forward(tables->num_tables, tables->dim, nullptr, tables->weights,
                                    idx, L, Bcap, n_valid, gamma, beta, eps, y, mean, rstd,
                                    static_cast<hipStream_t>(stream));
}

size_t ss_layernorm_backward_workspace_bytes(int32_t num_tables, int32_t dim, int32_t Bcap)
{
    if (num_tables < 1 || num_tables > 65535 || dim < 4 || dim % 4 != 0 || dim > 1024 ||
        Bcap < 1)
        return 0;
    return layernorm_backward_ws_bytes(num_tables, dim, Bcap);
}

int32_t ss_layernorm_backward(int32_t num_tables, int32_t dim, const float *dy,
                              const float *x, int32_t Bcap, const int32_t *n_valid,
                              const float *gamma, const float *mean, const float *rstd,
                              float *dx, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream)
{
    const char *who = "ss_layernorm_backward";
    int32_t rc = check_ln(who, num_tables, dim, Bcap);
    if (rc) return rc;
    if (!dy || !x || !mean || !rstd || !dx)
        return fail(SS_ERR_INVALID_ARG, "%s: dy, x, mean, rstd or dx is NULL", who);
    if (dgamma || dbeta) {
        rc = check_ws(who, ws, ws_bytes, layernorm_backward_ws_bytes(num_tables, dim, Bcap));
        if (rc) return rc;
    }
    {
        const void *const ptrs[] = {dy, x, dx, gamma, dgamma, dbeta};
        const char *const names[] = {"dy", "x", "dx", "gamma", "dgamma", "dbeta"};
        rc = check_f4_all(who, ptrs, names, 6);
        if (rc) return rc;
    }
    return launch_layernorm_backward(num_tables, dim, dy, x, nullptr, nullptr, 1, Bcap, n_valid,
                                     gamma, mean, rstd, dx, dgamma, dbeta, ws,
                                     static_cast<hipStream_t>(stream));
}

int32_t ss_embbag_ln_backward(const ss_tables *tables, const int32_t *idx, int32_t Bcap,
                              int32_t L, const int32_t *n_valid, const float *dy,
                              const float *gamma, const float *mean, const float *rstd,
                              float *dx, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream)
{
    const char *who = "ss_embbag_ln_backward";
    int32_t rc = check_tables(tables, who);
    if (rc) return rc;
    rc = check_batch(who, idx, Bcap, L, tables->num_tables);
    if (rc) return rc;
    if (!dy || !mean || !rstd || !dx)
        return fail(SS_ERR_INVALID_ARG, "%s: dy, mean, rstd or dx is NULL", who);
    if (dgamma || dbeta) {
        rc = check_ws(who, ws, ws_bytes,
                      layernorm_backward_ws_bytes(tables->num_tables, tables->dim, Bcap));
        if (rc) return rc;
    }
    {
        const void *const ptrs[] = {dy, dx, gamma, dgamma, dbeta};
        const char *const names[] = {"dy", "dx", "gamma", "dgamma", "dbeta"};
        rc = check_f4_all(who, ptrs, names, 5);
        if (rc) return rc;
    }
    rc = checked_indices(who, tables->num_tables, tables->rows, idx, Bcap, L, n_valid,
                         static_cast<hipStream_t>(stream));
    if (rc) return rc;
    return launch_layernorm_backward(tables->num_tables, tables->dim, dy, nullptr,
                                     tables->weights, idx, L, Bcap, n_valid, gamma, mean, rstd,
                                     dx, dgamma, dbeta, ws, static_cast<hipStream_t>(stream));
}

}  // extern "C"
