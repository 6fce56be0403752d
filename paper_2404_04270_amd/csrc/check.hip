// Range check of lookup indices and hot row ids.
//
// The kernels of this library do not range-check row ids: an id outside
// [0, rows) makes them read or write outside a table.  Two aids for finding
// such an input without a fault:
//   - ss_check_indices: one pass over an index tensor that only reads the
//     indices themselves and leaves a report in device memory (how many entries
//     are out of range, and where the first one is); enqueued like any other
//     call, the caller reads the report when it likes.
//   - checked mode (environment SS_CHECK=1 when the library is loaded, or
//     ss_check_enable): every entry point that takes indices or hot row ids runs
//     that pass first, WAITS for it on the host, and returns SS_ERR_INVALID_ARG
//     without enqueueing anything else if an id is out of range.  A debugging
//     mode: it synchronises with the host on every call and holds 16 bytes of
//     device memory per GPU.
#include <stdlib.h>

#include <atomic>
#include <mutex>

#include "ss_common.h"

namespace ss {

namespace {

constexpr int kCheckWG = 256;
constexpr int kCheckItems = 8;       // entries per thread

// report[0] = out-of-range entries, report[1] = (table << 32 | position in the
// table) of the first one, all ones if there is none
__global__ void check_init_kernel(unsigned long long *report)
{
    report[0] = 0ull;
    report[1] = ~0ull;
}

// Entries [0, n * per_item) of each of the T lists; list t starts at
// base + t * stride (ptrs == nullptr) or at ptrs[t].
__global__ __launch_bounds__(kCheckWG) void check_range_kernel(
    const int32_t *__restrict__ base, int64_t stride, const int32_t *const *__restrict__ ptrs,
    int cap, int per_item, const int32_t *__restrict__ n_valid, int64_t rows,
    unsigned long long *__restrict__ report)
{
    const int t = blockIdx.y;
    const int64_t n = (int64_t)clamp_valid(n_valid, cap) * per_item;
    const int32_t *__restrict__ p = ptrs ? ptrs[t] : base + (int64_t)t * stride;
    const int64_t first = ((int64_t)blockIdx.x * kCheckWG * kCheckItems) + threadIdx.x;
    unsigned bad = 0;
    unsigned long long where = ~0ull;
#pragma unroll
    for (int i = 0; i < kCheckItems; ++i) {
        const int64_t q = first + (int64_t)i * kCheckWG;
        if (q < n) {
            const int64_t v = p[q];
            if (v < 0 || v >= rows) {
                ++bad;
                const unsigned long long key = ((unsigned long long)t << 32) | (unsigned long long)q;
                where = key < where ? key : where;
            }
        }
    }
    // few inputs are bad: one pair of atomics per lane that saw one
    if (bad) {
        atomicAdd(&report[0], (unsigned long long)bad);
        atomicMin(&report[1], where);
    }
}

std::atomic<int> g_check_mode{-1};           // -1: not read from the environment yet
std::mutex g_mu;
constexpr int kMaxDevices = 64;
unsigned long long *g_report[kMaxDevices] = {};

int32_t launch_check(const int32_t *base, int64_t stride, const int32_t *const *ptrs, int T,
                     int cap, int per_item, const int32_t *n_valid, int64_t rows,
                     unsigned long long *report, hipStream_t s)
{
    hipLaunchKernelGGL(check_init_kernel, dim3(1), dim3(1), 0, s, report);
    const int64_t per_block = (int64_t)kCheckWG * kCheckItems;
    const int64_t blocks = ((int64_t)cap * per_item + per_block - 1) / per_block;
    if (blocks > 0x7fffffffLL || T > 65535)
        return fail(SS_ERR_UNSUPPORTED, "ss_check_indices: grid too large");
    if (blocks > 0)
        hipLaunchKernelGGL(check_range_kernel, dim3((unsigned)blocks, T), dim3(kCheckWG), 0, s,
                           base, stride, ptrs, cap, per_item, n_valid, rows, report);
    return check_launch("ss_check_indices");
}

// The report buffer of checked mode on the current device (allocated on first use).
int32_t mode_report(const char *who, unsigned long long **out)
{
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices)
        return fail(SS_ERR_HIP, "%s: no usable current device", who);
    std::lock_guard<std::mutex> lk(g_mu);
    if (!g_report[dev]) {
        void *p = nullptr;
        if (hipMalloc(&p, 2 * sizeof(unsigned long long)) != hipSuccess)
            return fail(SS_ERR_HIP, "%s: checked mode could not allocate its report", who);
        g_report[dev] = static_cast<unsigned long long *>(p);
    }
    *out = g_report[dev];
    return SS_OK;
}

int32_t run_and_read(const char *who, const char *what, const int32_t *base, int64_t stride,
                     const int32_t *const *ptrs, int T, int cap, int per_item,
                     const int32_t *n_valid, int64_t rows, hipStream_t s)
{
    unsigned long long *report = nullptr;
    int32_t rc = mode_report(who, &report);
    if (rc) return rc;
    rc = launch_check(base, stride, ptrs, T, cap, per_item, n_valid, rows, report, s);
    if (rc) return rc;
    unsigned long long host[2] = {0, 0};
    if (hipMemcpyAsync(host, report, sizeof(host), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess)
        return fail(SS_ERR_HIP, "%s: checked mode could not read its report", who);
    if (host[0] == 0) return SS_OK;
    const long long t = (long long)(host[1] >> 32), q = (long long)(host[1] & 0xFFFFFFFFull);
    return fail(SS_ERR_INVALID_ARG,
                "%s: %llu %s outside [0, %lld); the first is in table %lld at position %lld "
                "(entry %lld, lookup %lld); nothing was enqueued",
                who, host[0], what, (long long)rows, t, q, q / per_item, q % per_item);
}

}  // namespace

bool check_mode()
{
    int m = g_check_mode.load(std::memory_order_relaxed);
    if (m < 0) {
        const char *e = getenv("SS_CHECK");
        m = (e && e[0] && !(e[0] == '0' && !e[1])) ? 1 : 0;
        g_check_mode.store(m, std::memory_order_relaxed);
    }
    return m != 0;
}

int32_t checked_indices(const char *who, int T, int64_t rows, const int32_t *idx, int cap,
                        int L, const int32_t *n_valid, hipStream_t s)
{
    if (!check_mode()) return SS_OK;
    return run_and_read(who, "lookup indices are", idx, (int64_t)cap * L, nullptr, T, cap, L,
                        n_valid, rows, s);
}

int32_t checked_hot_ids(const char *who, int T, int64_t rows, int32_t *const *hot_ids, int H,
                        hipStream_t s)
{
    if (!check_mode()) return SS_OK;
    return run_and_read(who, "hot row ids are", nullptr, 0, hot_ids, T, H, 1, nullptr, rows, s);
}

}  // namespace ss

using namespace ss;

extern "C" {

void ss_check_enable(int32_t on) { g_check_mode.store(on != 0 ? 1 : 0); }

int32_t ss_check_indices(int32_t num_tables, int64_t rows, const int32_t *idx, int32_t B,
                         int32_t L, const int32_t *n_valid, uint64_t *report, void *stream)
{
    const char *who = "ss_check_indices";
    if (num_tables < 1 || num_tables > 65535)
        return fail(SS_ERR_INVALID_ARG, "%s: num_tables = %d (need 1..65535)", who, num_tables);
    if (rows < 1 || rows >= (1LL << 31))
        return fail(SS_ERR_INVALID_ARG, "%s: rows = %lld (need 1 <= rows < 2^31)", who,
                    (long long)rows);
    if (!idx || !report) return fail(SS_ERR_INVALID_ARG, "%s: idx or report is NULL", who);
    if (reinterpret_cast<uintptr_t>(report) % 8 != 0)
        return fail(SS_ERR_INVALID_ARG, "%s: report is not 8-byte aligned", who);
    if (B < 1 || L < 1 || (int64_t)B * L >= (1LL << 31))
        return fail(SS_ERR_INVALID_ARG, "%s: B = %d, L = %d", who, B, L);
    return launch_check(idx, (int64_t)B * L, nullptr, num_tables, B, L, n_valid, rows,
                        reinterpret_cast<unsigned long long *>(report),
                        static_cast<hipStream_t>(stream));
}

}  // extern "C"
