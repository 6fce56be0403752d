// Internal helpers shared by the kernels of libslipstream (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>

#include <type_traits>
#include <hip/hip_ext.h>
#include <stdint.h>

#include "slipstream.h"

namespace ss {

constexpr int kWG = 256;                    // threads per workgroup (4 wavefronts)
constexpr uint32_t kNoRow = 0xFFFFFFFFu;    // sentinel key: "no lookup here"

// Records the calling thread's error text; returns `code`.
int32_t fail(int32_t code, const char *fmt, ...);
// Common checks of an ss_tables argument.
int32_t check_tables(const ss_tables *tb, const char *who);
// hipGetLastError() after a launch -> SS_OK / SS_ERR_HIP.
int32_t check_launch(const char *who);
// Host-side checks of the arguments of ss_filter_batch and of the backward calls.
int32_t check_filter(const char *who, const ss_tables *tables, const int32_t *idx,
                     int32_t B, int32_t L, const uint8_t *skip_mask,
                     const int32_t *kept_ids, const int32_t *n_kept,
                     const int32_t *idx_c, const void *ws, size_t ws_bytes);
int32_t check_backward(const char *who, const ss_tables *tables, int32_t Bcap,
                       int32_t L, const void *ws, size_t ws_bytes);

// Checked mode (SS_CHECK=1 / ss_check_enable): the ids are range-checked by a
// kernel that reads nothing else, the host waits for its report, and an id
// outside [0, rows) becomes SS_ERR_INVALID_ARG before anything else is
// enqueued.  Both return SS_OK at once when the mode is off.
bool check_mode();
int32_t checked_indices(const char *who, int T, int64_t rows, const int32_t *idx, int cap,
                        int L, const int32_t *n_valid, hipStream_t s);
int32_t checked_hot_ids(const char *who, int T, int64_t rows, int32_t *const *hot_ids, int H,
                        hipStream_t s);

// Optional per-kernel timing (ss_profile_enable).  While a ProfScope is alive on
// this thread and profiling is on, launch() attaches a pair of events to the
// kernel it dispatches; the runtime stamps them with the start and the end of
// that dispatch on the GPU, so their difference is the kernel's own duration
// (no launch gap, no neighbouring kernel).
class ProfScope {
public:
    ProfScope(const char *kernel, hipStream_t s);
    ~ProfScope();
};
// While one is alive on this thread, ProfScope records nothing (for entry points
// that must not create HIP objects).
class ProfMute {
public:
    ProfMute();
    ~ProfMute();
};
// Events of the innermost live ProfScope, or false when profiling is off.
bool prof_events(hipEvent_t *start, hipEvent_t *stop);
// While profiling is on, a stream that has just been made to wait for an event
// gets an empty kernel of its own.  The runtime attaches the wait to the next
// command of the stream, and the event pair of that command then spans the wait
// as well: the empty kernel takes it, so that the kernel after it is timed alone.
void after_stream_wait(hipStream_t s);

// Trace mode (ss_profile_enable(2)): the kernels of the training iteration stamp
// the GPU's constant-rate clock when their first workgroups start and when each
// workgroup ends, into a slot of a device buffer that belongs to the launch, so
// that the real overlap and the gaps of a free-running pipeline can be read
// afterwards; no event pair, no extra host cost.  Such a kernel has the type of
// its last parameter as a template parameter: TraceSlot in the variant that
// stamps, NoTrace (nothing at all) in the one that runs otherwise; launch() is
// given both and picks.  (One variant with a slot pointer that is null while
// tracing is off was measured: the test of the pointer, or the clock read that
// avoids it, costs 0.2-0.7 us per training step at 26 tables of 8192 lookups and
// 1.2 us at 8 tables of 81920.)
constexpr int kTraceLanes = 64;
constexpr size_t kTraceMax = 1u << 15;       // launches per trace
struct TraceSlot {
    // kTraceLanes start stamps of this launch; its end stamps lie kTraceMax * kTraceLanes
    // words further on (all start stamps first, then all end stamps: two fills set
    // the buffer up).  nullptr: tracing is off
    unsigned long long *p;
};
struct NoTrace {};
TraceSlot next_trace_slot();

__device__ __forceinline__ unsigned trace_block_id()
{
    return blockIdx.x + gridDim.x * (blockIdx.y + gridDim.y * blockIdx.z);
}
template <typename TS> __device__ __forceinline__ unsigned long long trace_begin()
{
    if constexpr (std::is_same<TS, TraceSlot>::value) return wall_clock64();
    return 0ull;
}
__device__ __forceinline__ void trace_end(NoTrace, unsigned long long) {}
__device__ __forceinline__ void trace_end(TraceSlot ts, unsigned long long t0)
{
    if (ts.p && threadIdx.x == 0) {
        const unsigned b = trace_block_id();
        if (b < (unsigned)kTraceLanes) ts.p[b] = t0;
        atomicMax(&ts.p[kTraceMax * kTraceLanes + (b & (kTraceLanes - 1))],
                  (unsigned long long)wall_clock64());
    }
}

// k<..., NoTrace>, k<..., TraceSlot>: the two variants of a kernel template, for launch()
#define SS_BOTH(kernel, ...) (kernel<__VA_ARGS__, NoTrace>), (kernel<__VA_ARGS__, TraceSlot>)

// The next launch of the calling thread also records `ev` when its kernel has
// ended: the event rides on the dispatch's own completion signal, and the stream
// gets no separate command for it (between two dependent kernels such a command
// costs the stream several microseconds).
void stop_event_for_next_launch(hipEvent_t ev);
hipEvent_t take_stop_event();

template <typename K, typename... Args>
inline void launch_with_events(K kernel, dim3 grid, dim3 block, hipStream_t s, Args... args)
{
    hipEvent_t e0, e1;
    const hipEvent_t stop = take_stop_event();
    if (prof_events(&e0, &e1)) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, e0, e1, 0, args...);
        if (stop) (void)hipEventRecord(stop, s);
    } else if (stop) {
        hipExtLaunchKernelGGL(kernel, grid, block, 0, s, nullptr, stop, 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, grid, block, 0, s, args...);
    }
}

template <typename... KArgs, typename... Args>
inline void launch(void (*kernel)(KArgs...), dim3 grid, dim3 block, hipStream_t s,
                   Args... args)
{
    launch_with_events(kernel, grid, block, s, args...);
}

// A kernel with a traced variant: `plain` takes a NoTrace after args, `traced` a TraceSlot.
template <typename... PArgs, typename... TArgs, typename... Args>
inline void launch(void (*plain)(PArgs...), void (*traced)(TArgs...), dim3 grid, dim3 block,
                   hipStream_t s, Args... args)
{
    static_assert(sizeof...(PArgs) == sizeof...(Args) + 1 && sizeof...(TArgs) == sizeof...(Args) + 1,
                  "both variants take the arguments plus the trace parameter");
    const TraceSlot ts = next_trace_slot();
    if (ts.p) launch_with_events(traced, grid, block, s, args..., ts);
    else launch_with_events(plain, grid, block, s, args..., NoTrace{});
}

// Lanes that cooperate on one row: one f4 per lane, a power of two <= 64.
inline int lanes_per_row(int dim)
{
    int d4 = dim / 4, g = 1;
    while (g < d4 && g < 64) g <<= 1;
    return g;
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Calls f.template operator()<G>() for the power of two G in [1, 64].
#define SS_DISPATCH_G(g, ...)                                   \
    switch (g) {                                                \
    case 1: { constexpr int G = 1; __VA_ARGS__; } break;        \
    case 2: { constexpr int G = 2; __VA_ARGS__; } break;        \
    case 4: { constexpr int G = 4; __VA_ARGS__; } break;        \
    case 8: { constexpr int G = 8; __VA_ARGS__; } break;        \
    case 16: { constexpr int G = 16; __VA_ARGS__; } break;      \
    case 32: { constexpr int G = 32; __VA_ARGS__; } break;      \
    default: { constexpr int G = 64; __VA_ARGS__; } break;      \
    }

__device__ __forceinline__ int clamp_valid(const int32_t *n_valid, int cap)
{
    if (!n_valid) return cap;
    int n = *n_valid;
    return n < 0 ? 0 : (n > cap ? cap : n);
}

// Four consecutive floats of a row: a native vector, so that it can be loaded
// and stored through pointers of any address space with one 16-byte access.
typedef float f4 __attribute__((ext_vector_type(4)));

// w - lr * g, element by element
__device__ __forceinline__ f4 sgd(f4 w, f4 g, float lr) { return w - lr * g; }

// Pointers read out of a device array of pointers (tables, bitmaps, snapshots)
// carry no address space, which would make every access through them a FLAT
// instruction.  They always point into global memory: say so.
template <typename T> using gptr = T __attribute__((address_space(1))) *;
template <typename T> __device__ __forceinline__ gptr<T> as_global(T *p)
{
    return (gptr<T>)p;
}

// log2 of a power of two, at compile time
constexpr int ilog2(int x) { return x <= 1 ? 0 : 1 + ilog2(x / 2); }

// Four registers that hold "nothing yet": a value loaded under a condition needs
// some content on the other path, and zeros would cost four moves each time.
__device__ __forceinline__ f4 unset_f4()
{
    f4 v;
    asm volatile("" : "=v"(v));
    return v;
}

// Address of one lane's f4 of row r, given the address of that f4 in row 0.
// When a row fills its group of lanes exactly (FULL), the row length is the
// constant G and the 64-bit product becomes two 32-bit shifts.
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
template <int G, bool FULL, typename P>
__device__ __forceinline__ P row_ptr(P lane_base, uint32_t r, uint32_t d4)
{
    if (FULL) {
        constexpr int SH = ilog2(G) + 4;
        const u32x2 off = {r << SH, r >> (32 - SH)};
        return (P)((gptr<char>)lane_base + __builtin_bit_cast(uint64_t, off));
    }
    return lane_base + (uint64_t)r * d4;
}


// Workgroups are handed to the eight XCDs in turn (block b runs on XCD b % 8),
// and each XCD has an L2 of its own.  Where the same lines of a table are read
// again and again (hot rows in a multi-hot forward pass, a table's gradient rows
// in the update), they should sit in ONE L2 and not in eight: the first
// `pinned_blocks` blocks (per_table blocks for each of a multiple of 8 tables)
// keep every table on one XCD, the other tables are spread as usual.
__device__ __forceinline__ void block_to_table_pinned(int b, int per_table,
                                                      int pinned_blocks, int &t, int &i)
{
    if (b < pinned_blocks) {
        const int xcd = b & 7, j = b >> 3;
        const int q = j / per_table;
        t = q * 8 + xcd;
        i = j - q * per_table;
    } else {
        t = b / per_table;
        i = b - t * per_table;
    }
}

__device__ __forceinline__ bool bit_set(gptr<const uint32_t> bits, uint32_t r)
{
    return (bits[r >> 5] >> (r & 31)) & 1u;
}

// Entry points of the kernel families (each in its own .hip file).
int32_t launch_forward(const ss_tables *tb, const int32_t *idx, int Bcap, int L,
                       const int32_t *n_valid, float *out, hipStream_t s);
int32_t launch_filter(const ss_tables *tb, const int32_t *idx, int B, int L,
                      int alpha, uint8_t *skip_mask, int32_t *kept_ids,
                      int32_t *n_kept, int32_t *idx_c, void *ws, hipStream_t s);
// The same with a second set of bitmaps (hot rows): hot_mask[b] = every lookup of
// sample b is a hot row.  hot_mask == nullptr: the plain filter.
int32_t launch_filter_split(const ss_tables *tb, uint32_t *const *hot_bits, const int32_t *idx,
                            int B, int L, int alpha, uint8_t *skip_mask, uint8_t *hot_mask,
                            int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c, void *ws,
                            hipStream_t s);
int32_t launch_detect(const ss_tables *tb, int32_t *const *hot_ids, int H,
                      float **snapshot, float threshold, int refresh,
                      uint8_t **stale_hot, double **drift,
                      uint32_t *stale_count, hipStream_t s);
// record_after (may be null): an event to record when the grouped lists are complete
int32_t launch_backward_prepare(const ss_tables *tb, const int32_t *idx, int Bcap,
                                int L, const int32_t *n_valid, void *ws,
                                hipStream_t s, hipEvent_t record_after = nullptr);
// ss_issue_index_batch with an event (may be null) that the job records behind its
// last launch
int32_t issue_index_batch(::ss_issue_queue *q, const ss_tables *tables, const int32_t *idx,
                          int32_t B, int32_t L, int32_t alpha, uint8_t *skip_mask,
                          int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c, void *ws_filter,
                          size_t ws_filter_bytes, void *ws_backward, size_t ws_backward_bytes,
                          void *stream, void *record_after, uint64_t *ticket);
// record_after (may be null): an event to record when the update is complete
int32_t launch_backward_apply(const ss_tables *tb, int Bcap, int L, const float *grad,
                              float lr, void *ws, hipStream_t s,
                              hipEvent_t record_after = nullptr);
size_t backward_ws_bytes(int T, int Bcap, int L, int dim);
// Where stage 1 of the backward pass leaves a table's grouped lookups when it
// takes the one-launch path (buffer 0 of the workspace), and the padded length.
void backward_first_buffers(int T, int Bcap, int L, int dim, void *ws, uint2 **ent,
                            int *NP);
bool can_fuse_forward_group(const ss_tables *tb, int Bcap, int L);
int32_t launch_forward_group(const ss_tables *tb, const int32_t *idx, int Bcap,
                             const int32_t *n_valid, float *out, uint2 *ent, int NP,
                             hipStream_t s);
size_t filter_ws_bytes(int T, int B, int L);
int32_t launch_sample_drop(int T, int32_t *const *hot_ids, int H, double *const *drift,
                           const int32_t *sidx, int S, int L, int alpha,
                           const float *thresholds, int n_thr, uint32_t *counts,
                           hipStream_t s);
int32_t launch_count_accesses(int T, const int32_t *idx, int Bcap, int L,
                              const int32_t *n_valid, uint32_t *const *counts,
                              hipStream_t s);
size_t select_hot_ws_bytes(int T, int64_t R);
// Rows with count > c, and the first e rows (by id) with count == c; with `top`
// set, c and e are first replaced by the outcome of a radix select for the e
// largest counts.
int32_t launch_select_hot(int T, int64_t R, uint32_t *const *counts, bool top, uint32_t c,
                          uint32_t e, int32_t *const *hot_ids, int cap,
                          uint32_t *const *hot_bits, uint32_t *n_hot, void *ws, hipStream_t s);
// x != nullptr: vectors are read from x; x == nullptr: they are pooled from
// weights / idx / L on the fly.
int32_t launch_layernorm_forward(int T, int dim, const float *x, const float *const *weights,
                                 const int32_t *idx, int L, int Bcap, const int32_t *n_valid,
                                 const float *gamma, const float *beta, float eps, float *y,
                                 float *mean, float *rstd, hipStream_t s);
size_t layernorm_backward_ws_bytes(int T, int dim, int Bcap);
int32_t launch_layernorm_backward(int T, int dim, const float *dy, const float *x,
                                  const float *const *weights, const int32_t *idx, int L,
                                  int Bcap, const int32_t *n_valid, const float *gamma,
                                  const float *mean, const float *rstd, float *dx,
                                  float *dgamma, float *dbeta, void *ws, hipStream_t s);
// p[0..n) = 0 by a small kernel (a memset node would not survive graph capture)
void launch_zero_u32(uint32_t *p, int n, hipStream_t s);

}  // namespace ss
