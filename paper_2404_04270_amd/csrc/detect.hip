// ss_detect_stale: drift of every hot row against its last snapshot (Eq. 1,
// Eq. 5 of the paper), thresholded into the stale bitmap, with the snapshot
// refresh fused in so the hot rows are read from HBM once.
//
// A group of G lanes owns one hot slot; each lane holds one f4 of the row
// and of its snapshot, squares the fp64 differences and the group reduces them
// with wavefront shuffles.  fp64 is used because the verdict is compared
// bit-exactly with a reference outside a 1e-6 relative band around T, which an
// fp32 sum of up to 128 squares cannot guarantee; the kernel moves 12 bytes per
// element, so the extra arithmetic is hidden behind the memory traffic.
// Verdicts are staged in LDS; one lane per bitmap word then merges the bits of
// neighbouring hot rows into a single atomic OR.
#include "ss_common.h"

namespace ss {

__global__ void zero_u32_kernel(uint32_t *p, int n)
{
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0;
}

void launch_zero_u32(uint32_t *p, int n, hipStream_t s)
{
    if (n > 0) launch(zero_u32_kernel, dim3((n + 255) / 256), dim3(256), s, p, n);
}

template <int G, typename TS>
__global__ __launch_bounds__(kWG) void detect_kernel(
    const float *const *__restrict__ weights, uint32_t *const *__restrict__ bits,
    const int32_t *const *__restrict__ hot_ids, int H,
    float *const *__restrict__ snapshot, float threshold, int refresh,
    uint8_t *const *__restrict__ stale_hot, double *const *__restrict__ drift,
    uint32_t *__restrict__ stale_count, int D4, int tiles_per_table, TS ts)
{
    constexpr int SLOTS = kWG / G;
    const unsigned long long trace_t0 = trace_begin<TS>();
    __shared__ uint32_t s_row[SLOTS];
    __shared__ uint8_t s_flag[SLOTS];
    const int t = blockIdx.x / tiles_per_table;
    const int tile = blockIdx.x - t * tiles_per_table;
    const int g = threadIdx.x / G, c = threadIdx.x % G;
    const int h = tile * SLOTS + g;
    const bool valid = h < H;
    uint32_t r = kNoRow;
    double acc = 0.0;
    if (valid) {
        r = (uint32_t)as_global(hot_ids[t])[h];
        const auto W =
            as_global(reinterpret_cast<const f4 *>(weights[t])) + (int64_t)r * D4;
        const auto S = as_global(reinterpret_cast<f4 *>(snapshot[t])) + (int64_t)h * D4;
        for (int col = c; col < D4; col += G) {
            const f4 w = W[col];
            const f4 s = S[col];
            const double ex = (double)w.x - (double)s.x;
            const double ey = (double)w.y - (double)s.y;
            const double ez = (double)w.z - (double)s.z;
            const double ew = (double)w.w - (double)s.w;
            acc += ex * ex;
            acc += ey * ey;
            acc += ez * ez;
            acc += ew * ew;
            if (refresh) S[col] = w;
        }
    }
#pragma unroll
    for (int off = G / 2; off > 0; off >>= 1) acc += __shfl_xor(acc, off, G);

    bool stale = false;
    if (valid && c == 0) {
        const double dist = sqrt(acc);
        stale = threshold > 0.0f && dist <= (double)threshold;
        if (stale_hot && stale_hot[t]) as_global(stale_hot[t])[h] = stale ? 1 : 0;
        if (drift && drift[t]) as_global(drift[t])[h] = dist;
    }
    if (c == 0) {
        s_row[g] = r;
        s_flag[g] = stale ? 1 : 0;
    }
    __syncthreads();
    if (threadIdx.x < SLOTS) {
        const int k = threadIdx.x;
        const uint32_t row = s_row[k];
        const uint32_t word = row >> 5;
        const bool first = row != kNoRow && (k == 0 || (s_row[k - 1] >> 5) != word);
        if (first) {
            uint32_t mask = 0;
            for (int q = k; q < SLOTS && s_row[q] != kNoRow && (s_row[q] >> 5) == word; ++q)
                if (s_flag[q]) mask |= 1u << (s_row[q] & 31);
            if (mask) atomicOr((uint32_t *)&as_global(bits[t])[word], mask);
        }
        if (stale_count) {
            const unsigned long long bal = __ballot(s_flag[k] != 0);
            if ((k & 63) == 0 && bal) atomicAdd(&stale_count[t], (uint32_t)__popcll(bal));
        }
    }
    trace_end(ts, trace_t0);
}

int32_t launch_detect(const ss_tables *tb, int32_t *const *hot_ids, int H,
                      float **snapshot, float threshold, int refresh,
                      uint8_t **stale_hot, double **drift,
                      uint32_t *stale_count, hipStream_t s)
{
    const int T = tb->num_tables;
    const int D4 = tb->dim / 4;
    const int g = lanes_per_row(tb->dim);
    const int slots = kWG / g;
    const int tiles = (H + slots - 1) / slots;
    if (stale_count) launch_zero_u32(stale_count, T, s);
    ProfScope prof("detect_kernel", s);
    SS_DISPATCH_G(g, launch(SS_BOTH(detect_kernel, G), dim3((unsigned)(tiles * T)), dim3(kWG), s,
                            tb->weights, tb->stale_bits, hot_ids, H, snapshot, threshold,
                            refresh, stale_hot, drift, stale_count, D4, tiles));
    return check_launch("ss_detect_stale");
}

}  // namespace ss
