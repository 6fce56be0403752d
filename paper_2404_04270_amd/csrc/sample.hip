// ss_sample_drop: the input sampling block (section 3.3, Eq. 1-2 of the paper).
//
// For a set of sampled inputs it counts, for every threshold of a ladder at
// once, how many of them could be dropped: those with at least alpha lookups
// that reach a stale hot row.  The paper evaluates one threshold per pass over
// the sampled rows; here the drift of every hot row is computed once (by
// ss_detect_stale, which can write it out) and this kernel only looks drifts
// up, so a pass costs 8 bytes per lookup whatever the row length, and up to 32
// thresholds share that pass.
//
// G lanes share one sampled input and split its T*L lookups between them.  A
// lookup maps its row to a hot slot by a branch-free lower-bound search in the
// ascending hot_ids of its table; a lane runs up to four such searches
// interleaved, since each step is one dependent load that only latency
// bounds.  Per-threshold stale-lookup counts are summed over the group with
// wavefront shuffles, turned into verdicts by the group's first lane, counted
// per wavefront with ballots, per workgroup in LDS and once per workgroup in
// global memory.
#include "ss_common.h"

namespace ss {

// Thresholds as the kernel compares them: widened to fp64 on the host, and -1
// where no row may be stale (threshold 0 or an unused slot), since a drift is
// never below 0.  They arrive as kernel arguments and stay in scalar registers.
struct Ladder {
    double thr[SS_MAX_THRESHOLDS];
};

constexpr int kBatch = 4;     // searches a lane keeps in flight

template <int G>
__global__ __launch_bounds__(kWG) void sample_drop_kernel(
    const int32_t *const *__restrict__ hot_ids, int H,
    const double *const *__restrict__ drift, const int32_t *__restrict__ sidx, int S,
    int L, int TL, int alpha, Ladder ladder, int n_thr, uint32_t *__restrict__ counts)
{
    __shared__ uint32_t s_cnt[SS_MAX_THRESHOLDS];
    if (threadIdx.x < SS_MAX_THRESHOLDS) s_cnt[threadIdx.x] = 0;
    __syncthreads();

    constexpr int GROUPS = kWG / G;
    const int g = threadIdx.x / G, c = threadIdx.x % G;
    const int s = blockIdx.x * GROUPS + g;
    const bool valid = s < S;

    uint32_t cnt[SS_MAX_THRESHOLDS];
#pragma unroll
    for (int k = 0; k < SS_MAX_THRESHOLDS; ++k) cnt[k] = 0;

    if (valid && H > 0) {
        for (int q0 = c; q0 < TL; q0 += G * kBatch) {
            int32_t row[kBatch];
            int base[kBatch];
            gptr<const int32_t> ids[kBatch];
            gptr<const double> dr[kBatch];
            bool live[kBatch];
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const int q = q0 + i * G;
                live[i] = q < TL;
                const int qq = live[i] ? q : c;         // c < TL whenever q0 < TL
                const int t = qq / L, l = qq - t * L;
                row[i] = sidx[((int64_t)t * S + s) * L + l];
                ids[i] = as_global(hot_ids[t]);
                dr[i] = as_global(drift[t]);
                base[i] = 0;
            }
            // lower bound: the last slot whose id is <= row (slot 0 if none is)
            for (int n = H; n > 1;) {
                const int half = n >> 1;
#pragma unroll
                for (int i = 0; i < kBatch; ++i)
                    if (ids[i][base[i] + half] <= row[i]) base[i] += half;
                n -= half;
            }
#pragma unroll
            for (int i = 0; i < kBatch; ++i) {
                const bool hot = live[i] && ids[i][base[i]] == row[i];
                const double d = dr[i][base[i]];
#pragma unroll
                for (int k = 0; k < SS_MAX_THRESHOLDS; ++k) {
                    // same verdict as ss_detect_stale; a NaN drift compares false
                    const bool stale = hot && d <= ladder.thr[k];
                    cnt[k] += stale ? 1u : 0u;
                }
            }
        }
    }

    const int lane = threadIdx.x & 63;
#pragma unroll
    for (int k = 0; k < SS_MAX_THRESHOLDS; ++k) {
        uint32_t v = cnt[k];
#pragma unroll
        for (int off = G / 2; off > 0; off >>= 1) v += __shfl_xor(v, off, G);
        const bool drop = valid && c == 0 && k < n_thr && (int64_t)v >= (int64_t)alpha;
        const unsigned long long bal = __ballot(drop);
        if (lane == 0 && bal) atomicAdd(&s_cnt[k], (uint32_t)__popcll(bal));
    }
    __syncthreads();
    if ((int)threadIdx.x < n_thr && s_cnt[threadIdx.x])
        atomicAdd(&counts[threadIdx.x], s_cnt[threadIdx.x]);
}

int32_t launch_sample_drop(int T, int32_t *const *hot_ids, int H, double *const *drift,
                           const int32_t *sidx, int S, int L, int alpha,
                           const float *thresholds, int n_thr, uint32_t *counts,
                           hipStream_t s)
{
    launch_zero_u32(counts, n_thr, s);
    if (S > 0) {
        Ladder ladder;
        for (int k = 0; k < SS_MAX_THRESHOLDS; ++k)
            ladder.thr[k] = k < n_thr && thresholds[k] > 0.0f ? (double)thresholds[k] : -1.0;
        const int TL = T * L;
        int g = 1;
        while (g < 64 && g * kBatch < TL) g <<= 1;
        const int groups = kWG / g;
        const unsigned grid = (unsigned)(((int64_t)S + groups - 1) / groups);
        ProfScope prof("sample_drop_kernel", s);
        SS_DISPATCH_G(g, launch(sample_drop_kernel<G>, dim3(grid), dim3(kWG), s,
                                (const int32_t *const *)hot_ids, H,
                                (const double *const *)drift, sidx, S, L, TL, alpha,
                                ladder, n_thr, counts));
    }
    return check_launch("ss_sample_drop");
}

}  // namespace ss
