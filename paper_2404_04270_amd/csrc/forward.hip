// ss_embbag_forward: sum-pooled gather (section 2.1 of the paper: one pooled
// vector per table and sample).
//
// Bound by HBM: every looked-up row is read once (duplicates hit L2 / MALL),
// every pooled row written once, no arithmetic for L = 1.  A group of G lanes
// owns one bag; each lane carries one float4 of the row, so a wavefront reads
// 64/G rows per load instruction with 16-byte accesses that cover whole rows.
// The indices of up to 8 lookups are fetched first and their row loads issued
// back to back, so each lane keeps 8 independent 16-byte loads in flight.
#include "ss_common.h"

namespace ss {

template <int G>
__global__ __launch_bounds__(kWG) void forward_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, int L, const int32_t *__restrict__ n_valid,
    float *__restrict__ out, int D4, int tiles_per_table)
{
    constexpr int BAGS = kWG / G;
    const int t = blockIdx.x / tiles_per_table;
    const int tile = blockIdx.x - t * tiles_per_table;
    const int n = clamp_valid(n_valid, Bcap);
    const int j = tile * BAGS + (int)threadIdx.x / G;
    if (j >= n) return;
    const int c = threadIdx.x % G;
    const float4 *__restrict__ W = reinterpret_cast<const float4 *>(weights[t]);
    const int32_t *__restrict__ ip = idx + ((int64_t)t * Bcap + j) * L;
    float4 *__restrict__ o =
        reinterpret_cast<float4 *>(out) + ((int64_t)t * Bcap + j) * D4;

    for (int col = c; col < D4; col += G) {
        // first row initialises the sum, so that L = 1 is a bit-exact copy
        float4 acc = W[(int64_t)ip[0] * D4 + col];
        int l = 1;
        for (; l + 8 <= L; l += 8) {
            int32_t r[8];
            float4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) r[k] = ip[l + k];
#pragma unroll
            for (int k = 0; k < 8; ++k) v[k] = W[(int64_t)r[k] * D4 + col];
#pragma unroll
            for (int k = 0; k < 8; ++k) acc = acc + v[k];
        }
        if (l < L) {
            int32_t r[8];
            float4 v[8];
#pragma unroll
            for (int k = 0; k < 8; ++k) r[k] = (l + k < L) ? ip[l + k] : 0;
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (l + k < L) v[k] = W[(int64_t)r[k] * D4 + col];
#pragma unroll
            for (int k = 0; k < 8; ++k)
                if (l + k < L) acc = acc + v[k];
        }
        o[col] = acc;
    }
}

int32_t launch_forward(const ss_tables *tb, const int32_t *idx, int Bcap, int L,
                       const int32_t *n_valid, float *out, hipStream_t s)
{
    const int D4 = tb->dim / 4;
    const int g = lanes_per_row(tb->dim);
    const int bags = kWG / g;
    const int tiles = (Bcap + bags - 1) / bags;
    const int64_t blocks = (int64_t)tiles * tb->num_tables;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_forward: grid too large");
    ProfScope prof("forward_kernel", s);
    SS_DISPATCH_G(g, hipLaunchKernelGGL(forward_kernel<G>, dim3((unsigned)blocks),
                                        dim3(kWG), 0, s, tb->weights, idx, Bcap,
                                        L, n_valid, out, D4, tiles));
    return check_launch("ss_embbag_forward");
}

}  // namespace ss
