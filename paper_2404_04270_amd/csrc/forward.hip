// ss_embbag_forward: sum-pooled gather (section 2.1 of the paper: one pooled
// vector per table and sample).
//
// Bound by HBM: every looked-up row is read once (duplicates hit L2 / MALL),
// every pooled row written once, no arithmetic for L = 1.  A group of G lanes
// owns a bag; each lane carries one f4 of the row, so a wavefront reads
// 64/G rows per load instruction with 16-byte accesses that cover whole rows.
// What limits a gather is the number of independent loads in flight, so
//   - one-hot bags (L = 1): a group takes 8 bags, fetches their 8 indices, then
//     issues the 8 row loads back to back before the first store;
//   - multi-hot bags: the indices of up to 24 lookups of the bag are fetched
//     first and their row loads issued together.
// Pinning all workgroups of a table to one XCD (so that its hot rows live in one
// L2 instead of eight) was measured and dropped: no change at 8 tables x 10M rows
// (29.1 vs 28.8 us), the 256 MB memory-side cache already absorbs the re-reads.
#include "forward_body.h"
#include "ss_common.h"

namespace ss {

template <int G>
__global__ __launch_bounds__(kWG) void forward_onehot_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, const int32_t *__restrict__ n_valid, float *__restrict__ out,
    int D4, int tiles_per_table)
{
    forward_onehot_body<G, kWG>(blockIdx.x, weights, idx, Bcap, n_valid, out, D4,
                                tiles_per_table);
}

// U = row loads issued together per lane.
template <int G, int U>
__global__ __launch_bounds__(kWG) void forward_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, int L, const int32_t *__restrict__ n_valid,
    float *__restrict__ out, int D4, int tiles_per_table)
{
    constexpr int BAGS = kWG / G;
    int t, tile;
    block_to_table_tile(blockIdx.x, tiles_per_table, t, tile);
    const int n = clamp_valid(n_valid, Bcap);
    const int j = tile * BAGS + (int)threadIdx.x / G;
    if (j >= n) return;
    const int c = threadIdx.x % G;
    const auto W = as_global(reinterpret_cast<const f4 *>(weights[t]));
    const int32_t *__restrict__ ip = idx + ((int64_t)t * Bcap + j) * L;
    f4 *__restrict__ o = reinterpret_cast<f4 *>(out) + ((int64_t)t * Bcap + j) * D4;

    for (int col = c; col < D4; col += G) {
        // the first row initialises the sum; later rows are added in bag order
        f4 acc = f4{0.f, 0.f, 0.f, 0.f};
        for (int l = 0; l < L; l += U) {
            int32_t r[U];
            f4 v[U];
#pragma unroll
            for (int k = 0; k < U; ++k) r[k] = ip[l + k < L ? l + k : l];
#pragma unroll
            for (int k = 0; k < U; ++k) v[k] = W[(int64_t)r[k] * D4 + col];
            if (l == 0) acc = v[0];
#pragma unroll
            for (int k = 0; k < U; ++k)
                if (l + k < L && (l + k) > 0) acc = acc + v[k];
        }
        o[col] = acc;
    }
}

int32_t launch_forward(const ss_tables *tb, const int32_t *idx, int Bcap, int L,
                       const int32_t *n_valid, float *out, hipStream_t s)
{
    const int D4 = tb->dim / 4;
    const int g = lanes_per_row(tb->dim);
    const int bags = (kWG / g) * (L == 1 ? 8 : 1);
    const int tiles = (Bcap + bags - 1) / bags;
    const int64_t blocks = (int64_t)tiles * tb->num_tables;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_forward: grid too large");
    ProfScope prof("forward_kernel", s);
    if (L == 1) {
        SS_DISPATCH_G(g, launch(forward_onehot_kernel<G>,
                                            dim3((unsigned)blocks), dim3(kWG), s,
                                            tb->weights, idx, Bcap, n_valid, out,
                                            D4, tiles));
    } else {
#define SS_FWD(U_)                                                                \
    SS_DISPATCH_G(g, launch((forward_kernel<G, U_>),                   \
                                        dim3((unsigned)blocks), dim3(kWG), s,   \
                                        tb->weights, idx, Bcap, L, n_valid, out,   \
                                        D4, tiles))
        // enough loads per lane to cover the bag in one or two rounds
        if (L <= 8) { SS_FWD(8); }
        else if (L <= 16 || L > 24) { SS_FWD(16); }
        else { SS_FWD(24); }
#undef SS_FWD
    }
    return check_launch("ss_embbag_forward");
}

}  // namespace ss
