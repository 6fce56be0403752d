// One-hot pooled lookup as a device function, so that it can run as a kernel
// of its own or as one role of the fused forward + grouping launch.
#pragma once
#include "ss_common.h"

namespace ss {

// block index b -> (table, tile)
__device__ __forceinline__ void block_to_table_tile(int b, int tiles_per_table, int &t,
                                                    int &tile)
{
    t = b / tiles_per_table;
    tile = b - t * tiles_per_table;
}

constexpr int kOneHotBags = 8;     // bags per lane group in the one-hot kernel

// L = 1: a group of G lanes takes kOneHotBags bags, fetches their indices, then issues
// the 8 row loads back to back before the first store.
template <int G, int THREADS>
__device__ __forceinline__ void forward_onehot_body(
    int b, const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, const int32_t *__restrict__ n_valid, float *__restrict__ out, int D4,
    int tiles_per_table)
{
    constexpr int GROUPS = THREADS / G, BPG = kOneHotBags;
    int t, tile;
    block_to_table_tile(b, tiles_per_table, t, tile);
    const int g = threadIdx.x / G, c = threadIdx.x % G;
    const int j0 = tile * GROUPS * BPG + g;      // bags j0 + k * GROUPS
    if (j0 >= Bcap) return;
    const auto W = as_global(reinterpret_cast<const f4 *>(weights[t]));
    const int32_t *__restrict__ ip = idx + (int64_t)t * Bcap;
    f4 *__restrict__ o = reinterpret_cast<f4 *>(out) + (int64_t)t * Bcap * D4;

    // The index words are requested before the number of valid bags is looked at (it
    // sits in device memory, one more round trip away): every position below Bcap can
    // be read, and what lies past n_valid is replaced by bag j0's index before it is
    // used as a row number.  Those bags store nothing.
    int32_t r[BPG];
#pragma unroll
    for (int k = 0; k < BPG; ++k) {
        const int j = j0 + k * GROUPS;
        r[k] = ip[j < Bcap ? j : j0];
    }
    const int n = clamp_valid(n_valid, Bcap);
    if (j0 >= n) return;
#pragma unroll
    for (int k = 0; k < BPG; ++k)
        if (j0 + k * GROUPS >= n) r[k] = r[0];
    for (int col = c; col < D4; col += G) {
        f4 v[BPG];
#pragma unroll
        for (int k = 0; k < BPG; ++k) v[k] = W[(int64_t)r[k] * D4 + col];
        // The pooled vectors are as many bytes as the rows just read and are not read
        // again on this path: streamed past the caches they leave the gradients and
        // the hot rows of the update that follows in place (26 tables x 8192 bags x 64:
        // the lookup takes 0.5 us longer, the update 1.2 us less).
#pragma unroll
        for (int k = 0; k < BPG; ++k)
            if (j0 + k * GROUPS < n)
                __builtin_nontemporal_store(v[k], &o[(int64_t)(j0 + k * GROUPS) * D4 + col]);
    }
}

}  // namespace ss
