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
//   - multi-hot bags: the row numbers of up to 31 lookups of the bag are fetched
//     first and their row loads issued together (see forward_kernel below).
// All workgroups of a table run on one XCD in the multi-hot kernel, so that its
// hot rows live in one L2 instead of eight: 64 instead of 89 MB fetched from HBM
// per launch at 8 tables x 10M rows x 128, at the same duration (26-27 us).
#include "forward_body.h"
#include "ss_common.h"

namespace ss {

template <int G, typename TS>
__global__ __launch_bounds__(kWG) void forward_onehot_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, const int32_t *__restrict__ n_valid, float *__restrict__ out,
    int D4, int tiles_per_table, int pinned_blocks, TS ts)
{
    const unsigned long long trace_t0 = trace_begin<TS>();
    // a table's hot rows are wanted by all its tiles: keep them in one L2
    int t, tile;
    block_to_table_pinned(blockIdx.x, tiles_per_table, pinned_blocks, t, tile);
    forward_onehot_body<G, kWG>(t * tiles_per_table + tile, weights, idx, Bcap, n_valid, out, D4,
                                tiles_per_table);
    trace_end(ts, trace_t0);
}

// Multi-hot bags.  All lanes of a workgroup see the same bag length, so the bag
// is cut into pieces of 16, 8, 4, 2 and 1 lookups by scalar branches on the bits
// of the length: every piece is straight-line code with a known number of row
// loads, all pieces are requested before the first add (up to 31 loads in
// flight per lane), and the rows are added in bag order.  Bags of 32 lookups or
// more first run full rounds of 16.  FULL (a row fills its group of lanes
// exactly) turns the row address into shifts.
template <int N>
__device__ __forceinline__ void fetch_ids(int32_t (&r)[N], const int32_t *__restrict__ ip)
{
#pragma unroll
    for (int k = 0; k < N; ++k) r[k] = ip[k];
}

template <int N, int G, bool FULL, typename P>
__device__ __forceinline__ void fetch_rows(f4 (&v)[N], const int32_t (&r)[N],
                                           P lane_base, uint32_t d4)
{
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] = *row_ptr<G, FULL>(lane_base, (uint32_t)r[k], d4);
}

template <int N> __device__ __forceinline__ void unset_rows(f4 (&v)[N])
{
#pragma unroll
    for (int k = 0; k < N; ++k) v[k] = unset_f4();
}

template <int N> __device__ __forceinline__ void add_rows(f4 &acc, const f4 (&v)[N])
{
#pragma unroll
    for (int k = 0; k < N; ++k) acc = acc + v[k];
}

template <int G, bool FULL, typename TS>
__global__ __launch_bounds__(kWG) void forward_kernel(
    const float *const *__restrict__ weights, const int32_t *__restrict__ idx,
    int Bcap, int L, const int32_t *__restrict__ n_valid,
    float *__restrict__ out, int D4, int tiles_per_table, int pinned_blocks, TS ts)
{
    constexpr int BAGS = kWG / G;
    const unsigned long long trace_t0 = trace_begin<TS>();
    int t, tile;
    block_to_table_pinned(blockIdx.x, tiles_per_table, pinned_blocks, t, tile);
    const int n = clamp_valid(n_valid, Bcap);
    const int j = tile * BAGS + (int)threadIdx.x / G;
    if (j >= n) return;
    const int c = threadIdx.x % G;
    const uint32_t d4 = FULL ? (uint32_t)G : (uint32_t)D4;
    const auto W = as_global(reinterpret_cast<const f4 *>(weights[t]));
    const int32_t *__restrict__ ip = idx + ((int64_t)t * Bcap + j) * L;
    f4 *__restrict__ o = reinterpret_cast<f4 *>(out) + ((int64_t)t * Bcap + j) * d4;

    for (int col = c; FULL ? col == c : col < D4; col += G) {
        const auto Wc = W + col;            // this lane's f4 of row 0
        f4 acc = f4{0.f, 0.f, 0.f, 0.f};
        const int32_t *__restrict__ q = ip;
        int m = L;
        for (; m >= 32; m -= 16, q += 16) {
            int32_t r[16];
            f4 a[16];
            fetch_ids(r, q);
            fetch_rows<16, G, FULL>(a, r, Wc, d4);
            add_rows(acc, a);
        }
        // loads come back in the order they were issued: all row numbers first,
        // so that no wait for a row number also waits for rows
        int32_t ra[16] = {}, rb[8] = {}, rd[4] = {}, re[2] = {}, rf[1] = {};
        if (m & 16) { fetch_ids(ra, q); q += 16; }
        if (m & 8) { fetch_ids(rb, q); q += 8; }
        if (m & 4) { fetch_ids(rd, q); q += 4; }
        if (m & 2) { fetch_ids(re, q); q += 2; }
        if (m & 1) { fetch_ids(rf, q); }
        f4 a[16], b[8], d[4], e[2], f[1];
        unset_rows(a); unset_rows(b); unset_rows(d); unset_rows(e); unset_rows(f);
        if (m & 16) fetch_rows<16, G, FULL>(a, ra, Wc, d4);
        if (m & 8) fetch_rows<8, G, FULL>(b, rb, Wc, d4);
        if (m & 4) fetch_rows<4, G, FULL>(d, rd, Wc, d4);
        if (m & 2) fetch_rows<2, G, FULL>(e, re, Wc, d4);
        if (m & 1) fetch_rows<1, G, FULL>(f, rf, Wc, d4);
        if (m & 16) add_rows(acc, a);
        if (m & 8) add_rows(acc, b);
        if (m & 4) add_rows(acc, d);
        if (m & 2) add_rows(acc, e);
        if (m & 1) add_rows(acc, f);
        o[col] = acc;
    }
    trace_end(ts, trace_t0);
}

int32_t launch_forward(const ss_tables *tb, const int32_t *idx, int Bcap, int L,
                       const int32_t *n_valid, float *out, hipStream_t s)
{
    const int D4 = tb->dim / 4;
    const int g = lanes_per_row(tb->dim);
    const int bags = (kWG / g) * (L == 1 ? kOneHotBags : 1);
    const int tiles = (Bcap + bags - 1) / bags;
    const int64_t blocks = (int64_t)tiles * tb->num_tables;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_forward: grid too large");
    ProfScope prof("forward_kernel", s);
    if (L == 1) {
        SS_DISPATCH_G(g, launch(SS_BOTH(forward_onehot_kernel, G),
                                            dim3((unsigned)blocks), dim3(kWG), s,
                                            tb->weights, idx, Bcap, n_valid, out,
                                            D4, tiles, (tb->num_tables / 8) * 8 * tiles));
    } else {
#define SS_FWD(F_)                                                                \
    SS_DISPATCH_G(g, launch(SS_BOTH(forward_kernel, G, F_), dim3((unsigned)blocks),       \
                            dim3(kWG), s, tb->weights, idx, Bcap, L, n_valid, out,  \
                            D4, tiles, (tb->num_tables / 8) * 8 * tiles))
        if (D4 == g) { SS_FWD(true); } else { SS_FWD(false); }
#undef SS_FWD
    }
    return check_launch("ss_embbag_forward");
}

}  // namespace ss
