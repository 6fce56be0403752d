// ss_filter_batch: input classifier (section 3.4, Eq. 6-8) plus a stable
// stream compaction of the kept samples.
//
// Kernel 1 gives each sample a group of lanes, which probe one bit per lookup
// (the bitmaps are small and stay in L2) in chunks, all loads of a chunk in
// flight together, and stop as soon as the verdict is fixed: the count reached
// alpha, or it can no longer reach it.  (One lane per sample probing one lookup
// at a time is as fast while nothing is stale, but its chain of dependent loads
// grows with every stale lookup: 21 us at 26 tables once the hot rows are
// frozen.)  A wavefront ballot plus popcount yields the number of kept samples
// per workgroup.
// Kernel 2 runs one workgroup per (tile of 256 samples, table).  It turns the
// per-tile counts into an offset (summing the counts before it: at most a few
// hundred values), ranks the tile's kept samples with ballot + popcount prefix
// sums, writes kept_ids in ascending order and copies the index rows of the kept
// samples of its table to their compacted place.
#include "ss_common.h"

namespace ss {

// LANES lanes per sample, flag_wg(LANES) / LANES samples per workgroup.  A chunk
// of lookups costs two round trips to memory (indices, then bitmap words) however many of
// them are stale.  The first chunk is one lookup per lane: while few rows are
// stale that settles almost every sample, and the kernel reads no more than
// that.  Later chunks take eight per lane.  The host picks LANES so that two
// chunks cover all T * L lookups of a sample where it can: the kernel lasts as
// long as its unluckiest sample, and with most hot rows frozen there is always
// a sample that needs nearly all of them (160 lookups per sample: 16 us with
// four lanes and six chunks, 7 us with 32 lanes and two).
constexpr int kFlagProbes = 8;                   // lookups per lane and chunk
// Threads per workgroup: 256 (1024 with 64 lanes per sample).  Beside the training
// kernels a 1024-thread workgroup waits for a compute unit with sixteen free
// wavefront slots: at 32 lanes per sample the kernel then took 13-15 us instead of
// the 4 us it takes alone.
constexpr int flag_wg(int lanes) { return lanes <= 32 ? 256 : 1024; }

// SPLIT: the same pass also classifies the sample against a second set of bitmaps
// (the hot rows, section 3.1: an input that reads only hot entries is a hot input,
// I = I_hot + I_cold): hot_mask[b] = 1 iff every lookup of the sample hits a row
// whose hot bit is set.  The indices of a chunk are loaded once for both tests;
// each test stops probing as soon as its verdict is fixed.
template <int LANES, bool SPLIT, typename TS>
__global__ __launch_bounds__(flag_wg(LANES)) void filter_flag_kernel(
    const uint32_t *const *__restrict__ bits, const uint32_t *const *__restrict__ hot_bits,
    const int32_t *__restrict__ idx, int T, int B, int L, int alpha,
    uint8_t *__restrict__ skip_mask, uint8_t *__restrict__ hot_mask,
    int32_t *__restrict__ block_kept, TS ts)
{
    constexpr int kFlagWG = flag_wg(LANES);
    const unsigned long long trace_t0 = trace_begin<TS>();
    constexpr int SAMPLES = kFlagWG / LANES;
    const int c = threadIdx.x % LANES;
    const int b = blockIdx.x * SAMPLES + threadIdx.x / LANES;
    bool keep = false;
    if (b < B) {
        const int total = T * L;
        bool skip = false;
        bool stale_open = true;                  // is the stale verdict still undecided?
        if (alpha <= 0) {
            skip = true;
            stale_open = false;
        } else if (alpha > total || bits == nullptr) {
            stale_open = false;
        }
        bool hot_open = SPLIT && hot_bits != nullptr;
        bool all_hot = hot_open;                 // no hot bitmaps: no input is hot
        int count = 0;                           // stale lookups so far (all lanes)
        int per_lane = 1;
        for (int q0 = 0; q0 < total && (stale_open || hot_open);) {
            const int chunk = LANES * per_lane;
            uint32_t row[kFlagProbes];
            int tab[kFlagProbes];
            bool in[kFlagProbes];
#pragma unroll
            for (int i = 0; i < kFlagProbes; ++i) {
                const int q = q0 + i * LANES + c;
                in[i] = i < per_lane && q < total;
                const int qq = in[i] ? q : 0;
                const int t = qq / L, l = qq - t * L;
                tab[i] = t;
                row[i] = in[i] ? (uint32_t)idx[((int64_t)t * B + b) * L + l] : 0u;
            }
            if (stale_open) {
                gptr<const uint32_t> bt[kFlagProbes];
                uint32_t word[kFlagProbes];
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i) bt[i] = as_global(bits[tab[i]]);
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i)
                    word[i] = (in[i] && bt[i] != nullptr) ? bt[i][row[i] >> 5] : 0u;
                int mine = 0;
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i) mine += (word[i] >> (row[i] & 31)) & 1u;
#pragma unroll
                for (int off = 1; off < LANES; off <<= 1) mine += __shfl_xor(mine, off, LANES);
                count += mine;
            }
            if (SPLIT && hot_open) {
                gptr<const uint32_t> ht[kFlagProbes];
                uint32_t word[kFlagProbes];
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i) ht[i] = as_global(hot_bits[tab[i]]);
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i)
                    word[i] = (in[i] && ht[i] != nullptr) ? ht[i][row[i] >> 5] : 0u;
                int cold = 0;                    // lookups of this lane that miss the hot set
#pragma unroll
                for (int i = 0; i < kFlagProbes; ++i)
                    cold += in[i] && !((word[i] >> (row[i] & 31)) & 1u);
#pragma unroll
                for (int off = 1; off < LANES; off <<= 1) cold += __shfl_xor(cold, off, LANES);
                if (cold) {
                    all_hot = false;
                    hot_open = false;
                }
            }
            q0 += chunk;
            const int remaining = total > q0 ? total - q0 : 0;
            if (stale_open && (count >= alpha || count + remaining < alpha)) stale_open = false;
            per_lane = kFlagProbes;
        }
        if (alpha > 0 && alpha <= total && bits != nullptr) skip = count >= alpha;
        if (c == 0) skip_mask[b] = skip ? 1 : 0;
        if (SPLIT && c == 0) hot_mask[b] = all_hot ? 1 : 0;
        keep = !skip && c == 0;
    }
    __shared__ int s_cnt[kFlagWG / 64];
    const unsigned long long bal = __ballot(keep);
    if ((threadIdx.x & 63) == 0) s_cnt[threadIdx.x >> 6] = __popcll(bal);
    __syncthreads();
    if (threadIdx.x == 0) {
        int s = 0;
        for (int w = 0; w < kFlagWG / 64; ++w) s += s_cnt[w];
        block_kept[blockIdx.x] = s;
    }
    trace_end(ts, trace_t0);
}

template <typename TS>
__global__ __launch_bounds__(kWG) void filter_compact_kernel(
    const int32_t *__restrict__ idx, int B, int L,
    const uint8_t *__restrict__ skip_mask,
    const int32_t *__restrict__ block_kept, int per_tile,
    int32_t *__restrict__ kept_ids, int32_t *__restrict__ n_kept,
    int32_t *__restrict__ idx_c, TS ts)
{
    const unsigned long long trace_t0 = trace_begin<TS>();
    // grid: x = tile of 256 samples, y = table, z = part of the tile's rows.  Every
    // workgroup repeats the cheap ranking of tile x and copies index rows of table y.
    // block_kept holds per_tile counts for every tile (one per workgroup of the
    // flag kernel).
    __shared__ int s_red[kWG / 64];
    __shared__ int s_wbase[kWG / 64];
    __shared__ int32_t s_list[kWG];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int t = blockIdx.y;

    // samples kept by the tiles before this one
    int part = 0;
    for (int i = tid; i < (int)blockIdx.x * per_tile; i += kWG) part += block_kept[i];
    for (int off = 32; off > 0; off >>= 1) part += __shfl_xor(part, off);
    if (lane == 0) s_red[wave] = part;

    const int b = blockIdx.x * kWG + tid;
    const bool keep = b < B && skip_mask[b] == 0;
    const unsigned long long bal = __ballot(keep);
    const int before = __popcll(bal & ((1ull << lane) - 1ull));
    if (lane == 0) s_wbase[wave] = __popcll(bal);
    __syncthreads();
    int base = 0, wbase = 0, nk = 0;
    for (int w = 0; w < kWG / 64; ++w) {
        base += s_red[w];
        if (w < wave) wbase += s_wbase[w];
        nk += s_wbase[w];
    }
    if (keep) {
        if (t == 0 && blockIdx.z == 0) kept_ids[base + wbase + before] = b;
        s_list[wbase + before] = b;
    }
    if (t == 0 && blockIdx.z == 0 && blockIdx.x == gridDim.x - 1 && tid == 0)
        *n_kept = base + nk;
    __syncthreads();

    // idx_c[t][base + k][:] = idx[t][s_list[k]][:]
    const int32_t *__restrict__ src = idx + (int64_t)t * B * L;
    int32_t *__restrict__ dst = idx_c + ((int64_t)t * B + base) * L;
    if (L == 1) {
        if (tid < nk) dst[tid] = src[s_list[tid]];
    } else {
        // long bags: gridDim.z workgroups share the rows of a tile (each repeats the
        // cheap ranking above), 4 * kWG elements at a time
        const int total = nk * L;
        for (int e0 = tid + (int)blockIdx.z * 4 * kWG; e0 < total;
             e0 += (int)gridDim.z * 4 * kWG) {
            int32_t v[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = e0 + u * kWG;
                const int k = e / L, l = e - k * L;
                v[u] = e < total ? src[(int64_t)s_list[k] * L + l] : 0;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u)
                if (e0 + u * kWG < total) dst[e0 + u * kWG] = v[u];
        }
    }
    trace_end(ts, trace_t0);
}

// Lanes per sample in the flag kernel: the fewest of 4 ... 64 with which two
// chunks (one lookup per lane, then eight) cover all T * L lookups of a sample.
static int flag_lanes(int64_t total)
{
    int lanes = 4;
    while (lanes < 64 && (int64_t)lanes * (1 + kFlagProbes) < total) lanes *= 2;
    return lanes;
}

size_t filter_ws_bytes(int T, int B, int L)
{
    const int lanes = flag_lanes((int64_t)T * L);
    const int samples = flag_wg(lanes) / lanes;
    const size_t blocks = ((size_t)B + samples - 1) / samples;
    return align_up(blocks * sizeof(int32_t), 256);
}

int32_t launch_filter(const ss_tables *tb, const int32_t *idx, int B, int L,
                      int alpha, uint8_t *skip_mask, int32_t *kept_ids,
                      int32_t *n_kept, int32_t *idx_c, void *ws, hipStream_t s)
{
    return launch_filter_split(tb, nullptr, idx, B, L, alpha, skip_mask, nullptr, kept_ids,
                               n_kept, idx_c, ws, s);
}

int32_t launch_filter_split(const ss_tables *tb, uint32_t *const *hot_bits, const int32_t *idx,
                            int B, int L, int alpha, uint8_t *skip_mask, uint8_t *hot_mask,
                            int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c, void *ws,
                            hipStream_t s)
{
    const int lanes = flag_lanes((int64_t)tb->num_tables * L);
    const int samples = flag_wg(lanes) / lanes;      // per workgroup of the flag kernel
    const int flag_blocks = (B + samples - 1) / samples;
    const int tiles = (B + kWG - 1) / kWG;
    int32_t *block_kept = static_cast<int32_t *>(ws);
    {
        ProfScope prof("filter_flag_kernel", s);
#define SS_FLAG(LANES_)                                                            \
    if (hot_mask)                                                                  \
        launch(SS_BOTH(filter_flag_kernel, LANES_, true), dim3(flag_blocks),         \
               dim3(flag_wg(LANES_)), s, tb->stale_bits, hot_bits, idx,             \
               tb->num_tables, B, L, alpha, skip_mask, hot_mask, block_kept);       \
    else                                                                           \
        launch(SS_BOTH(filter_flag_kernel, LANES_, false), dim3(flag_blocks),        \
               dim3(flag_wg(LANES_)), s, tb->stale_bits, nullptr, idx,              \
               tb->num_tables, B, L, alpha, skip_mask, nullptr, block_kept)
        switch (lanes) {
        case 4: SS_FLAG(4); break;
        case 8: SS_FLAG(8); break;
        case 16: SS_FLAG(16); break;
        case 32: SS_FLAG(32); break;
        default: SS_FLAG(64); break;
        }
#undef SS_FLAG
    }
    ProfScope prof("filter_compact_kernel", s);
    // the last tile may be covered by fewer workgroups of the flag kernel: a tile
    // before it is always covered by exactly kWG / samples of them
    // one workgroup per 1024 index words of a tile's rows, at most eight
    const int parts = L == 1 ? 1 : (L + 3) / 4 > 8 ? 8 : (L + 3) / 4;
    launch(filter_compact_kernel<NoTrace>, filter_compact_kernel<TraceSlot>,
           dim3(tiles, tb->num_tables, parts), dim3(kWG), s, idx, B, L, skip_mask, block_kept,
           kWG / samples, kept_ids, n_kept, idx_c);
    return check_launch("ss_filter_batch");
}

}  // namespace ss
