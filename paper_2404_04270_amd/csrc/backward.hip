// ss_embbag_backward_update: gradient scatter of the pooled lookup fused with
// sparse SGD that skips stale rows (abstract and section 3.6 of the paper).
//
// Three stages, all tables in every launch:
//
//  1. GROUP the lookups of each table by row id (the apply stage needs equal rows
//     adjacent, not ascending; the order inside a group is the same from run to
//     run).  The lists hold (row, sample) pairs: the sample number is all the
//     gradient gather needs.
//       - up to 16384 lookups per table: one launch; the table is cut into
//         classes by the low bits of the row id and a 1024-thread workgroup per
//         class runs an LSD radix sort on the remaining bits with keys and
//         sample numbers in registers and the exchange buffers in LDS;
//       - more: one pass of a global LSD radix sort on the low bits (two
//         launches: per-tile digit histograms, then a stable scatter whose
//         workgroups each derive their own offsets from the histograms; the
//         histogram launch also writes the (row, sample) pairs, so the scatter
//         reads pairs and the bitmap is probed once per lookup), which leaves
//         the table in buckets; then one launch in which a 256-thread workgroup
//         per bucket sorts it by the remaining bits in LDS, in place;
//       - row ids of 10 bits or fewer with that many lookups: the one global
//         pass is all it takes (further passes of the same kind exist for row
//         ids whose remaining bits would not leave a bucket anything to sort).
//     A lookup whose row is stale is given the sentinel key when the keys are
//     first read, so it sorts behind all real lookups and costs nothing later.
//     Ranking inside a wavefront uses ballots: the lanes that hold the same
//     digit are found with one ballot per digit bit, a popcount of the lower
//     lanes gives the rank, and one lane per digit bumps the wavefront's LDS
//     counter.  Tables are padded with sentinel keys to a multiple of 2048.
//
//  2. APPLY walks the sorted list in strips of S lookups per group of G lanes
//     (one f4 of the row per lane).  All gradient rows of the strip and the
//     weight rows of the runs that end in it are requested up front, then the
//     runs are summed in order.  A run that lies inside one strip is applied
//     right away.  Runs that cross strip borders leave a leading / trailing
//     piece in LDS and are stitched together inside the workgroup in strip
//     order; runs that cross workgroup borders leave their piece in the
//     workspace.
//
//  3. FIXUP: a lane group per workgroup of the apply stage checks whether a run
//     left it; short runs are finished by that group, the few long ones by the
//     whole workgroup, pieces added in a fixed order.
//
// Rows whose stale bit is set drop out in stage 1, before any gradient or
// weight of theirs is read.  There are no floating-point atomics: every sum has a fixed
// order, so the result is reproducible.
#include "group_body.h"
#include "ss_common.h"

namespace ss {

namespace {

constexpr int kPad = 2048;             // per-table padding of the sorted arrays
constexpr int kLdsSortMax = 16384;     // largest table the one-launch sort takes
constexpr uint32_t kNoPrev = 0xFFFFFFFEu;
constexpr int kRsHistThreads = 256;    // global radix sort, histogram: threads per tile
constexpr int kRsHistItems = 8;        // ... keys per thread (tile = 2048 = kPad)
constexpr int kRsThreads = 512;        // scatter: threads per tile (its chain of ranking
constexpr int kRsItems = 4;            // steps per thread is what it waits for: 9.3 us
                                       // against 12.4 us with 256 x 8 at one table x 65536)
constexpr int kRsMaxBits = 10;         // ... widest digit
constexpr int kRsMaxDig = 1 << kRsMaxBits;
constexpr int kBucketThreads = 256;    // bucket sort: a workgroup no larger than those of the
constexpr int kBucketItems = 16;       // training kernels it runs beside; keys per thread
constexpr int kBucketCap = kBucketThreads * kBucketItems;
constexpr int kBsStride = kRsMaxDig + 4;   // per table: where each bucket starts
constexpr int kApplyWG = 256;           // apply stage: threads per workgroup (512 and
                                        // 1024 were measured slower: 22 and 38 us vs 18)

// Stage 1a (class sort, one launch for up to 16384 lookups per table) lives in
// group_body.h, shared with the fused forward + grouping launch.
template <int ITEMS, bool PACKED, typename TS>
__global__ __launch_bounds__(1024) void class_sort_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, const uint32_t *const *__restrict__ bits,
    int key_bits, int class_bits, int val_bits, uint2 *__restrict__ out_ent, int NP,
    TS ts)
{
    const unsigned long long trace_t0 = trace_begin<TS>();
    class_sort_body<ITEMS, PACKED>(blockIdx.x, blockIdx.y, idx, Bcap, L, n_valid, bits,
                                   key_bits, class_bits, val_bits, out_ent, NP);
    trace_end(ts, trace_t0);
}

// ---------------------------------------------------------------------------
// Stage 1b: one global radix pass on the low nb bits of the row id = histogram, then
// scatter.  Tile = 2048 keys; hist layout [table][tile][digit].
// ---------------------------------------------------------------------------
// Digit of a key.  sent (0 or 1): the sentinel key gets a digit of its own behind all
// others, so that every other bucket holds real rows only.
__device__ __forceinline__ uint32_t rs_digit(uint32_t key, uint32_t dmask, int sent)
{
    return sent && key == kNoRow ? dmask + 1u : key & dmask;
}

// Reads the index tensor, turns it into (row, sample) pairs with the sentinel for stale
// rows and padding (the sample number is the position divided by the bag length), leaves
// them for the scatter, which then needs neither the bitmap probes nor the division, and
// counts the digits of its tile.
template <typename TS>
__global__ __launch_bounds__(kRsHistThreads) void rs_hist_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, const uint32_t *const *__restrict__ bits,
    uint2 *__restrict__ pairs, int NP, int nb, int sent, uint32_t *__restrict__ hist,
    int tiles, TS ts)
{
    __shared__ uint32_t s_hist[kRsMaxDig];
    const unsigned long long trace_t0 = trace_begin<TS>();
    const int t = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
    const int n = clamp_valid(n_valid, Bcap) * L;
    const int ndig = (1 << nb) + sent;
    const uint32_t dmask = (1u << nb) - 1;
    const int32_t *__restrict__ ip = idx + (int64_t)t * Bcap * L;
    const auto bt = as_global(bits ? bits[t] : nullptr);
    for (int i = tid; i < ndig; i += kRsHistThreads) s_hist[i] = 0;
    __syncthreads();
    uint32_t key[kRsHistItems], val[kRsHistItems];
#pragma unroll
    for (int r = 0; r < kRsHistItems; ++r) {
        const int pos = tile * kPad + r * kRsHistThreads + tid;
        key[r] = pos < n ? (uint32_t)ip[pos] : kNoRow;
        val[r] = pos < n ? (uint32_t)(L == 1 ? pos : pos / L) : 0u;
    }
    drop_stale(bt, key);
    uint2 *__restrict__ eo = pairs + (int64_t)t * NP;
#pragma unroll
    for (int r = 0; r < kRsHistItems; ++r)
        eo[tile * kPad + r * kRsHistThreads + tid] = make_uint2(key[r], val[r]);
#pragma unroll
    for (int r = 0; r < kRsHistItems; ++r)
        atomicAdd(&s_hist[rs_digit(key[r], dmask, sent)], 1u);
    __syncthreads();
    for (int i = tid; i < ndig; i += kRsHistThreads)
        hist[((int64_t)t * tiles + tile) * kRsMaxDig + i] = s_hist[i];
    trace_end(ts, trace_t0);
}

// Stable scatter of one tile.  The workgroup first turns the table's histograms
// into the start offset of each of its digits: (keys with a smaller digit in
// the whole table) + (keys with this digit in earlier tiles).
template <typename TS>
__global__ __launch_bounds__(kRsThreads) void rs_scatter_kernel(
    const uint2 *__restrict__ in_ent, uint2 *__restrict__ out_ent, int NP, int nb, int sent,
    uint32_t *__restrict__ bucket_out, const uint32_t *__restrict__ hist, int tiles, TS ts)
{
    constexpr int NW = kRsThreads / 64;
    const unsigned long long trace_t0 = trace_begin<TS>();
    __shared__ uint32_t s_cnt[NW * kRsMaxDig];   // per wavefront and digit
    __shared__ uint32_t s_base[kRsMaxDig];       // start offset of each digit
    __shared__ uint32_t s_wsum[NW];
    const int t = blockIdx.y, tile = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int ndig = (1 << nb) + sent;
    const int nbits = nb + sent;                 // bits that tell the digits apart
    const uint32_t dmask = (1u << nb) - 1;
    const uint2 *__restrict__ ein = in_ent + (int64_t)t * NP;

    uint32_t key[kRsItems], val[kRsItems], rank[kRsItems];
#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {  // wavefront w owns a contiguous part of the tile
        const uint2 e = ein[tile * kPad + wave * (kRsItems * 64) + r * 64 + lane];
        key[r] = e.x;
        val[r] = e.y;
    }

    // Digit offsets from the histograms; each thread owns ndig / 256 digits.
    // This kernel runs about one wavefront per SIMD, so what it costs is the
    // number of instructions a wavefront executes one after the other, not
    // bytes: the loops over a thread's digits are unrolled (their sums stay in
    // fixed registers), and a tile's histogram is addressed as (base common to
    // all lanes) + (this lane's digit), which keeps the base in scalar registers.
    for (int i = tid; i < NW * ndig; i += kRsThreads) s_cnt[i] = 0;
    const int dpt = (ndig + kRsThreads - 1) / kRsThreads;   // 1 or 2
    uint32_t tot[4] = {0, 0, 0, 0}, early[4] = {0, 0, 0, 0}, run = 0;
    const uint32_t *__restrict__ ht = hist + (int64_t)t * tiles * kRsMaxDig;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int d = tid * dpt + q;
        if (q < dpt && d < ndig) {
            uint32_t all = 0, before = 0;
            int k = 0;
            // each round of loads is a trip to memory: 32 tiles per round first
            for (; k + 32 <= tiles; k += 32) {
                uint32_t c[32];
#pragma unroll
                for (int u = 0; u < 32; ++u) c[u] = (ht + (k + u) * kRsMaxDig)[d];
#pragma unroll
                for (int u = 0; u < 32; ++u) {
                    all += c[u];
                    before += k + u < tile ? c[u] : 0u;
                }
            }
            for (; k + 8 <= tiles; k += 8) {
                uint32_t c[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) c[u] = (ht + (k + u) * kRsMaxDig)[d];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    all += c[u];
                    before += k + u < tile ? c[u] : 0u;
                }
            }
            if (k < tiles) {        // up to seven more, requested together
                uint32_t c[8];
#pragma unroll
                for (int u = 0; u < 7; ++u)
                    c[u] = (ht + (k + u < tiles ? k + u : k) * kRsMaxDig)[d];
#pragma unroll
                for (int u = 0; u < 7; ++u) {
                    all += k + u < tiles ? c[u] : 0u;
                    before += k + u < tile ? c[u] : 0u;
                }
            }
            tot[q] = all;
            early[q] = before;
        }
        run += tot[q];
    }
    uint32_t incl = run;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == 63) s_wsum[wave] = incl;
    __syncthreads();
    uint32_t start = incl - run;
    for (int w = 0; w < wave; ++w) start += s_wsum[w];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int d = tid * dpt + q;
        if (q < dpt && d < ndig) s_base[d] = start + early[q];
        start += tot[q];
    }

#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {
        const uint32_t d = rs_digit(key[r], dmask, sent);
        rank[r] = wave_rank(s_cnt + wave * ndig, d, nbits, lane);
    }
    __syncthreads();
    if (bucket_out && tile == 0) {
        // The pass ahead of a bucket sort: where each bucket starts (for tile 0 the
        // digit offsets are just that; the last digit is the sentinels').
        uint32_t *__restrict__ bo = bucket_out + t * kBsStride;
        for (int d = tid; d < ndig; d += kRsThreads) bo[d] = s_base[d];
    }
    for (int d = tid; d < ndig; d += kRsThreads) {
        uint32_t acc = s_base[d];
        for (int w = 0; w < NW; ++w) {
            const uint32_t c = s_cnt[w * ndig + d];
            s_cnt[w * ndig + d] = acc;
            acc += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {
        const uint32_t d = rs_digit(key[r], dmask, sent);
        const int64_t p = (int64_t)t * NP + s_cnt[wave * ndig + d] + rank[r];
        out_ent[p] = make_uint2(key[r], val[r]);      // one 8-byte store, not two of 4
    }
    trace_end(ts, trace_t0);
}

// Stage 1c: after one global pass on the low nb0 bits a table lies in 2^nb0 buckets
// (plus the sentinels behind them).  The apply stage needs equal rows adjacent, not
// ascending, so all that is left to do is to sort every bucket by the remaining bits,
// in place, and a bucket fits the LDS of a workgroup: one launch instead of two or three
// more global passes of two launches each.  The workgroups are as small as those of the
// training kernels this runs beside (a workgroup that needs a whole compute unit waits
// there until those have all but left it).  Remaining row bits and sample number are
// packed into one word where they fit one, as in the class sort.
// A bucket of more than kBucketCap lookups nearly always owes its size to one row (the
// hottest row of a Zipf table holds a fifth of all lookups): that row is found by a
// vote among 64 samples and its lookups are moved to the end of the bucket while the
// others are collected in LDS and sorted.  The bucket is read from its end, so that the
// heavy row's lookups land on places that have been read already.  Others that LDS has
// no room for are parked in the spare buffer; with those the workgroup falls back on
// an LSD sort of its own through global memory (slow, and rare: it takes several rows
// of thousands of lookups each with the same low bits).

// n pairs from `from` to `to` (which do not overlap), by all NT threads, eight loads
// in flight per thread.
template <int NT>
__device__ __forceinline__ void copy_pairs(const uint2 *__restrict__ from,
                                           uint2 *__restrict__ to, uint32_t n, int tid)
{
    for (uint32_t i0 = 0; i0 < n; i0 += NT * 8) {
        uint2 e[8];
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t i = i0 + u * NT + tid;
            e[u] = from[i < n ? i : n - 1];
        }
#pragma unroll
        for (int u = 0; u < 8; ++u) {
            const uint32_t i = i0 + u * NT + tid;
            if (i < n) to[i] = e[u];
        }
    }
}

// LSD sort of the n pairs at a (global memory) by key bits [shift, shift + bits), by one
// workgroup of NT threads; b is scratch of the same size; the result is left in a.
// s_cnt: NW * 64 words, s_run: 64 words.  1024 pairs at a time.
template <int NT>
__device__ __forceinline__ void wg_lsd_global(uint2 *a, uint2 *b, uint32_t n, int shift,
                                              int bits, uint32_t *s_cnt, uint32_t *s_run)
{
    constexpr int NW = NT / 64, V = 1024 / NT;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int npass = (bits + 5) / 6;
    uint2 *cur = a, *oth = b;
    for (int pass = 0; pass < npass; ++pass) {
        const int nb = pass_bits(bits, npass, pass);
        const uint32_t dmask = (1u << nb) - 1u;
        // digit totals, then where each digit starts
        if (tid < 64) s_run[tid] = 0;
        __syncthreads();
        for (uint32_t i = tid; i < n; i += NT) atomicAdd(&s_run[(cur[i].x >> shift) & dmask], 1u);
        __syncthreads();
        if (wave == 0) {
            const uint32_t c = s_run[lane];
            uint32_t incl = c;
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            s_run[lane] = incl - c;
        }
        __syncthreads();
        for (uint32_t c0 = 0; c0 < n; c0 += NT * V) {
            for (int i = tid; i < NW * 64; i += NT) s_cnt[i] = 0;
            __syncthreads();
            uint2 e[V];
            uint32_t rank[V];
#pragma unroll
            for (int u = 0; u < V; ++u) {
                const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
                e[u] = cur[pos < n ? pos : n - 1];
            }
#pragma unroll
            for (int u = 0; u < V; ++u) {
                const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
                const bool valid = pos < n;
                const uint32_t d = (e[u].x >> shift) & dmask;
                const uint64_t mm = match_digit(d, nb) & __ballot(valid);
                const uint32_t before = __popcll(mm & lanes_below(lane));
                uint32_t base = 0;
                if (valid && before == 0) base = atomicAdd(&s_cnt[wave * 64 + d], (uint32_t)__popcll(mm));
                base = __shfl(base, mm ? __ffsll((long long)mm) - 1 : 0);
                rank[u] = base + before;
            }
            __syncthreads();
            if (wave == 0) {
                uint32_t acc = s_run[lane];
                for (int w = 0; w < NW; ++w) {
                    const uint32_t c = s_cnt[w * 64 + lane];
                    s_cnt[w * 64 + lane] = acc;
                    acc += c;
                }
                s_run[lane] = acc;
            }
            __syncthreads();
#pragma unroll
            for (int u = 0; u < V; ++u) {
                const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
                if (pos < n) {
                    const uint32_t d = (e[u].x >> shift) & dmask;
                    const uint32_t p = s_cnt[wave * 64 + d] + rank[u];
                    if (p < n) oth[p] = e[u];
                }
            }
            __syncthreads();
        }
        // what this workgroup wrote is read by all of it in the next pass
        __threadfence_block();
        __syncthreads();
        uint2 *x = cur;
        cur = oth;
        oth = x;
        shift += nb;
    }
    if (cur != a) {
        copy_pairs<NT>(cur, a, n, tid);
        __threadfence_block();
        __syncthreads();
    }
}

template <bool PACKED, typename TS>
__global__ __launch_bounds__(kBucketThreads) void bucket_sort_kernel(
    uint2 *ent, uint2 *spare, int NP, const uint32_t *__restrict__ bucket, int nb0,
    int rem_bits, int val_bits, TS ts)
{
    constexpr int NT = kBucketThreads, NW = NT / 64, CAP = kBucketCap, U = 8, V = 16;
    __shared__ uint32_t s_keys[CAP];
    __shared__ uint32_t s_vals[PACKED ? 1 : CAP];
    __shared__ uint32_t s_cnt[2 * NW * 64];
    __shared__ uint32_t s_dig[64];
    __shared__ uint32_t s_w[2][NW];      // per wavefront: the heavy row's / other lookups of a chunk
    __shared__ uint32_t s_heavy;
    const unsigned long long trace_t0 = trace_begin<TS>();
    const int d = blockIdx.x, t = blockIdx.y;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const uint32_t *__restrict__ bo = bucket + t * kBsStride;
    const uint32_t b0 = bo[d], b1 = bo[d + 1];
    if (b0 >= b1 || b1 > (uint32_t)NP) {         // empty (b0 > b1, b1 > NP: cannot happen)
        trace_end(ts, trace_t0);
        return;
    }
    const uint32_t m = b1 - b0;
    uint2 *io = ent + (int64_t)t * NP + b0;
    // in LDS: (row bits above the bucket's, sample) in one word, or the pair as it is
    const uint32_t vmask = PACKED ? (1u << val_bits) - 1u : 0u;
    const int lds_shift = PACKED ? val_bits : nb0;
    const auto put = [&](uint32_t i, uint2 e) {
        if (PACKED) {
            s_keys[i] = ((e.x >> nb0) << val_bits) | e.y;
        } else {
            s_keys[i] = e.x;
            s_vals[i] = e.y;
        }
    };
    const auto get = [&](uint32_t i) {
        const uint32_t w = s_keys[i];
        return PACKED ? make_uint2(((w >> val_bits) << nb0) | (uint32_t)d, w & vmask)
                      : make_uint2(w, s_vals[i]);
    };

    if (m <= (uint32_t)CAP) {
        for (uint32_t i0 = 0; i0 < m; i0 += NT * U) {
            uint2 e[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t i = i0 + u * NT + tid;
                e[u] = io[i < m ? i : m - 1];
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const uint32_t i = i0 + u * NT + tid;
                if (i < m) put(i, e[u]);
            }
        }
        __syncthreads();
        lds_lsd_sort<NT, kBucketItems, PACKED>(s_keys, s_vals, s_cnt, s_dig, m, rem_bits,
                                               lds_shift);
        for (uint32_t i = tid; i < m; i += NT) io[i] = get(i);
        trace_end(ts, trace_t0);
        return;
    }

    // the row most of 64 evenly spaced lookups hit (the lowest lane among equals)
    if (wave == 0) {
        const uint32_t mine = io[(uint32_t)(((uint64_t)lane * m) >> 6)].x;
        uint32_t votes = 0;
        for (int i = 0; i < 64; ++i) votes += __shfl(mine, i) == mine ? 1u : 0u;
        uint32_t best = (votes << 6) | (uint32_t)(63 - lane);
        for (int off = 32; off; off >>= 1) {
            const uint32_t o = __shfl_xor(best, off);
            best = o > best ? o : best;
        }
        const uint32_t heavy = __shfl(mine, 63 - (int)(best & 63u));
        if (lane == 0) s_heavy = heavy;
    }
    __syncthreads();
    const uint32_t heavy = s_heavy;
    // The split, 4096 lookups at a time, from the end of the bucket to its start: by the
    // time n_eq lookups of the heavy row have been found, at least n_eq places at the end
    // have been read.  Others: the first CAP into LDS (packed), the rest into the spare buffer.
    uint2 *park = spare + (int64_t)t * NP + b0;
    uint32_t n_eq = 0, n_ne = 0;
    const uint32_t nchunks = (m + NT * V - 1) / (NT * V);
    for (uint32_t c = 0; c < nchunks; ++c) {
        const uint32_t c0 = (nchunks - 1 - c) * (NT * V);
        uint2 e[V];
        uint32_t rank[V];
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
            e[u] = io[pos < m ? pos : m - 1];
        }
        uint32_t w_eq = 0, w_ne = 0;
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
            const bool eq = pos < m && e[u].x == heavy, ne = pos < m && e[u].x != heavy;
            const unsigned long long beq = __ballot(eq), bne = __ballot(ne);
            rank[u] = eq ? w_eq + __popcll(beq & lanes_below(lane))
                         : w_ne + __popcll(bne & lanes_below(lane));
            w_eq += __popcll(beq);
            w_ne += __popcll(bne);
        }
        if (lane == 0) {
            s_w[0][wave] = w_eq;
            s_w[1][wave] = w_ne;
        }
        __syncthreads();        // every wavefront has its part of the chunk in registers
        uint32_t off_eq = n_eq, off_ne = n_ne;
        for (int w = 0; w < NW; ++w) {
            if (w < wave) {
                off_eq += s_w[0][w];
                off_ne += s_w[1][w];
            }
            n_eq += s_w[0][w];
            n_ne += s_w[1][w];
        }
#pragma unroll
        for (int u = 0; u < V; ++u) {
            const uint32_t pos = c0 + wave * (64 * V) + u * 64 + lane;
            if (pos < m) {
                const uint32_t k = (e[u].x == heavy ? off_eq : off_ne) + rank[u];
                if (e[u].x == heavy) io[m - 1 - k] = e[u];
                else if (k < (uint32_t)CAP) put(k, e[u]);
                else park[k - CAP] = e[u];
            }
        }
        __syncthreads();
    }
    if (n_ne <= (uint32_t)CAP) {
        lds_lsd_sort<NT, kBucketItems, PACKED>(s_keys, s_vals, s_cnt, s_dig, n_ne, rem_bits,
                                               lds_shift);
        for (uint32_t i = tid; i < n_ne; i += NT) io[i] = get(i);
    } else {
        // all others back in front of the heavy row's lookups, then sorted through
        // global memory (what this workgroup wrote is read by all of it)
        for (uint32_t i = tid; i < (uint32_t)CAP; i += NT) io[i] = get(i);
        __threadfence_block();
        __syncthreads();
        copy_pairs<NT>(park, io + CAP, n_ne - CAP, tid);
        __threadfence_block();
        __syncthreads();
        wg_lsd_global<NT>(io, park, n_ne, nb0, rem_bits, s_cnt, s_dig);
    }
    trace_end(ts, trace_t0);
}

// ---------------------------------------------------------------------------
// Stage 2: apply.
// Workspace per (table, workgroup): trail_row (row whose run starts in this
// workgroup and continues into the next one, or kNoRow), lead_state (0: the
// workgroup starts with a new run; 1: it starts inside a run that ends in it;
// 2: that run covers the whole workgroup and goes on), and the two partial
// sums part_lead / part_trail of dim floats each.
// ---------------------------------------------------------------------------
// Address of one lane's f4 of a gradient row.  A table's block of gradient rows is below 4 GiB
// in the FULL variant (the host checks), so the offset fits 32 bits and the base
// can stay in scalar registers.
template <int G, bool FULL>
__device__ __forceinline__ const f4 *grad_ptr(const f4 *table_base, uint32_t smp,
                                              uint32_t col, uint32_t d4)
{
    if (FULL) {
        constexpr int SH = ilog2(G) + 4;
        const uint32_t off = (smp << SH) + (col << 4);
        return reinterpret_cast<const f4 *>(reinterpret_cast<const char *>(table_base) +
                                            off);
    }
    return table_base + ((uint64_t)smp * d4 + col);
}

template <int G, int S, bool FULL, typename TS>
__global__ __launch_bounds__(kApplyWG) void apply_kernel(
    float *const *__restrict__ weights, const uint2 *__restrict__ ent, int NP,
    const float *__restrict__ grad,
    int Bcap, int D4, float lr, int wgs_per_table, int pinned_blocks,
    bool stream_grads, uint32_t *__restrict__ meta_trail_row,
    uint8_t *__restrict__ meta_lead_state, f4 *__restrict__ part_lead,
    f4 *__restrict__ part_trail, TS ts)
{
    constexpr int NG = kApplyWG / G;
    const unsigned long long trace_t0 = trace_begin<TS>();
    // sum of the run that enters the strip from the left: up to its end, or
    // over the whole strip when it goes on to the right
    __shared__ f4 s_lead[kApplyWG];
    __shared__ uint8_t s_lead_state[NG];

    int t, wg;
    // multi-hot bags: a table's gradient block is re-read by every lookup of a bag,
    // in the order of the sorted rows; it only stays in L2 if the table has one
    block_to_table_pinned(blockIdx.x, wgs_per_table, pinned_blocks, t, wg);
    const int tid = threadIdx.x, g = tid / G, c = tid % G;
    const uint2 *__restrict__ ep = ent + (int64_t)t * NP;       // (row, sample) pairs
    const auto W = as_global(reinterpret_cast<f4 *>(weights[t]));
    const f4 *__restrict__ G4 =
        reinterpret_cast<const f4 *>(grad) + (int64_t)t * Bcap * D4;
    const int wg_base = wg * NG * S;
    const int base = wg_base + g * S;
    // f4 per row: a constant in the FULL variant, so that row * d4 is a shift
    const uint32_t d4 = FULL ? (uint32_t)G : (uint32_t)D4;

    uint32_t row[S], smp[S];
#pragma unroll
    for (int i = 0; i < S; i += 2) {
        const uint4 e2 = *reinterpret_cast<const uint4 *>(ep + base + i);   // two pairs
        row[i] = e2.x; smp[i] = e2.y;
        row[i + 1] = e2.z; smp[i + 1] = e2.w;
    }
    const uint32_t prev = base > 0 ? ep[base - 1].x : kNoPrev;
    const uint32_t next = base + S < NP ? ep[base + S].x : kNoRow;
    // only the last group looks at it: does its last run come from an earlier workgroup?
    const uint32_t before_wg = (g == NG - 1 && wg_base > 0) ? ep[wg_base - 1].x : kNoPrev;

    // Stale and padding lookups carry the sentinel key, the largest there is:
    // they form the last run of the table, which never ends and is never stored.
    // Their second word is a valid sample number, so gradient loads need no guard.
    //   end[i]: a run ends at lookup i;  put[i]: ... and it began in this strip,
    //   so its sum is complete here and the row is updated right away.
    const bool cont = row[0] == prev;       // the first run began before the strip
    bool end[S], put[S];
    bool open = cont;
#pragma unroll
    for (int i = 0; i < S; ++i) {
        end[i] = (i < S - 1 ? row[i + 1] : next) != row[i];
        put[i] = end[i] && !open && row[i] != kNoRow;
        open = open && !end[i];
    }
    const bool through = open;              // one run covers the strip and goes on
    const bool has_trail = !end[S - 1] && !through && row[S - 1] != kNoRow;
    // 0: the strip starts a new run; 1: it starts inside a run that ends in it; 2: through
    const uint8_t state = (cont && row[0] != kNoRow) ? (through ? 2 : 1) : 0;
    if (c == 0) s_lead_state[g] = state;
    // workgroup-level metadata, written by every workgroup on every call
    if (g == NG - 1 && c == 0) {
        const bool wg_trail = row[S - 1] != kNoRow && !end[S - 1] &&
                              before_wg != row[S - 1];
        meta_trail_row[t * wgs_per_table + wg] = wg_trail ? row[S - 1] : kNoRow;
    }

    for (int cb = 0; FULL ? cb == 0 : cb < D4; cb += G) {
        const int col = cb + c;
        const bool active = FULL || col < D4;
        const auto Wc = W + col;            // this lane's f4 of row 0
        f4 gv[S], wv[S];
#pragma unroll
        for (int i = 0; i < S; ++i) {
            f4 v = unset_f4();
            if (active) {
                // with one lookup per bag a gradient row is read exactly once
                const f4 *gp = grad_ptr<G, FULL>(G4, smp[i], (uint32_t)col, d4);
                v = stream_grads ? __builtin_nontemporal_load(gp) : *gp;
            }
            gv[i] = v;
        }
#pragma unroll
        for (int i = 0; i < S; ++i) {
            f4 w = unset_f4();
            if (put[i] && active) w = *row_ptr<G, FULL>(Wc, row[i], d4);
            wv[i] = w;
        }
        f4 w_trail = unset_f4();
        if (has_trail && active) w_trail = *row_ptr<G, FULL>(Wc, row[S - 1], d4);

        f4 acc = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int i = 0; i < S; ++i) {
            if (active) acc = i == 0 ? gv[0] : acc + gv[i];
            const f4 run = acc;
            acc = end[i] ? f4{0.f, 0.f, 0.f, 0.f} : acc;
            if (put[i] && active)
                *row_ptr<G, FULL>(Wc, row[i], d4) = sgd(wv[i], run, lr);
            // the only other run that can end is the one that came in from the left
            if (end[i] && !put[i]) s_lead[tid] = run;
        }
        if (through) s_lead[tid] = acc;
        __syncthreads();

        // stitch the runs that cross strip borders, in strip order; acc is the
        // sum of the run that leaves the strip to the right
        if (has_trail) {
            f4 sum = acc;
            bool ended = false;
            for (int q = g + 1; q < NG; ++q) {
                sum = sum + s_lead[q * G + c];
                if (s_lead_state[q] == 1) { ended = true; break; }
            }
            if (ended) {
                if (active)
                    *row_ptr<G, FULL>(Wc, row[S - 1], d4) = sgd(w_trail, sum, lr);
            } else if (active) {
                part_trail[((int64_t)t * wgs_per_table + wg) * D4 + col] = sum;
            }
        }
        if (g == 0) {
            uint8_t st = state;
            if (st != 0) {
                f4 sum = s_lead[c];
                int q = 0;
                while (st == 2 && q + 1 < NG) {
                    ++q;
                    sum = sum + s_lead[q * G + c];
                    st = s_lead_state[q];
                }
                if (active)
                    part_lead[((int64_t)t * wgs_per_table + wg) * D4 + col] = sum;
            }
            if (c == 0 && cb == 0) meta_lead_state[t * wgs_per_table + wg] = st;
        }
        if (!FULL) __syncthreads();
    }
    trace_end(ts, trace_t0);
}

// ---------------------------------------------------------------------------
// Stage 3: runs that cross workgroup borders.
// One thread group (G lanes) per workgroup of the apply stage: it looks up
// whether a run starts there and leaves it.  Most such runs end within the next
// few workgroups; the group then adds the pieces itself (everything it needs is
// requested at once: two round trips to memory in all).  The runs of the hottest
// rows cover hundreds of workgroups: those are queued in LDS and afterwards
// taken one at a time by all threads of the workgroup together.
// ---------------------------------------------------------------------------
// Pieces g, g + NG, g + 2 NG, ... of a run, added in that order, UN loads at a
// time.  Piece 0 is the trailing sum of the workgroup the run starts in (*pt),
// piece k the leading sum of the k-th workgroup after it (pl[k * D4]).
template <int UN, int NG>
__device__ __forceinline__ f4 sum_pieces(const f4 *__restrict__ pt,
                                         const f4 *__restrict__ pl, int D4, int g,
                                         int npieces)
{
    f4 sum = f4{0.f, 0.f, 0.f, 0.f};
    for (int k0 = g; k0 < npieces; k0 += NG * UN) {
        f4 v[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int k = k0 + u * NG;
            const int kk = k < npieces ? k : k0;      // in range, value unused
            v[u] = kk == 0 ? *pt : pl[(int64_t)kk * D4];
        }
#pragma unroll
        for (int u = 0; u < UN; ++u)
            if (k0 + u * NG < npieces) sum = sum + v[u];
    }
    return sum;
}

constexpr int kNear = 8;     // a run that ends this many workgroups on is "short"

template <int G, typename TS>
__global__ __launch_bounds__(kWG) void fixup_kernel(
    float *const *__restrict__ weights, int D4, float lr, int wgs_per_table,
    int chunks_per_table, int per_chunk, const uint32_t *__restrict__ meta_trail_row,
    const uint8_t *__restrict__ meta_lead_state,
    const f4 *__restrict__ part_lead, const f4 *__restrict__ part_trail, TS ts)
{
    constexpr int NG = kWG / G;
    __shared__ uint8_t s_state[kWG];     // lead states of the kWG workgroups after the first
    const unsigned long long trace_t0 = trace_begin<TS>();
    __shared__ int s_long[NG];           // queue of long runs: workgroup they start in
    __shared__ uint32_t s_long_row[NG];  // ... and their row
    __shared__ int s_nlong;
    __shared__ int s_end;
    __shared__ f4 s_part[kWG];
    const int t = blockIdx.x / chunks_per_table;
    const int chunk = blockIdx.x - t * chunks_per_table;
    const int tid = threadIdx.x, g = tid / G, c = tid % G;
    // per_chunk = NG: every group checks a workgroup of the apply stage;
    // per_chunk = 1: only the first does (for launches so small that one
    // workgroup per run costs nothing and spares a long run the wait for short ones)
    const int wg_first = chunk * per_chunk;
    const int wg = wg_first + g;              // the apply workgroup this group checks
    const uint8_t *__restrict__ ls = meta_lead_state + (int64_t)t * wgs_per_table;
    const f4 *__restrict__ PL = part_lead + (int64_t)t * wgs_per_table * D4;
    const f4 *__restrict__ PT = part_trail + (int64_t)t * wgs_per_table * D4;
    const auto W = as_global(reinterpret_cast<f4 *>(weights[t]));

    // One round trip: the row of the run that leaves each workgroup, and the lead
    // states of the next kWG workgroups (enough to see where nearly every run ends).
    const uint32_t row = (g < per_chunk && wg < wgs_per_table)
                             ? meta_trail_row[t * wgs_per_table + wg]
                             : kNoRow;
    {
        const int q = wg_first + 1 + tid;
        s_state[tid] = q < wgs_per_table ? ls[q] : (uint8_t)2;
    }
    if (tid == 0) s_nlong = 0;
    __syncthreads();

    // the run ends in the first later workgroup whose leading run stops there
    int last = -1;
#pragma unroll
    for (int u = kNear - 1; u >= 0; --u)
        if (g + u < kWG && s_state[g + u] != 2) last = u;
    const bool mine = row != kNoRow;
    const bool near = mine && last >= 0;
    if (mine && !near && c == 0) {
        const int slot = atomicAdd(&s_nlong, 1);
        s_long[slot] = wg;
        s_long_row[slot] = row;
    }

    if (near) {
        for (int cb = 0; cb < D4; cb += G) {
            const int col = cb + c;
            if (col < D4) {
                f4 v[kNear];
                const f4 tr = PT[(int64_t)wg * D4 + col];
#pragma unroll
                for (int u = 0; u < kNear; ++u) {
                    f4 x = f4{0.f, 0.f, 0.f, 0.f};
                    if (u <= last) x = PL[(int64_t)(wg + 1 + u) * D4 + col];
                    v[u] = x;
                }
                const int64_t o = (int64_t)row * D4 + col;
                const f4 w0 = W[o];
                f4 sum = tr;
#pragma unroll
                for (int u = 0; u < kNear; ++u)
                    if (u <= last) sum = sum + v[u];
                W[o] = sgd(w0, sum, lr);
            }
        }
    }
    __syncthreads();

    // long runs: all threads together, one run after the other
    const int nlong = s_nlong;
    for (int i = 0; i < nlong; ++i) {
        const int w0g = s_long[i];
        const uint32_t lrow = s_long_row[i];
        if (tid == 0) s_end = 0x7fffffff;
        __syncthreads();
        // first among the states already in LDS ...  (One LDS atomic per wavefront:
        // its first lane that sees the run end, found with a ballot.  An atomic per
        // lane on the one address took 2 us, a third of this kernel's duration.)
        {
            const int k = w0g - wg_first + tid;
            const unsigned long long hits = __ballot(k < kWG && s_state[k] != 2);
            if (hits && (tid & 63) == 0)
                atomicMin(&s_end, w0g + 1 + tid + (int)__builtin_ctzll(hits));
        }
        __syncthreads();
        int end = s_end;
        __syncthreads();
        // ... then, for the few runs longer than that, in memory
        for (int b0 = wg_first + 1 + kWG; end == 0x7fffffff && b0 < wgs_per_table;
             b0 += kWG) {
            const int q = b0 + tid;
            const uint8_t s2 = q < wgs_per_table ? ls[q] : (uint8_t)2;
            const unsigned long long hits = __ballot(q < wgs_per_table && s2 != 2);
            if (hits && (tid & 63) == 0) atomicMin(&s_end, q + (int)__builtin_ctzll(hits));
            __syncthreads();
            end = s_end;
            __syncthreads();
        }
        if (end == 0x7fffffff) continue;   // cannot happen for a sorted list

        // pieces: trail(w0g), lead(w0g + 1), ..., lead(end); group g adds every NG-th
        const int npieces = end - w0g + 1;
        for (int cb = 0; cb < D4; cb += G) {
            const int col = cb + c;
            const bool active = col < D4;
            const int64_t o = (int64_t)lrow * D4 + col;
            f4 w0 = f4{0.f, 0.f, 0.f, 0.f};
            if (g == 0 && active) w0 = W[o];
            f4 sum = f4{0.f, 0.f, 0.f, 0.f};
            if (active) {
                const f4 *pt = PT + (int64_t)w0g * D4 + col;
                const f4 *pl = PL + (int64_t)w0g * D4 + col;
                sum = sum_pieces<8, NG>(pt, pl, D4, g, npieces);
            }
            s_part[tid] = sum;
            __syncthreads();
            if (g == 0 && active) {
                f4 tot = s_part[c];
                const int used = npieces < NG ? npieces : NG;
                for (int q = 1; q < used; ++q) tot = tot + s_part[q * G + c];
                W[o] = sgd(w0, tot, lr);
            }
            __syncthreads();
        }
    }
    trace_end(ts, trace_t0);
}

struct Layout {
    int NP, tiles, max_wgs;
    size_t ent0, ent1, hist, bucket, trail_row, lead_state, part_lead,
        part_trail, total;
};

Layout make_layout(int T, int Bcap, int L, int dim)
{
    Layout y;
    const int64_t nnz = (int64_t)Bcap * L;
    y.NP = (int)align_up((size_t)nnz, kPad);
    y.tiles = y.NP / kPad;
    const int g = lanes_per_row(dim);
    const int ng = kApplyWG / g;
    y.max_wgs = y.NP / (ng * 4);          // smallest strip is 4 lookups
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    const size_t arr = (size_t)T * y.NP * sizeof(uint2);      // (row, sample) pairs
    y.ent0 = take(arr);
    y.ent1 = take(arr);
    y.hist = take((size_t)T * kRsMaxDig * y.tiles * sizeof(uint32_t));
    y.bucket = take((size_t)T * kBsStride * sizeof(uint32_t));
    y.trail_row = take((size_t)T * y.max_wgs * sizeof(uint32_t));
    y.lead_state = take((size_t)T * y.max_wgs);
    y.part_lead = take((size_t)T * y.max_wgs * dim * sizeof(float));
    y.part_trail = take((size_t)T * y.max_wgs * dim * sizeof(float));
    y.total = off;
    return y;
}

int key_bits_for(int64_t rows)
{
    int b = 1;
    while (b < 31 && (1LL << b) < rows) ++b;
    return b;
}

// Bits the global radix sort has to order.  The sentinel key of dropped and padding
// lookups is all ones, so it must differ from every row id within these bits, or a
// single-pass sort would file it with the last row and cut that row's run into
// pieces: one more bit than the row ids need when rows is a power of two.
int radix_bits_for(int64_t rows) { return key_bits_for(rows + 1); }

// Strip length (lookups per lane group in the apply stage), as measured: 4 for
// rows of 256 bytes (18.3 against 18.8 us at 26 tables x 8192 lookups), 8 for
// longer rows (40.2 against 42.1 us at 8 tables x 81920 lookups of 512 bytes:
// fewer pieces to stitch) and for shorter ones (8.3 against 10.2 us at 26 tables
// x 2048 lookups of 64 bytes, where a workgroup holds 64 groups).
int pick_strip(int lanes_per_group) { return lanes_per_group == 16 ? 4 : 8; }

}  // namespace

size_t backward_ws_bytes(int T, int Bcap, int L, int dim)
{
    return make_layout(T, Bcap, L, dim).total;
}

void backward_first_buffers(int T, int Bcap, int L, int dim, void *ws, uint2 **ent,
                            int *NP)
{
    const Layout y = make_layout(T, Bcap, L, dim);
    char *w8 = static_cast<char *>(ws);
    *ent = reinterpret_cast<uint2 *>(w8 + y.ent0);
    *NP = y.NP;
}

// Which of the two pair buffers holds the sorted lists after stage 1.
// How the lists of a table that is too large for the one-launch sort get grouped: one
// global pass on the low nb0 bits of the row id, and, if the row id has more bits than
// that, a sort of every bucket by the remaining bits (bucket_sort_kernel).
struct RadixPlan {
    int nb0;            // digit bits of the global pass (at most kRsMaxBits; 9 with buckets)
    bool buckets;
    int rem_bits;       // row bits left to sort in the buckets
    int val_bits;       // bits of a sample number
    bool packed;        // the two fit one word
};

static RadixPlan plan_radix(const Layout &y, int T, int Bcap, int64_t rows)
{
    RadixPlan p = {};
    const int sort_bits = radix_bits_for(rows);
    if (sort_bits <= kRsMaxBits) {
        p.nb0 = sort_bits;
        return p;
    }
    // Buckets of 2048 to 4096 lookups on average (at 8 tables x 81920 lookups, us per
    // training step: 87.4 with 32 buckets per table, 88.8 with 64, 90.8 with 128, 92.9
    // with 256; 95.1 with three global passes instead of the buckets.  In place of two
    // global passes: 52.6 instead of 54.0 at 8 tables x 32768 lookups of 500 000 rows,
    // 20.6 instead of 24.1 at one table x 65536 of 800 000), more buckets where the
    // tables are so few that this would leave compute units without one.
    int nb0 = 4;
    while (nb0 < 9 && (4096 << nb0) < y.NP) ++nb0;
    while (nb0 < 9 && ((int64_t)T << nb0) < 256 && (64 << nb0) < y.NP) ++nb0;
    p.nb0 = nb0;
    p.buckets = true;
    p.rem_bits = sort_bits - nb0;
    p.val_bits = 1;
    while ((1 << p.val_bits) < Bcap) ++p.val_bits;
    p.packed = p.rem_bits + p.val_bits <= 31;
    return p;
}

int32_t launch_backward_prepare(const ss_tables *tb, const int32_t *idx, int Bcap,
                                int L, const int32_t *n_valid, void *ws,
                                hipStream_t s, hipEvent_t record_after)
{
    const int T = tb->num_tables;
    const Layout y = make_layout(T, Bcap, L, tb->dim);
    char *w8 = static_cast<char *>(ws);
    uint2 *ent[2] = {reinterpret_cast<uint2 *>(w8 + y.ent0),
                     reinterpret_cast<uint2 *>(w8 + y.ent1)};
    uint32_t *hist = reinterpret_cast<uint32_t *>(w8 + y.hist);
    const int key_bits = key_bits_for(tb->rows);

    if (y.NP <= kLdsSortMax) {
        const ClassSortPlan cp = plan_class_sort(y.NP, Bcap, key_bits);
        const dim3 grid(1 << cp.class_bits, T);
        ProfScope prof("class_sort_kernel", s);
        if (record_after) stop_event_for_next_launch(record_after);     // the only launch
#define SS_LDS_SORT(I, P)                                                          \
    launch(SS_BOTH(class_sort_kernel, I, P), grid, dim3(1024), s, idx, Bcap, L, n_valid,     \
           tb->stale_bits, key_bits, cp.class_bits, cp.val_bits, ent[0],            \
           y.NP)
        if (cp.packed) {
            if (cp.items == 2) { SS_LDS_SORT(2, true); }
            else if (cp.items == 4) { SS_LDS_SORT(4, true); }
            else if (cp.items == 8) { SS_LDS_SORT(8, true); }
            else { SS_LDS_SORT(16, true); }
        } else {
            if (cp.items == 2) { SS_LDS_SORT(2, false); }
            else if (cp.items == 4) { SS_LDS_SORT(4, false); }
            else if (cp.items == 8) { SS_LDS_SORT(8, false); }
            else { SS_LDS_SORT(16, false); }
        }
#undef SS_LDS_SORT
    } else {
        // the (row, sample) pairs go to buffer 1 and are scattered into buffer 0, where
        // the buckets are then sorted in place (buffer 1 is their spare)
        const RadixPlan rp = plan_radix(y, T, Bcap, tb->rows);
        uint32_t *bucket = reinterpret_cast<uint32_t *>(w8 + y.bucket);
        const dim3 grid(y.tiles, T);
        const int sent = rp.buckets ? 1 : 0;
        {
            ProfScope prof("rs_hist_kernel", s);
            launch(rs_hist_kernel<NoTrace>, rs_hist_kernel<TraceSlot>, grid, dim3(kRsHistThreads),
                   s, idx, Bcap, L, n_valid, tb->stale_bits, ent[1], y.NP, rp.nb0, sent, hist,
                   y.tiles);
        }
        {
            ProfScope prof("rs_scatter_kernel", s);
            if (record_after && !rp.buckets) stop_event_for_next_launch(record_after);
            launch(rs_scatter_kernel<NoTrace>, rs_scatter_kernel<TraceSlot>, grid,
                   dim3(kRsThreads), s, (const uint2 *)ent[1], ent[0], y.NP, rp.nb0, sent,
                   rp.buckets ? bucket : nullptr, (const uint32_t *)hist, y.tiles);
        }
        if (rp.buckets) {
            ProfScope prof("bucket_sort_kernel", s);
            if (record_after) stop_event_for_next_launch(record_after);
            if (rp.packed)
                launch(SS_BOTH(bucket_sort_kernel, true), dim3(1u << rp.nb0, T),
                       dim3(kBucketThreads), s, ent[0], ent[1], y.NP,
                       (const uint32_t *)bucket, rp.nb0, rp.rem_bits, rp.val_bits);
            else
                launch(SS_BOTH(bucket_sort_kernel, false), dim3(1u << rp.nb0, T),
                       dim3(kBucketThreads), s, ent[0], ent[1], y.NP,
                       (const uint32_t *)bucket, rp.nb0, rp.rem_bits, rp.val_bits);
        }
    }
    return check_launch("ss_embbag_backward_prepare");
}

int32_t launch_backward_apply(const ss_tables *tb, int Bcap, int L, const float *grad,
                              float lr, void *ws, hipStream_t s, hipEvent_t record_after)
{
    const int T = tb->num_tables, D4 = tb->dim / 4;
    const Layout y = make_layout(T, Bcap, L, tb->dim);
    char *w8 = static_cast<char *>(ws);
    const uint2 *ent = reinterpret_cast<const uint2 *>(w8 + y.ent0);      // the grouped lists

    const int g = lanes_per_row(tb->dim);
    const int ng = kApplyWG / g;
    const int strip = pick_strip(g);
    const int wgs = y.NP / (ng * strip);
    uint32_t *trail_row = reinterpret_cast<uint32_t *>(w8 + y.trail_row);
    uint8_t *lead_state = reinterpret_cast<uint8_t *>(w8 + y.lead_state);
    f4 *part_lead = reinterpret_cast<f4 *>(w8 + y.part_lead);
    f4 *part_trail = reinterpret_cast<f4 *>(w8 + y.part_trail);
    const int64_t blocks = (int64_t)wgs * T;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_backward_apply: grid too large");
    // one gradient block per L2: only worth it when gradient rows are re-read
    const int pinned = L > 1 ? (T / 8) * 8 * wgs : 0;
#define SS_APPLY(S_, F_)                                                          \
    SS_DISPATCH_G(g, launch(SS_BOTH(apply_kernel, G, S_, F_), dim3((unsigned)blocks),    \
                            dim3(kApplyWG), s, tb->weights, ent, y.NP, grad,    \
                            Bcap, D4, lr, wgs, pinned, L == 1, trail_row,         \
                            lead_state, part_lead, part_trail))
    {
        ProfScope prof("apply_kernel", s);
        // a row that fills its group of lanes exactly needs no column loop and no guard
        const bool full = D4 == g && (int64_t)Bcap * tb->dim * 4 <= 0xFFFFFFFFLL;
        if (strip == 8) {
            if (full) { SS_APPLY(8, true); } else { SS_APPLY(8, false); }
        } else {
            if (full) { SS_APPLY(4, true); } else { SS_APPLY(4, false); }
        }
    }
#undef SS_APPLY
    ProfScope prof("fixup_kernel", s);
    // apply workgroups looked at per workgroup of this launch
    const int per_chunk = (int64_t)wgs * T <= 2048 ? 1 : kWG / g;
    const int chunks = (wgs + per_chunk - 1) / per_chunk;
    if (record_after) stop_event_for_next_launch(record_after);     // the last launch of the update
    SS_DISPATCH_G(g, launch(SS_BOTH(fixup_kernel, G), dim3((unsigned)(chunks * T)),
                                        dim3(kWG), s, tb->weights, D4, lr, wgs,
                                        chunks, per_chunk, trail_row, lead_state,
                                        part_lead, part_trail));
    return check_launch("ss_embbag_backward_apply");
}

}  // namespace ss
