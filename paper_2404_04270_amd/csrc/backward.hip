// ss_embbag_backward_update: gradient scatter of the pooled lookup fused with
// sparse SGD that skips stale rows (abstract and section 3.6 of the paper).
//
// Three stages, all tables in every launch:
//
//  1. SORT the lookups of each table by row id (stable, so equal rows keep the
//     order "ascending sample, then position in bag").  The payload is the
//     sample number, which is all the gradient gather needs.
//       - up to 16384 lookups per table: one 1024-thread workgroup per table
//         holds keys and payloads in registers and runs an LSD radix sort whose
//         exchange buffers live in LDS (one launch);
//       - more: a global LSD radix sort, 8 bits per pass, three launches per
//         pass (per-tile digit histogram, scan, stable scatter).
//     Ranking inside a wavefront uses ballots: the lanes that hold the same
//     digit are found with one ballot per digit bit, a popcount of the lower
//     lanes gives the rank, and one lane per digit bumps the wavefront's LDS
//     counter.  Tables are padded with sentinel keys to a multiple of 2048.
//
//  2. APPLY walks the sorted list in strips of S lookups per group of G lanes
//     (one float4 of the row per lane).  All gradient rows of the strip and the
//     weight rows of the runs that end in it are requested up front, then the
//     runs are summed in order.  A run that lies inside one strip is applied
//     right away.  Runs that cross strip borders leave a leading / trailing
//     piece in LDS and are stitched together inside the workgroup in strip
//     order; runs that cross workgroup borders leave their piece in the
//     workspace.
//
//  3. FIXUP: one workgroup per run that crossed a workgroup border adds its
//     pieces in a fixed order and applies the update.
//
// Rows whose stale bit is set are skipped before any gradient or weight of
// theirs is read.  There are no floating-point atomics: every sum has a fixed
// order, so the result is reproducible.
#include "ss_common.h"

namespace ss {

namespace {

constexpr int kPad = 2048;             // per-table padding of the sorted arrays
constexpr int kLdsSortMax = 16384;     // largest table the one-launch sort takes
constexpr uint32_t kNoPrev = 0xFFFFFFFEu;
constexpr int kRsThreads = 256;        // global radix sort: threads per tile
constexpr int kRsItems = 8;            // ... keys per thread (tile = 2048 = kPad)

__device__ __forceinline__ uint64_t lanes_below(int lane)
{
    return (1ull << lane) - 1ull;
}

// Lanes of this wavefront whose digit equals mine (all 64 lanes must call).
__device__ __forceinline__ uint64_t match_digit(uint32_t d, int nbits)
{
    uint64_t m = ~0ull;
    for (int b = 0; b < nbits; ++b) {
        const bool one = (d >> b) & 1u;
        const uint64_t bal = __ballot(one);
        m &= one ? bal : ~bal;
    }
    return m;
}

// Bits of the pass-th of npass digits when key_bits are split as evenly as
// possible (earlier passes take the extra bits).
__host__ __device__ inline int pass_bits(int key_bits, int npass, int pass)
{
    return key_bits / npass + (pass < key_bits % npass ? 1 : 0);
}

// ---------------------------------------------------------------------------
// Stage 1a: whole table in one workgroup.
// ---------------------------------------------------------------------------
template <int ITEMS>
__global__ __launch_bounds__(1024) void lds_sort_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, int key_bits,
    uint32_t *__restrict__ out_keys, uint32_t *__restrict__ out_vals, int NP)
{
    constexpr int NW = 16, CAP = 1024 * ITEMS;
    __shared__ uint32_t s_keys[CAP];
    __shared__ uint32_t s_vals[CAP];
    __shared__ uint32_t s_cnt[NW * 256];
    __shared__ uint32_t s_dig[256];
    __shared__ uint32_t s_wsum[4];
    volatile uint32_t *v_cnt = s_cnt;

    const int t = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = clamp_valid(n_valid, Bcap) * L;
    const int32_t *__restrict__ ip = idx + (int64_t)t * Bcap * L;

    uint32_t key[ITEMS], val[ITEMS], rank[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int pos = wave * ITEMS * 64 + r * 64 + lane;
        if (pos < n) {
            key[r] = (uint32_t)ip[pos];
            val[r] = (uint32_t)(pos / L);
        } else {
            key[r] = kNoRow;
            val[r] = 0;
        }
    }

    const int npass = (key_bits + 7) / 8;
    int shift = 0;
    for (int pass = 0; pass < npass; ++pass) {
        const int nb = pass_bits(key_bits, npass, pass);
        const uint32_t dmask = (1u << nb) - 1u;
        for (int i = tid; i < NW * 256; i += 1024) s_cnt[i] = 0;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const uint32_t d = (key[r] >> shift) & dmask;
            const uint64_t m = match_digit(d, nb);
            const uint32_t before = __popcll(m & lanes_below(lane));
            const uint32_t base = v_cnt[wave * 256 + d];
            rank[r] = base + before;
            if (before == 0) v_cnt[wave * 256 + d] = base + (uint32_t)__popcll(m);
        }
        __syncthreads();
        // per digit: exclusive offsets of the wavefronts, total of the digit
        if (tid <= (int)dmask) {
            uint32_t run = 0;
            for (int w = 0; w < NW; ++w) {
                const uint32_t c = s_cnt[w * 256 + tid];
                s_cnt[w * 256 + tid] = run;
                run += c;
            }
            s_dig[tid] = run;
        }
        __syncthreads();
        // exclusive scan of the digit totals (first four wavefronts)
        uint32_t incl = 0, mine = 0;
        if (tid < 256) {
            mine = tid <= (int)dmask ? s_dig[tid] : 0;
            incl = mine;
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            if (lane == 63) s_wsum[wave] = incl;
        }
        __syncthreads();
        if (tid < 256) {
            uint32_t wb = 0;
            for (int w = 0; w < wave; ++w) wb += s_wsum[w];
            s_dig[tid] = wb + incl - mine;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < ITEMS; ++r) {
            const uint32_t d = (key[r] >> shift) & dmask;
            const uint32_t p = s_dig[d] + s_cnt[wave * 256 + d] + rank[r];
            s_keys[p] = key[r];
            s_vals[p] = val[r];
        }
        __syncthreads();
        if (pass + 1 < npass) {
#pragma unroll
            for (int r = 0; r < ITEMS; ++r) {
                const int pos = wave * ITEMS * 64 + r * 64 + lane;
                key[r] = s_keys[pos];
                val[r] = s_vals[pos];
            }
        }
        shift += nb;
    }
    const int lim = CAP < NP ? CAP : NP;
    for (int i = tid; i < lim; i += 1024) {
        out_keys[(int64_t)t * NP + i] = s_keys[i];
        out_vals[(int64_t)t * NP + i] = s_vals[i];
    }
}

// ---------------------------------------------------------------------------
// Stage 1b: global LSD radix sort, one pass = histogram, scan, scatter.
// Tile = 2048 keys; hist layout [table][digit][tile].
// ---------------------------------------------------------------------------
template <bool FIRST>
__device__ __forceinline__ void rs_load(const int32_t *__restrict__ idx, int L, int n,
                                        const uint32_t *__restrict__ in_keys,
                                        const uint32_t *__restrict__ in_vals,
                                        int64_t table_off_idx, int64_t table_off,
                                        int pos, uint32_t &key, uint32_t &val)
{
    if (FIRST) {
        if (pos < n) {
            key = (uint32_t)idx[table_off_idx + pos];
            val = (uint32_t)(pos / L);
        } else {
            key = kNoRow;
            val = 0;
        }
    } else {
        key = in_keys[table_off + pos];
        val = in_vals[table_off + pos];
    }
}

template <bool FIRST>
__global__ __launch_bounds__(kRsThreads) void rs_hist_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, const uint32_t *__restrict__ in_keys,
    int NP, int shift, int nb, uint32_t *__restrict__ hist, int tiles)
{
    __shared__ uint32_t s_hist[256];
    const int t = blockIdx.y, tile = blockIdx.x, tid = threadIdx.x;
    const int n = clamp_valid(n_valid, Bcap) * L;
    const uint32_t dmask = (1u << nb) - 1u;
    s_hist[tid] = 0;
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {
        const int pos = tile * kPad + r * kRsThreads + tid;
        uint32_t key, val;
        rs_load<FIRST>(idx, L, n, in_keys, in_keys, (int64_t)t * Bcap * L,
                       (int64_t)t * NP, pos, key, val);
        atomicAdd(&s_hist[(key >> shift) & dmask], 1u);
    }
    __syncthreads();
    if (tid <= (int)dmask)
        hist[((int64_t)t * 256 + tid) * tiles + tile] = s_hist[tid];
}

// Exclusive scan over the (digit-major, tile-minor) histogram of each table.
__global__ __launch_bounds__(1024) void rs_scan_kernel(uint32_t *__restrict__ hist,
                                                       int tiles, int nb)
{
    __shared__ uint32_t s_wsum[16];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t *h = hist + (int64_t)t * 256 * tiles;
    const int len = (1 << nb) * tiles;
    const int per = (len + 1023) / 1024;
    const int lo = tid * per, hi = lo + per < len ? lo + per : len;
    uint32_t sum = 0;
    for (int i = lo; i < hi; ++i) sum += h[i];
    uint32_t incl = sum;
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t up = __shfl_up(incl, off);
        if (lane >= off) incl += up;
    }
    if (lane == 63) s_wsum[wave] = incl;
    __syncthreads();
    uint32_t run = incl - sum;
    for (int w = 0; w < wave; ++w) run += s_wsum[w];
    for (int i = lo; i < hi; ++i) {
        const uint32_t c = h[i];
        h[i] = run;
        run += c;
    }
}

template <bool FIRST>
__global__ __launch_bounds__(kRsThreads) void rs_scatter_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, const uint32_t *__restrict__ in_keys,
    const uint32_t *__restrict__ in_vals, uint32_t *__restrict__ out_keys,
    uint32_t *__restrict__ out_vals, int NP, int shift, int nb,
    const uint32_t *__restrict__ hist, int tiles)
{
    constexpr int NW = kRsThreads / 64;
    __shared__ uint32_t s_cnt[NW * 256];
    volatile uint32_t *v_cnt = s_cnt;
    const int t = blockIdx.y, tile = blockIdx.x;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = clamp_valid(n_valid, Bcap) * L;
    const uint32_t dmask = (1u << nb) - 1u;
    for (int i = tid; i < NW * 256; i += kRsThreads) s_cnt[i] = 0;
    __syncthreads();
    uint32_t key[kRsItems], val[kRsItems], rank[kRsItems];
#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {
        // wavefront w owns the contiguous quarter w of the tile, in order
        const int pos = tile * kPad + wave * (kRsItems * 64) + r * 64 + lane;
        rs_load<FIRST>(idx, L, n, in_keys, in_vals, (int64_t)t * Bcap * L,
                       (int64_t)t * NP, pos, key[r], val[r]);
        const uint32_t d = (key[r] >> shift) & dmask;
        const uint64_t m = match_digit(d, nb);
        const uint32_t before = __popcll(m & lanes_below(lane));
        const uint32_t base = v_cnt[wave * 256 + d];
        rank[r] = base + before;
        if (before == 0) v_cnt[wave * 256 + d] = base + (uint32_t)__popcll(m);
    }
    __syncthreads();
    if (tid <= (int)dmask) {
        uint32_t run = hist[((int64_t)t * 256 + tid) * tiles + tile];
        for (int w = 0; w < NW; ++w) {
            const uint32_t c = s_cnt[w * 256 + tid];
            s_cnt[w * 256 + tid] = run;
            run += c;
        }
    }
    __syncthreads();
#pragma unroll
    for (int r = 0; r < kRsItems; ++r) {
        const uint32_t d = (key[r] >> shift) & dmask;
        const int64_t p = (int64_t)t * NP + s_cnt[wave * 256 + d] + rank[r];
        out_keys[p] = key[r];
        out_vals[p] = val[r];
    }
}

// ---------------------------------------------------------------------------
// Stage 2: apply.
// Workspace per (table, workgroup): trail_row (row whose run starts in this
// workgroup and continues into the next one, or kNoRow), lead_state (0: the
// workgroup starts with a new run; 1: it starts inside a run that ends in it;
// 2: that run covers the whole workgroup and goes on), and the two partial
// sums part_lead / part_trail of dim floats each.
// ---------------------------------------------------------------------------
template <int G, int S>
__global__ __launch_bounds__(kWG) void apply_kernel(
    float *const *__restrict__ weights, const uint32_t *const *__restrict__ bits,
    const uint32_t *__restrict__ keys, const uint32_t *__restrict__ vals, int NP,
    const float *__restrict__ grad, int Bcap, int D4, float lr,
    int wgs_per_table, uint32_t *__restrict__ meta_trail_row,
    uint8_t *__restrict__ meta_lead_state, float4 *__restrict__ part_lead,
    float4 *__restrict__ part_trail)
{
    constexpr int NG = kWG / G;
    __shared__ float4 s_lead[kWG];
    __shared__ float4 s_trail[kWG];
    __shared__ uint32_t s_trail_row[NG];
    __shared__ uint8_t s_lead_state[NG];

    const int t = blockIdx.x / wgs_per_table;
    const int wg = blockIdx.x - t * wgs_per_table;
    const int tid = threadIdx.x, g = tid / G, c = tid % G;
    const uint32_t *__restrict__ kp = keys + (int64_t)t * NP;
    const uint32_t *__restrict__ vp = vals + (int64_t)t * NP;
    const uint32_t *__restrict__ bt = bits ? bits[t] : nullptr;
    float4 *__restrict__ W = reinterpret_cast<float4 *>(weights[t]);
    const float4 *__restrict__ G4 =
        reinterpret_cast<const float4 *>(grad) + (int64_t)t * Bcap * D4;
    const int wg_base = wg * NG * S;
    const int base = wg_base + g * S;

    uint32_t row[S], smp[S];
#pragma unroll
    for (int i = 0; i < S; i += 4) {
        const uint4 k4 = *reinterpret_cast<const uint4 *>(kp + base + i);
        const uint4 v4 = *reinterpret_cast<const uint4 *>(vp + base + i);
        row[i] = k4.x; row[i + 1] = k4.y; row[i + 2] = k4.z; row[i + 3] = k4.w;
        smp[i] = v4.x; smp[i + 1] = v4.y; smp[i + 2] = v4.z; smp[i + 3] = v4.w;
    }
    const uint32_t prev = base > 0 ? kp[base - 1] : kNoPrev;
    const uint32_t next = base + S < NP ? kp[base + S] : kNoRow;

    // live: a real lookup whose row is not stale.  Equal within a run.
    bool live[S], is_end[S], whole[S];
    {
        bool has_head = row[0] != prev;
#pragma unroll
        for (int i = 0; i < S; ++i) {
            live[i] = row[i] != kNoRow && !(bt && bit_set(bt, row[i]));
            is_end[i] = (i == S - 1) || row[i + 1] != row[i];
            const bool ends_here = (i < S - 1) || next != row[i];
            whole[i] = is_end[i] && has_head && ends_here;   // run inside the strip
            if (is_end[i]) has_head = true;
        }
    }
    // Run that ends the strip: does it start here, does it go on?
    bool last_has_head = row[0] != prev;
#pragma unroll
    for (int i = 0; i < S - 1; ++i)
        if (row[i + 1] != row[i]) last_has_head = true;
    const bool last_real = row[S - 1] != kNoRow;
    const bool has_trail = last_real && last_has_head && next == row[S - 1];
    // Run that begins the strip: is it a continuation?
    const bool has_lead = row[0] != kNoRow && row[0] == prev;

    if (c == 0) {
        s_trail_row[g] = has_trail ? row[S - 1] : kNoRow;
        uint8_t st = 0;
        if (has_lead) {
            // ends here unless the whole strip is this run and it continues
            bool through = next == row[0];
#pragma unroll
            for (int i = 0; i < S - 1; ++i)
                if (row[i + 1] != row[i]) through = false;
            st = through ? 2 : 1;
        }
        s_lead_state[g] = st;
    }
    // workgroup-level metadata, written by every workgroup on every call
    if (g == NG - 1 && c == 0) {
        const bool from_before = wg_base > 0 && kp[wg_base - 1] == row[S - 1];
        const bool wg_trail = last_real && next == row[S - 1] && !from_before;
        meta_trail_row[t * wgs_per_table + wg] = wg_trail ? row[S - 1] : kNoRow;
    }

    for (int cb = 0; cb < D4; cb += G) {
        const int col = cb + c;
        const bool active = col < D4;
        float4 gv[S], wv[S];
#pragma unroll
        for (int i = 0; i < S; ++i)
            if (live[i] && active) gv[i] = G4[(int64_t)smp[i] * D4 + col];
#pragma unroll
        for (int i = 0; i < S; ++i)
            if (whole[i] && live[i] && active) wv[i] = W[(int64_t)row[i] * D4 + col];
        float4 w_trail = make_float4(0.f, 0.f, 0.f, 0.f);
        if (has_trail && live[S - 1] && active)
            w_trail = W[(int64_t)row[S - 1] * D4 + col];

        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float4 lead_sum = acc, trail_sum = acc;
        bool first_run = true;
#pragma unroll
        for (int i = 0; i < S; ++i) {
            if (live[i] && active) acc = acc + gv[i];
            if (is_end[i]) {
                if (whole[i]) {
                    if (live[i] && active)
                        W[(int64_t)row[i] * D4 + col] = sgd(wv[i], acc, lr);
                } else if (first_run && has_lead) {
                    lead_sum = acc;
                } else {
                    trail_sum = acc;   // only the last run can get here
                }
                acc = make_float4(0.f, 0.f, 0.f, 0.f);
                first_run = false;
            }
        }
        s_lead[tid] = lead_sum;
        s_trail[tid] = trail_sum;
        __syncthreads();

        // stitch the runs that cross strip borders, in strip order
        if (s_trail_row[g] != kNoRow) {
            float4 sum = s_trail[tid];
            bool ended = false;
            for (int q = g + 1; q < NG; ++q) {
                sum = sum + s_lead[q * G + c];
                if (s_lead_state[q] == 1) { ended = true; break; }
            }
            if (ended) {
                if (live[S - 1] && active)
                    W[(int64_t)row[S - 1] * D4 + col] = sgd(w_trail, sum, lr);
            } else if (active) {
                part_trail[((int64_t)t * wgs_per_table + wg) * D4 + col] = sum;
            }
        }
        if (g == 0) {
            uint8_t st = s_lead_state[0];
            if (st != 0) {
                float4 sum = s_lead[c];
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
        __syncthreads();
    }
}

// ---------------------------------------------------------------------------
// Stage 3: runs that cross workgroup borders.
// ---------------------------------------------------------------------------
template <int G>
__global__ __launch_bounds__(kWG) void fixup_kernel(
    float *const *__restrict__ weights, const uint32_t *const *__restrict__ bits,
    int D4, float lr, int wgs_per_table,
    const uint32_t *__restrict__ meta_trail_row,
    const uint8_t *__restrict__ meta_lead_state,
    const float4 *__restrict__ part_lead, const float4 *__restrict__ part_trail)
{
    constexpr int NG = kWG / G;
    __shared__ int s_end;
    __shared__ float4 s_part[kWG];
    const int t = blockIdx.x / wgs_per_table;
    const int wg = blockIdx.x - t * wgs_per_table;
    const uint32_t row = meta_trail_row[t * wgs_per_table + wg];
    if (row == kNoRow) return;
    const uint32_t *__restrict__ bt = bits ? bits[t] : nullptr;
    if (bt && bit_set(bt, row)) return;

    const int tid = threadIdx.x, g = tid / G, c = tid % G;
    const uint8_t *__restrict__ ls = meta_lead_state + (int64_t)t * wgs_per_table;
    // the run ends in the first later workgroup whose leading run stops there
    if (tid == 0) s_end = 0x7fffffff;
    __syncthreads();
    int end = 0x7fffffff;
    for (int b0 = wg + 1; b0 < wgs_per_table; b0 += kWG) {
        const int q = b0 + tid;
        if (q < wgs_per_table && ls[q] != 2) atomicMin(&s_end, q);
        __syncthreads();
        end = s_end;
        __syncthreads();
        if (end != 0x7fffffff) break;
    }
    if (end == 0x7fffffff) return;   // cannot happen for a sorted list

    // pieces: trail(wg), lead(wg+1), ..., lead(end); group g sums every NG-th
    const int npieces = end - wg + 1;
    float4 *__restrict__ W = reinterpret_cast<float4 *>(weights[t]);
    const float4 *__restrict__ PL = part_lead + (int64_t)t * wgs_per_table * D4;
    const float4 *__restrict__ PT = part_trail + (int64_t)t * wgs_per_table * D4;
    for (int cb = 0; cb < D4; cb += G) {
        const int col = cb + c;
        const bool active = col < D4;
        float4 sum = make_float4(0.f, 0.f, 0.f, 0.f);
        if (active)
            for (int k = g; k < npieces; k += NG)
                sum = sum + (k == 0 ? PT[(int64_t)wg * D4 + col]
                                    : PL[(int64_t)(wg + k) * D4 + col]);
        s_part[tid] = sum;
        __syncthreads();
        if (g == 0 && active) {
            float4 tot = s_part[c];
            const int used = npieces < NG ? npieces : NG;
            for (int q = 1; q < used; ++q) tot = tot + s_part[q * G + c];
            const int64_t o = (int64_t)row * D4 + col;
            W[o] = sgd(W[o], tot, lr);
        }
        __syncthreads();
    }
}

struct Layout {
    int NP, tiles, max_wgs;
    size_t keys0, vals0, keys1, vals1, hist, trail_row, lead_state, part_lead,
        part_trail, total;
};

Layout make_layout(int T, int Bcap, int L, int dim)
{
    Layout y;
    const int64_t nnz = (int64_t)Bcap * L;
    y.NP = (int)align_up((size_t)nnz, kPad);
    y.tiles = y.NP / kPad;
    const int g = lanes_per_row(dim);
    const int ng = kWG / g;
    y.max_wgs = y.NP / (ng * 4);          // smallest strip is 4 lookups
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    const size_t arr = (size_t)T * y.NP * sizeof(uint32_t);
    y.keys0 = take(arr);
    y.vals0 = take(arr);
    y.keys1 = take(arr);
    y.vals1 = take(arr);
    y.hist = take((size_t)T * 256 * y.tiles * sizeof(uint32_t));
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

// Strip length: long strips cut the number of pieces, short ones give a small
// problem enough workgroups to occupy the chip.
int pick_strip(int64_t total_lookups, int ng)
{
    if (total_lookups / (ng * 16) >= 1024) return 16;
    if (total_lookups / (ng * 8) >= 1024) return 8;
    return 4;
}

}  // namespace

size_t backward_ws_bytes(int T, int Bcap, int L, int dim)
{
    return make_layout(T, Bcap, L, dim).total;
}

int32_t launch_backward(const ss_tables *tb, const int32_t *idx, int Bcap, int L,
                        const int32_t *n_valid, const float *grad, float lr,
                        void *ws, hipStream_t s)
{
    const int T = tb->num_tables, D4 = tb->dim / 4;
    const Layout y = make_layout(T, Bcap, L, tb->dim);
    char *w8 = static_cast<char *>(ws);
    uint32_t *keys[2] = {reinterpret_cast<uint32_t *>(w8 + y.keys0),
                         reinterpret_cast<uint32_t *>(w8 + y.keys1)};
    uint32_t *vals[2] = {reinterpret_cast<uint32_t *>(w8 + y.vals0),
                         reinterpret_cast<uint32_t *>(w8 + y.vals1)};
    uint32_t *hist = reinterpret_cast<uint32_t *>(w8 + y.hist);
    const int key_bits = key_bits_for(tb->rows);
    int cur = 0;   // buffer that holds the sorted lists

    if (y.NP <= kLdsSortMax) {
        const int items = y.NP / 1024;   // NP is a multiple of 2048
#define SS_LDS_SORT(I)                                                          \
    ProfScope prof("lds_sort_kernel", s);                                        \
    hipLaunchKernelGGL(lds_sort_kernel<I>, dim3(T), dim3(1024), 0, s, idx, Bcap, \
                       L, n_valid, key_bits, keys[0], vals[0], y.NP)
        if (items <= 2) { SS_LDS_SORT(2); }
        else if (items <= 4) { SS_LDS_SORT(4); }
        else if (items <= 8) { SS_LDS_SORT(8); }
        else { SS_LDS_SORT(16); }
#undef SS_LDS_SORT
    } else {
        const int npass = (key_bits + 7) / 8;
        const dim3 grid(y.tiles, T);
        int shift = 0;
        for (int pass = 0; pass < npass; ++pass) {
            const int nb = pass_bits(key_bits, npass, pass);
            const int in = cur, out = pass == 0 ? 0 : 1 - cur;
            {
            ProfScope prof("rs_hist_kernel", s);
            if (pass == 0) {
                hipLaunchKernelGGL(rs_hist_kernel<true>, grid, dim3(kRsThreads), 0,
                                   s, idx, Bcap, L, n_valid, nullptr, y.NP, shift,
                                   nb, hist, y.tiles);
            } else {
                hipLaunchKernelGGL(rs_hist_kernel<false>, grid, dim3(kRsThreads), 0,
                                   s, idx, Bcap, L, n_valid, keys[in], y.NP, shift,
                                   nb, hist, y.tiles);
            }
            }
            {
            ProfScope prof("rs_scan_kernel", s);
            hipLaunchKernelGGL(rs_scan_kernel, dim3(T), dim3(1024), 0, s, hist,
                               y.tiles, nb);
            }
            ProfScope prof("rs_scatter_kernel", s);
            if (pass == 0) {
                hipLaunchKernelGGL(rs_scatter_kernel<true>, grid, dim3(kRsThreads),
                                   0, s, idx, Bcap, L, n_valid, nullptr, nullptr,
                                   keys[out], vals[out], y.NP, shift, nb, hist,
                                   y.tiles);
            } else {
                hipLaunchKernelGGL(rs_scatter_kernel<false>, grid, dim3(kRsThreads),
                                   0, s, idx, Bcap, L, n_valid, keys[in], vals[in],
                                   keys[out], vals[out], y.NP, shift, nb, hist,
                                   y.tiles);
            }
            cur = out;
            shift += nb;
        }
    }

    const int g = lanes_per_row(tb->dim);
    const int ng = kWG / g;
    const int strip = pick_strip((int64_t)T * y.NP, ng);
    const int wgs = y.NP / (ng * strip);
    uint32_t *trail_row = reinterpret_cast<uint32_t *>(w8 + y.trail_row);
    uint8_t *lead_state = reinterpret_cast<uint8_t *>(w8 + y.lead_state);
    float4 *part_lead = reinterpret_cast<float4 *>(w8 + y.part_lead);
    float4 *part_trail = reinterpret_cast<float4 *>(w8 + y.part_trail);
    const int64_t blocks = (int64_t)wgs * T;
    if (blocks > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_embbag_backward_update: grid too large");
#define SS_APPLY(S_)                                                             \
    SS_DISPATCH_G(g, hipLaunchKernelGGL(                                         \
                         (apply_kernel<G, S_>), dim3((unsigned)blocks), dim3(kWG), \
                         0, s, tb->weights, tb->stale_bits, keys[cur], vals[cur],  \
                         y.NP, grad, Bcap, D4, lr, wgs, trail_row, lead_state,     \
                         part_lead, part_trail))
    {
    ProfScope prof("apply_kernel", s);
    if (strip == 16) { SS_APPLY(16); }
    else if (strip == 8) { SS_APPLY(8); }
    else { SS_APPLY(4); }
    }
#undef SS_APPLY
    ProfScope prof("fixup_kernel", s);
    SS_DISPATCH_G(g, hipLaunchKernelGGL(fixup_kernel<G>, dim3((unsigned)blocks),
                                        dim3(kWG), 0, s, tb->weights,
                                        tb->stale_bits, D4, lr, wgs, trail_row,
                                        lead_state, part_lead, part_trail));
    return check_launch("ss_embbag_backward_update");
}

}  // namespace ss
