// Hot-set identification (section 3.1 of the paper and the preprocessing loop of
// Algorithm 1): per-row access counters over the sampled inputs, then the set of
// hot rows of every table, either by the paper's share rule (C_r / total >=
// lambda) or as the H most accessed rows (ties to the lower row id), written as
// an ascending id list and as a bitmap.
//
// Counting.  Accesses are Zipf-like, so a few rows of a table take most of its
// lookups; sent to memory as they come, those would be thousands of atomics on
// one address.  Each workgroup therefore counts its chunk of lookups in a small
// LDS table first (open slot per row, claimed with a compare-and-swap on the
// tag; a lookup that finds its slot taken by another row goes to memory
// directly) and adds the table to the global counters at the end.  Integer
// adds commute, so the counters do not depend on the order of anything.
//
// Selecting.  Both rules reduce to "count > c, or count == c and fewer than e
// such rows came before": for the share rule c = (smallest passing count) - 1
// and e = 0, computed on the host; for top-H, c is the H-th largest count, found
// by a four-pass radix select over the 8-bit digits of the counters (histogram
// per pass in LDS, one pick step per pass), and e is what is left of H after the
// rows above c.  A three-step ordered compaction (block totals, scan, write)
// then emits the ids in ascending order; 64 consecutive rows per wavefront step
// make the bitmap words fall out of the same ballots.
#include "ss_common.h"

namespace ss {
namespace {

constexpr int kCountSlots = 1024;        // LDS counters per workgroup
constexpr int kCountChunk = 2048;        // lookups per workgroup
constexpr int kSelSteps = 16;            // 64-row steps per wavefront
constexpr int kSelRows = kSelSteps * kWG;   // rows per workgroup: 4096

__global__ __launch_bounds__(kWG) void count_kernel(
    const int32_t *__restrict__ idx, int Bcap, int L, const int32_t *__restrict__ n_valid,
    uint32_t *const *__restrict__ counts, int chunks_per_table)
{
    __shared__ uint32_t s_tag[kCountSlots];
    __shared__ uint32_t s_cnt[kCountSlots];
    const int t = blockIdx.x / chunks_per_table;
    const int chunk = blockIdx.x - t * chunks_per_table;
    const int64_t n = (int64_t)clamp_valid(n_valid, Bcap) * L;     // lookups of this table
    const int64_t first = (int64_t)chunk * kCountChunk;
    if (first >= n) return;
    for (int i = threadIdx.x; i < kCountSlots; i += kWG) {
        s_tag[i] = kNoRow;
        s_cnt[i] = 0;
    }
    __syncthreads();
    const int32_t *__restrict__ ip = idx + (int64_t)t * Bcap * L;
    uint32_t *cg = counts[t];
    const int64_t last = first + kCountChunk < n ? first + kCountChunk : n;
    for (int64_t q = first + threadIdx.x; q < last; q += kWG) {
        const uint32_t r = (uint32_t)ip[q];
        const uint32_t slot = (r * 2654435761u) >> 22;            // 10 bits
        const uint32_t seen = atomicCAS(&s_tag[slot], kNoRow, r);
        if (seen == kNoRow || seen == r)
            atomicAdd(&s_cnt[slot], 1u);
        else
            atomicAdd(&cg[r], 1u);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < kCountSlots; i += kWG) {
        const uint32_t r = s_tag[i];
        if (r != kNoRow) atomicAdd(&cg[r], s_cnt[i]);
    }
}

// ---- selection ---------------------------------------------------------
// state[t] = { c, e }: rows with count > c are taken, and the first e rows (by
// row id) with count == c.
struct SelState {
    uint32_t c, e;
};

__global__ void sel_set_state_kernel(SelState *state, int T, uint32_t c, uint32_t e)
{
    const int t = blockIdx.x * blockDim.x + threadIdx.x;
    if (t < T) state[t] = SelState{c, e};
}

// Radix select, pass p (0 = top digit).  While the passes run, state[t].c holds
// the digits decided so far (lower digits zero) and state[t].e what is still to
// be found among the rows that match them.
__global__ __launch_bounds__(kWG) void sel_hist_kernel(
    uint32_t *const *__restrict__ counts, int64_t R, const SelState *__restrict__ state,
    int pass, uint32_t *__restrict__ hist)
{
    __shared__ uint32_t s_hist[256];
    const int t = blockIdx.y;
    s_hist[threadIdx.x] = 0;
    __syncthreads();
    const int shift = 24 - 8 * pass;
    const uint32_t prefix = state[t].c;
    const auto cg = as_global((const uint32_t *)counts[t]);
    const int64_t base = (int64_t)blockIdx.x * kSelRows;
    const int lane = threadIdx.x & 63;
#pragma unroll 4
    for (int k = 0; k < kSelSteps; ++k) {
        const int64_t r = base + k * kWG + threadIdx.x;
        uint32_t c = 0;
        if (r < R) c = cg[r];
        // rows whose higher digits differ from the prefix are out of the race
        const bool in = r < R && (pass == 0 || (c >> (shift + 8)) == (prefix >> (shift + 8)));
        const uint32_t d = (c >> shift) & 255u;
        // Counters are mostly small, so most lanes of a wavefront share a digit:
        // the first lane in the race adds for all that agree with it.
        const unsigned long long racing = __ballot(in);
        if (racing) {
            const int lead = __ffsll((long long)racing) - 1;
            const uint32_t d_lead = __shfl(d, lead);
            const unsigned long long same = __ballot(in && d == d_lead);
            if (lane == lead) atomicAdd(&s_hist[d_lead], (uint32_t)__popcll(same));
            if (in && d != d_lead) atomicAdd(&s_hist[d], 1u);
        }
    }
    __syncthreads();
    const uint32_t v = s_hist[threadIdx.x];
    if (v) atomicAdd(&hist[((int64_t)t * 4 + pass) * 256 + threadIdx.x], v);
}

// Largest digit d with  #(rows above d) < e <= #(rows at or above d): every
// thread owns a digit, the counts above it come from a suffix scan in LDS, and
// the one thread whose digit satisfies the condition writes the state.
__global__ __launch_bounds__(256) void sel_pick_kernel(SelState *__restrict__ state,
                                                        int pass,
                                                        const uint32_t *__restrict__ hist)
{
    __shared__ uint32_t s_suf[256];
    const int t = blockIdx.x, d = threadIdx.x;
    const uint32_t h = hist[((int64_t)t * 4 + pass) * 256 + d];
    const SelState st = state[t];
    s_suf[d] = h;
    __syncthreads();
    // inclusive suffix sums: s_suf[d] = sum of h over digits >= d
    for (int off = 1; off < 256; off <<= 1) {
        const uint32_t add = d + off < 256 ? s_suf[d + off] : 0u;
        __syncthreads();
        s_suf[d] += add;
        __syncthreads();
    }
    const uint32_t at_or_above = s_suf[d], above = at_or_above - h;
    // e >= 1 and the rows still in the race number at least e, so exactly one digit
    // qualifies (and it is present: h > 0)
    if (above < st.e && st.e <= at_or_above)
        state[t] = SelState{st.c | ((uint32_t)d << (24 - 8 * pass)), st.e - above};
}

// Wavefront w of the workgroup takes rows base + (k * 4 + w) * 64 + lane in step
// k; `gt` and `eq` are the ballots of that step.
__device__ __forceinline__ void sel_ballots(gptr<const uint32_t> cg, int64_t R, int64_t row,
                                            SelState st, unsigned long long &gt,
                                            unsigned long long &eq)
{
    uint32_t c = 0;
    const bool in = row < R;
    if (in) c = cg[row];
    gt = __ballot(in && c > st.c);
    eq = __ballot(in && c == st.c);
}

__global__ __launch_bounds__(kWG) void sel_count_kernel(
    uint32_t *const *__restrict__ counts, int64_t R, const SelState *__restrict__ state,
    uint2 *__restrict__ block_counts, int nb)
{
    __shared__ uint32_t s_gt, s_eq;
    const int t = blockIdx.y;
    if (threadIdx.x == 0) s_gt = s_eq = 0;
    __syncthreads();
    const SelState st = state[t];
    const auto cg = as_global((const uint32_t *)counts[t]);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t base = (int64_t)blockIdx.x * kSelRows;
    uint32_t n_gt = 0, n_eq = 0;
#pragma unroll 4
    for (int k = 0; k < kSelSteps; ++k) {
        unsigned long long gt, eq;
        sel_ballots(cg, R, base + (k * 4 + wave) * 64 + lane, st, gt, eq);
        n_gt += (uint32_t)__popcll(gt);
        n_eq += (uint32_t)__popcll(eq);
    }
    if (lane == 0) {
        atomicAdd(&s_gt, n_gt);
        atomicAdd(&s_eq, n_eq);
    }
    __syncthreads();
    if (threadIdx.x == 0) block_counts[(int64_t)t * nb + blockIdx.x] = make_uint2(s_gt, s_eq);
}

// Exclusive scan of the block totals of one table; n_hot = what the write step
// will emit (before any cap).  Each thread owns a contiguous piece of the
// blocks; the 256 piece totals are scanned with wavefront shuffles.
__global__ __launch_bounds__(kWG) void sel_scan_kernel(
    const uint2 *__restrict__ block_counts, uint2 *__restrict__ block_before, int nb,
    const SelState *__restrict__ state, uint32_t *__restrict__ n_hot)
{
    __shared__ uint32_t s_wgt[4], s_weq[4];
    const int t = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int per = (nb + kWG - 1) / kWG;
    const int b0 = tid * per, b1 = b0 + per < nb ? b0 + per : nb;
    const uint2 *__restrict__ bc = block_counts + (int64_t)t * nb;
    uint2 *__restrict__ bb = block_before + (int64_t)t * nb;
    uint32_t gt = 0, eq = 0;
    for (int b = b0; b < b1; ++b) {
        gt += bc[b].x;
        eq += bc[b].y;
    }
    uint32_t inc_gt = gt, inc_eq = eq;                  // inclusive within the wavefront
    for (int off = 1; off < 64; off <<= 1) {
        const uint32_t a = __shfl_up(inc_gt, off), c = __shfl_up(inc_eq, off);
        if (lane >= off) {
            inc_gt += a;
            inc_eq += c;
        }
    }
    if (lane == 63) {
        s_wgt[wave] = inc_gt;
        s_weq[wave] = inc_eq;
    }
    __syncthreads();
    uint32_t run_gt = inc_gt - gt, run_eq = inc_eq - eq, tot_gt = 0, tot_eq = 0;
    for (int w = 0; w < 4; ++w) {
        if (w < wave) {
            run_gt += s_wgt[w];
            run_eq += s_weq[w];
        }
        tot_gt += s_wgt[w];
        tot_eq += s_weq[w];
    }
    for (int b = b0; b < b1; ++b) {
        const uint2 v = bc[b];
        bb[b] = make_uint2(run_gt, run_eq);
        run_gt += v.x;
        run_eq += v.y;
    }
    if (tid == 0 && n_hot) {
        const uint32_t e = state[t].e;
        n_hot[t] = tot_gt + (tot_eq < e ? tot_eq : e);
    }
}

__global__ __launch_bounds__(kWG) void sel_write_kernel(
    uint32_t *const *__restrict__ counts, int64_t R, const SelState *__restrict__ state,
    const uint2 *__restrict__ block_before, int nb, int32_t *const *__restrict__ hot_ids,
    int cap, uint32_t *const *__restrict__ hot_bits)
{
    // totals of every (step, wavefront) cell, then their exclusive prefix in row order
    __shared__ uint32_t s_gt[kSelSteps * 4], s_eq[kSelSteps * 4];
    const int t = blockIdx.y;
    const SelState st = state[t];
    const auto cg = as_global((const uint32_t *)counts[t]);
    const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
    const int64_t base = (int64_t)blockIdx.x * kSelRows;
    unsigned long long gts[kSelSteps], eqs[kSelSteps];
#pragma unroll
    for (int k = 0; k < kSelSteps; ++k) {
        sel_ballots(cg, R, base + (k * 4 + wave) * 64 + lane, st, gts[k], eqs[k]);
        if (lane == 0) {
            s_gt[k * 4 + wave] = (uint32_t)__popcll(gts[k]);
            s_eq[k * 4 + wave] = (uint32_t)__popcll(eqs[k]);
        }
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint2 before = block_before[(int64_t)t * nb + blockIdx.x];
        uint32_t g = before.x, q = before.y;
        for (int i = 0; i < kSelSteps * 4; ++i) {
            const uint32_t a = s_gt[i], b = s_eq[i];
            s_gt[i] = g;
            s_eq[i] = q;
            g += a;
            q += b;
        }
    }
    __syncthreads();
    const unsigned long long below = lane == 0 ? 0ull : (~0ull >> (64 - lane));
    int32_t *ids = hot_ids ? hot_ids[t] : nullptr;
    uint32_t *bits = hot_bits ? hot_bits[t] : nullptr;
    const int64_t words = (R + 31) >> 5;
#pragma unroll
    for (int k = 0; k < kSelSteps; ++k) {
        const int64_t row0 = base + (k * 4 + wave) * 64;
        if (row0 >= R) break;                     // uniform within the wavefront
        const uint32_t g_before = s_gt[k * 4 + wave] + (uint32_t)__popcll(gts[k] & below);
        const uint32_t q_before = s_eq[k * 4 + wave] + (uint32_t)__popcll(eqs[k] & below);
        const bool is_gt = (gts[k] >> lane) & 1ull;
        const bool is_eq = (eqs[k] >> lane) & 1ull;
        const bool take = is_gt || (is_eq && q_before < st.e);
        if (take && ids) {
            const uint64_t pos = (uint64_t)g_before + (q_before < st.e ? q_before : st.e);
            if (pos < (uint64_t)cap) ids[pos] = (int32_t)(row0 + lane);
        }
        if (bits) {
            const unsigned long long sel = __ballot(take);
            const int64_t w0 = row0 >> 5;
            if (lane == 0) bits[w0] = (uint32_t)sel;
            if (lane == 1 && w0 + 1 < words) bits[w0 + 1] = (uint32_t)(sel >> 32);
        }
    }
}

struct SelLayout {
    int nb;
    size_t hist, state, block_counts, block_before, total;
};

SelLayout make_sel_layout(int T, int64_t R)
{
    SelLayout y;
    y.nb = (int)((R + kSelRows - 1) / kSelRows);
    size_t off = 0;
    auto take = [&](size_t bytes) {
        const size_t o = off;
        off += align_up(bytes, 256);
        return o;
    };
    y.hist = take((size_t)T * 4 * 256 * sizeof(uint32_t));
    y.state = take((size_t)T * sizeof(SelState));
    y.block_counts = take((size_t)T * y.nb * sizeof(uint2));
    y.block_before = take((size_t)T * y.nb * sizeof(uint2));
    y.total = off;
    return y;
}

void compact(int T, int64_t R, uint32_t *const *counts, const SelLayout &y, char *w8,
             int32_t *const *hot_ids, int cap, uint32_t *const *hot_bits, uint32_t *n_hot,
             hipStream_t s)
{
    SelState *state = reinterpret_cast<SelState *>(w8 + y.state);
    uint2 *bc = reinterpret_cast<uint2 *>(w8 + y.block_counts);
    uint2 *bb = reinterpret_cast<uint2 *>(w8 + y.block_before);
    launch(sel_count_kernel, dim3(y.nb, T), dim3(kWG), s, counts, R, (const SelState *)state,
           bc, y.nb);
    launch(sel_scan_kernel, dim3(T), dim3(kWG), s, (const uint2 *)bc, bb, y.nb,
           (const SelState *)state, n_hot);
    ProfScope prof("sel_write_kernel", s);
    launch(sel_write_kernel, dim3(y.nb, T), dim3(kWG), s, counts, R, (const SelState *)state,
           (const uint2 *)bb, y.nb, hot_ids, cap, hot_bits);
}

}  // namespace

int32_t launch_count_accesses(int T, const int32_t *idx, int Bcap, int L,
                              const int32_t *n_valid, uint32_t *const *counts,
                              hipStream_t s)
{
    const int64_t nnz = (int64_t)Bcap * L;
    const int64_t chunks = (nnz + kCountChunk - 1) / kCountChunk;
    if (chunks * T > 0x7fffffffLL)
        return fail(SS_ERR_UNSUPPORTED, "ss_count_accesses: grid too large");
    ProfScope prof("count_kernel", s);
    launch(count_kernel, dim3((unsigned)(chunks * T)), dim3(kWG), s, idx, Bcap, L, n_valid,
           counts, (int)chunks);
    return check_launch("ss_count_accesses");
}

size_t select_hot_ws_bytes(int T, int64_t R) { return make_sel_layout(T, R).total; }

int32_t launch_select_hot(int T, int64_t R, uint32_t *const *counts, bool top, uint32_t c,
                          uint32_t e, int32_t *const *hot_ids, int cap,
                          uint32_t *const *hot_bits, uint32_t *n_hot, void *ws, hipStream_t s)
{
    const SelLayout y = make_sel_layout(T, R);
    char *w8 = static_cast<char *>(ws);
    SelState *state = reinterpret_cast<SelState *>(w8 + y.state);
    // top-H starts from "nothing decided, e = H still to find"
    launch(sel_set_state_kernel, dim3((T + 255) / 256), dim3(256), s, state, T, c, e);
    if (top && e > 0) {
        uint32_t *hist = reinterpret_cast<uint32_t *>(w8 + y.hist);
        launch_zero_u32(hist, T * 4 * 256, s);
        for (int pass = 0; pass < 4; ++pass) {
            {
                ProfScope prof("sel_hist_kernel", s);
                launch(sel_hist_kernel, dim3(y.nb, T), dim3(kWG), s, counts, R,
                       (const SelState *)state, pass, hist);
            }
            launch(sel_pick_kernel, dim3(T), dim3(256), s, state, pass,
                   (const uint32_t *)hist);
        }
    }
    compact(T, R, counts, y, w8, hot_ids, cap, hot_bits, n_hot, s);
    return check_launch("ss_select_hot");
}

}  // namespace ss
