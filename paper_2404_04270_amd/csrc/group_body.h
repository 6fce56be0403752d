// Grouping of one table's lookups by row, for tables of up to 16384 lookups
// (stage 1 of the backward pass), as a device function so that it can run as a
// kernel of its own or as one role of the fused forward + grouping launch; and the
// pieces it shares with the grouping of larger tables: ranking inside a wavefront,
// the sentinel for stale rows, the LDS radix sort of one workgroup.
#pragma once
#include "ss_common.h"

namespace ss {

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

// Stable rank of this lane's key among the keys its wavefront has seen so far
// with the same digit: the lowest lane of each digit group bumps the
// wavefront's LDS counter once for the whole group and hands the old value to
// the others.  cnt points at the wavefront's counters (one per digit).
__device__ __forceinline__ uint32_t wave_rank(uint32_t *cnt, uint32_t d, int nbits,
                                              int lane)
{
    const uint64_t m = match_digit(d, nbits);
    const uint32_t before = __popcll(m & lanes_below(lane));
    uint32_t base = 0;
    if (before == 0) base = atomicAdd(&cnt[d], (uint32_t)__popcll(m));
    base = __shfl(base, __ffsll((long long)m) - 1);
    return base + before;
}

// Gives the sentinel key to lookups of stale rows.  All bitmap words are
// requested before the first one is used.
template <int N>
__device__ __forceinline__ void drop_stale(gptr<const uint32_t> bt, uint32_t (&key)[N])
{
    if (!bt) return;
    uint32_t word[N];
#pragma unroll
    for (int r = 0; r < N; ++r) word[r] = bt[key[r] == kNoRow ? 0u : key[r] >> 5];
#pragma unroll
    for (int r = 0; r < N; ++r)
        if (key[r] != kNoRow && ((word[r] >> (key[r] & 31)) & 1u)) key[r] = kNoRow;
}

// Bits of the pass-th of npass digits when key_bits are split as evenly as
// possible (earlier passes take the extra bits).
__host__ __device__ inline int pass_bits(int key_bits, int npass, int pass)
{
    return key_bits / npass + (pass < key_bits % npass ? 1 : 0);
}

// LSD radix sort, by a workgroup of NT threads, of m <= NT * ITEMS keys that lie in LDS,
// on `bits` key bits from bit `shift` up; stable.  PACKED: s_keys alone is permuted,
// else s_vals with it.  s_cnt: 2 * (NT / 64) * 64 words, s_dig: 64 words.  All threads
// call; on return the sorted keys are visible to all of them.
// Digits of at most 6 bits: one wavefront can then turn the per-wavefront counters into
// offsets with shuffles alone, which leaves three barriers per pass.
template <int NT, int ITEMS, bool PACKED>
__device__ __forceinline__ void lds_lsd_sort(uint32_t *s_keys, uint32_t *s_vals,
                                             uint32_t *s_cnt, uint32_t *s_dig, uint32_t m,
                                             int bits, int shift)
{
    constexpr int NW = NT / 64;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    uint32_t key[ITEMS], val[PACKED ? 1 : ITEMS], rank[ITEMS];
    const int rounds = ((int)m + NT - 1) / NT;       // keys per thread, <= ITEMS
    const int npass = (bits + 5) / 6;
    for (int i = tid; i < 2 * NW * 64; i += NT) s_cnt[i] = 0;
    __syncthreads();
    for (int pass = 0; pass < npass; ++pass) {
        uint32_t *cnt = s_cnt + (pass & 1) * (NW * 64);       // this pass
        uint32_t *cnt_next = s_cnt + ((pass + 1) & 1) * (NW * 64);
#pragma unroll
        for (int r = 0; r < ITEMS; ++r)
            if (r < rounds) {
                const uint32_t pos = wave * rounds * 64 + r * 64 + lane;
                key[r] = pos < m ? s_keys[pos] : kNoRow;
                if (!PACKED) val[r] = pos < m ? s_vals[pos] : 0u;
            }
        const int nb = pass_bits(bits, npass, pass);
        const uint32_t dmask = (1u << nb) - 1u;
#pragma unroll
        for (int r = 0; r < ITEMS; ++r)
            if (r < rounds) {
                const uint32_t d = (key[r] >> shift) & dmask;
                rank[r] = wave_rank(cnt + wave * 64, d, nb, lane);
            }
        __syncthreads();
        if (wave == 0) {
            // lane d: offsets of the wavefronts for digit d, then digit starts
            uint32_t run = 0;
            if (lane <= (int)dmask)
                for (int w = 0; w < NW; ++w) {
                    const uint32_t c = cnt[w * 64 + lane];
                    cnt[w * 64 + lane] = run;
                    run += c;
                }
            uint32_t incl = run;
            for (int off = 1; off < 64; off <<= 1) {
                const uint32_t up = __shfl_up(incl, off);
                if (lane >= off) incl += up;
            }
            s_dig[lane] = incl - run;
        }
        if (NW == 1 || wave != 0)
            for (int i = NW == 1 ? tid : tid - 64; i < NW * 64; i += NW == 1 ? NT : NT - 64)
                cnt_next[i] = 0;
        __syncthreads();
#pragma unroll
        for (int r = 0; r < ITEMS; ++r)
            if (r < rounds) {
                const uint32_t d = (key[r] >> shift) & dmask;
                const uint32_t p = s_dig[d] + cnt[wave * 64 + d] + rank[r];
                if (p < m) {            // padding keys rank behind every real key
                    s_keys[p] = key[r];
                    if (!PACKED) s_vals[p] = val[r];
                }
            }
        __syncthreads();
        shift += nb;
    }
}

// ---------------------------------------------------------------------------
// The apply stage needs equal rows to be neighbours, not ascending rows, so a
// table is cut into P classes by the low bits of the row id and each class is
// sorted by the remaining bits by its own 1024-thread workgroup: P times the
// parallelism of a whole-table sort and fewer digit passes.  Every workgroup
// reads all lookups of its table (cheap at this size), keeps its class in the
// original order, and learns from the same read where its class starts in the
// output (the number of lookups in lower classes).  Output order: class,
// remaining bits, original position; sentinels last.
//
// PACKED: the remaining row bits and the sample number fit one 31-bit word
// (rem_bits + val_bits <= 31), which is then all that is sorted: half the LDS
// and half the registers.
// ---------------------------------------------------------------------------
template <int ITEMS, bool PACKED>
__device__ __forceinline__ void class_sort_body(
    int cls, int t, const int32_t *__restrict__ idx, int Bcap, int L,
    const int32_t *__restrict__ n_valid, const uint32_t *const *__restrict__ bits,
    int key_bits, int class_bits, int val_bits, uint2 *__restrict__ out_ent, int NP)
{
    constexpr int NW = 16, CAP = 1024 * ITEMS;
    __shared__ uint32_t s_keys[CAP];
    __shared__ uint32_t s_vals[PACKED ? 1 : CAP];
    __shared__ uint32_t s_cnt[2 * NW * 64];   // two sets: one is cleared while the
    __shared__ uint32_t s_dig[64];            // other is in use
    __shared__ uint32_t s_mine[NW], s_below[NW], s_real[NW];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n = clamp_valid(n_valid, Bcap) * L;
    const int32_t *__restrict__ ip = idx + (int64_t)t * Bcap * L;
    const auto bt = as_global(bits ? bits[t] : nullptr);
    const uint32_t cmask = (1u << class_bits) - 1u;

    uint32_t key[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const int pos = wave * ITEMS * 64 + r * 64 + lane;
        // requested before n is known (it comes from device memory); used only below n
        const uint32_t word = (uint32_t)ip[pos < Bcap * L ? pos : 0];
        key[r] = pos < n ? word : kNoRow;
    }
    drop_stale(bt, key);

    // keep my class, in order; count the lookups of lower classes
    uint32_t c_mine = 0, c_below = 0, c_real = 0, slot[ITEMS];
#pragma unroll
    for (int r = 0; r < ITEMS; ++r) {
        const bool real = key[r] != kNoRow;
        const uint32_t kc = key[r] & cmask;
        const uint64_t bm = __ballot(real && kc == (uint32_t)cls);
        slot[r] = c_mine + __popcll(bm & lanes_below(lane));
        c_mine += __popcll(bm);
        c_below += __popcll(__ballot(real && kc < (uint32_t)cls));
        c_real += __popcll(__ballot(real));
    }
    if (lane == 0) {
        s_mine[wave] = c_mine;
        s_below[wave] = c_below;
        s_real[wave] = c_real;
    }
    __syncthreads();
    uint32_t woff = 0, m = 0, n_below = 0, n_real = 0;
    for (int w = 0; w < NW; ++w) {
        if (w < wave) woff += s_mine[w];
        m += s_mine[w];
        n_below += s_below[w];
        n_real += s_real[w];
    }
#pragma unroll
    for (int r = 0; r < ITEMS; ++r)
        if (key[r] != kNoRow && (key[r] & cmask) == (uint32_t)cls) {
            const int pos = wave * ITEMS * 64 + r * 64 + lane;
            const uint32_t smp = (uint32_t)(L == 1 ? pos : pos / L);
            if (PACKED) {
                s_keys[woff + slot[r]] = ((key[r] >> class_bits) << val_bits) | smp;
            } else {
                s_keys[woff + slot[r]] = key[r];
                s_vals[woff + slot[r]] = smp;
            }
        }
    __syncthreads();

    lds_lsd_sort<1024, ITEMS, PACKED>(s_keys, s_vals, s_cnt, s_dig, m, key_bits - class_bits,
                                      PACKED ? val_bits : class_bits);
    uint2 *__restrict__ oe = out_ent + (int64_t)t * NP;
    const uint32_t vmask = PACKED ? (1u << val_bits) - 1u : 0u;
    for (uint32_t i = tid; i < m; i += 1024) {
        const uint32_t w = s_keys[i];
        if (PACKED)
            oe[n_below + i] = make_uint2(((w >> val_bits) << class_bits) | (uint32_t)cls,
                                         w & vmask);
        else
            oe[n_below + i] = make_uint2(w, s_vals[i]);
    }
    if (cls == 0)
        for (uint32_t i = n_real + tid; i < (uint32_t)NP; i += 1024)
            oe[i] = make_uint2(kNoRow, 0u);
}

// Host side: how the class sort is configured for a table geometry.
struct ClassSortPlan {
    int items;        // template ITEMS: 2, 4, 8 or 16
    int class_bits;   // log2 of the number of classes
    int val_bits;     // bits of a sample number
    bool packed;      // row bits above the class bits + sample number fit 31 bits
};

inline ClassSortPlan plan_class_sort(int NP, int Bcap, int key_bits)
{
    ClassSortPlan p;
    const int it = NP / 1024;
    p.items = it <= 2 ? 2 : it <= 4 ? 4 : it <= 8 ? 8 : 16;
    p.class_bits = 0;              // about 1024 lookups per class
    while ((1024 << p.class_bits) < NP && p.class_bits < key_bits) ++p.class_bits;
    p.val_bits = 1;
    while ((1 << p.val_bits) < Bcap) ++p.val_bits;
    p.packed = (key_bits - p.class_bits) + p.val_bits <= 31;
    return p;
}

}  // namespace ss
