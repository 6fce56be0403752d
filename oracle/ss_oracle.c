/*
 * CPU oracle for the embedding-table side of a Slipstream training step.
 *
 * TEST INFRASTRUCTURE ONLY.  This file defines what the GPU library must
 * compute; it is slow on purpose (scalar loops, fp64 accumulation, one table
 * and one lookup at a time) so that it can be checked against the paper by
 * eye.  Only the tests, the smoke check and the benchmark's CPU-baseline leg
 * may call it.  It shares no code, header or table with the HIP library.
 *
 * Every function works on HOST memory.  Tables are fp32, row-major [R][D].
 * A stale bitmap holds one bit per row: row r is bit (r & 31) of 32-bit word
 * (r >> 5).  Lookup indices are int32 [T][B][L].
 *
 * Parity pins (tests that tie each function to something other than itself):
 *   forward          - brute force, gather identity for L = 1, library
 *                      embedding-bag sum, m copies of a row = m * row
 *   backward_update  - dense scatter-add SGD (textbook), closed forms for
 *                      duplicates, frozen stale rows
 *   detect_stale     - closed-form Euclidean norms with exact ties,
 *                      threshold 0 / infinity, monotone bitmap
 *   filter_batch     - brute force, alpha = 0 drops everything (the first
 *                      column of the paper's alpha table), partition identity
 *   general alpha between 1 and T*L-1: the paper's own drop percentages need
 *   its datasets, so for those values parity is pinned by brute force only.
 *   sample_drop      - exact counts from constructed drifts, T = 0 / infinity,
 *                      monotone in T, agreement with detect_stale + filter_batch
 *   drop_stats       - binomial closed forms, vanishing interval for a full
 *                      sample, the paper's critical value 3.340
 *   the search for T over the sampled drop estimates has no stated stopping
 *   rule in the paper: parity unpinned for it (it is host control flow).
 *   count_accesses   - library histogram (bincount), additivity over calls
 *   select_hot_ratio - brute force with exact rationals, the paper's reading of
 *                      lambda = 1e-6 as "one access in a million"
 *   select_hot_top   - brute force (repeated arg-max), library lexicographic
 *                      sort, ties to the lower row id, the harness's own hot set
 *   layernorm        - zero mean / unit variance of the output, the library's
 *                      layer norm and its autograd, central differences
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

static int bit_is_set(const uint32_t *bits, int64_t r)
{
    if (!bits)
        return 0;
    return (int)((bits[r >> 5] >> (r & 31)) & 1u);
}

/*
 * Pooled lookup (section 2.1: every sparse feature yields one vector per
 * table; the multi-hot workload fixes the pooling to a sum):
 *     out[t][j][:] = sum_{l < L} W_t[ idx[t][j][l] ][:]        j < n_valid
 * A row that occurs m times in a bag is added m times.  Sums are taken in
 * fp64 and rounded once.  Returns 0, or -1 on an out-of-range index.
 */
int oracle_embbag_forward(int T, int64_t R, int D, float *const *W,
                          const int32_t *idx, int Bcap, int L, int n_valid,
                          float *out)
{
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < n_valid; ++j) {
            for (int d = 0; d < D; ++d) {
                double s = 0.0;
                for (int l = 0; l < L; ++l) {
                    int64_t r = idx[((int64_t)t * Bcap + j) * L + l];
                    if (r < 0 || r >= R)
                        return -1;
                    s += (double)W[t][r * D + d];
                }
                out[((int64_t)t * Bcap + j) * D + d] = (float)s;
            }
        }
    }
    return 0;
}

/*
 * Sparse SGD that leaves stale rows alone (abstract and section 3.6: stale
 * embeddings are found on the fly and their updates are skipped).
 *
 * With sum pooling the gradient of bag (t, j) flows unchanged to each of its
 * L lookups, so for every row r of table t that was looked up at least once
 *     acc[r][:] = sum over lookups (j, l) with idx[t][j][l] == r of g[t][j][:]
 * and, when r's stale bit is clear,
 *     W_t[r][:] <- W_t[r][:] - lr * acc[r][:]
 * (fp64 throughout, one rounding to fp32).  Rows whose bit is set are neither
 * read nor written.  Bitmaps are not modified.
 */
int oracle_embbag_backward_update(int T, int64_t R, int D, float *const *W,
                                  uint32_t *const *stale_bits,
                                  const int32_t *idx, int Bcap, int L,
                                  int n_valid, const float *grad, float lr)
{
    int64_t nnz = (int64_t)n_valid * L;
    if (nnz == 0)
        return 0;
    /* slot[r] = position of row r's accumulator, or -1 */
    int32_t *slot = (int32_t *)malloc((size_t)R * sizeof(int32_t));
    int64_t *rows = (int64_t *)malloc((size_t)nnz * sizeof(int64_t));
    double *acc = (double *)malloc((size_t)nnz * D * sizeof(double));
    if (!slot || !rows || !acc) {
        free(slot); free(rows); free(acc);
        return -2;
    }
    memset(slot, 0xff, (size_t)R * sizeof(int32_t));
    int rc = 0;
    for (int t = 0; t < T && rc == 0; ++t) {
        const uint32_t *bits = stale_bits ? stale_bits[t] : NULL;
        int64_t n_touched = 0;
        for (int j = 0; j < n_valid && rc == 0; ++j) {
            const float *g = grad + ((int64_t)t * Bcap + j) * D;
            for (int l = 0; l < L; ++l) {
                int64_t r = idx[((int64_t)t * Bcap + j) * L + l];
                if (r < 0 || r >= R) { rc = -1; break; }
                if (slot[r] < 0) {
                    slot[r] = (int32_t)n_touched;
                    rows[n_touched] = r;
                    for (int d = 0; d < D; ++d)
                        acc[n_touched * D + d] = 0.0;
                    ++n_touched;
                }
                double *a = acc + (int64_t)slot[r] * D;
                for (int d = 0; d < D; ++d)
                    a[d] += (double)g[d];
            }
        }
        for (int64_t k = 0; k < n_touched; ++k) {
            int64_t r = rows[k];
            slot[r] = -1;
            if (rc != 0 || bit_is_set(bits, r))
                continue;
            float *w = W[t] + r * D;
            for (int d = 0; d < D; ++d)
                w[d] = (float)((double)w[d] - (double)lr * acc[k * D + d]);
        }
    }
    free(slot); free(rows); free(acc);
    return rc;
}

/*
 * Drift test of hot rows against their last snapshot (Eq. 1 and Eq. 5: a hot
 * row is "varying" when the Euclidean distance between two consecutive
 * snapshots of it exceeds T, and stale otherwise).
 *
 * For hot slot h of table t, r = hot_ids[t][h]:
 *     drift = || W_t[r][:] - S_t[h][:] ||_2                       (fp64)
 *     stale = (T > 0) and (drift <= T)
 * Readings where the paper is silent: equality counts as stale ("> T" is
 * varying); T = 0 switches detection off so that a zero threshold means plain
 * training; a stale bit, once set, is never cleared (section 1: a stale row stays
 * skipped until training ends), so the bitmap is OR-ed; a NaN
 * drift compares false and leaves the row varying.
 * If refresh != 0 the snapshot row is then overwritten with the current row.
 * stale_hot[t][h] (0/1), drift[t][h] and stale_count[t] (rows flagged by this
 * call, whether or not their bit was already set) are optional outputs.
 */
int oracle_detect_stale(int T, int64_t R, int D, float *const *W,
                        uint32_t *const *stale_bits, int32_t *const *hot_ids,
                        int H, float *const *snapshot, float threshold,
                        int refresh, uint8_t *const *stale_hot,
                        double *const *drift, uint32_t *stale_count)
{
    double thr = (double)threshold;
    for (int t = 0; t < T; ++t) {
        uint32_t count = 0;
        for (int h = 0; h < H; ++h) {
            int64_t r = hot_ids[t][h];
            if (r < 0 || r >= R)
                return -1;
            const float *w = W[t] + r * D;
            float *s = snapshot[t] + (int64_t)h * D;
            double d2 = 0.0;
            for (int d = 0; d < D; ++d) {
                double e = (double)w[d] - (double)s[d];
                d2 += e * e;
            }
            double dist = sqrt(d2);
            int stale = (thr > 0.0) && (dist <= thr);
            if (stale) {
                stale_bits[t][r >> 5] |= (1u << (r & 31));
                ++count;
            }
            if (stale_hot && stale_hot[t])
                stale_hot[t][h] = (uint8_t)stale;
            if (drift && drift[t])
                drift[t][h] = dist;
            if (refresh)
                memcpy(s, w, (size_t)D * sizeof(float));
        }
        if (stale_count)
            stale_count[t] = count;
    }
    return 0;
}

/*
 * Input classifier (section 3.4, Eq. 6-8): an input is dropped when the
 * number of stale embeddings it accesses reaches alpha; the rest are kept, in
 * their original order.
 *     c_b    = #{ (t, l) : stale_t[ idx[t][b][l] ] }
 *     skip_b = (c_b >= alpha)
 * alpha = T*L drops the inputs whose every lookup is stale; alpha <= 0 drops
 * every input (the alpha = 0 column of the paper's alpha table reads 100 %).
 * Outputs: skip_mask[B]; kept_ids[0..n_kept) ascending; *n_kept;
 * idx_c[t][j][:] = idx[t][kept_ids[j]][:] with the same [T][B][L] strides
 * (entries j >= n_kept are left as they were).
 */
int oracle_filter_batch(int T, int64_t R, uint32_t *const *stale_bits,
                        const int32_t *idx, int B, int L, int alpha,
                        uint8_t *skip_mask, int32_t *kept_ids, int32_t *n_kept,
                        int32_t *idx_c)
{
    int32_t nk = 0;
    for (int b = 0; b < B; ++b) {
        int c = 0;
        for (int t = 0; t < T; ++t) {
            const uint32_t *bits = stale_bits ? stale_bits[t] : NULL;
            for (int l = 0; l < L; ++l) {
                int64_t r = idx[((int64_t)t * B + b) * L + l];
                if (r < 0 || r >= R)
                    return -1;
                c += bit_is_set(bits, r);
            }
        }
        int skip = (c >= alpha);
        skip_mask[b] = (uint8_t)skip;
        if (!skip)
            kept_ids[nk++] = b;
    }
    for (int t = 0; t < T; ++t)
        for (int32_t j = 0; j < nk; ++j)
            for (int l = 0; l < L; ++l)
                idx_c[((int64_t)t * B + j) * L + l] =
                    idx[((int64_t)t * B + kept_ids[j]) * L + l];
    *n_kept = nk;
    return 0;
}

/*
 * Sampling block (section 3.3): how many of a sample of inputs could be dropped
 * at each of several candidate thresholds.
 *
 * For sampled input s (its lookups sidx[t][s][l]) and threshold T_k, a lookup
 * counts as stale when its row is a hot row (it has a snapshot) and the Euclidean
 * distance between the row and its snapshot does not exceed T_k (Eq. 1, with the
 * same readings as oracle_detect_stale: equality is stale, T_k = 0 flags nothing,
 * rows outside the hot set are never stale).  The input is droppable when at
 * least alpha of its T*L lookups are stale (section 3.4), and
 *     counts[k] = number of droppable inputs among the n_samples sampled ones,
 * which is |S| * D of Eq. 2.  Eq. 2 as printed sums the indicator of "varying"
 * while calling the result the dropped share; the dropped share is what is
 * wanted, so the indicator of "stale" is summed.  Nothing is modified.
 * Whether a row is hot, and which snapshot slot it has, is read from a plain
 * table with one entry per row, filled from hot_ids before the loops.
 */
int oracle_sample_drop(int T, int64_t R, int D, float *const *W,
                       int32_t *const *hot_ids, int H, float *const *snapshot,
                       const int32_t *sidx, int n_samples, int L, int alpha,
                       const float *thresholds, int n_thr, uint32_t *counts)
{
    for (int k = 0; k < n_thr; ++k)
        counts[k] = 0;
    /* slot_of[t][r] = hot slot of row r of table t, or -1 */
    int32_t *slot_of = (int32_t *)malloc((size_t)T * (size_t)R * sizeof(int32_t));
    if (!slot_of)
        return -2;
    for (int64_t i = 0; i < (int64_t)T * R; ++i)
        slot_of[i] = -1;
    for (int t = 0; t < T; ++t)
        for (int h = 0; h < H; ++h) {
            int64_t r = hot_ids[t][h];
            if (r < 0 || r >= R) {
                free(slot_of);
                return -1;
            }
            slot_of[(int64_t)t * R + r] = h;
        }
    for (int s = 0; s < n_samples; ++s) {
        for (int k = 0; k < n_thr; ++k) {
            double thr = (double)thresholds[k];
            int stale_lookups = 0;
            for (int t = 0; t < T; ++t) {
                for (int l = 0; l < L; ++l) {
                    int64_t r = sidx[((int64_t)t * n_samples + s) * L + l];
                    if (r < 0 || r >= R) {
                        free(slot_of);
                        return -1;
                    }
                    int h = slot_of[(int64_t)t * R + r];
                    if (h < 0)
                        continue;                /* not a hot row: never stale */
                    const float *w = W[t] + r * D;
                    const float *sn = snapshot[t] + (int64_t)h * D;
                    double d2 = 0.0;
                    for (int d = 0; d < D; ++d) {
                        double e = (double)w[d] - (double)sn[d];
                        d2 += e * e;
                    }
                    if (thr > 0.0 && sqrt(d2) <= thr)
                        ++stale_lookups;
                }
            }
            if (stale_lookups >= alpha)
                ++counts[k];
        }
    }
    free(slot_of);
    return 0;
}

/*
 * Estimate of the dropped share with its confidence interval (Eq. 2-4).
 *     D    = count / |S|                                   (Eq. 2)
 *     sd   = sqrt( (1/|S|) * sum_s (delta_s - D)^2 )        (Eq. 3)
 *          = sqrt( D (1 - D) )   because delta_s is 0 or 1
 *     half = t * sqrt( ((I - |S|) / I) * (sd^2 / |S|) )     (Eq. 4; the paper writes
 *            both |S| and m for the sample size: they are the same number)
 * on the scale of the share D.  The paper states the interval around
 * D_bar = D * I_hot, the expected number of dropped hot inputs; that interval is
 * out[0..1] scaled by I_hot and is returned too.  t is the critical value the
 * caller supplies (the paper uses 3.340 for 99.9 %).  I is the population the
 * sample was drawn from.
 * out = { D, sd, half, D - half, D + half, D_bar, D_bar - half*I_hot, D_bar + half*I_hot }
 */
int oracle_drop_stats(uint32_t count, int64_t n_samples, int64_t population,
                      int64_t n_hot_inputs, double t_crit, double *out)
{
    if (n_samples <= 0 || population < n_samples || count > (uint64_t)n_samples)
        return -3;
    double n = (double)n_samples;
    double Dk = (double)count / n;
    /* Eq. 3 written out over the two kinds of samples */
    double ss = (double)count * (1.0 - Dk) * (1.0 - Dk) +
                ((double)n_samples - (double)count) * (0.0 - Dk) * (0.0 - Dk);
    double sd = sqrt(ss / n);
    double fpc = ((double)population - n) / (double)population;
    double half = t_crit * sqrt(fpc * (sd * sd / n));
    out[0] = Dk;
    out[1] = sd;
    out[2] = half;
    out[3] = Dk - half;
    out[4] = Dk + half;
    out[5] = Dk * (double)n_hot_inputs;
    out[6] = (Dk - half) * (double)n_hot_inputs;
    out[7] = (Dk + half) * (double)n_hot_inputs;
    return 0;
}

/*
 * Access counters of the preprocessing phase (section 3.1 and the first loop of
 * Algorithm 1: one counter C_i per embedding entry, advanced for every sampled
 * input that reads entry i):
 *     counts[t][r] += #{ (j, l) : j < n_valid, idx[t][j][l] == r }
 * Counters accumulate over calls; the caller zeroes them once.
 */
int oracle_count_accesses(int T, int64_t R, const int32_t *idx, int B, int L,
                          int n_valid, uint32_t *const *counts)
{
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < n_valid; ++j) {
            for (int l = 0; l < L; ++l) {
                int64_t r = idx[((int64_t)t * B + j) * L + l];
                if (r < 0 || r >= R)
                    return -1;
                counts[t][r] += 1u;
            }
        }
    }
    return 0;
}

static void write_hot_set(int64_t R, const uint8_t *is_hot, int cap, int32_t *ids,
                          uint32_t *bits, uint32_t *n_hot)
{
    uint32_t n = 0;
    if (bits)
        memset(bits, 0, (size_t)((R + 31) / 32) * sizeof(uint32_t));
    for (int64_t r = 0; r < R; ++r) {
        if (!is_hot[r])
            continue;
        if (bits)
            bits[r >> 5] |= 1u << (r & 31);
        if ((int64_t)n < cap)
            ids[n] = (int32_t)r;
        ++n;
    }
    *n_hot = n;
}

/*
 * Hotness rule of section 3.1 / Algorithm 1: entry r of table t is hot when its
 * share of the accesses reaches lambda,
 *     C_r / total >= lambda
 * with the quotient taken in fp64 (correctly rounded, so that a share written
 * as a decimal, say 30 of 10000 against lambda = 0.003, compares as equal).
 * total >= 1 is the number of accesses each table received (inputs * L).
 * Outputs per table: the hot row ids in ascending order (the first `cap` of
 * them), the hot bitmap (bits[t] may be NULL; overwritten, not OR-ed), and the
 * number of hot rows n_hot[t] (which may exceed cap).
 */
int oracle_select_hot_ratio(int T, int64_t R, uint32_t *const *counts, double lambda,
                            int64_t total, int cap, int32_t *const *hot_ids,
                            uint32_t *const *hot_bits, uint32_t *n_hot)
{
    if (total < 1)
        return -3;
    uint8_t *is_hot = (uint8_t *)malloc((size_t)R);
    if (!is_hot)
        return -2;
    for (int t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r)
            is_hot[r] = (double)counts[t][r] / (double)total >= lambda;
        write_hot_set(R, is_hot, cap, hot_ids[t], hot_bits ? hot_bits[t] : NULL,
                      &n_hot[t]);
    }
    free(is_hot);
    return 0;
}

/* order: larger count first, lower row id first among equal counts */
typedef struct {
    uint32_t count;
    int32_t row;
} counted_row;

static int by_count_then_row(const void *a, const void *b)
{
    const counted_row *x = (const counted_row *)a, *y = (const counted_row *)b;
    if (x->count != y->count)
        return x->count > y->count ? -1 : 1;
    return x->row < y->row ? -1 : (x->row > y->row ? 1 : 0);
}

/*
 * "Hot set = the H most accessed rows of each table" (the workloads state the
 * hot set as a share of the rows): rank the rows by count, larger first, equal
 * counts by lower row id, keep the first H, and report them in ascending row
 * order.  H <= R.
 */
int oracle_select_hot_top(int T, int64_t R, uint32_t *const *counts, int H,
                          int32_t *const *hot_ids, uint32_t *const *hot_bits)
{
    if (H < 0 || H > R)
        return -3;
    counted_row *rank = (counted_row *)malloc((size_t)R * sizeof(counted_row));
    uint8_t *is_hot = (uint8_t *)malloc((size_t)R);
    if (!rank || !is_hot) {
        free(rank); free(is_hot);
        return -2;
    }
    for (int t = 0; t < T; ++t) {
        for (int64_t r = 0; r < R; ++r) {
            rank[r].count = counts[t][r];
            rank[r].row = (int32_t)r;
        }
        qsort(rank, (size_t)R, sizeof(counted_row), by_count_then_row);
        memset(is_hot, 0, (size_t)R);
        for (int k = 0; k < H; ++k)
            is_hot[rank[k].row] = 1;
        uint32_t n;
        write_hot_set(R, is_hot, H, hot_ids[t], hot_bits ? hot_bits[t] : NULL, &n);
    }
    free(rank);
    free(is_hot);
    return 0;
}

/*
 * Feature normalization of the pooled vectors (section 3.5: every sparse vector
 * is brought to zero mean and unit variance by a LayerNorm layer).  For each
 * vector x = x[t][j][:] of length D, j < n_valid:
 *     mu    = (1/D) sum_d x_d
 *     var   = (1/D) sum_d (x_d - mu)^2
 *     rstd  = 1 / sqrt(var + eps)
 *     y_d   = gamma[t][d] * (x_d - mu) * rstd + beta[t][d]
 * gamma / beta may be NULL (1 and 0).  mean and rstd are returned per vector.
 * All arithmetic in fp64, one rounding on store.
 */
int oracle_layernorm_forward(int T, int D, const float *x, int Bcap, int n_valid,
                             const float *gamma, const float *beta, double eps,
                             float *y, float *mean, float *rstd)
{
    for (int t = 0; t < T; ++t) {
        for (int j = 0; j < n_valid; ++j) {
            const float *xv = x + ((int64_t)t * Bcap + j) * D;
            float *yv = y + ((int64_t)t * Bcap + j) * D;
            double mu = 0.0, var = 0.0;
            for (int d = 0; d < D; ++d)
                mu += (double)xv[d];
            mu /= D;
            for (int d = 0; d < D; ++d)
                var += ((double)xv[d] - mu) * ((double)xv[d] - mu);
            var /= D;
            double rs = 1.0 / sqrt(var + eps);
            for (int d = 0; d < D; ++d) {
                double g = gamma ? (double)gamma[(int64_t)t * D + d] : 1.0;
                double b = beta ? (double)beta[(int64_t)t * D + d] : 0.0;
                yv[d] = (float)(g * ((double)xv[d] - mu) * rs + b);
            }
            mean[(int64_t)t * Bcap + j] = (float)mu;
            rstd[(int64_t)t * Bcap + j] = (float)rs;
        }
    }
    return 0;
}

/*
 * Gradient of the above.  With xh_d = (x_d - mu) * rstd and g_d = gamma_d * dy_d:
 *     dx_d      = rstd * ( g_d - mean_d(g) - xh_d * mean_d(g * xh) )
 *     dgamma_d  = sum_{j < n_valid} dy[t][j][d] * xh[t][j][d]
 *     dbeta_d   = sum_{j < n_valid} dy[t][j][d]
 * mu and rstd are recomputed from x in fp64 (they are not inputs here), so the
 * result does not inherit the rounding of a stored fp32 rstd.
 */
int oracle_layernorm_backward(int T, int D, const float *dy, const float *x, int Bcap,
                              int n_valid, const float *gamma, double eps, float *dx,
                              float *dgamma, float *dbeta)
{
    double *xh = (double *)malloc((size_t)D * sizeof(double));
    double *dg = (double *)malloc((size_t)D * sizeof(double));
    double *db = (double *)malloc((size_t)D * sizeof(double));
    if (!xh || !dg || !db) {
        free(xh); free(dg); free(db);
        return -2;
    }
    for (int t = 0; t < T; ++t) {
        for (int d = 0; d < D; ++d)
            dg[d] = db[d] = 0.0;
        for (int j = 0; j < n_valid; ++j) {
            const float *xv = x + ((int64_t)t * Bcap + j) * D;
            const float *dv = dy + ((int64_t)t * Bcap + j) * D;
            float *ov = dx + ((int64_t)t * Bcap + j) * D;
            double mu = 0.0, var = 0.0;
            for (int d = 0; d < D; ++d)
                mu += (double)xv[d];
            mu /= D;
            for (int d = 0; d < D; ++d)
                var += ((double)xv[d] - mu) * ((double)xv[d] - mu);
            var /= D;
            double rs = 1.0 / sqrt(var + eps);
            double m_g = 0.0, m_gx = 0.0;
            for (int d = 0; d < D; ++d) {
                double g = (gamma ? (double)gamma[(int64_t)t * D + d] : 1.0) * (double)dv[d];
                xh[d] = ((double)xv[d] - mu) * rs;
                m_g += g;
                m_gx += g * xh[d];
                dg[d] += (double)dv[d] * xh[d];
                db[d] += (double)dv[d];
            }
            m_g /= D;
            m_gx /= D;
            for (int d = 0; d < D; ++d) {
                double g = (gamma ? (double)gamma[(int64_t)t * D + d] : 1.0) * (double)dv[d];
                ov[d] = (float)(rs * (g - m_g - xh[d] * m_gx));
            }
        }
        for (int d = 0; d < D; ++d) {
            if (dgamma) dgamma[(int64_t)t * D + d] = (float)dg[d];
            if (dbeta) dbeta[(int64_t)t * D + d] = (float)db[d];
        }
    }
    free(xh); free(dg); free(db);
    return 0;
}
