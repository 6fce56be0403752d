/*
 * libslipstream - embedding-table side of a Slipstream training step on one
 * AMD MI355X (gfx950).  C ABI; every kernel behind it is hand-written HIP.
 *
 * The paper (arXiv 2404.04270) trains recommendation models whose embedding
 * tables E (m rows x d columns, section 2.4.1) dominate memory traffic.  It
 * keeps periodic snapshots of the frequently accessed ("hot") rows, marks a hot
 * row stale once the Euclidean distance between two consecutive snapshots of it
 * no longer exceeds a threshold T (Eq. 1, Eq. 5), stops updating stale rows and
 * drops the inputs that only reach stale rows (Eq. 6-8).  ss_filter_batch,
 * ss_embbag_forward, ss_embbag_backward_update and ss_detect_stale are the pieces
 * of one training iteration that touch the tables; the calls after them set the
 * method up: the sampling block that prices candidate thresholds (section 3.3)
 * and the identification of the hot rows (section 3.1).
 *
 * Conventions common to all calls
 *   - Return value: SS_OK or an SS_ERR_* code; ss_last_error() gives the text
 *     of the calling thread's last error.  On an error nothing was enqueued.
 *   - Arguments are validated on the host.  Row indices are NOT range-checked
 *     by the kernels: an index outside [0, rows) is undefined behaviour, unless
 *     the checked mode is on (ss_check_enable below), which turns it into an
 *     error return.
 *   - Every pointer marked "device" is device memory owned by the caller; the
 *     library allocates nothing, keeps no state between calls and never
 *     synchronises with the host.  (Exceptions, each stated at its declaration:
 *     the issue queue, the profiling aid and the checked mode hold state;
 *     ss_embbag_backward_update_noalloc uses a buffer inside the library's
 *     device image; the checked mode waits for the GPU.)  Work is enqueued on `stream`
 *     (a hipStream_t passed as void*; NULL is the default stream) and the
 *     buffers must stay alive until that work has finished.
 *   - The ss_tables struct itself lives in HOST memory and is only read.
 *   - Tables are fp32, row-major [rows][dim], 16-byte aligned, dim % 4 == 0.
 *   - A stale bitmap has one bit per row: row r is bit (r & 31) of 32-bit
 *     word (r >> 5); ceil(rows / 32) words per table.
 *   - Lookup indices are int32 [T][B][L]: table-major, then sample, then the
 *     L lookups of that sample's bag (L = 1 for one-hot features).
 */
#ifndef SLIPSTREAM_H
#define SLIPSTREAM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
    SS_OK = 0,
    SS_ERR_INVALID_ARG = 1,
    SS_ERR_UNSUPPORTED = 2,
    SS_ERR_WORKSPACE = 3, /* workspace missing, misaligned or too small */
    SS_ERR_HIP = 4        /* a HIP runtime call or kernel launch failed */
};

/* Text of the calling thread's last error ("" if none).  Static storage. */
const char *ss_last_error(void);

typedef struct {
    int32_t num_tables;    /* 1 <= T <= 65535 */
    int32_t dim;           /* d: floats per row, multiple of 4, <= 1024 */
    int64_t rows;          /* m: rows of every table, 1 <= rows < 2^31 */
    float **weights;       /* device array of T device pointers, each [rows][dim] */
    uint32_t **stale_bits; /* device array of T device pointers to bitmaps, or
                              NULL when no row of any table is stale */
} ss_tables;

/*
 * Input classifier (section 3.4, Eq. 6-8; alpha as in the notation table and
 * the alpha ablation).  For sample b let c_b be the number of its T*L lookups
 * that hit a row whose stale bit is set.  The sample is skipped iff
 * c_b >= alpha.  alpha = T*L skips the samples whose every lookup is stale;
 * alpha <= 0 skips every sample; alpha > T*L skips none.
 *
 *   idx        device, int32 [T][B][L], read only
 *   skip_mask  device, uint8 [B]: 1 = skipped
 *   kept_ids   device, int32 [B]: the kept sample numbers in ascending order
 *              in entries [0, n_kept); the rest is left untouched
 *   n_kept     device, one int32
 *   idx_c      device, int32 [T][B][L]: idx_c[t][j][:] = idx[t][kept_ids[j]][:]
 *              for j < n_kept (same strides as idx); rows j >= n_kept are
 *              left untouched.  Must not alias idx.
 *   ws         device workspace of ss_filter_batch_workspace_bytes(T, B, L)
 *              bytes, 256-byte aligned
 */
int32_t ss_filter_batch(const ss_tables *tables, const int32_t *idx, int32_t B,
                        int32_t L, int32_t alpha, uint8_t *skip_mask,
                        int32_t *kept_ids, int32_t *n_kept, int32_t *idx_c,
                        void *ws, size_t ws_bytes, void *stream);
size_t ss_filter_batch_workspace_bytes(int32_t T, int32_t B, int32_t L);

/*
 * ss_filter_batch, and in the same pass the split of the inputs into hot and
 * cold ones (section 3.1: the hot inputs are those that read only hot entries;
 * I = I_hot + I_cold): with hot_bits a second set of bitmaps in the layout of
 * stale_bits (bit r of hot_bits[t] set iff row r of table t is hot, e.g. as
 * ss_select_hot_top / ss_select_hot_ratio write them),
 *     hot_mask[b] = 1 iff every one of the T*L lookups of sample b hits a hot row
 * for every sample of the batch, skipped or kept (device uint8 [B]).  hot_bits:
 * device array of T device pointers; NULL, or a NULL entry, means no hot row
 * (in that table), so no input is hot.  Everything else as ss_filter_batch, same
 * workspace; the indices are read once for both tests.
 */
int32_t ss_filter_batch_split(const ss_tables *tables, uint32_t *const *hot_bits,
                              const int32_t *idx, int32_t B, int32_t L, int32_t alpha,
                              uint8_t *skip_mask, uint8_t *hot_mask, int32_t *kept_ids,
                              int32_t *n_kept, int32_t *idx_c, void *ws, size_t ws_bytes,
                              void *stream);

/*
 * Pooled embedding lookup (section 2.1: the lookup of one sparse feature
 * yields a single vector per table; bags are pooled by summation):
 *     out[t][j][:] = sum_{l < L} W_t[ idx[t][j][l] ][:]      for j < n_valid
 * A row that appears m times in a bag is added m times.  With L = 1 the
 * result is a bit-exact copy of the row.
 *
 *   idx      device, int32 [T][Bcap][L]
 *   n_valid  device, one int32 in [0, Bcap] (e.g. ss_filter_batch's n_kept),
 *            or NULL meaning Bcap
 *   out      device, fp32 [T][Bcap][dim], 16-byte aligned; rows j >= n_valid
 *            are left untouched
 */
int32_t ss_embbag_forward(const ss_tables *tables, const int32_t *idx,
                          int32_t Bcap, int32_t L, const int32_t *n_valid,
                          float *out, void *stream);

/*
 * Backward of the pooled lookup fused with sparse SGD that skips stale rows
 * (abstract, section 3.6: stale embeddings are identified and their updates
 * skipped; section 2.3.1 counts the optimizer's embedding update among the
 * dominant costs).  With sum pooling every lookup (t, j, l) receives
 * grad[t][j][:].  For each row r of table t that is looked up at least once
 * by a sample j < n_valid and whose stale bit is clear
 *     W_t[r][:] -= lr * sum_{(j,l): idx[t][j][l] == r} grad[t][j][:]
 * Rows whose stale bit is set are neither read nor written; bitmaps are not
 * modified.  The sum is taken in fp32 in a fixed order (ascending sample, then
 * position in the bag; long runs are split at fixed boundaries), so results
 * are reproducible run to run.
 *
 *   grad  device, fp32 [T][Bcap][dim], 16-byte aligned, read only
 *   ws    device workspace of ss_backward_workspace_bytes(T, Bcap, L, dim)
 *         bytes, 256-byte aligned; contents on entry are ignored
 */
int32_t ss_embbag_backward_update(const ss_tables *tables, const int32_t *idx,
                                  int32_t Bcap, int32_t L,
                                  const int32_t *n_valid, const float *grad,
                                  float lr, void *ws, size_t ws_bytes,
                                  void *stream);
size_t ss_backward_workspace_bytes(int32_t T, int32_t Bcap, int32_t L,
                                   int32_t dim);

/*
 * ss_embbag_backward_update for callers that cannot allocate device memory and
 * have no workspace to pass: code under HIP stream capture, tight serving loops,
 * harnesses that forbid hipMalloc.  The call allocates nothing and creates no HIP
 * object (also while ss_profile_enable is on: its launches are not timed).  What
 * the update keeps between its launches (sorted lookup lists, histograms, partial
 * sums) lives in a buffer of SS_NOALLOC_SCRATCH_BYTES that is part of the
 * library's device image: every GPU the library is used on holds one copy of it
 * until the process ends.  Same arguments, kernels and results (bit for bit) as
 * ss_embbag_backward_update without ws / ws_bytes.
 *   - Shapes with ss_backward_workspace_bytes(T, Bcap, L, dim) above
 *     SS_NOALLOC_SCRATCH_BYTES are rejected with SS_ERR_WORKSPACE; nothing is
 *     enqueued.  (26 tables x 8192 one-hot lookups x dim 64 need 5.6 MB.)
 *   - All calls on one GPU share that GPU's buffer: two calls whose work overlaps
 *     on one GPU (different streams, or threads) race.  Calls on one stream, one
 *     after the other, are safe; a call never reads what an earlier one left.
 *   - The buffer's device address is looked up on the first call on each device
 *     (a symbol lookup, no allocation): make that first call outside a capture.
 */
#define SS_NOALLOC_SCRATCH_BYTES (16u << 20)
int32_t ss_embbag_backward_update_noalloc(const ss_tables *tables, const int32_t *idx,
                                          int32_t Bcap, int32_t L,
                                          const int32_t *n_valid, const float *grad,
                                          float lr, void *stream);

/*
 * The same update in two halves, for callers that want to overlap them with
 * other work.  ss_embbag_backward_prepare groups the lookups of every table by
 * row (and drops the lookups of stale rows); it depends only on idx, n_valid
 * and the stale bitmaps, not on the gradients, so it can run on a second stream
 * next to the forward pass and the dense part of the model.
 * ss_embbag_backward_apply then sums the gradients per row and applies the SGD
 * step.  ss_embbag_backward_update(...) is exactly prepare(...) followed by
 * apply(...) on one stream.  The caller orders the two halves (same stream, or
 * an event), passes the same tables, Bcap, L and workspace to both, and leaves
 * the workspace and the bitmaps untouched in between.
 */
int32_t ss_embbag_backward_prepare(const ss_tables *tables, const int32_t *idx,
                                   int32_t Bcap, int32_t L, const int32_t *n_valid,
                                   void *ws, size_t ws_bytes, void *stream);
int32_t ss_embbag_backward_apply(const ss_tables *tables, int32_t Bcap, int32_t L,
                                 const float *grad, float lr, void *ws,
                                 size_t ws_bytes, void *stream);

/*
 * ss_embbag_forward(...) and ss_embbag_backward_prepare(...) of the same batch in
 * one call: out receives the pooled vectors, bwd_ws is left ready for
 * ss_embbag_backward_apply.  Both halves read the same indices, and the grouping
 * is bound by latency while the gather is bound by HBM, so for one-hot batches
 * of at most 16384 lookups per table (and row ids + sample numbers that fit 31
 * bits together) a single launch runs the grouping in the shadow of the gather;
 * other shapes get the two launches back to back.  Results are identical to the
 * separate calls.
 */
int32_t ss_embbag_forward_grouped(const ss_tables *tables, const int32_t *idx,
                                  int32_t Bcap, int32_t L, const int32_t *n_valid,
                                  float *out, void *bwd_ws, size_t bwd_ws_bytes,
                                  void *stream);

/*
 * Snapshot comparison (section 3.1.2 snapshots; Eq. 1 and Eq. 5).  For hot
 * slot h of table t with r = hot_ids[t][h]:
 *     drift = || W_t[r][:] - snapshot_t[h][:] ||_2        (accumulated in fp64)
 *     stale = (threshold > 0) && (drift <= threshold)
 * and if stale, bit r of stale_bits[t] is set (bits are only ever OR-ed in:
 * once stale, a row stays stale).  Equality counts as stale because Eq. 1 calls
 * a row varying only when the distance exceeds T.  threshold = 0 disables
 * detection (plain training); threshold = +inf flags every hot row.  A NaN
 * drift leaves the row varying.  If refresh_snapshot != 0, snapshot_t[h][:] is
 * then overwritten with W_t[r][:].  To capture a first snapshot, call with
 * threshold = 0 and refresh_snapshot = 1.
 *
 *   tables->stale_bits must not be NULL
 *   hot_ids      device array of T device pointers, each int32 [H]; the row
 *                ids of one table must be distinct (ascending order lets
 *                neighbouring rows share one bitmap update, but is not needed)
 *   snapshot     device array of T device pointers, each fp32 [H][dim]
 *   stale_hot    NULL, or device array of T device pointers, each uint8 [H]:
 *                this call's verdict per hot slot
 *   drift        NULL, or device array of T device pointers, each fp64 [H]
 *   stale_count  NULL, or device uint32 [T]: slots flagged stale by this call
 *                (zeroed by the call, then one atomic add per workgroup that
 *                flags a row: a diagnostic, it slows a pass in which most rows
 *                are flagged; pass NULL on the training path)
 */
int32_t ss_detect_stale(const ss_tables *tables, int32_t *const *hot_ids,
                        int32_t H, float **snapshot, float threshold,
                        int32_t refresh_snapshot, uint8_t **stale_hot,
                        double **drift, uint32_t *stale_count, void *stream);

/*
 * Input sampling block (section 3.3.2-3.3.3, Eq. 1 and the count of Eq. 2): on
 * a sample of S inputs, how many could be dropped under each of n_thr candidate
 * thresholds.  With stale_k(row) = row is hot, T_k > 0 and drift(row) <= T_k
 * (the verdict ss_detect_stale would reach with threshold T_k),
 *     counts[k] = #{ sampled inputs with at least alpha lookups (out of their
 *                    T*L) for which stale_k holds }
 * Eq. 2 as printed sums the "varying" indicator while its text asks for the
 * dropped share; the dropped share is what the search over T needs, so the
 * stale indicator is counted.  Rows outside the hot set are never stale.
 * The drifts come from a call of ss_detect_stale with a non-NULL drift argument
 * (threshold 0 and refresh_snapshot 0 leave bitmaps and snapshots untouched), so
 * the hot rows are read once however many thresholds and samples follow.
 * Nothing but counts is written.
 *
 *   num_tables   T, 1..65535
 *   hot_ids      device array of T device pointers, each int32 [H], strictly
 *                ascending (rows are mapped to hot slots by bisection; the
 *                order is not checked)
 *   drift        device array of T device pointers, each fp64 [H]: drift of hot
 *                slot h of table t, none NULL
 *   sidx         device int32 [T][S][L]: lookups of the sampled inputs; a value
 *                that is no hot row id (out-of-range ones included) counts as
 *                not stale
 *   alpha        >= 0; alpha = 0 makes every sampled input droppable, alpha >
 *                T*L none, alpha = T*L is the "every lookup stale" rule of Eq. 6-8
 *   thresholds   HOST array of n_thr floats (1 <= n_thr <= SS_MAX_THRESHOLDS),
 *                read before the call returns; any order; NaN is rejected
 *   counts       device uint32 [n_thr], overwritten
 * S = 0 or H = 0 are allowed (no row is stale then).
 */
#define SS_MAX_THRESHOLDS 32
int32_t ss_sample_drop(int32_t num_tables, int32_t *const *hot_ids, int32_t H,
                       double *const *drift, const int32_t *sidx, int32_t S,
                       int32_t L, int32_t alpha, const float *thresholds,
                       int32_t n_thr, uint32_t *counts, void *stream);

/*
 * Estimate of the dropped share from one count of ss_sample_drop, with its
 * confidence interval (Eq. 2-4).  Host arithmetic only, fp64; no GPU work.
 *     D    = count / n_samples                                         (Eq. 2)
 *     sd   = sqrt( mean over the sample of (indicator - D)^2 )          (Eq. 3)
 *     half = t_crit * sqrt( (population - n_samples) / population
 *                           * sd^2 / n_samples )                        (Eq. 4)
 * Eq. 4 writes the sample size both as |S| and as m: one number, n_samples.
 * population is the number of inputs the sample was drawn from without
 * replacement; n_hot_inputs scales the share to the expected number of dropped
 * hot inputs, the quantity the paper's interval is centred on (normally equal
 * to population).  t_crit is the critical value, 3.340 in the paper for 99.9 %.
 *   out   HOST double[8]: D, sd, half, D - half, D + half,
 *         D * n_hot_inputs, (D - half) * n_hot_inputs, (D + half) * n_hot_inputs
 * Errors: n_samples < 1, population < n_samples, count > n_samples,
 * n_hot_inputs < 0, t_crit negative or NaN, out NULL.
 */
int32_t ss_drop_stats(uint32_t count, int64_t n_samples, int64_t population,
                      int64_t n_hot_inputs, double t_crit, double *out);

/*
 * Access counters of the preprocessing phase (section 3.1; first loop of
 * Algorithm 1: one counter per embedding entry, advanced for every sampled
 * input that reads the entry):
 *     counts[t][r] += #{ (j, l) : j < n_valid, idx[t][j][l] == r }
 * Counters accumulate over calls (32-bit, wrapping); the caller zeroes them once.
 *   idx       device int32 [T][B][L]
 *   n_valid   NULL (all B inputs count) or device int32: inputs j >= *n_valid are
 *             not read
 *   counts    device array of T device pointers, each uint32 [rows]
 */
int32_t ss_count_accesses(int32_t num_tables, int64_t rows, const int32_t *idx,
                          int32_t B, int32_t L, const int32_t *n_valid,
                          uint32_t *const *counts, void *stream);

/* Bytes of 256-byte-aligned device scratch the two selections below need
 * (0 for arguments they would reject). */
size_t ss_select_hot_workspace_bytes(int32_t num_tables, int64_t rows);

/*
 * Hot rows by the paper's share rule (section 3.1, Algorithm 1): row r of
 * table t is hot when
 *     counts[t][r] / total >= lambda        (the quotient taken in fp64)
 * where total >= 1 is the number of accesses each table received (inputs * L).
 * lambda <= 0 makes every row hot.  Per table the call writes
 *   hot_ids[t]   int32 [cap]: the hot row ids in ascending order; if there are
 *                more than cap, the cap lowest; entries past n_hot[t] untouched
 *                (hot_ids may be NULL when cap = 0)
 *   hot_bits[t]  NULL array, or bitmaps of ceil(rows/32) words each, overwritten
 *                (not OR-ed): bit r set iff row r is hot; usable as the second
 *                bitmap of ss_filter_batch to split inputs into hot and cold
 *   n_hot        NULL, or device uint32 [T]: number of hot rows (may exceed cap)
 * All device memory; ws as sized by ss_select_hot_workspace_bytes.
 */
int32_t ss_select_hot_ratio(int32_t num_tables, int64_t rows, uint32_t *const *counts,
                            double lambda, int64_t total, int32_t cap,
                            int32_t *const *hot_ids, uint32_t *const *hot_bits,
                            uint32_t *n_hot, void *ws, size_t ws_bytes, void *stream);

/*
 * Hot rows as the H most accessed rows of each table (how the workloads of this
 * build state their hot sets: a share of the rows).  Rows are ranked by count,
 * larger first, equal counts by lower row id; the first H form the hot set,
 * written to hot_ids[t] (int32 [H]) in ascending row order and, if hot_bits is
 * not NULL, as bitmaps (overwritten).  0 <= H <= rows.  The result has the
 * layout ss_detect_stale and ss_sample_drop expect of hot_ids.
 */
int32_t ss_select_hot_top(int32_t num_tables, int64_t rows, uint32_t *const *counts,
                          int32_t H, int32_t *const *hot_ids, uint32_t *const *hot_bits,
                          void *ws, size_t ws_bytes, void *stream);

/*
 * Feature normalization of the pooled vectors (section 3.5: a LayerNorm layer
 * brings every sparse vector to zero mean and unit variance; one layer per
 * table).  For each vector v = x[t][j][:], j < n_valid:
 *     mu = mean_d(v),  var = mean_d((v - mu)^2),  rstd = 1 / sqrt(var + eps)
 *     y[t][j][d] = gamma[t][d] * (v_d - mu) * rstd + beta[t][d]
 *   x, y      device fp32 [T][Bcap][dim], 16-byte aligned (the layout of
 *             ss_embbag_forward's output); y may be x itself
 *   gamma, beta  device fp32 [T][dim], or NULL for 1 and 0
 *   mean, rstd   device fp32 [T][Bcap], written for j < n_valid (the backward
 *             pass reads them)
 *   n_valid   as for ss_embbag_forward; vectors j >= n_valid are left untouched
 *   eps >= 0
 */
int32_t ss_layernorm_forward(int32_t num_tables, int32_t dim, const float *x,
                             int32_t Bcap, const int32_t *n_valid, const float *gamma,
                             const float *beta, float eps, float *y, float *mean,
                             float *rstd, void *stream);

/*
 * Gradient of ss_layernorm_forward.  With xh = (x - mu) * rstd and g = gamma * dy:
 *     dx[t][j][d]  = rstd * ( g_d - mean_d(g) - xh_d * mean_d(g * xh) )
 *     dgamma[t][d] = sum_{j < n_valid} dy[t][j][d] * xh[t][j][d]
 *     dbeta[t][d]  = sum_{j < n_valid} dy[t][j][d]
 * dx is the gradient ss_embbag_backward_update expects.  dx may be dy itself.
 * dgamma / dbeta (device fp32 [T][dim]) may be NULL; if either is given, ws must
 * hold ss_layernorm_backward_workspace_bytes(...) bytes, 256-byte aligned.  The
 * sums over the batch are taken in a fixed order.
 */
int32_t ss_layernorm_backward(int32_t num_tables, int32_t dim, const float *dy,
                              const float *x, int32_t Bcap, const int32_t *n_valid,
                              const float *gamma, const float *mean, const float *rstd,
                              float *dx, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream);
size_t ss_layernorm_backward_workspace_bytes(int32_t num_tables, int32_t dim,
                                             int32_t Bcap);

/*
 * The pooled lookup (section 2.1) and its feature normalization (section 3.5) in
 * one pass each way, without the pooled tensor ever being stored:
 *   ss_embbag_forward_ln(...)  = ss_embbag_forward into a temporary x, then
 *                                ss_layernorm_forward(x) -> y, mean, rstd
 *   ss_embbag_ln_backward(...) = the same temporary x formed again from the
 *                                tables, then ss_layernorm_backward(dy, x) -> dx,
 *                                dgamma, dbeta
 * Results are bit-identical to the separate calls.  ss_embbag_ln_backward must
 * see the tables as the forward pass saw them, i.e. it runs before
 * ss_embbag_backward_update of the same batch, whose gradient argument dx is.
 * Arguments as in the separate calls; ws as for ss_layernorm_backward (dim and
 * num_tables taken from tables).
 */
int32_t ss_embbag_forward_ln(const ss_tables *tables, const int32_t *idx, int32_t Bcap,
                             int32_t L, const int32_t *n_valid, const float *gamma,
                             const float *beta, float eps, float *y, float *mean,
                             float *rstd, void *stream);
int32_t ss_embbag_ln_backward(const ss_tables *tables, const int32_t *idx, int32_t Bcap,
                              int32_t L, const int32_t *n_valid, const float *dy,
                              const float *gamma, const float *mean, const float *rstd,
                              float *dx, float *dgamma, float *dbeta, void *ws,
                              size_t ws_bytes, void *stream);

/*
 * Issue queue: a host thread of the library's own that enqueues work on HIP
 * streams, for callers whose single host thread cannot enqueue a batch as fast
 * as the GPU finishes it (enqueueing one kernel costs the host about 3 us here;
 * the index work of a batch - section 3.4, the input classifier, and the grouping
 * half of the update - is up to eight kernels).  Jobs are issued in submission
 * order.  Nothing here waits for the GPU or touches device memory.  A caller
 * may hold several queues (say one per stream it feeds); they share nothing, so
 * an event must outlive every queue that holds a job naming it: destroy the
 * queues first, then the events.
 *
 *   ss_issue_queue_create   starts the thread, bound to the device that is
 *                           current in the calling thread; *out owns it
 *   ss_issue_queue_destroy  issues what is still queued, joins, frees
 *   ss_issue_index_batch    = ss_filter_batch, then ss_embbag_backward_prepare on
 *                           the idx_c / n_kept it produced, both on `stream`.
 *                           Arguments as in those two calls (validated here, on
 *                           the calling thread: an error is returned at once and
 *                           nothing is queued); every buffer and the arrays that
 *                           `tables` points to must stay valid until the job has
 *                           run (the struct itself is copied)
 *   ss_issue_wait_event     hipStreamWaitEvent(stream, event) as a job
 *   ss_issue_record_event   hipEventRecord(event, stream) as a job
 *   ss_issue_wait           blocks the calling host thread until job `ticket` has
 *                           been ISSUED (not executed); returns the first error
 *                           any job met.  Needed before another stream is made
 *                           to wait for an event that the queue records: waiting
 *                           for an event that has not been recorded yet is a no-op
 *   ticket                  NULL, or host address that receives the job's number
 *
 * Events are plain HIP events without timing, as void *: ss_event_create /
 * ss_event_destroy, and the two immediate calls a caller needs on its own
 * streams, ss_event_record(event, stream) and ss_stream_wait_event(stream, event).
 */
typedef struct ss_issue_queue ss_issue_queue;
int32_t ss_issue_queue_create(ss_issue_queue **out);
int32_t ss_issue_queue_destroy(ss_issue_queue *queue);
int32_t ss_issue_index_batch(ss_issue_queue *queue, const ss_tables *tables,
                             const int32_t *idx, int32_t B, int32_t L, int32_t alpha,
                             uint8_t *skip_mask, int32_t *kept_ids, int32_t *n_kept,
                             int32_t *idx_c, void *ws_filter, size_t ws_filter_bytes,
                             void *ws_backward, size_t ws_backward_bytes, void *stream,
                             uint64_t *ticket);
int32_t ss_issue_wait_event(ss_issue_queue *queue, void *event, void *stream,
                            uint64_t *ticket);
int32_t ss_issue_record_event(ss_issue_queue *queue, void *event, void *stream,
                              uint64_t *ticket);
int32_t ss_issue_wait(ss_issue_queue *queue, uint64_t ticket);
int32_t ss_event_create(void **event);
int32_t ss_event_destroy(void *event);
int32_t ss_event_record(void *event, void *stream);
int32_t ss_stream_wait_event(void *stream, void *event);

/*
 * The training iteration as a whole (Algorithm 1: drop the inputs that only
 * reach stale entries, train on the rest, every K iterations compare the hot rows
 * with their last snapshot; the first period is the warm-up of section 3.1.1 and
 * ends with the capture of the first snapshot), scheduled so that the index work
 * of the coming batches (ss_filter_batch, ss_embbag_backward_prepare: they read
 * indices and stale bitmaps only) runs on index streams of the object's own while
 * the current batch is in its lookup and update kernels on the caller's training
 * stream.  Results are those of the calls issued one after the other on one
 * stream, bit for bit: the only reordering is that index work of later batches
 * runs before the update of earlier ones, which it does not read; batches after
 * one that ends with a detect pass are held back until that pass is enqueued.
 *
 * An ss_step is a stateful host object: it owns its index streams (default
 * priority), a fixed pool of events created at ss_step_create, and, if the plan
 * asks for them, issue threads (ss_issue_queue).  It allocates no device memory:
 * the caller hands over a ring of buffer sets and the pooled output.  Use from
 * one host thread.  Per batch, in this order:
 *     ss_step_submit(idx)      as far ahead as ss_step_room() allows (up to two
 *                              thirds of the ring); idx must stay untouched until
 *                              the batch's ss_step_backward has been called.  If
 *                              idx is still being produced on some stream, pass
 *                              the event recorded after its producer (a
 *                              hipEvent_t as void *), else NULL.  The wait for it
 *                              may be enqueued later than this call (by an issue
 *                              thread, or after a detect pass): the event must
 *                              not be destroyed or recorded again before the
 *                              batch's ss_step_forward has returned
 *     ss_step_forward          pooled lookup of the oldest submitted batch into
 *                              `pooled` on the training stream; *set_used (may be
 *                              NULL) = the buffer set that holds this batch's
 *                              skip_mask, kept_ids, n_kept and idx_c
 *     ss_step_backward(grad)   update with the gradients of the kept samples
 *                              (layout of ss_embbag_backward_update), then, when
 *                              the snapshot period ends, the capture or the
 *                              detect pass; *detected (may be NULL) = 1 after a
 *                              detect pass
 * ss_step_flush returns once everything submitted so far has been handed to its
 * stream (with issue threads; a no-op otherwise), so that a device
 * synchronisation after it covers that work.  ss_step_destroy ends the threads,
 * waits for the index streams and releases streams and events (the one call of
 * this group that waits for the GPU).  Calls out of order return
 * SS_ERR_INVALID_ARG and enqueue nothing.
 *
 * The plan: `every` batches between two cross-stream events, `index_streams`,
 * `issue_threads` (0: the calling thread enqueues everything) and the number of
 * buffer sets, 3 * every * index_streams.  host_wait_us: when the index work of
 * the batch that ss_step_forward is about to look up has not finished, and the
 * training stream still has a few batches of work queued, the call may keep the
 * calling thread polling for it for up to this many microseconds instead of
 * giving the training stream a wait command (which costs the stream time between
 * two kernels); the thread then stays at most a ring of batches ahead of the GPU.
 * 0: never, ss_step_forward only ever enqueues.  dim: floats per row, an input
 * of ss_step_plan_for only (0: unknown; with it the choice of index_streams can
 * weigh the training kernels of a batch against its index work).
 * ss_step_plan_for fills in what the caller left at 0 (every, index_streams) or
 * -1 (issue_threads, host_wait_us) with the measured choices for the shape, and
 * sets num_sets.
 */
typedef struct {
    int32_t every;
    int32_t index_streams;
    int32_t issue_threads;
    int32_t num_sets;
    int32_t host_wait_us;
    int32_t dim;
} ss_step_plan;

/* One buffer set of the ring: the outputs of ss_filter_batch for the batch that
 * occupies it and the workspaces of that batch (sizes as the workspace queries
 * give them for T, B, L, dim); all device memory owned by the caller. */
typedef struct {
    uint8_t *skip_mask;    /* [B] */
    int32_t *kept_ids;     /* [B] */
    int32_t *n_kept;       /* one int32 */
    int32_t *idx_c;        /* [T][B][L] */
    void *ws_filter;
    size_t ws_filter_bytes;
    void *ws_backward;
    size_t ws_backward_bytes;
} ss_step_set;

typedef struct ss_step ss_step;
int32_t ss_step_plan_for(int32_t T, int32_t B, int32_t L, ss_step_plan *plan);
/* hot_ids, snapshot, stale_hot, drift, stale_count: as for ss_detect_stale;
 * sets: HOST array of plan->num_sets entries (copied); pooled: device fp32
 * [T][B][dim]; train_stream: the caller's stream (NULL: the default stream);
 * alpha as for ss_filter_batch (T * L: drop the inputs whose every lookup is stale). */
int32_t ss_step_create(const ss_tables *tables, int32_t B, int32_t L, int32_t alpha, float lr,
                       float threshold, int32_t snapshot_every, int32_t *const *hot_ids,
                       int32_t H, float **snapshot, uint8_t **stale_hot, double **drift,
                       uint32_t *stale_count, const ss_step_plan *plan, const ss_step_set *sets,
                       float *pooled, void *train_stream, ss_step **out);
int32_t ss_step_destroy(ss_step *step);
int32_t ss_step_room(const ss_step *step);
int32_t ss_step_submit(ss_step *step, const int32_t *idx, void *ready_event);
int32_t ss_step_forward(ss_step *step, int32_t *set_used);
int32_t ss_step_backward(ss_step *step, const float *grad, int32_t *detected);
int32_t ss_step_flush(ss_step *step);
/* What the scheduler has done so far, for diagnosis (host memory, four values):
 * out[0] = lookups enqueued, out[1] = wait commands given to the training stream
 * for index work, out[2] = times the calling thread polled for index work
 * (host_wait_us), out[3] = polls that ended with the index work finished. */
int32_t ss_step_counters(const ss_step *step, int64_t *out);

/*
 * The same scheduler with every operation it would enqueue handed to a callback
 * instead (no GPU work at all): a test can record the program of streams, event
 * records and waits that a sequence of ss_step_* calls produces, execute it under
 * a scheduler of its own and check that every kernel would find its inputs
 * complete.  Streams are numbered 0 .. index_streams - 1, the training stream is
 * -1; events are numbered from 1; sets are ring positions.  The q_* callbacks
 * stand for jobs handed to issue queue `queue` (they may be issued later; *ticket
 * receives the job's number) and q_wait_issued for "block until that job has been
 * issued".  Every callback returns SS_OK or an error code, which the call in
 * progress passes on.
 */
typedef struct {
    void *user;
    int32_t (*index_now)(void *user, int32_t stream, int32_t set);
    int32_t (*q_index)(void *user, int32_t queue, int32_t stream, int32_t set, uint64_t *ticket);
    int32_t (*lookup)(void *user, int32_t set);
    int32_t (*update)(void *user, int32_t set);
    int32_t (*detect)(void *user, int32_t with_threshold);
    int32_t (*record_now)(void *user, int32_t event, int32_t stream);
    int32_t (*wait_now)(void *user, int32_t stream, int32_t event);
    int32_t (*q_record)(void *user, int32_t queue, int32_t event, int32_t stream,
                        uint64_t *ticket);
    int32_t (*q_wait)(void *user, int32_t queue, int32_t event, int32_t stream, uint64_t *ticket);
    int32_t (*q_wait_issued)(void *user, int32_t queue, uint64_t ticket);
} ss_step_trace_ops;
int32_t ss_step_create_traced(const ss_step_plan *plan, int32_t snapshot_every,
                              const ss_step_trace_ops *callbacks, ss_step **out);

/*
 * Range check of lookup indices (a debugging aid, not part of the method).
 *
 * ss_check_indices is one pass over an index tensor that reads nothing but the
 * indices (and *n_valid): it cannot fault on a bad index.  It is enqueued like
 * any other call and leaves in `report` (device, uint64 [2], 8-byte aligned)
 *     report[0] = number of entries idx[t][j][l], j < n_valid, outside [0, rows)
 *     report[1] = (t << 32) | (j * L + l) of the first such entry in (t, j, l)
 *                 order, or all ones if there is none
 * for the caller to read when it likes.
 *
 * Checked mode: on when the environment holds SS_CHECK=1 at the library's first
 * call, or after ss_check_enable(1).  While it is on, every entry point that
 * takes lookup indices or hot row ids (ss_filter_batch, ss_embbag_forward*,
 * ss_embbag_backward_update / _prepare, ss_embbag_ln_backward, ss_count_accesses,
 * ss_detect_stale, the jobs of ss_issue_index_batch) first runs that pass on
 * `stream`, WAITS for it on the host and, if an id is out of range, returns
 * SS_ERR_INVALID_ARG with the place in ss_last_error(); nothing else has been
 * enqueued then, so no kernel of the library faults on the input.  The mode
 * costs a host synchronisation per call and 16 bytes of device memory per GPU
 * (allocated on first use); ss_embbag_backward_update_noalloc is not covered.
 */
int32_t ss_check_indices(int32_t num_tables, int64_t rows, const int32_t *idx, int32_t B,
                         int32_t L, const int32_t *n_valid, uint64_t *report, void *stream);
void ss_check_enable(int32_t on);

/*
 * Measurement aids, off by default (not part of the method).  Process-wide; meant
 * for a single benchmarking thread.
 *
 * ss_profile_enable(1): every kernel the library launches carries a pair of HIP
 * events that the runtime stamps with the start and end of that kernel's execution
 * (this and trace mode are the cases in which the library creates HIP objects or
 * allocates).  ss_profile_report waits for the recorded events, writes one line
 * "kernel_name launches total_milliseconds" per kernel into buf (host memory, NUL
 * terminated), and forgets them.  At most 2^20 launches are recorded between two
 * reports.  A launch with an event pair costs the host about 20 us, so a pipeline
 * of several streams does not run at its own pace while this is on.
 *
 * ss_profile_enable(2): trace mode.  The kernels of the training iteration
 * (classifier, grouping, lookup, update, fixup, detect) stamp the GPU's
 * constant-rate clock themselves, when their first workgroups start and when each
 * workgroup ends, into a device buffer of the library (32 MB, allocated at the
 * first use); launches cost the host nothing extra, so the pipeline runs as it
 * does untraced.  ss_profile_trace stops tracing, waits for the device and writes
 * one line "kernel_name start_ns end_ns" per traced launch, in launch order,
 * times relative to the earliest start (resolution 10 ns).  At most 32768
 * launches per trace.
 *
 * ss_profile_enable(0) switches both off.
 */
void ss_profile_enable(int32_t mode);
int32_t ss_profile_report(char *buf, size_t buf_bytes);
int32_t ss_profile_trace(char *buf, size_t buf_bytes);

#ifdef __cplusplus
}
#endif
#endif /* SLIPSTREAM_H */
