/*
 * icq.h -- C ABI of the MI355X (gfx950) query-time path of Interleaved
 * Composite Quantization (arxiv 1912.08756).
 *
 * Notation follows the paper: K codebooks ("quantizers") C_k of m codewords in
 * R^d; every database item i is stored as K one-byte sub-codes code_k(i); the
 * first Kf codebooks are the fast set (script-K of Sec. 1 / Eq. 8; the caller
 * orders the codebooks so that the fast ones come first).  N items, Q queries.
 *
 * General rules
 *  - Every pointer is a DEVICE pointer owned by the caller unless marked
 *    "host".  The library never frees or keeps caller memory beyond a call,
 *    except that an index keeps private device copies it allocates itself.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    Every call only enqueues work on `stream` and returns; results are valid
 *    once the stream has been synchronised (icq_index_create also waits for
 *    its own counting pass before it sizes the grouped layouts).  Calls on one
 *    index from several host threads, or on several streams, are safe as long
 *    as they do not share output or workspace buffers (with stage timing off):
 *    searches of different query batches on two streams overlap -- the short
 *    kernels of one call run behind the long ones of the other.
 *  - Return value: ICQ_OK (0) or a negative ICQ_ERR_* code.  Arguments are
 *    checked on the host before anything is launched; an argument or
 *    workspace error means nothing has been enqueued (ICQ_ERR_HIP can come from
 *    a launch in the middle of a call).
 *  - Layouts are row-major with the last index contiguous.
 *  - Candidate lists: cand_ids / cand_partial are [Q][cap]; list q holds
 *    min(cand_count[q], cap) valid entries in UNSPECIFIED order (compare as
 *    sets).  cand_count[q] is the true number of survivors even when it
 *    exceeds cap; in that case which survivors were kept is unspecified and
 *    the caller must retry with a larger cap.
 *  - Results: out_ids / out_dist are [Q][topk], ascending by (distance, id);
 *    when fewer than topk items survive, the tail is (0xFFFFFFFF, +inf).
 *  - The distance returned is the table sum on the left of Eq. 1,
 *    sum_k ||q - c_{k,code_k(i)}||^2, not corrected by the constant
 *    -(K-1)||q||^2 + eps that relates it to ||q - xbar_i||^2.
 */
#ifndef ICQ_H
#define ICQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define ICQ_OK 0
#define ICQ_ERR_ARG (-1)       /* null pointer, or K/m/d/Kf/N/Q/topk/cap out of range   */
#define ICQ_ERR_WORKSPACE (-2) /* workspace missing, misaligned (256 B) or too small    */
#define ICQ_ERR_HIP (-3)       /* a HIP runtime call failed (allocation, launch)        */
#define ICQ_ERR_CAPACITY (-4)  /* reserved for synchronous helpers; async calls report
                                  overflow through cand_count / out_survivors            */

#define ICQ_ERR_SCRATCH (-5)   /* icq_search_static: the call needs more than the built-in
                                  scratch array of ICQ_STATIC_SCRATCH_BYTES holds           */

#define ICQ_MAX_K 64      /* codebooks                         */
#define ICQ_MAX_M 256     /* codewords per codebook (one byte) */
#define ICQ_MAX_TOPK 1024 /* result list length                */
#define ICQ_MAX_N 0xFFF00000ll /* items per index (ids are 32-bit) */
#define ICQ_MAX_Q (1 << 22) /* queries per call                  */
#define ICQ_MAX_SAMPLE 4096 /* items icq_sample_thresholds looks at */
#define ICQ_PAD_ID 0xFFFFFFFFu

typedef struct icq_index icq_index;

/* Human-readable text for an ICQ_* code (host pointer to a static string). */
const char *icq_strerror(int code);

/*
 * Build a search index from codebooks and codes (Sec. 1: x_i is quantised to
 * xbar_i = sum_k c_{k,code_k(i)}; the codes are the K codeword indices).
 *   codebooks [K][m][d] fp32;  codes [K][N] uint8, codebook-major, every value < m;
 *   1 <= Kf <= K <= ICQ_MAX_K, 1 <= m <= 256, d >= 1, 0 <= N <= ICQ_MAX_N.
 * The index copies what it needs into private device arrays laid out for the
 * kernels (fast sub-codes [Kf][N] padded and 16-byte aligned per row, all K
 * sub-codes of an item as one item-major record [N][stride], codewords padded
 * in d, codeword norms), so
 * the caller may release `codebooks` and `codes` once `stream` has been
 * synchronised.  Sub-codes >= m are not detected; tables are always 256
 * entries wide with +inf beyond m, so such an item simply gets distance +inf.  *out is set only on success.
 */
int icq_index_create(icq_index **out /*host*/, const float *codebooks, const uint8_t *codes,
                     int K, int m, int d, int Kf, int64_t N, void *stream);

/* Free the index and its private device arrays (host call; the caller makes
 * sure no enqueued work still uses it).  NULL is ignored. */
void icq_index_destroy(icq_index *index);

/* Write the index's private copy of the codes back in the input layout
 * [K][N] (bit-exact round trip of the storage layout; a debugging aid).
 * from_items == 0: fast rows from the stage-1 array, slow rows from the item
 * records; 1: every row from the item records; 2: from the grouped layout alone
 * through its position -> id map (Kf <= 2: the grouped item records; Kf = 3, 4:
 * rows 0, 1 from the pair each group of 16 positions is labelled with, the other
 * fast rows from the streamed rows, the rest from the grouped records);
 * ICQ_ERR_ARG if the index has no grouped layout (Kf > 4 or N == 0). */
int icq_index_export_codes(const icq_index *index, int from_items, uint8_t *codes_out, void *stream);

/*
 * Stage-1 strategy.  An item's crude distance (Eq. 2) depends only on its Kf fast
 * sub-codes.  Kf <= 2: when N is much larger than 256^Kf the index also keeps the
 * items grouped by that tuple, and for calls with more than 4 queries stage 1
 * evaluates each tuple once per query instead of each item.  Kf = 3, 4: the index
 * also keeps the items ordered by their first two fast sub-codes (every pair's run
 * padded to 16 positions); stage 1 then forms the pair's table sum once per 16
 * positions and streams only the remaining fast rows.  Values, survivors and
 * results are identical in every form (same additions in the same order).
 * ICQ_SCAN_AUTO picks a grouped form when it is available and cheaper (Kf = 3, 4:
 * from 64 * 65536 items on), ICQ_SCAN_STREAMED always walks all Kf fast rows item
 * by item, ICQ_SCAN_GROUPED uses the grouped form whenever the index has it.
 */
#define ICQ_SCAN_AUTO 0
#define ICQ_SCAN_STREAMED 1
#define ICQ_SCAN_GROUPED 2
int icq_index_set_scan_mode(icq_index *index, int mode);

/*
 * Number of positions stage 1 walks per pass over the index in its current scan
 * mode (host call; a measurement aid for work and traffic models): N for the
 * item-by-item scan; the 65536 runs' padded total, rounded up to whole block
 * steps, when the items grouped by their first two fast sub-codes are walked
 * (Kf = 3, 4); 256^Kf (one evaluation per tuple) for the grouped form of
 * Kf <= 2 with more than 4 queries.  *out is a host pointer.
 */
int icq_index_scan_positions(const icq_index *index, int Q, int64_t *out /*host*/);

/*
 * Stage timing, a measurement aid for icq_search (for profiling only: it adds
 * four event records per call and is not thread-safe).  With enable != 0 every
 * later icq_search on this index records events on its stream around the
 * kernels of its FIRST query sub-batch: before the table build, after it, after
 * stage 1 (scan, plus the survivors' distances where the scan is fused with
 * them; the interval starts once the survivor counters are zeroed) and after
 * the nearest-neighbour lists are written.  icq_scan_fast records the same
 * events (its stage-1 interval is its scan kernel, stage 2 is empty).  The
 * latest ICQ_TIMED_CALLS calls are kept.  enable == 0 stops that and releases the
 * events.
 * icq_index_stage_times waits for the last recorded call to finish and writes
 * ms[0..2] (host) = milliseconds of table build, stage 1, stage 2 + list,
 * averaged over the calls recorded since timing was switched on or last read
 * (*calls, host, may be NULL); *batches (host, may be NULL) = the largest number
 * of sub-batches one of those calls was split into (the times cover whole calls
 * only when it is 1).  Reading resets the record.  ICQ_ERR_ARG when timing is
 * off or no search has run since it was switched on or last read.
 */
#define ICQ_TIMED_CALLS 64
int icq_index_set_stage_timing(icq_index *index, int enable);
int icq_index_stage_times(const icq_index *index, float *ms /*host [3]*/, int *calls /*host*/,
                          int *batches /*host*/);

/* Bytes of 256-byte-aligned device workspace that icq_scan_fast, icq_refine
 * and icq_search need for up to Q queries per call, candidate capacity `cap`
 * per query and result length `topk`.  *out is a host pointer. */
int icq_workspace_bytes(const icq_index *index, int Q, int64_t cap, int topk, size_t *out /*host*/);

/*
 * Lookup-table precompute (Sec. 1, text after Eq. 1: all ||q - c_{k,j}||^2 are
 * computed once per query so that a distance costs K additions):
 *   lut[q][k][j] = ||q||^2 - 2<q, c_{k,j}> + ||c_{k,j}||^2,   fp32, [Q][K][256]
 * (rows are always 256 wide; entries j >= m are +inf).  queries [Q][d] fp32;
 * lut 16-byte aligned (ICQ_ERR_ARG otherwise).  The inner products run on the
 * fp32 matrix cores.  Q >= 0.
 */
int icq_build_lut(const icq_index *index, const float *queries, int Q, float *lut, void *stream);

/*
 * Stage 1, crude comparison (Eq. 2 with a static per-query threshold in place
 * of "furthest list element + sigma"): for every item
 *   P[q][i] = sum_{k<Kf} lut[q][k][code_k(i)]   (k ascending, fp32)
 * and item i survives for query q iff P[q][i] < thresholds[q] (strict; +inf
 * keeps every item, NaN keeps none).  Survivors are appended to query q's
 * candidate list as (cand_ids, cand_partial = P).  cand_partial may be NULL
 * when the caller does not need the crude distances (the kernels list ids and
 * fill in P afterwards, so this saves a pass).  cand_count [Q] is written
 * (not accumulated).  lut is [Q][K][256] as written by icq_build_lut.
 * 0 <= Q, 1 <= cap, Q*cap < 2^40.  Needs icq_workspace_bytes(index, Q, cap, 1).
 */
int icq_scan_fast(const icq_index *index, const float *lut, int Q, const float *thresholds,
                  uint32_t *cand_ids, float *cand_partial, uint32_t *cand_count, int64_t cap,
                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * Stage 2, exact comparison for the survivors only (Eq. 1, left side) and the
 * nearest-neighbour list (Sec. 3.4):
 *   D[q][i] = cand_partial + sum_{k=Kf..K-1} lut[q][k][code_k(i)]   (k ascending, fp32)
 * then the topk smallest (D, id) per query.  Reads min(cand_count[q], cap)
 * entries of each list; every listed id must be below N (ids are not checked:
 * a larger one reads outside the index's item records).  With cand_partial == NULL the same D is formed as the
 * whole K-term sum (same order of additions, identical bits).
 * 1 <= topk <= ICQ_MAX_TOPK.
 */
int icq_refine(const icq_index *index, const float *lut, int Q, const uint32_t *cand_ids,
               const float *cand_partial, const uint32_t *cand_count, int64_t cap, int topk,
               uint32_t *out_ids, float *out_dist, void *workspace, size_t workspace_bytes,
               void *stream);

/*
 * The whole path for a batch of queries: table precompute, stage 1, stage 2,
 * nearest-neighbour list.  queries [Q][d], thresholds [Q]; `cap` is the
 * per-query candidate capacity carved out of the workspace (needs
 * icq_workspace_bytes(index, Q, cap, topk)).  out_survivors [Q] (may be NULL)
 * receives the true survivor count of each query; a value above cap means
 * that query's list overflowed and its result may miss neighbours.  (Two forms
 * keep no candidate lists and are complete for far more survivors than cap:
 * the grouped stage 1 of Kf <= 2 with records of at most 16 bytes and
 * topk <= 256, where the candidates never leave the chip; and, from 2^22 items
 * on with K <= 16 and topk <= 512, the item-by-item stage 1, which hands stage 2
 * one hit bit per item and query and keeps only the keys that can still reach
 * the result.)  Calls with more than 32768 queries are worked off in slices.
 */
int icq_search(const icq_index *index, const float *queries, int Q, const float *thresholds,
               int64_t cap, int topk, uint32_t *out_ids, float *out_dist, uint32_t *out_survivors,
               void *workspace, size_t workspace_bytes, void *stream);

/*
 * icq_search for callers that cannot allocate device memory or hand over a
 * workspace: code under HIP graph capture, tight serving loops, harnesses that
 * forbid hipMalloc.  Same arguments, results and kernels as icq_search, but the
 * workspace is a fixed array of ICQ_STATIC_SCRATCH_BYTES inside the library's
 * device image (every GPU the library runs on holds its copy until the process
 * ends).  The call allocates nothing and frees nothing.  The whole call must
 * fit the array at once -- icq_workspace_bytes(index, Q, cap, topk) <=
 * ICQ_STATIC_SCRATCH_BYTES -- else ICQ_ERR_SCRATCH and nothing is enqueued
 * (lower Q, cap or topk, or use icq_search with a workspace of your own).  The
 * index must live on the current device (ICQ_ERR_ARG otherwise).  All calls on
 * one GPU share that GPU's array: calls that overlap in time on one GPU -- from
 * different streams or host threads -- race; run them on one stream or order
 * them with events.  The array keeps the last call's contents; everything a
 * call reads it writes first.
 */
#define ICQ_STATIC_SCRATCH_BYTES (32 << 20)
int icq_search_static(const icq_index *index, const float *queries, int Q, const float *thresholds,
                      int64_t cap, int topk, uint32_t *out_ids, float *out_dist, uint32_t *out_survivors,
                      void *stream);

/*
 * A static threshold with the meaning of the running one of Sec. 3.4 (right
 * side of Eq. 2: crude distance of the furthest element of the nearest-
 * neighbour list, plus the margin sigma of Eq. 11).  For every query the first
 * min(M, N) items of the index all get the exact comparison; with f the
 * topk-th nearest of them by (D, id),
 *     thresholds_out[q] = P[q][f] + sigma[q]            (fp32)
 * i.e. what the paper's loop would hold after its first M items had none of
 * them been pruned.  Fewer than topk items: +inf (the list never fills).
 * sigma [Q] may be NULL (zero margin); the caller derives it from the variance
 * of its data in the subspace the slow codebooks cover.  lut [Q][K][256] as
 * written by icq_build_lut.  1 <= M <= ICQ_MAX_SAMPLE, 1 <= topk <= ICQ_MAX_TOPK.
 * Feed the result to icq_scan_fast / icq_search.
 */
int icq_sample_thresholds(const icq_index *index, const float *lut, int Q, const float *sigma, int topk,
                          int64_t M, float *thresholds_out, void *stream);

/*
 * The search loop of Sec. 3.4 with its running threshold refreshed per tile of
 * items.  The paper visits the items one by one and lets an item through to the
 * exact comparison when its crude distance is below that of the furthest
 * element f of the nearest-neighbour list plus the margin (right side of Eq. 2,
 * sigma as in Eq. 11).  Here the database is given as R tiles -- indexes over
 * consecutive ranges of item ids, created by the caller from the same codebooks
 * with the same Kf (ICQ_ERR_ARG when K, Kf, d or m differ), tile r holding the
 * items id_base[r] .. id_base[r] + N_r - 1 -- and tile r is searched like
 * icq_search with
 *     t_q = P[q][f] + sigma[q],   f = furthest element (largest (D, id)) of the
 *                                 list after tiles 0 .. r-1,
 * or t_q = +inf while that list holds fewer than topk items (every item of the
 * tile then gets the exact comparison); the tile's survivors are merged into
 * the list by (D, id) and the threshold is refreshed.  Tiles of one item each
 * would be the paper's loop itself; one tile is the exhaustive search.
 *   out_ids/out_dist [Q][topk]: the list after the last tile, ids global, as
 *                    icq_search writes them (padding included);
 *   out_refined [Q]: items that got the exact comparison, summed over the tiles
 *                    (the `refined` of icq_op_counts, which takes N from the
 *                    index it is given: one over the whole database);
 *   sigma [Q] fp32, may be NULL (zero margin); id_base is a HOST array [R];
 *   cap: candidate capacity per query and tile as in icq_search (a tile never
 *        needs more than its own item count; tiles searched while the list is
 *        not full need all of it);
 *   workspace: icq_running_workspace_bytes(tiles, R, Q, cap, topk) bytes, 256-byte
 *        aligned; tiles is a HOST array of R index handles.
 * Work is enqueued on `stream`: one table build, then per tile the two-step
 * search and one merge kernel.
 */
int icq_running_workspace_bytes(const icq_index *const *tiles /*host [R]*/, int R, int Q, int64_t cap, int topk,
                                size_t *out /*host*/);
int icq_search_running(const icq_index *const *tiles /*host [R]*/, const uint32_t *id_base /*host [R]*/, int R,
                       const float *queries, int Q, const float *sigma, int64_t cap, int topk, uint32_t *out_ids,
                       float *out_dist, uint32_t *out_refined, void *workspace, size_t workspace_bytes,
                       void *stream);

/*
 * Operation counts of the two-step search (Sec. 1: Kf table additions for every
 * item, K - Kf more for each item that gets the exact comparison, against K per
 * item for the one-step search) and the effective code length of Sec. 4.2.
 * refined [Q] = items that got the exact comparison (the out_survivors /
 * cand_count of a search); values above N count as N.
 *   ops_out[q]     = N*Kf + refined[q]*(K-Kf)            (64-bit, device)
 *   summary_out[0] = mean over the queries of ops_out    (double, device [4])
 *   summary_out[1] = N*K, [2] = [0]/[1],
 *   summary_out[3] = K*log2(m) * [2]: the code length at which the one-step
 *                    search would cost the same.
 */
int icq_op_counts(const icq_index *index, const uint32_t *refined, int Q, unsigned long long *ops_out,
                  double *summary_out, void *stream);

/*
 * Encoding, the step before the search path (Sec. 1: an item is stored as one
 * codeword index per codebook, xbar_i = sum_k c_{k,code_k(i)}).  The paper
 * gives no assignment algorithm; this is the greedy residual assignment in
 * codebook order:  r_0 = x_i;  code_k(i) = argmin_j ||r_k - c_{k,j}||^2
 * (ties: smallest j);  r_{k+1} = r_k - c_{k,code_k(i)}.  On codebooks with
 * pairwise-disjoint supports every step is the exact nearest codeword in its
 * subspace.  Scores are formed in fp32 on the matrix cores.
 * index: any index over the codebooks (it may hold no items: N = 0 at create).
 * x [N][d] fp32, codes_out [K][N] (the layout icq_index_create takes),
 * workspace of icq_encode_workspace_bytes(index, N) bytes (the residuals).
 */
int icq_encode_workspace_bytes(const icq_index *index, int64_t N, size_t *out /*host*/);
int icq_encode(const icq_index *index, const float *x, int64_t N, uint8_t *codes_out, void *workspace,
               size_t workspace_bytes, void *stream);

/*
 * Refinement of given codes by coordinate descent over the codebooks (iterated
 * conditional modes; the greedy assignment above never revisits a choice).  One
 * sweep takes the codebooks in order; with the item's other sub-codes fixed,
 *     r = x_i - sum_{l != k} c_{l,code_l(i)},   j* = argmin_j ||r - c_{k,j}||^2,
 * and code_k(i) becomes j* only if it is strictly nearer than the current
 * codeword (equal scores keep what is there), so ||x_i - xbar_i||^2 does not
 * grow beyond the rounding of the fp32 scores.  codes [K][N] in and out;
 * 0 <= sweeps <= ICQ_MAX_SWEEPS; changed_out: device [sweeps] or NULL, the
 * number of sub-codes replaced in each sweep (a sweep that replaces none has
 * reached a point no single change improves); workspace as icq_encode.
 *
 * icq_quantization_error: err_out[i] = ||x_i - xbar_i||^2 of given codes,
 * accumulated in double (device [N]).
 */
#define ICQ_MAX_SWEEPS 64
int icq_encode_refine(const icq_index *index, const float *x, int64_t N, uint8_t *codes, int sweeps,
                      uint32_t *changed_out, void *workspace, size_t workspace_bytes, void *stream);
int icq_quantization_error(const icq_index *index, const float *x, int64_t N, const uint8_t *codes,
                           double *err_out, void *stream);

/*
 * Quantities around the fast set (Sec. 3.1 - 3.4).  Small utilities, none on
 * the search path; all arrays are device memory, variances and the prior are
 * handled in double.
 *
 * icq_batch_moments: population mean and variance per dimension of a batch
 *   x [n][d] fp32 (the batch statistics of Sec. 3.2).
 * icq_online_variance_update: the two update equations of Sec. 3.2 for batch
 *   number b (1-based), in place on mean / var [d]:
 *     var  += (batch_var - var)/b + (1/b)(1 - 1/b)(batch_mean - mean)^2
 *     mean += (batch_mean - mean)/b
 * icq_subspace_mask: the vector xi of Sec. 3.1, xi_i = 1 iff
 *     pi2 * SN(lambda_i; mu2, sigma2, alpha2) > pi1 * N(lambda_i; 0, sigma1)
 *   (SN(x; mu, s, a) = (2/s) phi((x-mu)/s) Phi(a (x-mu)/s)); sigma1, sigma2 > 0.
 * icq_fast_set: the defining condition of the fast set (Sec. 3.1): codebook k
 *   is fast iff every one of its codewords c has ||c o (1-xi)|| < ||c o xi||.
 *   xi [d], fast_out [K] (1 / 0).  The caller reorders the codebooks so that
 *   the fast ones come first before it builds a search index.
 * icq_margin: sigma of Sec. 3.4's last equation with proportionality constant
 *   1, sigma_out[0] = sum of lambda_i over the dimensions with xi_i = 0: the
 *   value icq_sample_thresholds takes as margin.
 */
int icq_batch_moments(const float *x, int64_t n, int d, double *mean_out, double *var_out, void *stream);
int icq_online_variance_update(double *mean, double *var, const double *batch_mean, const double *batch_var,
                               int d, int64_t b, void *stream);
int icq_subspace_mask(const double *lambda, int d, double pi1, double sigma1, double pi2, double mu2,
                      double sigma2, double alpha2, uint8_t *xi_out, void *stream);
int icq_fast_set(const icq_index *index, const uint8_t *xi, uint8_t *fast_out, void *stream);
int icq_margin(const double *lambda, const uint8_t *xi, int d, double *sigma_out, void *stream);

/*
 * Machine-limit probe, a measurement aid (nothing on the search path uses it): runs one of a few
 * plain kernels `reps` times on `stream`, WAITS for them, and reports the mean launch time in
 * milliseconds (*ms_out, host) and the work one launch did (*units_out, host): bytes read
 * (ICQ_PROBE_READ: 128-bit loads over `buffer`, one block per CU; ICQ_PROBE_READ_NT: the same with
 * the non-temporal hint), lane reads of a conflict-free 128 KB LDS table in 4-, 8- or 16-byte
 * accesses (ICQ_PROBE_LDS_B32/B64/B128), plain single-precision vector additions
 * (ICQ_PROBE_VALU), atomic additions on one word (ICQ_PROBE_ATOMIC), or the single-precision
 * 32x32x2 matrix instruction on register operands (ICQ_PROBE_MFMA_F32: two small integers as
 * operands; ICQ_PROBE_MFMA_F32_RANDOM: pseudo-random values with full mantissas; units =
 * floating-point operations).  buffer: device memory
 * of `bytes` >= 4 MiB, 16-byte aligned; every kind may overwrite its first 4 MiB.
 */
#define ICQ_PROBE_READ 0
#define ICQ_PROBE_READ_NT 1
#define ICQ_PROBE_LDS_B32 2
#define ICQ_PROBE_LDS_B64 3
#define ICQ_PROBE_LDS_B128 4
#define ICQ_PROBE_VALU 5
#define ICQ_PROBE_ATOMIC 6
#define ICQ_PROBE_MFMA_F32 7
#define ICQ_PROBE_MFMA_F32_RANDOM 8
int icq_machine_probe(int kind, void *buffer, size_t bytes, int reps, double *ms_out /*host*/,
                      double *units_out /*host*/, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* ICQ_H */
