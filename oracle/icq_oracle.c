/*
 * icq_oracle.c -- TEST INFRASTRUCTURE, not part of the product.
 *
 * A plain, slow, double-precision CPU statement of what the ICQ query-time
 * path computes (arxiv 1912.08756): the per-query table of squared
 * query-to-codeword distances, the crude sum over the fast codebooks
 * (left side of Eq. 2), the threshold filter, the full K-term sum (left side
 * of Eq. 1) for the survivors, and the nearest-neighbour list (Sec. 3.4).
 *
 * The method reaches a result that has a plain definition (sum table entries,
 * filter, select), so every function below is that definition written out with
 * no blocking, fusion or reordering.  Nothing here is shared with the GPU
 * library: no headers, no helpers, no tables.  Only tests, the smoke check
 * and the benchmark's cpu_baseline leg may call it.
 *
 * Pins (tests/test_oracle_pins.py): the composite-quantization distance
 * identity on constant-inner-product codebooks, infinite threshold ==
 * exhaustive ADC, brute-force k-NN over reconstructions on tiny inputs, the
 * product-quantization special case, filter/select commutation, the
 * lossless-pruning invariant on codebooks with the ICQ zero pattern, Kf == K,
 * padding, and a hand-worked micro example; for the paper's serial loop:
 * infinite margin == exhaustive ADC, a margin above the spread of the slow
 * terms loses nothing, a margin of -inf keeps the first topk items, closed
 * forms on items visited in ascending order of distance, and a hand-worked
 * trace; for the sample threshold and the operation counts: closed forms; for
 * the greedy encoding: K = 1 is the plain nearest codeword, disjoint supports
 * give the sub-vector assignment and the brute-force optimum over all code
 * combinations, reconstructions encode back to their own codes; for the
 * fast-set quantities: the online variance equals the variance of the
 * concatenated batches, the two prior densities integrate to their weights and
 * the skew-normal mean has its textbook value, a symmetric special case puts the
 * boundary of psi at mu/2, codebooks built inside / outside psi are classified
 * as such.  No function here is unpinned.
 *
 * Conventions: codebooks [K][m][d] float; codes [K][N] uint8, codebook-major,
 * rows 0..Kf-1 are the fast codebooks; T [Q][K][m] double; ids are uint32;
 * an empty result slot is (0xFFFFFFFF, +inf).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

typedef struct {
    double dist;
    uint32_t id;
} pair_t;

/* Order of the nearest-neighbour list: ascending distance, ties by ascending
 * id (the paper is silent on ties; Sec. 3.4 only keeps "the nearest"). */
static int pair_cmp(const void *a, const void *b)
{
    const pair_t *x = (const pair_t *)a, *y = (const pair_t *)b;
    if (x->dist < y->dist) return -1;
    if (x->dist > y->dist) return 1;
    if (x->id < y->id) return -1;
    if (x->id > y->id) return 1;
    return 0;
}

/* Table precompute (Sec. 1, paragraph after Eq. 1; the norm is squared as in
 * Eq. 1 and Eq. 2):  T[q][k][j] = sum_e (q_e - c_{k,j,e})^2, direct form. */
void icq_oracle_lut(const float *codebooks, int K, int m, int d,
                    const float *queries, int Q, double *T)
{
#pragma omp parallel for schedule(static)
    for (int q = 0; q < Q; ++q) {
        const float *qv = queries + (size_t)q * d;
        for (int k = 0; k < K; ++k) {
            for (int j = 0; j < m; ++j) {
                const float *c = codebooks + ((size_t)k * m + j) * d;
                double s = 0.0;
                for (int e = 0; e < d; ++e) {
                    double diff = (double)qv[e] - (double)c[e];
                    s += diff * diff;
                }
                T[((size_t)q * K + k) * m + j] = s;
            }
        }
    }
}

/* Crude distance (left side of Eq. 2): P[q][i] = sum_{k in fast set} T[q][k][code_k(i)],
 * fast set = codebooks 0..Kf-1, k ascending. */
void icq_oracle_partial(const double *T, int K, int m, const uint8_t *codes,
                        int64_t N, int Kf, int Q, double *P)
{
#pragma omp parallel for schedule(static)
    for (int q = 0; q < Q; ++q) {
        const double *Tq = T + (size_t)q * K * m;
        for (int64_t i = 0; i < N; ++i) {
            double s = 0.0;
            for (int k = 0; k < Kf; ++k)
                s += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
            P[(size_t)q * N + i] = s;
        }
    }
}

/* Two-step search (Sec. 1 after Eq. 2, Sec. 3.4) with a static per-query
 * threshold in place of the running "furthest list element + sigma":
 *   survivor  <=>  P[q][i] < t_q            (strict, as in Eq. 2)
 *   D[q][i]   =    P[q][i] + sum_{k=Kf..K-1} T[q][k][code_k(i)]   (Eq. 1, left side)
 *   result    =    the topk smallest (D, id) among survivors, ascending,
 *                  padded with (0xFFFFFFFF, +inf).
 * out_count[q] = number of survivors.  P_out / D_out (each [Q][N], may be
 * NULL) receive every item's crude distance and the survivors' full distance
 * (NaN for pruned items). */
void icq_oracle_search(const double *T, int K, int m, const uint8_t *codes,
                       int64_t N, int Kf, int Q, const float *thresholds,
                       int topk, uint32_t *out_ids, double *out_dist,
                       int64_t *out_count, double *P_out, double *D_out)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < Q; ++q) {
        const double *Tq = T + (size_t)q * K * m;
        const double t = (double)thresholds[q];
        pair_t *surv = (pair_t *)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
        int64_t ns = 0;
        for (int64_t i = 0; i < N; ++i) {
            double p = 0.0;
            for (int k = 0; k < Kf; ++k)
                p += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
            if (P_out) P_out[(size_t)q * N + i] = p;
            if (D_out) D_out[(size_t)q * N + i] = NAN;
            if (p < t) {
                double dfull = p;
                for (int k = Kf; k < K; ++k)
                    dfull += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
                if (D_out) D_out[(size_t)q * N + i] = dfull;
                surv[ns].dist = dfull;
                surv[ns].id = (uint32_t)i;
                ++ns;
            }
        }
        qsort(surv, (size_t)ns, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < topk; ++r) {
            if (r < ns) {
                out_ids[(size_t)q * topk + r] = surv[r].id;
                out_dist[(size_t)q * topk + r] = surv[r].dist;
            } else {
                out_ids[(size_t)q * topk + r] = 0xFFFFFFFFu;
                out_dist[(size_t)q * topk + r] = INFINITY;
            }
        }
        out_count[q] = ns;
        free(surv);
    }
}

/* One-step exhaustive ADC (the conventional search of Sec. 3.4, first
 * paragraph): every item gets all K table terms in a single loop and the
 * whole list is sorted.  Written separately from icq_oracle_search on
 * purpose; D_all ([Q][N], may be NULL) receives every distance. */
void icq_oracle_adc_exhaustive(const double *T, int K, int m,
                               const uint8_t *codes, int64_t N, int Q, int topk,
                               uint32_t *out_ids, double *out_dist, double *D_all)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < Q; ++q) {
        pair_t *all = (pair_t *)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
        for (int64_t i = 0; i < N; ++i) {
            double s = 0.0;
            for (int k = 0; k < K; ++k) {
                int code = codes[(size_t)k * N + i];
                s += T[((size_t)q * K + k) * m + code];
            }
            all[i].dist = s;
            all[i].id = (uint32_t)i;
            if (D_all) D_all[(size_t)q * N + i] = s;
        }
        qsort(all, (size_t)N, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < topk; ++r) {
            int has = r < N;
            out_ids[(size_t)q * topk + r] = has ? all[r].id : 0xFFFFFFFFu;
            out_dist[(size_t)q * topk + r] = has ? all[r].dist : INFINITY;
        }
        free(all);
    }
}

/* The search operation as the paper states it (Sec. 3.4), a serial loop over
 * the items in index order with a list of the topk nearest found so far:
 *   - while the list is not full, an item gets the exact comparison at once
 *     (the paper does not say what "the furthest element" is before the list
 *     is full; this is the reading taken here);
 *   - afterwards let f be the furthest element of the list (largest (D, id)).
 *     Crude comparison (Eq. 2):  P(i) < P(f) + sigma_q.  Only if it holds, the
 *     exact comparison (Eq. 1, left sides): D(i) < D(f); if that holds too,
 *     i replaces f.
 * P is the sum over the fast codebooks 0..Kf-1, D adds the other K-Kf terms.
 * sigma [Q] is the margin of Eq. 2 / Eq. 11, supplied by the caller (double;
 * +inf makes the crude comparison always hold).  Output: the list ascending by
 * (D, id), padded with (0xFFFFFFFF, +inf); out_refined[q] = how many items got
 * the exact comparison (the quantity behind the paper's "average ops"). */
void icq_oracle_running_search(const double *T, int K, int m, const uint8_t *codes,
                               int64_t N, int Kf, int Q, const double *sigma, int topk,
                               uint32_t *out_ids, double *out_dist, int64_t *out_refined)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < Q; ++q) {
        const double *Tq = T + (size_t)q * K * m;
        pair_t *list = (pair_t *)malloc(sizeof(pair_t) * (size_t)topk);   /* (D, id) */
        double *listP = (double *)malloc(sizeof(double) * (size_t)topk);  /* P of the same entries */
        int len = 0;
        int64_t refined = 0;
        for (int64_t i = 0; i < N; ++i) {
            double p = 0.0;
            for (int k = 0; k < Kf; ++k)
                p += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
            int f = -1;                       /* slot of the furthest element */
            if (len == topk) {
                f = 0;
                for (int r = 1; r < len; ++r)
                    if (pair_cmp(&list[r], &list[f]) > 0) f = r;
                if (!(p < listP[f] + sigma[q])) continue;      /* pruned by the crude comparison */
            }
            double dfull = p;
            for (int k = Kf; k < K; ++k)
                dfull += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
            ++refined;
            if (f < 0) {                      /* list not full yet */
                list[len].dist = dfull; list[len].id = (uint32_t)i; listP[len] = p;
                ++len;
            } else if (dfull < list[f].dist) {
                list[f].dist = dfull; list[f].id = (uint32_t)i; listP[f] = p;
            }
        }
        qsort(list, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < topk; ++r) {
            out_ids[(size_t)q * topk + r] = r < len ? list[r].id : 0xFFFFFFFFu;
            out_dist[(size_t)q * topk + r] = r < len ? list[r].dist : INFINITY;
        }
        out_refined[q] = refined;
        free(list);
        free(listP);
    }
}

/* The loop of Sec. 3.4 with the right side of its crude comparison refreshed per
 * tile of items instead of per item (what a machine that scans a tile of items
 * in parallel can do): tile r covers the items bounds[r] .. bounds[r+1]-1
 * (bounds[0] = 0, ascending, bounds[R] = N).  At the start of a tile let f be the
 * furthest element of the list as it stands; every item of the tile meets the
 * crude comparison P(i) < P(f) + sigma_q with THAT f (no comparison while the
 * list was not full at the start of the tile: every item of the tile then gets
 * the exact comparison).  The exact comparison D(i) < D(furthest now) and the
 * replacement run item by item as in the loop.  Tiles of one item each are the
 * paper's loop itself; one tile over everything is the exhaustive search.
 * Outputs as icq_oracle_running_search. */
void icq_oracle_running_search_tiled(const double *T, int K, int m, const uint8_t *codes,
                                     int64_t N, int Kf, int Q, const double *sigma, int topk,
                                     const int64_t *bounds, int R,
                                     uint32_t *out_ids, double *out_dist, int64_t *out_refined)
{
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < Q; ++q) {
        const double *Tq = T + (size_t)q * K * m;
        pair_t *list = (pair_t *)malloc(sizeof(pair_t) * (size_t)topk);
        double *listP = (double *)malloc(sizeof(double) * (size_t)topk);
        int len = 0;
        int64_t refined = 0;
        for (int r = 0; r < R; ++r) {
            const int full_at_start = len == topk;
            double t = INFINITY;
            if (full_at_start) {
                int f = 0;
                for (int e = 1; e < len; ++e)
                    if (pair_cmp(&list[e], &list[f]) > 0) f = e;
                t = listP[f] + sigma[q];
            }
            for (int64_t i = bounds[r]; i < bounds[r + 1]; ++i) {
                double p = 0.0;
                for (int k = 0; k < Kf; ++k)
                    p += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
                if (full_at_start && !(p < t)) continue;
                double dfull = p;
                for (int k = Kf; k < K; ++k)
                    dfull += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
                ++refined;
                if (len < topk) {
                    list[len].dist = dfull; list[len].id = (uint32_t)i; listP[len] = p;
                    ++len;
                } else {
                    int f = 0;
                    for (int e = 1; e < len; ++e)
                        if (pair_cmp(&list[e], &list[f]) > 0) f = e;
                    if (dfull < list[f].dist) {
                        list[f].dist = dfull; list[f].id = (uint32_t)i; listP[f] = p;
                    }
                }
            }
        }
        qsort(list, (size_t)len, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < topk; ++r) {
            out_ids[(size_t)q * topk + r] = r < len ? list[r].id : 0xFFFFFFFFu;
            out_dist[(size_t)q * topk + r] = r < len ? list[r].dist : INFINITY;
        }
        out_refined[q] = refined;
        free(list);
        free(listP);
    }
}

/* A static threshold with the meaning of Sec. 3.4's running one: look at the
 * first M items only, give every one of them the exact comparison, let f be
 * the topk-th nearest of them by (D, id), and set
 *     t_q = P(f) + sigma_q
 * -- the right side of Eq. 2 as the paper's loop would hold it after its first
 * M items had none of them been pruned.  Fewer than topk items in the sample:
 * t_q = +inf (the list would not be full).  thr_out [Q] double. */
void icq_oracle_sample_thresholds(const double *T, int K, int m, const uint8_t *codes,
                                  int64_t N, int Kf, int Q, const double *sigma, int topk,
                                  int64_t M, double *thr_out)
{
    const int64_t n = M < N ? M : N;
#pragma omp parallel for schedule(dynamic, 1)
    for (int q = 0; q < Q; ++q) {
        if (n < topk) { thr_out[q] = INFINITY; continue; }
        const double *Tq = T + (size_t)q * K * m;
        pair_t *all = (pair_t *)malloc(sizeof(pair_t) * (size_t)n);
        for (int64_t i = 0; i < n; ++i) {
            double s = 0.0;
            for (int k = 0; k < K; ++k)
                s += Tq[(size_t)k * m + codes[(size_t)k * N + i]];
            all[i].dist = s;
            all[i].id = (uint32_t)i;
        }
        qsort(all, (size_t)n, sizeof(pair_t), pair_cmp);
        const int64_t f = all[topk - 1].id;
        double p = 0.0;
        for (int k = 0; k < Kf; ++k)
            p += Tq[(size_t)k * m + codes[(size_t)k * N + f]];
        thr_out[q] = p + sigma[q];
        free(all);
    }
}

/* Operation counts behind the paper's speed axis (Sec. 1, last sentences before
 * the contributions; Sec. 4.2, effective code length): a two-step search spends
 * Kf table additions on every item and K-Kf more on each item that gets the
 * exact comparison, the one-step search spends K on every item:
 *     ops_icq[q] = N*Kf + refined[q]*(K-Kf),      ops_adc = N*K.
 * summary[0] = mean_q ops_icq, [1] = ops_adc, [2] = their ratio,
 * [3] = effective code length  code_bits * ratio  (Sec. 4.2's l-hat with the
 * one-step search at the same code length as the reference). */
void icq_oracle_op_counts(int64_t N, int K, int Kf, int Q, const int64_t *refined,
                          double code_bits, double *ops_icq, double *summary)
{
    double sum = 0.0;
    for (int q = 0; q < Q; ++q) {
        ops_icq[q] = (double)N * (double)Kf + (double)refined[q] * (double)(K - Kf);
        sum += ops_icq[q];
    }
    summary[0] = Q > 0 ? sum / Q : 0.0;
    summary[1] = (double)N * (double)K;
    summary[2] = summary[1] > 0.0 ? summary[0] / summary[1] : 0.0;
    summary[3] = code_bits * summary[2];
}

/* Encoding (the step before the search path, Sec. 1: an item is stored as one
 * codeword index per codebook so that xbar_i = sum_k c_{k,code_k(i)}).  The
 * paper gives no assignment algorithm; this build takes the greedy residual
 * assignment in codebook order:
 *     r_0 = x_i;   code_k(i) = argmin_j || r_k - c_{k,j} ||^2  (ties: smallest j);
 *     r_{k+1} = r_k - c_{k,code_k(i)}.
 * On codebooks with pairwise-disjoint supports (the ICQ zero pattern taken to
 * its limit) a codeword only touches its own coordinates, so every step is the
 * exact nearest codeword in its subspace and the result minimises
 * ||x_i - xbar_i||^2 over all code combinations.  x [N][d] float;
 * codes_out [K][N]; err_out [N] (may be NULL) = ||r_K||^2 = ||x_i - xbar_i||^2. */
void icq_oracle_encode(const float *codebooks, int K, int m, int d, const float *x,
                       int64_t N, uint8_t *codes_out, double *err_out)
{
#pragma omp parallel
    {
        double *r = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static)
        for (int64_t i = 0; i < N; ++i) {
            for (int e = 0; e < d; ++e) r[e] = (double)x[(size_t)i * d + e];
            for (int k = 0; k < K; ++k) {
                int best = 0;
                double best_s = INFINITY;
                for (int j = 0; j < m; ++j) {
                    const float *c = codebooks + ((size_t)k * m + j) * d;
                    double s = 0.0;
                    for (int e = 0; e < d; ++e) {
                        double diff = r[e] - (double)c[e];
                        s += diff * diff;
                    }
                    if (s < best_s) { best_s = s; best = j; }
                }
                codes_out[(size_t)k * N + i] = (uint8_t)best;
                const float *c = codebooks + ((size_t)k * m + best) * d;
                for (int e = 0; e < d; ++e) r[e] -= (double)c[e];
            }
            if (err_out) {
                double s = 0.0;
                for (int e = 0; e < d; ++e) s += r[e] * r[e];
                err_out[i] = s;
            }
        }
        free(r);
    }
}

/* ||x_i - xbar_i||^2 of given codes (Sec. 1: xbar_i = sum_k c_{k,code_k(i)}; the quantity
 * the quantizers of Sec. 2 minimise).  codes [K][N]; err_out [N]. */
void icq_oracle_quantization_error(const float *codebooks, int K, int m, int d, const float *x,
                                   int64_t N, const uint8_t *codes, double *err_out)
{
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; ++i) {
        double s = 0.0;
        for (int e = 0; e < d; ++e) {
            double xb = 0.0;
            for (int k = 0; k < K; ++k)
                xb += (double)codebooks[((size_t)k * m + codes[(size_t)k * N + i]) * d + e];
            const double diff = (double)x[(size_t)i * d + e] - xb;
            s += diff * diff;
        }
        err_out[i] = s;
    }
}

/* Refinement of given codes by coordinate descent over the codebooks (iterated
 * conditional modes; the paper gives no assignment algorithm, and the greedy
 * assignment above never revisits a choice).  One sweep takes the codebooks in
 * order k = 0 .. K-1; with all other sub-codes of the item fixed,
 *     r = x_i - sum_{l != k} c_{l,code_l(i)},
 *     j* = argmin_j || r - c_{k,j} ||^2   (smallest j among exact minima),
 * and code_k(i) becomes j* only if that is strictly nearer than the current
 * codeword (so ||x_i - xbar_i||^2 never grows, and equal choices keep what is
 * there).  r is formed from scratch for every step.  codes [K][N] in and out;
 * changed_out [sweeps] (may be NULL) = sub-codes changed in each sweep. */
void icq_oracle_encode_icm(const float *codebooks, int K, int m, int d, const float *x,
                           int64_t N, uint8_t *codes, int sweeps, int64_t *changed_out)
{
    for (int sw = 0; sw < sweeps; ++sw) {
        int64_t changed = 0;
#pragma omp parallel
        {
            double *r = (double *)malloc(sizeof(double) * (size_t)d);
#pragma omp for schedule(static) reduction(+ : changed)
            for (int64_t i = 0; i < N; ++i) {
                for (int k = 0; k < K; ++k) {
                    for (int e = 0; e < d; ++e) {
                        double others = 0.0;
                        for (int l = 0; l < K; ++l)
                            if (l != k)
                                others += (double)codebooks[((size_t)l * m + codes[(size_t)l * N + i]) * d + e];
                        r[e] = (double)x[(size_t)i * d + e] - others;
                    }
                    const int old = codes[(size_t)k * N + i];
                    int best = 0;
                    double best_s = INFINITY, old_s = INFINITY;
                    for (int j = 0; j < m; ++j) {
                        const float *c = codebooks + ((size_t)k * m + j) * d;
                        double sq = 0.0;
                        for (int e = 0; e < d; ++e) {
                            const double diff = r[e] - (double)c[e];
                            sq += diff * diff;
                        }
                        if (sq < best_s) { best_s = sq; best = j; }
                        if (j == old) old_s = sq;
                    }
                    if (best_s < old_s) {
                        codes[(size_t)k * N + i] = (uint8_t)best;
                        ++changed;
                    }
                }
            }
            free(r);
        }
        if (changed_out) changed_out[sw] = changed;
    }
}

/* ---- quantities around the fast set (Sec. 3.1 - 3.4); none is on the search path ---- */

/* Population mean and variance of a batch per dimension (what Sec. 3.2 calls the
 * sample mean and variance of a batch), two passes.  x [n][d]. */
void icq_oracle_batch_moments(const float *x, int64_t n, int d, double *mean, double *var)
{
    for (int e = 0; e < d; ++e) {
        double s = 0.0;
        for (int64_t i = 0; i < n; ++i) s += (double)x[(size_t)i * d + e];
        const double mu = n > 0 ? s / (double)n : 0.0;
        double v = 0.0;
        for (int64_t i = 0; i < n; ++i) {
            const double t = (double)x[(size_t)i * d + e] - mu;
            v += t * t;
        }
        mean[e] = mu;
        var[e] = n > 0 ? v / (double)n : 0.0;
    }
}

/* Online estimate of the dataset variance from batch statistics (Sec. 3.2, the
 * two update equations): with b the 1-based number of the batch just seen,
 *   Lambda_b = Lambda_{b-1} + (Lambda_batch - Lambda_{b-1})/b + (1/b)(1 - 1/b)(M_batch - M_{b-1})^2
 *   M_b      = M_{b-1} + (M_batch - M_{b-1})/b
 * (b = 1 makes the state equal to the batch).  mean / var [d] are updated in place. */
void icq_oracle_online_variance(double *mean, double *var, const double *batch_mean,
                                const double *batch_var, int d, int64_t b)
{
    const double w = 1.0 / (double)b;
    for (int e = 0; e < d; ++e) {
        const double dm = batch_mean[e] - mean[e];
        var[e] = var[e] + w * (batch_var[e] - var[e]) + w * (1.0 - w) * dm * dm;
        mean[e] = mean[e] + w * dm;
    }
}

/* High-variance subspace psi (Sec. 3.1): dimension i belongs to psi iff the minor,
 * skew-normal mode of the prior explains its variance better than the major, zero-centred
 * normal mode:  pi2 * SN(lambda_i; mu2, sigma2, alpha2) > pi1 * N(lambda_i; 0, sigma1), with
 *   N(x; 0, s)       = exp(-x^2 / (2 s^2)) / (s sqrt(2 pi))
 *   SN(x; mu, s, a)  = (2/s) phi(z) Phi(a z),  z = (x - mu)/s,  phi / Phi the standard normal
 *                      density / distribution function.
 * xi [d] = 1 inside psi, 0 outside (the vector xi of the paper); p_major / p_minor [d] (may be
 * NULL) receive the two weighted densities. */
void icq_oracle_subspace_mask(const double *lambda, int d, double pi1, double sigma1, double pi2,
                              double mu2, double sigma2, double alpha2, uint8_t *xi,
                              double *p_major, double *p_minor)
{
    const double inv_sqrt_2pi = 0.3989422804014327;
    for (int i = 0; i < d; ++i) {
        const double x = lambda[i];
        const double pm = pi1 * inv_sqrt_2pi / sigma1 * exp(-0.5 * (x / sigma1) * (x / sigma1));
        const double z = (x - mu2) / sigma2;
        const double phi = inv_sqrt_2pi * exp(-0.5 * z * z);
        const double Phi = 0.5 * erfc(-alpha2 * z / 1.4142135623730951);
        const double pn = pi2 * 2.0 / sigma2 * phi * Phi;
        xi[i] = pn > pm ? 1 : 0;
        if (p_major) p_major[i] = pm;
        if (p_minor) p_minor[i] = pn;
    }
}

/* The fast set (Sec. 3.1, the definition after the joint objective): codebook k is fast iff
 * EVERY one of its codewords has more norm inside psi than outside,
 *   || c o (1 - xi) || < || c o xi ||.   fast [K] = 1 / 0. */
void icq_oracle_fast_set(const float *codebooks, int K, int m, int d, const uint8_t *xi,
                         uint8_t *fast)
{
    for (int k = 0; k < K; ++k) {
        int all = 1;
        for (int j = 0; j < m; ++j) {
            const float *c = codebooks + ((size_t)k * m + j) * d;
            double in = 0.0, out = 0.0;
            for (int e = 0; e < d; ++e) {
                const double v = (double)c[e] * (double)c[e];
                if (xi[e]) in += v; else out += v;
            }
            if (!(out < in)) all = 0;
        }
        fast[k] = (uint8_t)all;
    }
}

/* Margin of the crude comparison (Sec. 3.4, last equation; the constant of proportionality
 * taken as 1, the index set read as the dimensions outside psi):  sigma = sum_{xi_i = 0} lambda_i. */
double icq_oracle_margin(const double *lambda, const uint8_t *xi, int d)
{
    double s = 0.0;
    for (int i = 0; i < d; ++i)
        if (!xi[i]) s += lambda[i];
    return s;
}

/* Reconstruction (Sec. 1): xbar_i = sum_k c_{k, code_k(i)} for the listed items. */
void icq_oracle_reconstruct(const float *codebooks, int K, int m, int d,
                            const uint8_t *codes, int64_t N, const int64_t *items,
                            int64_t n_items, double *xbar)
{
    for (int64_t r = 0; r < n_items; ++r) {
        int64_t i = items[r];
        double *x = xbar + (size_t)r * d;
        for (int e = 0; e < d; ++e) x[e] = 0.0;
        for (int k = 0; k < K; ++k) {
            const float *c = codebooks + ((size_t)k * m + codes[(size_t)k * N + i]) * d;
            for (int e = 0; e < d; ++e) x[e] += (double)c[e];
        }
    }
}

/* Exact k-NN over the reconstructions: ||q - xbar_i||^2 by brute force
 * (right side of Eq. 1), sorted by (distance, id). */
void icq_oracle_bruteforce_knn(const float *codebooks, int K, int m, int d,
                               const uint8_t *codes, int64_t N, const float *queries,
                               int Q, int topk, uint32_t *out_ids, double *out_dist)
{
    double *x = (double *)malloc(sizeof(double) * (size_t)d);
    pair_t *all = (pair_t *)malloc(sizeof(pair_t) * (size_t)(N > 0 ? N : 1));
    for (int q = 0; q < Q; ++q) {
        const float *qv = queries + (size_t)q * d;
        for (int64_t i = 0; i < N; ++i) {
            icq_oracle_reconstruct(codebooks, K, m, d, codes, N, &i, 1, x);
            double s = 0.0;
            for (int e = 0; e < d; ++e) {
                double diff = (double)qv[e] - x[e];
                s += diff * diff;
            }
            all[i].dist = s;
            all[i].id = (uint32_t)i;
        }
        qsort(all, (size_t)N, sizeof(pair_t), pair_cmp);
        for (int r = 0; r < topk; ++r) {
            int has = r < N;
            out_ids[(size_t)q * topk + r] = has ? all[r].id : 0xFFFFFFFFu;
            out_dist[(size_t)q * topk + r] = has ? all[r].dist : INFINITY;
        }
    }
    free(all);
    free(x);
}

/* Number of OpenMP threads a parallel region here would use (for reporting). */
#ifdef _OPENMP
#include <omp.h>
int icq_oracle_threads(void) { return omp_get_max_threads(); }
#else
int icq_oracle_threads(void) { return 1; }
#endif
