/* Host-side sanitizer run of the CPU oracle.  TEST INFRASTRUCTURE, like the oracle itself.
 *
 * This program includes icq_oracle.c (one translation unit), calls every oracle function on small
 * seeded inputs whose sizes sit on the awkward spots -- no items, one item, fewer items than the
 * list is long, thresholds that keep nothing / everything, many equal distances, a sample larger
 * than the index -- and prints every result.  The test builds it twice, plainly and with
 * -fsanitize=address,undefined -fno-sanitize-recover=all, runs both and compares the output: the
 * sanitized run must end with status 0 (no out-of-bounds access, no undefined behaviour in the
 * qsort comparators, the [K][N] index arithmetic or the OpenMP loops) and print the same numbers.
 * Inputs come from a 64-bit linear congruential generator: data only, none of the method's steps.
 */
#include "icq_oracle.c"

#include <stdio.h>

static uint64_t rng_state = 0x1912087560000001ull;
static uint32_t rnd(void)
{
    rng_state = rng_state * 6364136223846793005ull + 1442695040888963407ull;
    return (uint32_t)(rng_state >> 33);
}
static float rnd_float(void) { return (float)((double)rnd() / 2147483648.0 * 2.0 - 1.0); }

static void print_u32(const char *tag, const uint32_t *v, size_t n)
{
    printf("%s", tag);
    for (size_t i = 0; i < n; ++i) printf(" %u", v[i]);
    printf("\n");
}
static void print_f64(const char *tag, const double *v, size_t n)
{
    printf("%s", tag);
    for (size_t i = 0; i < n; ++i) printf(" %.17g", v[i]);
    printf("\n");
}
static void print_i64(const char *tag, const int64_t *v, size_t n)
{
    printf("%s", tag);
    for (size_t i = 0; i < n; ++i) printf(" %lld", (long long)v[i]);
    printf("\n");
}

static void one_case(int K, int Kf, int m, int d, int64_t N, int Q, int topk, int coarse)
{
    printf("case K=%d Kf=%d m=%d d=%d N=%lld Q=%d topk=%d coarse=%d\n", K, Kf, m, d, (long long)N, Q, topk, coarse);
    const size_t nn = (size_t)(N > 0 ? N : 1);
    float *cb = (float *)malloc(sizeof(float) * (size_t)K * m * d);
    uint8_t *codes = (uint8_t *)malloc((size_t)K * nn);
    float *queries = (float *)malloc(sizeof(float) * (size_t)Q * d);
    /* coarse: codeword entries from {-1, 0, 1}, so that many table sums are exactly equal (ties) */
    for (size_t i = 0; i < (size_t)K * m * d; ++i) cb[i] = coarse ? (float)((int)(rnd() % 3) - 1) : rnd_float();
    for (size_t i = 0; i < (size_t)K * nn; ++i) codes[i] = (uint8_t)(rnd() % (uint32_t)m);
    for (size_t i = 0; i < (size_t)Q * d; ++i) queries[i] = coarse ? (float)((int)(rnd() % 3) - 1) : rnd_float();

    double *T = (double *)malloc(sizeof(double) * (size_t)Q * K * m);
    icq_oracle_lut(cb, K, m, d, queries, Q, T);
    print_f64("lut", T, (size_t)Q * K * m < 24 ? (size_t)Q * K * m : 24);

    double *P = (double *)malloc(sizeof(double) * (size_t)Q * nn);
    double *D = (double *)malloc(sizeof(double) * (size_t)Q * nn);
    icq_oracle_partial(T, K, m, codes, N, Kf, Q, P);
    if (N > 0) print_f64("partial", P, (size_t)Q * N < 16 ? (size_t)Q * N : 16);

    float *thr = (float *)malloc(sizeof(float) * (size_t)Q);
    for (int q = 0; q < Q; ++q) {
        /* the median crude distance, then the special values in turn */
        float t = N > 0 ? (float)P[(size_t)q * N + (size_t)(N / 2)] : 0.0f;
        if (q % 5 == 1) t = INFINITY;
        if (q % 5 == 2) t = -INFINITY;
        if (q % 5 == 3) t = NAN;
        thr[q] = t;
    }
    uint32_t *ids = (uint32_t *)malloc(sizeof(uint32_t) * (size_t)Q * topk);
    double *dist = (double *)malloc(sizeof(double) * (size_t)Q * topk);
    int64_t *cnt = (int64_t *)malloc(sizeof(int64_t) * (size_t)Q);
    icq_oracle_search(T, K, m, codes, N, Kf, Q, thr, topk, ids, dist, cnt, P, D);
    print_u32("search ids", ids, (size_t)Q * topk);
    print_f64("search dist", dist, (size_t)Q * topk);
    print_i64("search count", cnt, (size_t)Q);
    icq_oracle_search(T, K, m, codes, N, Kf, Q, thr, topk, ids, dist, cnt, NULL, NULL);
    print_i64("search count again", cnt, (size_t)Q);

    icq_oracle_adc_exhaustive(T, K, m, codes, N, Q, topk, ids, dist, D);
    print_u32("exhaustive ids", ids, (size_t)Q * topk);
    print_f64("exhaustive dist", dist, (size_t)Q * topk);

    double *sigma = (double *)malloc(sizeof(double) * (size_t)Q);
    for (int q = 0; q < Q; ++q) sigma[q] = q % 4 == 0 ? 0.0 : q % 4 == 1 ? 0.5 : q % 4 == 2 ? INFINITY : -INFINITY;
    int64_t *refined = (int64_t *)malloc(sizeof(int64_t) * (size_t)Q);
    icq_oracle_running_search(T, K, m, codes, N, Kf, Q, sigma, topk, ids, dist, refined);
    print_u32("running ids", ids, (size_t)Q * topk);
    print_i64("running refined", refined, (size_t)Q);
    {
        /* an empty tile, a tile shorter than the list, ragged ones, the rest */
        int64_t bounds[6];
        bounds[0] = 0; bounds[1] = 0; bounds[2] = topk / 2 < N ? topk / 2 : N; bounds[3] = N / 3 > bounds[2] ? N / 3 : bounds[2];
        bounds[4] = N / 3 * 2 + 1 > bounds[3] && N / 3 * 2 + 1 <= N ? N / 3 * 2 + 1 : bounds[3]; bounds[5] = N;
        icq_oracle_running_search_tiled(T, K, m, codes, N, Kf, Q, sigma, topk, bounds, 5, ids, dist, refined);
        print_u32("tiled running ids", ids, (size_t)Q * topk);
        print_i64("tiled running refined", refined, (size_t)Q);
    }

    double *thr_out = (double *)malloc(sizeof(double) * (size_t)Q);
    icq_oracle_sample_thresholds(T, K, m, codes, N, Kf, Q, sigma, topk, N / 2 + 3, thr_out);
    print_f64("sampled thresholds", thr_out, (size_t)Q);
    icq_oracle_sample_thresholds(T, K, m, codes, N, Kf, Q, sigma, topk, 4 * N + 7, thr_out);
    print_f64("sampled thresholds, whole index", thr_out, (size_t)Q);

    double *ops = (double *)malloc(sizeof(double) * (size_t)Q), summary[4];
    icq_oracle_op_counts(N, K, Kf, Q, refined, 8.0 * K, ops, summary);
    print_f64("ops", ops, (size_t)Q);
    print_f64("ops summary", summary, 4);

    if (N > 0) {
        const int64_t n_items = N < 5 ? N : 5;
        int64_t items[5];
        for (int64_t r = 0; r < n_items; ++r) items[r] = (int64_t)(rnd() % (uint32_t)N);
        double *xbar = (double *)malloc(sizeof(double) * (size_t)n_items * d);
        icq_oracle_reconstruct(cb, K, m, d, codes, N, items, n_items, xbar);
        print_f64("reconstruct", xbar, (size_t)n_items * d < 12 ? (size_t)n_items * d : 12);
        /* encode the reconstructions (as float) and a few random vectors */
        float *x = (float *)malloc(sizeof(float) * (size_t)(n_items + 3) * d);
        for (size_t i = 0; i < (size_t)n_items * d; ++i) x[i] = (float)xbar[i];
        for (size_t i = (size_t)n_items * d; i < (size_t)(n_items + 3) * d; ++i) x[i] = rnd_float();
        uint8_t *enc = (uint8_t *)malloc((size_t)K * (size_t)(n_items + 3));
        double *err = (double *)malloc(sizeof(double) * (size_t)(n_items + 3));
        icq_oracle_encode(cb, K, m, d, x, n_items + 3, enc, err);
        printf("encode");
        for (size_t i = 0; i < (size_t)K * (size_t)(n_items + 3); ++i) printf(" %u", enc[i]);
        printf("\n");
        print_f64("encode err", err, (size_t)(n_items + 3));
        icq_oracle_encode(cb, K, m, d, x, n_items + 3, enc, NULL);
        {
            int64_t changed[3];
            for (size_t i = 0; i < (size_t)K * (size_t)(n_items + 3); ++i) enc[i] = (uint8_t)(rnd() % (uint32_t)m);
            icq_oracle_quantization_error(cb, K, m, d, x, n_items + 3, enc, err);
            print_f64("error of random codes", err, (size_t)(n_items + 3));
            icq_oracle_encode_icm(cb, K, m, d, x, n_items + 3, enc, 3, changed);
            print_i64("icm changed", changed, 3);
            icq_oracle_encode_icm(cb, K, m, d, x, n_items + 3, enc, 0, NULL);
            icq_oracle_quantization_error(cb, K, m, d, x, n_items + 3, enc, err);
            print_f64("error after icm", err, (size_t)(n_items + 3));
        }
        free(xbar); free(x); free(enc); free(err);
    }
    icq_oracle_bruteforce_knn(cb, K, m, d, codes, N, queries, Q, topk, ids, dist);
    print_u32("bruteforce ids", ids, (size_t)Q * topk);

    /* the quantities around the fast set */
    double *mean = (double *)malloc(sizeof(double) * (size_t)d), *var = (double *)malloc(sizeof(double) * (size_t)d);
    double *bm = (double *)malloc(sizeof(double) * (size_t)d), *bv = (double *)malloc(sizeof(double) * (size_t)d);
    icq_oracle_batch_moments(queries, Q, d, mean, var);
    for (int b = 2; b <= 3; ++b) {
        icq_oracle_batch_moments(queries, Q / b + 1 <= Q ? Q / b + 1 : Q, d, bm, bv);
        icq_oracle_online_variance(mean, var, bm, bv, d, b);
    }
    print_f64("online mean", mean, (size_t)d < 8 ? (size_t)d : 8);
    print_f64("online var", var, (size_t)d < 8 ? (size_t)d : 8);
    uint8_t *xi = (uint8_t *)malloc((size_t)d), *fast = (uint8_t *)malloc((size_t)K);
    double *pa = (double *)malloc(sizeof(double) * (size_t)d), *pb = (double *)malloc(sizeof(double) * (size_t)d);
    icq_oracle_subspace_mask(var, d, 0.9, 0.05, 0.1, 0.3, 0.2, -10.0, xi, pa, pb);
    icq_oracle_subspace_mask(var, d, 0.9, 0.05, 0.1, 0.3, 0.2, -10.0, xi, NULL, NULL);
    printf("xi");
    for (int e = 0; e < d; ++e) printf(" %u", xi[e]);
    printf("\n");
    icq_oracle_fast_set(cb, K, m, d, xi, fast);
    printf("fast");
    for (int k = 0; k < K; ++k) printf(" %u", fast[k]);
    printf("\n");
    printf("margin %.17g\n", icq_oracle_margin(var, xi, d));

    free(cb); free(codes); free(queries); free(T); free(P); free(D); free(thr); free(ids); free(dist);
    free(cnt); free(sigma); free(refined); free(thr_out); free(ops); free(mean); free(var); free(bm);
    free(bv); free(xi); free(fast); free(pa); free(pb);
}

int main(void)
{
    one_case(4, 1, 256, 8, 1000, 7, 10, 0);
    one_case(8, 2, 256, 5, 333, 5, 100, 0);      /* ragged sizes */
    one_case(3, 3, 7, 3, 50, 6, 60, 1);          /* Kf == K, list longer than the index, ties */
    one_case(5, 2, 256, 4, 1, 3, 4, 0);          /* one item */
    one_case(2, 1, 2, 2, 0, 4, 3, 0);            /* no items */
    one_case(16, 4, 256, 6, 4097, 9, 100, 1);    /* K = 16, Kf = 4, many equal distances */
    printf("threads %d\n", icq_oracle_threads() > 0);
    return 0;
}
