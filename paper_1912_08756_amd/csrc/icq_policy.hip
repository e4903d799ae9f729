// Threshold policy and operation counts around the two-step search of arxiv
// 1912.08756.
//
// Sec. 3.4 prunes with a running threshold: the crude distance of the furthest
// element of the nearest-neighbour list plus the margin sigma (right side of
// Eq. 2, sigma as in Eq. 11).  The search kernels here take a static threshold
// per query instead, and icq_sample_thresholds derives one with the same
// meaning from the first M items: every one of them gets the exact comparison,
// f is the topk-th nearest of them by (D, id), and t_q = P(f) + sigma_q -- what
// the paper's loop would hold after its first M items had none been pruned.
//
// icq_op_counts turns survivor counts into the table additions the paper's speed
// axis counts (Sec. 1: Kf per item plus K - Kf per item that gets the exact
// comparison, against K per item for the one-step search) and the effective code
// length of Sec. 4.2.
#include "icq_internal.h"
#include "icq_sort.h"

#include <math.h>

namespace {

constexpr int SP_THREADS = ICQ_SORT_THREADS;

constexpr int SP_LPT = ICQ_MAX_SAMPLE / SP_THREADS;    // sample items per thread
static_assert(ICQ_MAX_SAMPLE % SP_THREADS == 0 && SP_LPT <= 32, "one flag bit per item of a thread");

// One block per query; thread t owns sample items u * SP_THREADS + t.  LDS: the K tables.
// The topk-th nearest by (D, id) comes from two exact radix selects: the topk-th smallest
// distance word, then -- among the items at exactly that distance -- the id that completes
// the count (usually the only one).
__global__ __launch_bounds__(SP_THREADS) void sample_threshold_kernel(
    const uint8_t *__restrict__ items, int stride, int K, int Kf, const float *__restrict__ lut,
    const float *__restrict__ sigma, int topk, int n, float *__restrict__ thr_out) {
    extern __shared__ __attribute__((aligned(16))) float sp_smem[];
    __shared__ IcqKthShared kth;
    __shared__ uint32_t s_below[SP_THREADS / 64];
    float *T = sp_smem;
    const int q = blockIdx.x, tid = threadIdx.x;
    const uint32_t lane = (uint32_t)tid & 63u;
    const int wave = tid >> 6;
    const float *Tq = lut + (int64_t)q * K * ICQ_LUT_W;
    for (int i = tid; i < K * ICQ_LUT_W; i += SP_THREADS) T[i] = Tq[i];
    __syncthreads();
    uint32_t v[SP_LPT], ok = 0;
#pragma unroll
    for (int u = 0; u < SP_LPT; ++u) {
        const int i = u * SP_THREADS + tid;
        v[u] = 0;
        if (i < n) {
            // the record word by word (records are 4-byte aligned); k ascending, as in the search kernels
            const uint32_t *rec = reinterpret_cast<const uint32_t *>(items + (size_t)i * stride);
            float d = 0.0f;
            for (int w = 0; w * 4 < K; ++w) {
                const uint32_t word = rec[w];
#pragma unroll
                for (int b = 0; b < 4; ++b) {
                    const int k = w * 4 + b;
                    if (k < K) {
                        const float e = T[k * ICQ_LUT_W + ((word >> (8 * b)) & 0xffu)];
                        d = k == 0 ? e : d + e;
                    }
                }
            }
            v[u] = icq_order_bits(d);
            ok |= 1u << u;
        }
    }
    const uint32_t cut = block_kth<SP_LPT>(kth, v, ok, (uint32_t)topk, true, tid, lane, wave);
    // items nearer than the cut, and the ids of those at it
    uint32_t below = 0, eq = 0, ids[SP_LPT];
#pragma unroll
    for (int u = 0; u < SP_LPT; ++u) {
        ids[u] = (uint32_t)(u * SP_THREADS + tid);
        if (((ok >> u) & 1u) && v[u] < cut) ++below;
        if (((ok >> u) & 1u) && v[u] == cut) eq |= 1u << u;
    }
#pragma unroll
    for (int d = 32; d > 0; d >>= 1) below += __shfl_xor(below, d, 64);
    __syncthreads();
    if (lane == 0) s_below[wave] = below;
    __syncthreads();
    uint32_t total_below = 0;
#pragma unroll
    for (int w = 0; w < SP_THREADS / 64; ++w) total_below += s_below[w];
    const uint32_t f = block_kth<SP_LPT>(kth, ids, eq, (uint32_t)topk - total_below, true, tid, lane, wave);
    if (tid == 0) {
        const uint8_t *rec = items + (size_t)f * stride;
        float p = T[rec[0]];
        for (int k = 1; k < Kf; ++k) p += T[k * ICQ_LUT_W + rec[k]];
        thr_out[q] = p + (sigma ? sigma[q] : 0.0f);
    }
}

__global__ void fill_float_kernel(float *__restrict__ p, int n, float v) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// One block: ops[q] for every query, then the summary from the exact integer sum.
__global__ __launch_bounds__(1024) void op_counts_kernel(const uint32_t *__restrict__ refined, int Q,
                                                         unsigned long long N, int K, int Kf, double code_bits,
                                                         unsigned long long *__restrict__ ops,
                                                         double *__restrict__ summary) {
    __shared__ unsigned long long part[1024];
    unsigned long long sum = 0;
    for (int q = threadIdx.x; q < Q; q += 1024) {
        unsigned long long r = refined[q];
        if (r > N) r = N;                              // a survivor count never exceeds N; guards stale input
        const unsigned long long o = N * (unsigned long long)Kf + r * (unsigned long long)(K - Kf);
        ops[q] = o;
        sum += o;
    }
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int d = 512; d > 0; d >>= 1) {
        if ((int)threadIdx.x < d) part[threadIdx.x] += part[threadIdx.x + d];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        const double mean = Q > 0 ? (double)part[0] / (double)Q : 0.0;
        const double adc = (double)N * (double)K;
        const double ratio = adc > 0.0 ? mean / adc : 0.0;
        summary[0] = mean;
        summary[1] = adc;
        summary[2] = ratio;
        summary[3] = code_bits * ratio;
    }
}

// ---- quantities around the fast set (Sec. 3.1 - 3.4); small, none on the search path

// One block per dimension: population mean and variance of x[:, e], two passes, double.
__global__ __launch_bounds__(256) void batch_moments_kernel(const float *__restrict__ x, long long n, int d,
                                                            double *__restrict__ mean, double *__restrict__ var) {
    __shared__ double part[256];
    const int e = blockIdx.x, tid = threadIdx.x;
    auto block_sum = [&](double v) {
        __syncthreads();
        part[tid] = v;
        __syncthreads();
        for (int s = 128; s > 0; s >>= 1) {
            if (tid < s) part[tid] += part[tid + s];
            __syncthreads();
        }
        return part[0];
    };
    double s = 0.0;
    for (long long i = tid; i < n; i += 256) s += (double)x[i * d + e];
    const double mu = n > 0 ? block_sum(s) / (double)n : 0.0;
    double v = 0.0;
    for (long long i = tid; i < n; i += 256) {
        const double t = (double)x[i * d + e] - mu;
        v += t * t;
    }
    const double vs = block_sum(v);
    if (tid == 0) {
        mean[e] = mu;
        var[e] = n > 0 ? vs / (double)n : 0.0;
    }
}

__global__ void online_variance_kernel(double *__restrict__ mean, double *__restrict__ var,
                                       const double *__restrict__ bmean, const double *__restrict__ bvar, int d,
                                       double w) {
    const int e = blockIdx.x * blockDim.x + threadIdx.x;
    if (e >= d) return;
    const double dm = bmean[e] - mean[e];
    var[e] = var[e] + w * (bvar[e] - var[e]) + w * (1.0 - w) * dm * dm;
    mean[e] = mean[e] + w * dm;
}

__global__ void subspace_mask_kernel(const double *__restrict__ lambda, int d, double pi1, double sigma1, double pi2,
                                     double mu2, double sigma2, double alpha2, uint8_t *__restrict__ xi) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= d) return;
    const double inv_sqrt_2pi = 0.3989422804014327;
    const double x = lambda[i];
    const double pm = pi1 * inv_sqrt_2pi / sigma1 * exp(-0.5 * (x / sigma1) * (x / sigma1));
    const double z = (x - mu2) / sigma2;
    const double phi = inv_sqrt_2pi * exp(-0.5 * z * z);
    const double Phi = 0.5 * erfc(-alpha2 * z / 1.4142135623730951);
    xi[i] = pi2 * 2.0 / sigma2 * phi * Phi > pm ? 1 : 0;
}

// One block per codebook, one wavefront per codeword at a time: norm inside / outside psi in double.
__global__ __launch_bounds__(256) void fast_set_kernel(const float *__restrict__ cb, int m, int d, int d_pad,
                                                       const uint8_t *__restrict__ xi, uint8_t *__restrict__ fast) {
    __shared__ int s_bad;
    const int k = blockIdx.x, tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    if (tid == 0) s_bad = 0;
    __syncthreads();
    for (int j = wave; j < m; j += 4) {
        const float *c = cb + ((size_t)k * ICQ_LUT_W + j) * d_pad;
        double in = 0.0, out = 0.0;
        for (int e = lane; e < d; e += 64) {
            const double v = (double)c[e] * (double)c[e];
            if (xi[e]) in += v; else out += v;
        }
        for (int off = 32; off > 0; off >>= 1) {
            in += __shfl_xor(in, off, 64);
            out += __shfl_xor(out, off, 64);
        }
        if (lane == 0 && !(out < in)) atomicOr(&s_bad, 1);
    }
    __syncthreads();
    if (tid == 0) fast[k] = s_bad ? 0 : 1;
}

__global__ __launch_bounds__(256) void margin_kernel(const double *__restrict__ lambda, const uint8_t *__restrict__ xi,
                                                     int d, double *__restrict__ out) {
    __shared__ double part[256];
    double s = 0.0;
    for (int i = threadIdx.x; i < d; i += 256)
        if (!xi[i]) s += lambda[i];
    part[threadIdx.x] = s;
    __syncthreads();
    for (int st = 128; st > 0; st >>= 1) {
        if ((int)threadIdx.x < st) part[threadIdx.x] += part[threadIdx.x + st];
        __syncthreads();
    }
    if (threadIdx.x == 0) out[0] = part[0];
}

}  // namespace

ICQ_EXPORT int icq_sample_thresholds(const icq_index *ix, const float *lut, int Q, const float *sigma,
                                     int topk, int64_t M, float *thresholds_out, void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || topk < 1 || topk > ICQ_MAX_TOPK || M < 1 || M > ICQ_MAX_SAMPLE)
        return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if (!lut || !thresholds_out) return ICQ_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    const int n = (int)(M < ix->N ? M : ix->N);
    if (n < topk) {   // the list would never fill: nothing is pruned
        fill_float_kernel<<<(Q + 255) / 256, 256, 0, s>>>(thresholds_out, Q, INFINITY);
        return icq_check_launch();
    }
    const size_t lds = sizeof(float) * (size_t)ix->K * ICQ_LUT_W;
    ICQ_HIP_TRY(icq_allow_lds(reinterpret_cast<const void *>(&sample_threshold_kernel), 65536));
    sample_threshold_kernel<<<Q, SP_THREADS, lds, s>>>(ix->items, ix->item_stride, ix->K, ix->Kf, lut, sigma,
                                                       topk, n, thresholds_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_op_counts(const icq_index *ix, const uint32_t *refined, int Q, unsigned long long *ops_out,
                             double *summary_out, void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || !summary_out) return ICQ_ERR_ARG;
    if (Q > 0 && (!refined || !ops_out)) return ICQ_ERR_ARG;
    const double code_bits = (double)ix->K * log2((double)ix->m);
    op_counts_kernel<<<1, 1024, 0, (hipStream_t)stream>>>(refined, Q, (unsigned long long)ix->N, ix->K, ix->Kf,
                                                          code_bits, ops_out, summary_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_batch_moments(const float *x, int64_t n, int d, double *mean_out, double *var_out, void *stream) {
    if (n < 0 || d < 1 || d > (1 << 20) || !mean_out || !var_out || (n > 0 && !x)) return ICQ_ERR_ARG;
    batch_moments_kernel<<<d, 256, 0, (hipStream_t)stream>>>(x, (long long)n, d, mean_out, var_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_online_variance_update(double *mean, double *var, const double *batch_mean,
                                          const double *batch_var, int d, int64_t b, void *stream) {
    if (!mean || !var || !batch_mean || !batch_var || d < 1 || b < 1) return ICQ_ERR_ARG;
    online_variance_kernel<<<(d + 255) / 256, 256, 0, (hipStream_t)stream>>>(mean, var, batch_mean, batch_var, d,
                                                                             1.0 / (double)b);
    return icq_check_launch();
}

ICQ_EXPORT int icq_subspace_mask(const double *lambda, int d, double pi1, double sigma1, double pi2, double mu2,
                                 double sigma2, double alpha2, uint8_t *xi_out, void *stream) {
    if (!lambda || !xi_out || d < 1 || !(sigma1 > 0.0) || !(sigma2 > 0.0)) return ICQ_ERR_ARG;
    subspace_mask_kernel<<<(d + 255) / 256, 256, 0, (hipStream_t)stream>>>(lambda, d, pi1, sigma1, pi2, mu2, sigma2,
                                                                           alpha2, xi_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_fast_set(const icq_index *ix, const uint8_t *xi, uint8_t *fast_out, void *stream) {
    if (!ix || !xi || !fast_out) return ICQ_ERR_ARG;
    fast_set_kernel<<<ix->K, 256, 0, (hipStream_t)stream>>>(ix->cb, ix->m, ix->d, ix->d_pad, xi, fast_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_margin(const double *lambda, const uint8_t *xi, int d, double *sigma_out, void *stream) {
    if (!lambda || !xi || !sigma_out || d < 1) return ICQ_ERR_ARG;
    margin_kernel<<<1, 256, 0, (hipStream_t)stream>>>(lambda, xi, d, sigma_out);
    return icq_check_launch();
}
