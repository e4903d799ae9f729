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
    static bool attr_set = false;
    if (!attr_set) {
        ICQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&sample_threshold_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 65536));
        attr_set = true;
    }
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
