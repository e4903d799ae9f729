// Index construction: private device copies of codebooks and codes in the
// layouts the search kernels stream (Sec. 1 of arxiv 1912.08756: an item is K
// codeword indices; the fast set is codebooks 0..Kf-1).
#include "icq_internal.h"

#include <math.h>
#include <mutex>
#include <new>
#include <set>
#include <utility>

namespace {

// fast[k][i] = codes[k][i] for k < Kf, zero beyond N (row stride Npad).
__global__ void copy_fast_kernel(const uint8_t *__restrict__ codes, int64_t N, int64_t Npad,
                                 uint8_t *__restrict__ fast) {
    int k = blockIdx.y;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < Npad) fast[(int64_t)k * Npad + i] = i < N ? codes[(int64_t)k * N + i] : (uint8_t)0;
}

// items[i][k] = codes[k][i] for k < K, zero for K <= k < stride.
__global__ void copy_items_kernel(const uint8_t *__restrict__ codes, int64_t N, int K, int stride,
                                  uint8_t *__restrict__ items) {
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    uint8_t *dst = items + i * stride;
    for (int k = 0; k < stride; ++k) dst[k] = k < K ? codes[(int64_t)k * N + i] : (uint8_t)0;
}

// One wavefront per table row r = k*256 + j: copy the codeword with zero padding
// in d and store its squared norm (accumulated in double, rounded once).
__global__ void copy_codebooks_kernel(const float *__restrict__ codebooks, int K, int m, int d,
                                      int d_pad, float *__restrict__ cb,
                                      float *__restrict__ cnorm) {
    int row = blockIdx.x * (blockDim.x / ICQ_WAVE) + threadIdx.x / ICQ_WAVE;
    int lane = threadIdx.x % ICQ_WAVE;
    if (row >= K * ICQ_LUT_W) return;
    int k = row / ICQ_LUT_W, j = row % ICQ_LUT_W;
    double s = 0.0;
    for (int e = lane; e < d_pad; e += ICQ_WAVE) {
        float v = (j < m && e < d) ? codebooks[((int64_t)k * m + j) * d + e] : 0.0f;
        cb[(int64_t)row * d_pad + e] = v;
        s += (double)v * (double)v;
    }
    for (int off = ICQ_WAVE / 2; off > 0; off >>= 1) s += __shfl_down(s, off, ICQ_WAVE);
    if (lane == 0) cnorm[row] = j < m ? (float)s : INFINITY;
}

// codes_out[k][perm[pos]] = items_grouped[pos][k]: the grouped layout written back in item order.
__global__ void export_grouped_kernel(const uint8_t *__restrict__ items_grouped,
                                      const uint32_t *__restrict__ perm, int64_t N, int stride,
                                      uint8_t *__restrict__ out) {
    int k = blockIdx.y;
    int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos >= N) return;
    out[(int64_t)k * N + perm[pos]] = items_grouped[pos * stride + k];
}

// codes_out[k][i] rebuilt from the private layouts: rows below `fast_rows` from
// the codebook-major fast array, the others from the item records.
__global__ void export_codes_kernel(const uint8_t *__restrict__ fast, const uint8_t *__restrict__ items,
                                    int64_t N, int64_t Npad, int fast_rows, int stride,
                                    uint8_t *__restrict__ out) {
    int k = blockIdx.y;
    int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    out[(int64_t)k * N + i] = k < fast_rows ? fast[(int64_t)k * Npad + i] : items[i * stride + k];
}

int item_stride_for(int K) {
    if (K <= 4) return 4;
    if (K <= 8) return 8;
    return (K + 15) / 16 * 16;
}

}  // namespace

hipError_t icq_allow_lds(const void *fn, int bytes, bool no_static_lds) {
    static std::mutex mu;
    static std::set<std::pair<int, const void *>> done;
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    std::lock_guard<std::mutex> lock(mu);
    if (done.count({dev, fn})) return hipSuccess;
    if (no_static_lds) {
        hipFuncAttributes attr;
        e = hipFuncGetAttributes(&attr, fn);
        if (e != hipSuccess) return e;
        if (attr.sharedSizeBytes != 0) return hipErrorInvalidValue;
    }
    e = hipFuncSetAttribute(fn, hipFuncAttributeMaxDynamicSharedMemorySize, bytes);
    if (e == hipSuccess) done.insert({dev, fn});
    return e;
}

ICQ_EXPORT const char *icq_strerror(int code) {
    switch (code) {
        case ICQ_OK: return "ok";
        case ICQ_ERR_ARG: return "invalid argument";
        case ICQ_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
        case ICQ_ERR_HIP: return "HIP runtime error";
        case ICQ_ERR_CAPACITY: return "candidate capacity exceeded";
        case ICQ_ERR_SCRATCH: return "the call needs more than the library's built-in scratch array (ICQ_STATIC_SCRATCH_BYTES)";
        default: return "unknown error code";
    }
}

ICQ_EXPORT void icq_index_destroy(icq_index *ix) {
    if (!ix) return;
    (void)hipFree(ix->cb);
    (void)hipFree(ix->cnorm);
    (void)hipFree(ix->fast);
    (void)hipFree(ix->items);
    (void)hipFree(ix->group_start);
    (void)hipFree(ix->group_cursor);
    (void)hipFree(ix->perm);
    (void)hipFree(ix->items_grouped);
    (void)hipFree(ix->g2_rows);
    (void)hipFree(ix->g2_info);
    if (ix->timer) {
        for (int i = 0; i < ICQ_TIMED_CALLS * 4; ++i) (void)hipEventDestroy(ix->timer->ev[i / 4][i % 4]);
        delete ix->timer;
    }
    delete ix;
}

ICQ_EXPORT int icq_index_create(icq_index **out, const float *codebooks, const uint8_t *codes,
                                int K, int m, int d, int Kf, int64_t N, void *stream) {
    if (!out || !codebooks) return ICQ_ERR_ARG;
    if (K < 1 || K > ICQ_MAX_K || Kf < 1 || Kf > K || m < 1 || m > ICQ_MAX_M || d < 1 ||
        d > (1 << 20))
        return ICQ_ERR_ARG;
    if (N < 0 || N > ICQ_MAX_N || (N > 0 && !codes)) return ICQ_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;

    icq_index *ix = new (std::nothrow) icq_index();
    if (!ix) return ICQ_ERR_HIP;
    ix->K = K; ix->m = m; ix->d = d; ix->Kf = Kf; ix->Ks = K - Kf;
    ix->d_pad = (d + 15) / 16 * 16;
    ix->item_stride = item_stride_for(K);
    ix->N = N;
    ix->Npad = (N + 16383) / 16384 * 16384 + 16384;   // spare so that whole-step reads stay in bounds
    ix->cb = nullptr; ix->cnorm = nullptr; ix->fast = nullptr; ix->items = nullptr;
    ix->groups = 0; ix->scan_mode = ICQ_SCAN_AUTO; ix->timer = nullptr;
    ix->group_start = nullptr; ix->group_cursor = nullptr; ix->perm = nullptr; ix->items_grouped = nullptr;
    ix->g2 = 0; ix->g2_npos = 0; ix->g2_npad = 0; ix->g2_rows = nullptr; ix->g2_info = nullptr;
    hipDeviceProp_t prop;
    if (hipGetDevice(&ix->device) != hipSuccess ||
        hipGetDeviceProperties(&prop, ix->device) != hipSuccess) {
        delete ix;
        return ICQ_ERR_HIP;
    }
    ix->num_cu = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;

    bool ok = hipMalloc(&ix->cb, sizeof(float) * (size_t)K * ICQ_LUT_W * ix->d_pad) == hipSuccess &&
              hipMalloc(&ix->cnorm, sizeof(float) * (size_t)K * ICQ_LUT_W) == hipSuccess &&
              hipMalloc(&ix->fast, (size_t)Kf * ix->Npad) == hipSuccess;
    if (ok && N > 0) ok = hipMalloc(&ix->items, (size_t)N * ix->item_stride) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        icq_index_destroy(ix);
        return ICQ_ERR_HIP;
    }

    const int T = 256;
    copy_codebooks_kernel<<<(K * ICQ_LUT_W + 3) / 4, T, 0, s>>>(codebooks, K, m, d, ix->d_pad,
                                                                 ix->cb, ix->cnorm);
    {
        dim3 g((unsigned)((ix->Npad + T - 1) / T), (unsigned)Kf);
        copy_fast_kernel<<<g, T, 0, s>>>(codes, N, ix->Npad, ix->fast);
    }
    if (N > 0)
        copy_items_kernel<<<(unsigned)((N + T - 1) / T), T, 0, s>>>(codes, N, K, ix->item_stride,
                                                                     ix->items);
    if (icq_check_launch() != ICQ_OK || icq_group_build(ix, s) != ICQ_OK || icq_group2_build(ix, s) != ICQ_OK) {
        icq_index_destroy(ix);
        return ICQ_ERR_HIP;
    }
    *out = ix;
    return ICQ_OK;
}

ICQ_EXPORT int icq_index_export_codes(const icq_index *ix, int from_items, uint8_t *codes_out,
                                      void *stream) {
    if (!ix || (!codes_out && ix->N > 0)) return ICQ_ERR_ARG;
    if (ix->N == 0) return ICQ_OK;
    const int T = 256;
    dim3 g((unsigned)((ix->N + T - 1) / T), (unsigned)ix->K);
    if (from_items == 2) {
        if (ix->g2) return icq_group2_export(ix, codes_out, (hipStream_t)stream);
        if (!ix->groups) return ICQ_ERR_ARG;
        export_grouped_kernel<<<g, T, 0, (hipStream_t)stream>>>(ix->items_grouped, ix->perm, ix->N,
                                                                ix->item_stride, codes_out);
        return icq_check_launch();
    }
    export_codes_kernel<<<g, T, 0, (hipStream_t)stream>>>(ix->fast, ix->items, ix->N, ix->Npad,
                                                          from_items ? 0 : ix->Kf, ix->item_stride,
                                                          codes_out);
    return icq_check_launch();
}

ICQ_EXPORT int icq_index_scan_positions(const icq_index *ix, int Q, int64_t *out) {
    if (!ix || !out || Q < 0) return ICQ_ERR_ARG;
    if (icq_group_usable(ix, Q)) *out = ix->groups;
    else if (icq_g2_usable(ix) && ix->Kf <= 4) *out = ix->g2_npos;
    else *out = ix->N;
    return ICQ_OK;
}

static void timer_free(icq_stage_timer *t, int created) {
    for (int i = 0; i < created; ++i) (void)hipEventDestroy(t->ev[i / 4][i % 4]);
    delete t;
}

ICQ_EXPORT int icq_index_set_stage_timing(icq_index *ix, int enable) {
    if (!ix) return ICQ_ERR_ARG;
    if (!enable) {
        if (ix->timer) timer_free(ix->timer, ICQ_TIMED_CALLS * 4);
        ix->timer = nullptr;
        return ICQ_OK;
    }
    if (ix->timer) return ICQ_OK;
    icq_stage_timer *t = new (std::nothrow) icq_stage_timer();
    if (!t) return ICQ_ERR_HIP;
    t->calls = 0;
    t->batches = 0;
    for (int i = 0; i < ICQ_TIMED_CALLS * 4; ++i) {
        if (hipEventCreate(&t->ev[i / 4][i % 4]) != hipSuccess) {
            (void)hipGetLastError();
            timer_free(t, i);
            return ICQ_ERR_HIP;
        }
    }
    ix->timer = t;
    return ICQ_OK;
}

ICQ_EXPORT int icq_index_stage_times(const icq_index *ix, float *ms, int *calls, int *batches) {
    if (!ix || !ms || !ix->timer || ix->timer->calls == 0) return ICQ_ERR_ARG;
    icq_stage_timer *t = ix->timer;
    const long long last = t->calls - 1;
    const int n = t->calls < ICQ_TIMED_CALLS ? (int)t->calls : ICQ_TIMED_CALLS;
    ICQ_HIP_TRY(hipEventSynchronize(t->ev[last % ICQ_TIMED_CALLS][3]));
    double sum[3] = {0.0, 0.0, 0.0};
    for (int c = 0; c < n; ++c) {
        const int slot = (int)((last - c) % ICQ_TIMED_CALLS);
        for (int i = 0; i < 3; ++i) {
            float v = 0.0f;
            ICQ_HIP_TRY(hipEventElapsedTime(&v, t->ev[slot][i], t->ev[slot][i + 1]));
            sum[i] += v;
        }
    }
    for (int i = 0; i < 3; ++i) ms[i] = (float)(sum[i] / n);
    if (calls) *calls = n;
    if (batches) *batches = t->batches;
    t->calls = 0;
    t->batches = 0;
    return ICQ_OK;
}
