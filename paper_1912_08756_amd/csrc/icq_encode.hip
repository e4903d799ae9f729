// Encoding, the step before the search path (arxiv 1912.08756, Sec. 1: an item is
// stored as one codeword index per codebook, xbar_i = sum_k c_{k,code_k(i)}).  The
// paper gives no assignment algorithm; this is the greedy residual assignment in
// codebook order:
//     r_0 = x_i;  code_k(i) = argmin_j ||r_k - c_{k,j}||^2 (ties: smallest j);
//     r_{k+1} = r_k - c_{k,code_k(i)}.
// ||r - c||^2 = ||r||^2 - 2<r,c> + ||c||^2 and ||r||^2 does not depend on j, so a level
// is one [N x d].[d x 256] contraction on the fp32 matrix cores with the epilogue
// argmin_j (||c_j||^2 - 2<r,c_j>), followed by the residual update of the block's own
// rows.
//
// icq_encode_refine revisits given codes by coordinate descent over the codebooks (iterated
// conditional modes): with the other sub-codes of an item fixed, codebook k's codeword becomes the
// nearest one to r = x - sum_{l != k} c_l, and only if that is strictly nearer than the current
// one.  The kernel is the same contraction: the residual array holds x - xbar, a level adds the
// current codeword back while staging its rows, the argmin prefers the current codeword among equal
// scores, and only rows whose sub-code changed are rewritten.
#include "icq_internal.h"
#include "icq_sort.h"

#include <math.h>

namespace {

// the smaller of a lane's key and its DPP neighbour's (a lane without a source keeps its own)
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ u64 dpp_min64(u64 key) {
    const uint32_t lo = icq_dpp<CTRL, ROW_MASK, 0xFFFFFFFFu>((uint32_t)key);
    const uint32_t hi = icq_dpp<CTRL, ROW_MASK, 0xFFFFFFFFu>((uint32_t)(key >> 32));
    const u64 o = ((u64)hi << 32) | lo;
    return o < key ? o : key;
}

typedef float float16v __attribute__((ext_vector_type(16)));
constexpr int EM = 64;            // items per block
constexpr int EN = ICQ_LUT_W;     // codewords per level: the whole codebook (rows j >= m have norm +inf)
constexpr int EK = 16;            // reduction slice staged in LDS
constexpr int E_THREADS = 256;

// One level for 64 items.  4 wavefronts, wavefront w owns codewords [64w, 64w + 64) as
// 2x2 accumulators of 32x32 (MFMA 32x32x2 layout: lane l supplies A[l%32][l/32] and
// B[l/32][l%32]; accumulator register v of lane l is C[(v%4) + 4*(l/32) + 8*(v/4)][l%32]).
// src: x (row stride d, level 0) or the residuals (row stride d_pad); dst: residuals.
// ICM: src = res holds x - xbar, codes_k holds the current sub-codes (in and out), *changed counts
// the sub-codes replaced.
template <bool ICM>
__global__ __launch_bounds__(E_THREADS) void encode_level_kernel(
    const float *src, int src_stride, int d, const float *__restrict__ cb_k, int d_pad,
    const float *__restrict__ cnorm_k, int64_t N, uint8_t *codes_k, float *res, int vec_ok, uint32_t *changed) {
    __shared__ float As[EK][EM + 1];
    __shared__ float Bs[EK][EN + 1];
    __shared__ u64 best[E_THREADS / 64][EM];
    __shared__ uint32_t s_code[EM];
    __shared__ uint32_t s_old[EM];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int64_t i0 = (int64_t)blockIdx.x * EM;
    const int le = tid & 15, lr = tid >> 4;       // reduction position and row (+16 per pass) of the staging loads
    if (ICM && tid < EM) s_old[tid] = codes_k[i0 + tid < N ? i0 + tid : N - 1];     // visible after the first slice's barrier

    float16v acc[2][2];
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.0f;

    // Rows past N read the last row instead (their codes and residuals are never stored) and
    // columns past d read column d - 1 (the codebook copy is zero there, the product vanishes):
    // no load depends on a condition, so a slice's twenty are in flight together.
    const float *arow[EM / 16];
    const float *orow[EM / 16];                   // ICM: the row's current codeword, added back while staging
#pragma unroll
    for (int p = 0; p < EM / 16; ++p) {
        const int64_t row = i0 + lr + 16 * p;
        const int64_t rc = row < N ? row : N - 1;
        arow[p] = src + rc * src_stride;
        orow[p] = ICM ? cb_k + (int64_t)codes_k[rc] * d_pad : cb_k;
    }
    for (int k0 = 0; k0 < d_pad; k0 += EK) {
        float a[EM / 16], b[EN / 16];
        const int e = k0 + le;
        const int ec = e < d ? e : d - 1;
#pragma unroll
        for (int p = 0; p < EM / 16; ++p) a[p] = ICM ? arow[p][ec] + orow[p][e] : arow[p][ec];
#pragma unroll
        for (int p = 0; p < EN / 16; ++p) b[p] = cb_k[(int64_t)(lr + 16 * p) * d_pad + e];
        __syncthreads();   // previous slice fully consumed
#pragma unroll
        for (int p = 0; p < EM / 16; ++p) As[le][lr + 16 * p] = a[p];
#pragma unroll
        for (int p = 0; p < EN / 16; ++p) Bs[le][lr + 16 * p] = b[p];
        __syncthreads();
#pragma unroll
        for (int s = 0; s < EK / 2; ++s) {
            float av[2], bv[2];
#pragma unroll
            for (int i = 0; i < 2; ++i) {
                av[i] = As[2 * s + (lane >> 5)][i * 32 + (lane & 31)];
                bv[i] = Bs[2 * s + (lane >> 5)][wave * 64 + i * 32 + (lane & 31)];
            }
#pragma unroll
            for (int i = 0; i < 2; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[i], bv[j], acc[i][j], 0, 0, 0);
        }
    }
    // argmin over the wavefront's 64 codewords for each of the 64 rows: key = (order-preserving bits
    // of ||c||^2 - 2<r,c>, codeword index), the smaller key wins, so equal scores go to the smaller index
    // (ICM: index + 1, and 0 for the row's current codeword, which so wins among equal scores)
    float cn[2];
#pragma unroll
    for (int j = 0; j < 2; ++j) cn[j] = cnorm_k[wave * 64 + j * 32 + (lane & 31)];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            u64 key = ~0ull;
            const uint32_t cur = ICM ? s_old[i * 32 + (v & 3) + 4 * (lane >> 5) + 8 * (v >> 2)] : 0u;
#pragma unroll
            for (int j = 0; j < 2; ++j) {
                const float score = cn[j] - 2.0f * acc[i][j][v];
                const uint32_t col = (uint32_t)(wave * 64 + j * 32 + (lane & 31));
                const uint32_t field = ICM ? (col == cur ? 0u : col + 1u) : col;
                const u64 kj = ((u64)icq_order_bits(score) << 32) | field;
                key = kj < key ? kj : key;
            }
            // minimum over each half of 32 lanes on the DPP path (row shifts, then lane 15 of rows 0 and 2
            // into rows 1 and 3): lanes 31 and 63 end up with their half's smallest key
            key = dpp_min64<0x111, 0xf>(key);
            key = dpp_min64<0x112, 0xf>(key);
            key = dpp_min64<0x114, 0xf>(key);
            key = dpp_min64<0x118, 0xf>(key);
            key = dpp_min64<0x142, 0xa>(key);
            if ((lane & 31) == 31) best[wave][i * 32 + (v & 3) + 4 * (lane >> 5) + 8 * (v >> 2)] = key;
        }
    }
    __syncthreads();
    if (tid < EM) {
        u64 key = best[0][tid];
#pragma unroll
        for (int w = 1; w < E_THREADS / 64; ++w) key = best[w][tid] < key ? best[w][tid] : key;
        const uint32_t field = (uint32_t)key;
        const uint32_t code = ICM ? (field == 0u ? s_old[tid] : field - 1u) : field;
        s_code[tid] = code;
        const bool store = i0 + tid < N && (!ICM || code != s_old[tid]);
        if (store) codes_k[i0 + tid] = (uint8_t)code;
        if (ICM && changed) {                      // tid < 64: the first wavefront, whole
            const int n = __builtin_popcountll(__ballot(store));
            if (tid == 0 && n > 0) atomicAdd(changed, (uint32_t)n);
        }
    }
    __syncthreads();
    // residual update of the block's rows (zero beyond d, so later levels can read whole slices)
    if (vec_ok && i0 + EM <= N) {
        // whole block, d == d_pad, 16-byte aligned rows: 128-bit accesses, four of a thread's in flight
        // together (one by one, each store would be waited for before the next load: stores count
        // with the loads)
        const int row4 = d_pad / 4;                       // 128-bit pieces per row; EM * row4 = 256 * (d_pad / 16)
        const int nit = d_pad / 16;
        const float4 *src4 = reinterpret_cast<const float4 *>(src);
        const float4 *cb4 = reinterpret_cast<const float4 *>(cb_k);
        float4 *res4 = reinterpret_cast<float4 *>(res);
        const int src_row4 = src_stride / 4;
        constexpr int U = 4;
        for (int it = 0; it < nit; it += U) {
            float4 xa[U], ca[U];
            int64_t off[U];
            bool keep[U];
#pragma unroll
            for (int u = 0; u < U; ++u) {
                const int idx = (it + u < nit ? it + u : it) * E_THREADS + tid;
                const int r = idx / row4, e4 = idx % row4;
                xa[u] = src4[(i0 + r) * src_row4 + e4];
                ca[u] = cb4[(int64_t)s_code[r] * row4 + e4];
                off[u] = (i0 + r) * row4 + e4;
                keep[u] = ICM && s_code[r] == s_old[r];
                if (ICM) {
                    const float4 co = cb4[(int64_t)s_old[r] * row4 + e4];
                    xa[u] = make_float4(xa[u].x + co.x, xa[u].y + co.y, xa[u].z + co.z, xa[u].w + co.w);
                }
            }
#pragma unroll
            for (int u = 0; u < U; ++u) {
                if (it + u < nit && !keep[u])             // the first condition is block-uniform
                    res4[off[u]] = make_float4(xa[u].x - ca[u].x, xa[u].y - ca[u].y, xa[u].z - ca[u].z, xa[u].w - ca[u].w);
            }
        }
        return;
    }
    for (int idx = tid; idx < EM * d_pad; idx += E_THREADS) {
        const int r = idx / d_pad, e = idx % d_pad;
        const int64_t row = i0 + r;
        if (row < N && !(ICM && s_code[r] == s_old[r])) {
            float xv = e < d ? src[row * src_stride + e] : 0.0f;
            if (ICM) xv += cb_k[(int64_t)s_old[r] * d_pad + e];
            res[row * d_pad + e] = xv - cb_k[(int64_t)s_code[r] * d_pad + e];
        }
    }
}

// res[n][e] = x[n][e] - sum_k c_{k,code_k(n)}[e] (k ascending), zero beyond d: what the refinement starts from.
__global__ void residual_kernel(const float *__restrict__ x, int d, int d_pad, const float *__restrict__ cb, int K,
                                const uint8_t *__restrict__ codes, int64_t N, float *__restrict__ res) {
    const int64_t idx = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (idx >= N * d_pad) return;
    const int64_t n = idx / d_pad;
    const int e = (int)(idx % d_pad);
    float r = e < d ? x[n * d + e] : 0.0f;
    for (int k = 0; k < K; ++k) r -= cb[((int64_t)k * ICQ_LUT_W + codes[(int64_t)k * N + n]) * d_pad + e];
    res[idx] = r;
}

__global__ void zero_words_kernel(uint32_t *p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// One wavefront per item: ||x - sum_k c_{k,code_k}||^2 accumulated in double.
__global__ __launch_bounds__(256) void quantization_error_kernel(const float *__restrict__ x, int d, int d_pad,
                                                                 const float *__restrict__ cb, int K,
                                                                 const uint8_t *__restrict__ codes, int64_t N,
                                                                 double *__restrict__ err) {
    const int64_t n = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (n >= N) return;                            // whole wavefronts leave together
    const int lane = threadIdx.x & 63;
    double s = 0.0;
    for (int e = lane; e < d; e += 64) {
        double xb = 0.0;
        for (int k = 0; k < K; ++k) xb += (double)cb[((int64_t)k * ICQ_LUT_W + codes[(int64_t)k * N + n]) * d_pad + e];
        const double diff = (double)x[n * d + e] - xb;
        s += diff * diff;
    }
    for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o);
    if (lane == 0) err[n] = s;
}

}  // namespace

ICQ_EXPORT int icq_encode_workspace_bytes(const icq_index *ix, int64_t N, size_t *out) {
    if (!ix || !out || N < 0 || N > ICQ_MAX_N) return ICQ_ERR_ARG;
    const size_t need = sizeof(float) * (size_t)N * (size_t)ix->d_pad;
    *out = need > ICQ_ALIGN ? icq_align_up(need, ICQ_ALIGN) : ICQ_ALIGN;
    return ICQ_OK;
}

ICQ_EXPORT int icq_encode(const icq_index *ix, const float *x, int64_t N, uint8_t *codes_out, void *workspace,
                          size_t workspace_bytes, void *stream) {
    if (!ix || N < 0 || N > ICQ_MAX_N) return ICQ_ERR_ARG;
    if (N == 0) return ICQ_OK;
    if (!x || !codes_out) return ICQ_ERR_ARG;
    size_t need = 0;
    (void)icq_encode_workspace_bytes(ix, N, &need);
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < need) return ICQ_ERR_WORKSPACE;
    float *res = static_cast<float *>(workspace);
    hipStream_t s = (hipStream_t)stream;
    const unsigned blocks = (unsigned)((N + EM - 1) / EM);
    for (int k = 0; k < ix->K; ++k) {
        const float *src = k == 0 ? x : res;
        const int stride = k == 0 ? ix->d : ix->d_pad;
        // in place for k > 0: a block reads and writes only its own rows, and every read of a row
        // (slices, then the update) precedes its write in program order behind a barrier
        const float *cbk = ix->cb + (size_t)k * ICQ_LUT_W * ix->d_pad;
        const int vec_ok = ix->d == ix->d_pad && stride % 4 == 0 && (uintptr_t)src % 16 == 0 && (uintptr_t)cbk % 16 == 0;
        encode_level_kernel<false><<<blocks, E_THREADS, 0, s>>>(src, stride, ix->d, cbk, ix->d_pad,
                                                                ix->cnorm + (size_t)k * ICQ_LUT_W, N,
                                                                codes_out + (size_t)k * N, res, vec_ok, nullptr);
    }
    return icq_check_launch();
}

ICQ_EXPORT int icq_encode_refine(const icq_index *ix, const float *x, int64_t N, uint8_t *codes, int sweeps,
                                 uint32_t *changed_out, void *workspace, size_t workspace_bytes, void *stream) {
    if (!ix || N < 0 || N > ICQ_MAX_N || sweeps < 0 || sweeps > ICQ_MAX_SWEEPS) return ICQ_ERR_ARG;
    if (N == 0 || sweeps == 0) return ICQ_OK;
    if (!x || !codes) return ICQ_ERR_ARG;
    size_t need = 0;
    (void)icq_encode_workspace_bytes(ix, N, &need);
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < need) return ICQ_ERR_WORKSPACE;
    float *res = static_cast<float *>(workspace);
    hipStream_t s = (hipStream_t)stream;
    const int64_t total = N * ix->d_pad;
    residual_kernel<<<(unsigned)((total + 255) / 256), 256, 0, s>>>(x, ix->d, ix->d_pad, ix->cb, ix->K, codes, N, res);
    if (changed_out) zero_words_kernel<<<(sweeps + 255) / 256, 256, 0, s>>>(changed_out, sweeps);
    const unsigned blocks = (unsigned)((N + EM - 1) / EM);
    for (int sw = 0; sw < sweeps; ++sw) {
        for (int k = 0; k < ix->K; ++k) {
            // in place: a block reads and writes only its own rows and sub-codes, reads first
            const float *cbk = ix->cb + (size_t)k * ICQ_LUT_W * ix->d_pad;
            const int vec_ok = ix->d == ix->d_pad && (uintptr_t)cbk % 16 == 0;
            encode_level_kernel<true><<<blocks, E_THREADS, 0, s>>>(res, ix->d_pad, ix->d, cbk, ix->d_pad,
                                                                   ix->cnorm + (size_t)k * ICQ_LUT_W, N,
                                                                   codes + (size_t)k * N, res, vec_ok,
                                                                   changed_out ? changed_out + sw : nullptr);
        }
    }
    return icq_check_launch();
}

ICQ_EXPORT int icq_quantization_error(const icq_index *ix, const float *x, int64_t N, const uint8_t *codes,
                                      double *err_out, void *stream) {
    if (!ix || N < 0 || N > ICQ_MAX_N) return ICQ_ERR_ARG;
    if (N == 0) return ICQ_OK;
    if (!x || !codes || !err_out) return ICQ_ERR_ARG;
    quantization_error_kernel<<<(unsigned)((N + 3) / 4), 256, 0, (hipStream_t)stream>>>(x, ix->d, ix->d_pad, ix->cb, ix->K,
                                                                                         codes, N, err_out);
    return icq_check_launch();
}
