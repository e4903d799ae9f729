// Stage 2 of the two-step search (arxiv 1912.08756, Eq. 1 and Sec. 3.4): for
// the survivors of the crude comparison only, finish the K-term table sum
//   D[q][i] = P[q][i] + sum_{k=Kf..K-1} lut[q][k][code_k(i)]
// and keep the per-query list of the topk nearest, ordered by (D, id).
//
// One block handles one slice of one query's candidate list.  The query's
// tables sit in LDS; each thread gathers one survivor's sub-codes (stored
// item-major, one aligned record per item) and forms D, either from the crude
// distance handed over by stage 1 plus the slow terms, or -- when stage 1 listed
// ids only -- as the whole K-term sum in the same order of additions.  Selection keeps a
// running bound: a 64-bit key (order-preserving bits of D, id) enters an LDS
// buffer only if it beats the current topk-th key; when the buffer fills it is
// sorted (bitonic) and cut back to topk, which tightens the bound.
#include "icq_internal.h"

namespace {

typedef unsigned long long u64;
constexpr int RF_THREADS = 256;
constexpr u64 KEY_PAD = ~0ull;

__device__ __forceinline__ uint32_t order_bits(float x) {
    uint32_t b = __float_as_uint(x);
    return (b & 0x80000000u) ? ~b : (b | 0x80000000u);
}
__device__ __forceinline__ float unorder_bits(uint32_t u) {
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

// Ascending bitonic sort of keys[0..len), len a power of two >= 2, whole block.
__device__ void block_sort(u64 *keys, int len) {
    for (int k = 2; k <= len; k <<= 1) {
        for (int j = k >> 1; j > 0; j >>= 1) {
            for (int i = threadIdx.x; i < len / 2; i += RF_THREADS) {
                int a = ((i / j) * 2 * j) + (i % j);
                int b = a + j;
                bool up = (a & k) == 0;
                u64 x = keys[a], y = keys[b];
                if ((x > y) == up) {
                    keys[a] = y;
                    keys[b] = x;
                }
            }
            __syncthreads();
        }
    }
}

// Sort the buffered keys and keep the best `topk`; returns the kept count.
// Every thread of the block must call it (contains barriers).
__device__ int compact_keys(u64 *keys, uint32_t *s_cnt, u64 *s_bound, int topk) {
    int n = (int)*s_cnt;
    __syncthreads();
    int len = 2;
    while (len < n) len <<= 1;
    for (int i = n + threadIdx.x; i < len; i += RF_THREADS) keys[i] = KEY_PAD;
    __syncthreads();
    block_sort(keys, len);
    int kept = n < topk ? n : topk;
    if (threadIdx.x == 0) {
        *s_cnt = (uint32_t)kept;
        *s_bound = n >= topk ? keys[topk - 1] : KEY_PAD;
    }
    __syncthreads();
    return kept;
}

__device__ __forceinline__ void write_result(const u64 *keys, int kept, int topk,
                                             uint32_t *out_ids, float *out_dist) {
    for (int r = threadIdx.x; r < topk; r += RF_THREADS) {
        if (r < kept) {
            out_ids[r] = (uint32_t)keys[r];
            out_dist[r] = unorder_bits((uint32_t)(keys[r] >> 32));
        } else {
            out_ids[r] = ICQ_PAD_ID;
            out_dist[r] = INFINITY;
        }
    }
}

// grid (Q * splits), block b = q * splits + slice.  LDS: keys[bufn] | tables k0..K-1,
// k0 = Kf when cand_part is given, else 0.
__global__ __launch_bounds__(RF_THREADS) void refine_kernel(
    const uint8_t *__restrict__ items, int stride, int K, int Kf, const float *__restrict__ lut,
    const uint32_t *__restrict__ cand_ids, const float *__restrict__ cand_part,
    const uint32_t *__restrict__ cand_count, int64_t cap, int topk, int bufn, int splits,
    u64 *__restrict__ keys_out, uint32_t *__restrict__ out_ids, float *__restrict__ out_dist) {
    extern __shared__ u64 smem64[];
    __shared__ uint32_t s_cnt;
    __shared__ u64 s_bound;
    u64 *keys = smem64;
    float *T = reinterpret_cast<float *>(keys + bufn);
    const int k0 = cand_part ? Kf : 0;
    const int q = blockIdx.x / splits, sp = blockIdx.x % splits;
    const int tid = threadIdx.x;

    for (int i = tid; i < (K - k0) * ICQ_LUT_W; i += RF_THREADS)
        T[i] = lut[((int64_t)q * K + k0) * ICQ_LUT_W + i];
    if (tid == 0) {
        s_cnt = 0;
        s_bound = KEY_PAD;
    }
    __syncthreads();

    u64 n = cand_count[q];
    if (n > (u64)cap) n = (u64)cap;
    const u64 lo = n * (u64)sp / (u64)splits, hi = n * (u64)(sp + 1) / (u64)splits;
    const uint32_t *ids = cand_ids + (int64_t)q * cap;
    const float *part = cand_part ? cand_part + (int64_t)q * cap : nullptr;
    const int w0 = k0 / 4;   // first record word that holds a needed sub-code

    for (u64 base = lo; base < hi; base += RF_THREADS) {
        const u64 idx = base + tid;
        if (idx < hi) {
            const uint32_t id = ids[idx];
            float D = part ? part[idx] : 0.0f;
            const uint32_t *rec = reinterpret_cast<const uint32_t *>(items + (size_t)id * stride);
            for (int w = w0; w * 4 < K; ++w) {
                const uint32_t word = rec[w];
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    const int k = w * 4 + j;
                    if (k >= k0 && k < K) {
                        const float v = T[(k - k0) * ICQ_LUT_W + ((word >> (8 * j)) & 0xffu)];
                        D = (k == 0) ? v : D + v;
                    }
                }
            }
            const u64 key = ((u64)order_bits(D) << 32) | id;
            if (key < s_bound) {
                uint32_t slot = atomicAdd(&s_cnt, 1u);
                keys[slot] = key;
            }
        }
        __syncthreads();
        const int filled = (int)s_cnt;
        __syncthreads();   // every thread has read the count before anyone appends again
        if (filled > bufn - RF_THREADS) compact_keys(keys, &s_cnt, &s_bound, topk);
    }
    const int kept = compact_keys(keys, &s_cnt, &s_bound, topk);
    if (splits == 1) {
        write_result(keys, kept, topk, out_ids + (int64_t)q * topk, out_dist + (int64_t)q * topk);
    } else {
        u64 *dst = keys_out + ((int64_t)q * splits + sp) * topk;
        for (int r = tid; r < topk; r += RF_THREADS) dst[r] = r < kept ? keys[r] : KEY_PAD;
    }
}

// grid (Q): merge the per-slice lists of one query.  LDS: keys[len], len >= splits*topk.
__global__ __launch_bounds__(RF_THREADS) void merge_kernel(const u64 *__restrict__ keys_in,
                                                           int splits, int topk, int len,
                                                           uint32_t *__restrict__ out_ids,
                                                           float *__restrict__ out_dist) {
    extern __shared__ u64 smem64[];
    u64 *keys = smem64;
    const int q = blockIdx.x;
    const int n = splits * topk;
    for (int i = threadIdx.x; i < len; i += RF_THREADS)
        keys[i] = i < n ? keys_in[(int64_t)q * n + i] : KEY_PAD;
    __syncthreads();
    block_sort(keys, len);
    // pads sort last; count the real keys among the first topk
    for (int r = threadIdx.x; r < topk; r += RF_THREADS) {
        const u64 key = keys[r];
        if (key != KEY_PAD) {
            out_ids[(int64_t)q * topk + r] = (uint32_t)key;
            out_dist[(int64_t)q * topk + r] = unorder_bits((uint32_t)(key >> 32));
        } else {
            out_ids[(int64_t)q * topk + r] = ICQ_PAD_ID;
            out_dist[(int64_t)q * topk + r] = INFINITY;
        }
    }
}

int bufn_for(int topk) { return topk <= 256 ? 2048 : 4096; }

}  // namespace

int icq_refine_splits(const icq_index *ix, int Q, int64_t cap, int topk) {
    if (Q <= 0) return 1;
    int64_t s = (4LL * ix->num_cu + Q - 1) / Q;
    int64_t by_len = cap / 2048 + 1;            // do not slice short lists
    int64_t by_merge = 4096 / topk;             // merge buffer holds splits*topk keys
    if (s > by_len) s = by_len;
    if (s > by_merge) s = by_merge;
    if (s > 64) s = 64;
    if (s < 1) s = 1;
    return (int)s;
}

int icq_launch_refine(const icq_index *ix, const float *lut, int Q, const uint32_t *cand_ids,
                      const float *cand_part, const uint32_t *cand_count, int64_t cap, int topk,
                      int splits, u64 *keys, uint32_t *out_ids, float *out_dist, hipStream_t s) {
    if (Q == 0) return ICQ_OK;
    const int bufn = bufn_for(topk);
    const size_t lds = sizeof(u64) * bufn + sizeof(float) * (size_t)(cand_part ? ix->Ks : ix->K) * ICQ_LUT_W;
    static bool attr_set = false;
    if (!attr_set) {
        ICQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&refine_kernel),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, 98304));
        attr_set = true;
    }
    const unsigned grid = (unsigned)Q * (unsigned)splits;
    refine_kernel<<<grid, RF_THREADS, lds, s>>>(ix->items, ix->item_stride, ix->K, ix->Kf, lut,
                                                cand_ids, cand_part, cand_count, cap, topk, bufn,
                                                splits, keys, out_ids, out_dist);
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    if (splits > 1) {
        int len = 2;
        while (len < splits * topk) len <<= 1;
        merge_kernel<<<Q, RF_THREADS, sizeof(u64) * len, s>>>(keys, splits, topk, len, out_ids,
                                                              out_dist);
        return icq_check_launch();
    }
    return ICQ_OK;
}

ICQ_EXPORT int icq_refine(const icq_index *ix, const float *lut, int Q, const uint32_t *cand_ids,
                          const float *cand_part, const uint32_t *cand_count, int64_t cap, int topk,
                          uint32_t *out_ids, float *out_dist, void *workspace,
                          size_t workspace_bytes, void *stream) {
    if (!ix || Q < 0 || Q > (1 << 22) || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK)
        return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if (!lut || !cand_ids || !cand_count || !out_ids || !out_dist) return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    icq_ws_layout L = icq_layout(ix, Q, cap, topk, false, false);
    if (L.total > 0 &&
        (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < L.total))
        return ICQ_ERR_WORKSPACE;
    u64 *keys = reinterpret_cast<u64 *>(static_cast<char *>(workspace) + L.keys_off);
    return icq_launch_refine(ix, lut, Q, cand_ids, cand_part, cand_count, cap, topk, L.splits, keys,
                             out_ids, out_dist, (hipStream_t)stream);
}
