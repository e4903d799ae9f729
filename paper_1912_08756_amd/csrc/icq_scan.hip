// Stage 1 of the two-step search (arxiv 1912.08756, Eq. 2 and Sec. 3.4): the
// crude distance P[q][i] = sum_{k<Kf} lut[q][k][code_k(i)] over the fast
// codebooks only, compared with a per-query threshold; survivors are appended
// to per-query candidate lists for stage 2.
//
// Two kernels share the contract:
//   scan_batch_kernel  - lanes = queries.  A tile of 64 queries keeps its fast
//       tables in LDS as [k][code][query]; a wavefront walks the items, the
//       sub-code is wave-uniform, so every table read is one conflict-free
//       256-byte LDS row.  One pass over the codes serves 64 queries.
//   scan_items_kernel  - lanes = items.  Any Kf; the tables of a few queries
//       sit in LDS as [query][k][code], each lane gathers with its own
//       sub-codes held in registers, survivors are compacted with a ballot.
#include "icq_internal.h"

#include <math.h>

namespace {

// ------------------------------------------------------------------ helpers
__device__ __forceinline__ uint32_t lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

// Zero the per-query survivor counters (a fill kernel rather than a memset
// node so that the call can sit inside a captured graph).
__global__ void zero_counts_kernel(uint32_t *__restrict__ cnt, int Q) {
    int q = blockIdx.x * blockDim.x + threadIdx.x;
    if (q < Q) cnt[q] = 0u;
}

// lutT[tile][k][code][lane] = lut[tile*64 + lane][k][code] for k < Kf; queries
// beyond Q get +inf (never below any threshold).  Block = (tile, k), 256 threads.
__global__ __launch_bounds__(256) void transpose_fast_lut_kernel(const float *__restrict__ lut,
                                                                 int Q, int K, int Kf,
                                                                 float *__restrict__ lutT) {
    __shared__ float tile[64][65];
    const int t = blockIdx.x, k = blockIdx.y;
    const int tx = threadIdx.x & 63, ty = threadIdx.x >> 6;
    for (int c0 = 0; c0 < ICQ_LUT_W; c0 += 64) {
        for (int r = ty; r < 64; r += 4) {
            int q = t * 64 + r;
            tile[r][tx] = q < Q ? lut[((int64_t)q * K + k) * ICQ_LUT_W + c0 + tx] : INFINITY;
        }
        __syncthreads();
        for (int c = ty; c < 64; c += 4)
            lutT[(((int64_t)t * Kf + k) * ICQ_LUT_W + c0 + c) * 64 + tx] = tile[tx][c];
        __syncthreads();
    }
}

// ------------------------------------------------------------------ lanes = queries
constexpr int SB_WAVES = 8;                 // wavefronts per block
constexpr int SB_THREADS = SB_WAVES * 64;
constexpr int SB_STAGE = 6;                 // staged survivors per lane before a flush
constexpr int SB_GROUP = 256;               // items per wavefront step (one dword per lane and row)

template <int KF>
__global__ __launch_bounds__(SB_THREADS, 1) void scan_batch_kernel(
    const uint8_t *__restrict__ fast, int64_t Npad, uint32_t N, const float *__restrict__ lutT,
    const float *__restrict__ thr, int Q, uint32_t *__restrict__ cand_ids,
    float *__restrict__ cand_part, uint32_t *__restrict__ cand_count, int64_t cap,
    uint32_t items_per_block) {
    extern __shared__ float smem[];
    constexpr int LUT_FLOATS = KF * ICQ_LUT_W * 64;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int tile = blockIdx.y;

    {   // tile's tables -> LDS, straight copy
        const float4 *src = reinterpret_cast<const float4 *>(lutT + (int64_t)tile * LUT_FLOATS);
        float4 *dst = reinterpret_cast<float4 *>(smem);
        for (int i = tid; i < LUT_FLOATS / 4; i += SB_THREADS) dst[i] = src[i];
    }
    __syncthreads();

    const int q = tile * 64 + lane;
    const float t = q < Q ? thr[q] : -INFINITY;
    uint32_t *my_ids = cand_ids + (int64_t)q * cap;
    float *my_part = cand_part + (int64_t)q * cap;
    // per-wavefront staging area [slot][lane] of (id, P) pairs
    uint2 *stage = reinterpret_cast<uint2 *>(smem + LUT_FLOATS) + wave * (64 * SB_STAGE);
    int my_cnt = 0;

    auto flush = [&]() {
        uint32_t base = 0;
        if (my_cnt > 0) base = atomicAdd(&cand_count[q], (uint32_t)my_cnt);
#pragma unroll
        for (int s = 0; s < SB_STAGE; ++s) {
            if (s < my_cnt) {
                uint64_t slot = (uint64_t)base + s;
                if (slot < (uint64_t)cap) {
                    uint2 e = stage[s * 64 + lane];
                    my_ids[slot] = e.x;
                    my_part[slot] = __uint_as_float(e.y);
                }
            }
        }
        my_cnt = 0;
    };

    const uint32_t begin = blockIdx.x * items_per_block;
    uint32_t end = begin + items_per_block;
    if (end > N || end < begin) end = N;
    const float *lds = smem;

    uint32_t w[KF], wn[KF];
    uint32_t g = begin + wave * SB_GROUP;
    if (g < end) {
#pragma unroll
        for (int k = 0; k < KF; ++k)
            w[k] = *reinterpret_cast<const uint32_t *>(fast + (int64_t)k * Npad + g + lane * 4);
    }
    for (; g < end; g += SB_WAVES * SB_GROUP) {
        const uint32_t gn = g + SB_WAVES * SB_GROUP;
        if (gn < end) {   // read ahead; rows are padded so a full group is always addressable
#pragma unroll
            for (int k = 0; k < KF; ++k)
                wn[k] = *reinterpret_cast<const uint32_t *>(fast + (int64_t)k * Npad + gn + lane * 4);
        }
        const int nl = (end - g + 3) / 4 < 64 ? (int)((end - g + 3) / 4) : 64;
#pragma unroll 2
        for (int l = 0; l < nl; ++l) {
            uint32_t s[KF];
#pragma unroll
            for (int k = 0; k < KF; ++k) s[k] = __builtin_amdgcn_readlane(w[k], l);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float P = lds[(0 * ICQ_LUT_W + ((s[0] >> (8 * j)) & 0xffu)) * 64 + lane];
#pragma unroll
                for (int k = 1; k < KF; ++k)
                    P += lds[(k * ICQ_LUT_W + ((s[k] >> (8 * j)) & 0xffu)) * 64 + lane];
                const uint32_t id = g + l * 4 + j;
                const bool hit = (P < t) && (id < end);
                if (__builtin_amdgcn_ballot_w64(hit) != 0) {
                    if (hit) {
                        stage[my_cnt * 64 + lane] = make_uint2(id, __float_as_uint(P));
                        ++my_cnt;
                    }
                    if (__builtin_amdgcn_ballot_w64(my_cnt == SB_STAGE) != 0) flush();
                }
            }
        }
#pragma unroll
        for (int k = 0; k < KF; ++k) w[k] = wn[k];
    }
    flush();
}

// ------------------------------------------------------------------ lanes = items
constexpr int SI_THREADS = 256;

// Block (x = item chunk, y = query group of up to `nb` queries).  LDS holds
// lut[q][k][*] for the group's queries and k < Kf.  Each thread owns 4
// consecutive items per step (one dword of sub-codes per fast row).
template <int KF_MAX>
__global__ __launch_bounds__(SI_THREADS) void scan_items_kernel(
    const uint8_t *__restrict__ fast, int64_t Npad, uint32_t N, const float *__restrict__ lut,
    int K, int Kf, const float *__restrict__ thr, int Q, int nb, uint32_t *__restrict__ cand_ids,
    float *__restrict__ cand_part, uint32_t *__restrict__ cand_count, int64_t cap,
    uint32_t items_per_block) {
    extern __shared__ float smem[];
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int qbase = blockIdx.y * nb;
    const int nq = (Q - qbase) < nb ? (Q - qbase) : nb;

    for (int i = tid; i < nq * Kf * ICQ_LUT_W; i += SI_THREADS) {
        int b = i / (Kf * ICQ_LUT_W), r = i % (Kf * ICQ_LUT_W);
        smem[i] = lut[((int64_t)(qbase + b) * K) * ICQ_LUT_W + r];
    }
    __syncthreads();

    const uint32_t begin = blockIdx.x * items_per_block;
    uint32_t end = begin + items_per_block;
    if (end > N || end < begin) end = N;

    for (uint32_t g = begin + tid * 4; g < end; g += SI_THREADS * 4) {
        uint32_t w[KF_MAX];
#pragma unroll
        for (int k = 0; k < KF_MAX; ++k)
            if (k < Kf) w[k] = *reinterpret_cast<const uint32_t *>(fast + (int64_t)k * Npad + g);
        for (int b = 0; b < nq; ++b) {
            const float *T = smem + b * Kf * ICQ_LUT_W;
            const float t = thr[qbase + b];
            const int64_t row = (int64_t)(qbase + b) * cap;
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                float P = T[(w[0] >> (8 * j)) & 0xffu];
#pragma unroll
                for (int k = 1; k < KF_MAX; ++k)
                    if (k < Kf) P += T[k * ICQ_LUT_W + ((w[k] >> (8 * j)) & 0xffu)];
                const uint32_t id = g + j;
                const bool hit = (P < t) && (id < end);
                const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
                if (mask != 0) {
                    uint32_t base = 0;
                    const int leader = __builtin_ctzll(mask);
                    if ((int)lane == leader)
                        base = atomicAdd(&cand_count[qbase + b], (uint32_t)__builtin_popcountll(mask));
                    base = __builtin_amdgcn_readlane(base, leader);
                    if (hit) {
                        uint64_t slot = (uint64_t)base + __builtin_popcountll(mask & ((1ull << lane) - 1));
                        if (slot < (uint64_t)cap) {
                            cand_ids[row + slot] = id;
                            cand_part[row + slot] = P;
                        }
                    }
                }
            }
        }
    }
}

template <int KF>
int launch_batch(const icq_index *ix, int Q, const float *thr, uint32_t *cand_ids, float *cand_part,
                 uint32_t *cand_count, int64_t cap, const float *lutT, hipStream_t s) {
    const int tiles = (Q + 63) / 64;
    const size_t lds = sizeof(float) * KF * ICQ_LUT_W * 64 + sizeof(uint2) * SB_WAVES * 64 * SB_STAGE;
    static bool attr_set = false;   // idempotent; a race only repeats the call
    if (!attr_set) {
        ICQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_batch_kernel<KF>),
                                        hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds));
        attr_set = true;
    }
    // enough blocks to fill the chip ~8 times over, chunk a multiple of one block step
    const uint32_t step = SB_WAVES * SB_GROUP;
    int64_t chunks = (8LL * ix->num_cu + tiles - 1) / tiles;
    int64_t max_chunks = (ix->N + step - 1) / step;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    uint32_t per = (uint32_t)(((ix->N + chunks - 1) / chunks + step - 1) / step * step);
    chunks = (ix->N + per - 1) / per;
    dim3 grid((unsigned)chunks, (unsigned)tiles);
    scan_batch_kernel<KF><<<grid, SB_THREADS, lds, s>>>(ix->fast, ix->Npad, (uint32_t)ix->N, lutT,
                                                        thr, Q, cand_ids, cand_part, cand_count,
                                                        cap, per);
    return icq_check_launch();
}

}  // namespace

int icq_launch_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                    uint32_t *cand_ids, float *cand_part, uint32_t *cand_count, int64_t cap,
                    float *lutT, hipStream_t s) {
    if (Q == 0) return ICQ_OK;
    zero_counts_kernel<<<(Q + 255) / 256, 256, 0, s>>>(cand_count, Q);
    if (ix->N == 0) return icq_check_launch();

    if (ix->Kf <= 2 && Q >= 8) {
        const int tiles = (Q + 63) / 64;
        dim3 g((unsigned)tiles, (unsigned)ix->Kf);
        transpose_fast_lut_kernel<<<g, 256, 0, s>>>(lut, Q, ix->K, ix->Kf, lutT);
        if (ix->Kf == 1)
            return launch_batch<1>(ix, Q, thr, cand_ids, cand_part, cand_count, cap, lutT, s);
        return launch_batch<2>(ix, Q, thr, cand_ids, cand_part, cand_count, cap, lutT, s);
    }

    // lanes = items: group size limited by LDS (64 KB of tables per block)
    int nb = 64 / ix->Kf;
    if (nb < 1) nb = 1;
    if (nb > 16) nb = 16;
    if (nb > Q) nb = Q;
    const int groups = (Q + nb - 1) / nb;
    const size_t lds = sizeof(float) * (size_t)nb * ix->Kf * ICQ_LUT_W;
    const uint32_t step = SI_THREADS * 4;
    int64_t chunks = (8LL * ix->num_cu + groups - 1) / groups;
    int64_t max_chunks = (ix->N + step - 1) / step;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    uint32_t per = (uint32_t)(((ix->N + chunks - 1) / chunks + step - 1) / step * step);
    chunks = (ix->N + per - 1) / per;
    dim3 grid((unsigned)chunks, (unsigned)groups);
#define ICQ_SI_LAUNCH(KFM)                                                                          \
    do {                                                                                            \
        static bool attr_set = false;                                                               \
        if (!attr_set) {                                                                            \
            ICQ_HIP_TRY(hipFuncSetAttribute(reinterpret_cast<const void *>(&scan_items_kernel<KFM>),\
                                            hipFuncAttributeMaxDynamicSharedMemorySize, 65536));    \
            attr_set = true;                                                                        \
        }                                                                                           \
        scan_items_kernel<KFM><<<grid, SI_THREADS, lds, s>>>(ix->fast, ix->Npad, (uint32_t)ix->N,   \
                                                             lut, ix->K, ix->Kf, thr, Q, nb,        \
                                                             cand_ids, cand_part, cand_count, cap,  \
                                                             per);                                  \
    } while (0)
    if (ix->Kf <= 4) ICQ_SI_LAUNCH(4);
    else if (ix->Kf <= 16) ICQ_SI_LAUNCH(16);
    else ICQ_SI_LAUNCH(64);
#undef ICQ_SI_LAUNCH
    return icq_check_launch();
}

ICQ_EXPORT int icq_scan_fast(const icq_index *ix, const float *lut, int Q, const float *thresholds,
                             uint32_t *cand_ids, float *cand_part, uint32_t *cand_count,
                             int64_t cap, void *workspace, size_t workspace_bytes, void *stream) {
    if (!ix || Q < 0 || Q > (1 << 22) || cap < 1) return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if (!lut || !thresholds || !cand_ids || !cand_part || !cand_count) return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    icq_ws_layout L = icq_layout(ix, Q, cap, 1, false, false);
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < L.total)
        return ICQ_ERR_WORKSPACE;
    float *lutT = reinterpret_cast<float *>(static_cast<char *>(workspace) + L.lutT_off);
    return icq_launch_scan(ix, lut, Q, thresholds, cand_ids, cand_part, cand_count, cap, lutT,
                           (hipStream_t)stream);
}
