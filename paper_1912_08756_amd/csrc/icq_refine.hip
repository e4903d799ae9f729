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
#include "icq_sort.h"

namespace {

constexpr int RF_THREADS = ICQ_SORT_THREADS;   // block_sort runs with the whole block

__device__ __forceinline__ uint32_t order_bits(float x) { return icq_order_bits(x); }
__device__ __forceinline__ float unorder_bits(uint32_t u) { return icq_unorder_bits(u); }

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
    const uint32_t *__restrict__ perm, const uint32_t *__restrict__ cand_count, int64_t cap, int topk,
    int bufn, int splits, u64 *__restrict__ keys_out, uint32_t *__restrict__ out_ids,
    float *__restrict__ out_dist) {
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
            const u64 key = ((u64)order_bits(D) << 32) | (perm ? perm[id] : id);
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

// grid (Q): join the lists of one query when every list is already ascending (pads last) and all
// keys differ: a key's row is the number of keys below it, one binary search per list, no sort.
// LDS: keys[parts * topk].
__global__ __launch_bounds__(RF_THREADS) void merge_sorted_kernel(const u64 *__restrict__ keys_in, int parts,
                                                                  int topk, uint32_t *__restrict__ out_ids,
                                                                  float *__restrict__ out_dist) {
    extern __shared__ u64 smem64[];
    u64 *keys = smem64;
    __shared__ int s_real;
    const int q = blockIdx.x;
    const int n = parts * topk;
    if (threadIdx.x == 0) s_real = 0;
    for (int i = threadIdx.x; i < n; i += RF_THREADS) keys[i] = keys_in[(int64_t)q * n + i];
    __syncthreads();
    auto below = [&](const u64 *list, u64 k) -> int {      // keys of an ascending list that are < k
        int lo = 0, hi = topk;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            if (list[mid] < k) lo = mid + 1;
            else hi = mid;
        }
        return lo;
    };
    if ((int)threadIdx.x < parts) atomicAdd(&s_real, below(keys + threadIdx.x * topk, KEY_PAD));
    for (int i = threadIdx.x; i < n; i += RF_THREADS) {
        const u64 k = keys[i];
        if (k == KEY_PAD) continue;
        int rank = 0;
        for (int p = 0; p < parts && rank < topk; ++p) rank += below(keys + p * topk, k);
        if (rank < topk) {
            out_ids[(int64_t)q * topk + rank] = (uint32_t)k;
            out_dist[(int64_t)q * topk + rank] = unorder_bits((uint32_t)(k >> 32));
        }
    }
    __syncthreads();
    for (int r = s_real + (int)threadIdx.x; r < topk; r += RF_THREADS) {
        out_ids[(int64_t)q * topk + r] = ICQ_PAD_ID;
        out_dist[(int64_t)q * topk + r] = INFINITY;
    }
}

int bufn_for(int topk) { return topk <= 256 ? 2048 : 4096; }

// ------------------------------------------------------------------ distances, then bounded select
// Stage 2 runs as two kernels.
//   refine_dist_kernel: flat over all candidates of all queries, many small blocks at
//     full occupancy.  A block owns RD_BLOCK consecutive candidates of one query,
//     keeps that query's tables in LDS (one table per record byte; tables that do not
//     take part are zero, so the sum has no conditions) and writes one 64-bit key
//     (order-preserving bits of D, item id) per candidate.
//   select_keys_kernel: one wavefront per (query, slice) streams the keys.  An exact
//     radix select (8-bit digits over the occupied range, LDS histogram) over the first
//     512 keys gives their topk-th distance, the bound; afterwards only keys at or
//     below the bound enter a key list (ballot compaction).  Whenever the list could
//     overflow it is bitonic-sorted, cut to topk and the bound tightened; the final
//     sort orders the result.
constexpr int RD_PER = 8;                            // candidates per thread and step
constexpr int RD_STEP = RF_THREADS * RD_PER;         // 2048
constexpr int RD_BLOCK = 2 * RD_STEP;                // candidates per block

template <int WORDS>
__global__ __launch_bounds__(RF_THREADS) void refine_dist_kernel(
    const uint8_t *__restrict__ items, int K, int Kf, const float *__restrict__ lut,
    const uint32_t *__restrict__ cand_ids, const float *__restrict__ cand_part,
    const uint32_t *__restrict__ cand_count, int64_t cap, int blocks_per_query, u64 *__restrict__ keys) {
    __shared__ float T[4 * WORDS * ICQ_LUT_W];
    constexpr int RW = WORDS;                         // words per item record
    // Blocks are numbered piece-major: blocks that run together take the same stretch of every
    // query's list.  The lists follow the scan order, so those stretches hold ids from the same
    // regions of the item records, and a record line fetched for one query is still cached when
    // the other queries' candidates in it are gathered.
    const int nq = gridDim.x / blocks_per_query;
    const int q = blockIdx.x % nq;
    const u64 c0 = (u64)(blockIdx.x / nq) * RD_BLOCK;
    const int tid = threadIdx.x;
    u64 n = cand_count[q];
    if (n > (u64)cap) n = (u64)cap;
    if (c0 >= n) return;                              // block-uniform
    const int k0 = cand_part ? Kf : 0;
    const uint32_t *ids = cand_ids + (int64_t)q * cap;
    const float *part = cand_part ? cand_part + (int64_t)q * cap : nullptr;
    u64 *out = keys + (int64_t)q * cap;

    // Loads are unconditional with the index clamped to the last candidate: without
    // branches around them they all go out back to back and are waited for once.
    uint32_t id[2][RD_PER], rec[2][RD_PER][RW];
    float D[2][RD_PER];
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int j = 0; j < RD_PER; ++j) {
            const u64 i = c0 + (u64)st * RD_STEP + j * RF_THREADS + tid;
            const u64 ic = i < n ? i : n - 1;
            id[st][j] = ids[ic];
            D[st][j] = part ? part[ic] : 0.0f;
        }
    }
    {   // tables -> LDS
        const float4 *src = reinterpret_cast<const float4 *>(lut + (int64_t)q * K * ICQ_LUT_W);
        float4 *dst = reinterpret_cast<float4 *>(T);
        constexpr int N4 = 4 * WORDS * (ICQ_LUT_W / 4);
        float4 v[(N4 + RF_THREADS - 1) / RF_THREADS];
#pragma unroll
        for (int r = 0; r < (N4 + RF_THREADS - 1) / RF_THREADS; ++r) {
            const int i = r * RF_THREADS + tid;
            const int k = i / (ICQ_LUT_W / 4);
            v[r] = (i < N4 && k >= k0 && k < K) ? src[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int r = 0; r < (N4 + RF_THREADS - 1) / RF_THREADS; ++r) {
            const int i = r * RF_THREADS + tid;
            if (i < N4) dst[i] = v[r];
        }
    }
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int j = 0; j < RD_PER; ++j) {
            const uint32_t *p = reinterpret_cast<const uint32_t *>(items + (size_t)id[st][j] * (RW * 4));
            if (RW == 1) {
                rec[st][j][0] = p[0];
            } else if (RW == 2) {
                const uint2 v = *reinterpret_cast<const uint2 *>(p);
                rec[st][j][0] = v.x;
                rec[st][j][1 % RW] = v.y;
            } else {
#pragma unroll
                for (int w4 = 0; w4 < RW / 4; ++w4) {
                    const uint4 v = reinterpret_cast<const uint4 *>(p)[w4];
                    rec[st][j][(4 * w4) % RW] = v.x;
                    rec[st][j][(4 * w4 + 1) % RW] = v.y;
                    rec[st][j][(4 * w4 + 2) % RW] = v.z;
                    rec[st][j][(4 * w4 + 3) % RW] = v.w;
                }
            }
        }
    }
    __syncthreads();
#pragma unroll
    for (int st = 0; st < 2; ++st) {
#pragma unroll
        for (int j = 0; j < RD_PER; ++j) {
            float d = D[st][j];
#pragma unroll
            for (int w = 0; w < WORDS; ++w) {
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    d += T[(w * 4 + b) * ICQ_LUT_W + ((rec[st][j][w] >> (8 * b)) & 0xffu)];
            }
            const u64 i = c0 + (u64)st * RD_STEP + j * RF_THREADS + tid;
            if (i < n) out[i] = ((u64)order_bits(d) << 32) | id[st][j];
        }
    }
}

// One WAVEFRONT per (query, slice): nothing in the select needs more than 64 lanes,
// and a one-wavefront block pays no barrier waits, so a CU keeps ~15 independent
// selects in flight instead of 3 barrier-bound blocks.
constexpr int SK_THREADS = 64;
constexpr int SK_CHUNK = 8;                           // keys per lane and chunk
constexpr int SK_FIRST = SK_THREADS * SK_CHUNK;       // 512

struct SelectShared {
    uint32_t hist[256];
    uint32_t bin, below, cnt;
};

// Locate the bin that holds the kr-th smallest element (1-based) of a complete
// 256-bin histogram with one wavefront (4 bins per lane).
__device__ __forceinline__ void find_bin(SelectShared *sh, uint32_t kr) {
    const int lane = threadIdx.x;
    uint32_t h[4], mine = 0;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        h[r] = sh->hist[lane * 4 + r];
        mine += h[r];
    }
    const uint32_t incl = wave_scan_add(mine);
    uint32_t run = incl - mine;
#pragma unroll
    for (int r = 0; r < 4; ++r) {
        if (run < kr && run + h[r] >= kr) {
            sh->bin = (uint32_t)(lane * 4 + r);
            sh->below = run;
        }
        run += h[r];
    }
    __syncthreads();
}

// The kr-th smallest (1-based) of U[0..n), n >= kr >= 1; vmin/vmax bound the values.
__device__ uint32_t wave_radix_select(SelectShared *sh, const uint32_t *U, uint32_t n, uint32_t kr,
                                      uint32_t vmin, uint32_t vmax) {
    const int tid = threadIdx.x;
    const uint32_t range = vmax - vmin;
    const int bits = range == 0 ? 0 : 32 - __builtin_clz(range);
    int shift = bits > 8 ? bits - 8 : 0;
    int width = bits < 8 ? bits : 8;
    uint32_t prefix = 0;       // chosen high digits of (value - vmin)
    int fixed_from = bits;     // bits [fixed_from, 32) of (value - vmin) are decided
    for (;;) {
#pragma unroll
        for (int r = 0; r < 4; ++r) sh->hist[tid * 4 + r] = 0;
        __syncthreads();
        const uint32_t dmask = (1u << width) - 1u;
        for (uint32_t i = tid; i < n; i += SK_THREADS) {
            const uint32_t y = U[i] - vmin;
            const bool match = fixed_from >= 32 ? true : (y >> fixed_from) == prefix;
            if (match) atomicAdd(&sh->hist[(y >> shift) & dmask], 1u);
        }
        __syncthreads();
        find_bin(sh, kr);
        kr -= sh->below;
        prefix = (prefix << width) | sh->bin;
        fixed_from = shift;
        if (shift == 0) break;
        const int ns = shift > 8 ? shift - 8 : 0;
        width = shift - ns;
        shift = ns;
        __syncthreads();
    }
    return vmin + prefix;
}

// Cut the list back to its topk smallest distances (ties at the cut kept): exact radix
// select of the topk-th distance, then an in-place ballot compaction.  One wavefront,
// cnt <= 1024 (wave-uniform), cnt > topk.  Returns the new count; *ubound = the cut.
__device__ uint32_t wave_cut_list(SelectShared *sh, u64 *list, uint32_t *U, uint32_t cnt, int topk,
                                  uint32_t *ubound) {
    const int lane = threadIdx.x;
    u64 x[16];
    uint32_t umin = 0xFFFFFFFFu, umax = 0u;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        const uint32_t i = r * 64 + lane;
        x[r] = i < cnt ? list[i] : KEY_PAD;
        if (i < cnt) {
            const uint32_t u = (uint32_t)(x[r] >> 32);
            U[i] = u;
            umin = u < umin ? u : umin;
            umax = u > umax ? u : umax;
        }
    }
    umin = wave_min_u32(umin);
    umax = wave_max_u32(umax);
    __syncthreads();
    const uint32_t cut = wave_radix_select(sh, U, cnt, (uint32_t)topk, umin, umax);
    __syncthreads();
    uint32_t kept = 0;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if ((uint32_t)(r * 64) < cnt) {   // wave-uniform
            const bool keep = (uint32_t)(r * 64 + lane) < cnt && (uint32_t)(x[r] >> 32) <= cut;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(keep);
            if (keep) list[kept + __builtin_popcountll(mask & ((1ull << lane) - 1))] = x[r];
            kept += (uint32_t)__builtin_popcountll(mask);
        }
    }
    __syncthreads();
    *ubound = cut;
    return kept;
}

// grid (Q * splits), block = one wavefront.  LDS: list[listcap] (u64) | U[listcap] (u32);
// listcap is a power of two, topk + SK_FIRST <= listcap <= 1024... 2048 (see launcher).
__global__ __launch_bounds__(SK_THREADS) __attribute__((amdgpu_waves_per_eu(3, 8))) void select_keys_kernel(
    const u64 *__restrict__ keys_in, const uint32_t *__restrict__ cand_count, int64_t cap, int topk,
    int listcap, int splits, u64 *__restrict__ keys_out, uint32_t *__restrict__ out_ids,
    float *__restrict__ out_dist) {
    extern __shared__ u64 smem64[];
    __shared__ SelectShared sh;
    u64 *list = smem64;
    uint32_t *U = reinterpret_cast<uint32_t *>(list + listcap);
    const int q = blockIdx.x / splits, sp = blockIdx.x % splits;
    const int tid = threadIdx.x;
    u64 ntot = cand_count[q];
    if (ntot > (u64)cap) ntot = (u64)cap;
    const u64 lo = ntot * (u64)sp / (u64)splits, hi = ntot * (u64)(sp + 1) / (u64)splits;
    const u64 n = hi - lo;
    const u64 *in = keys_in + (int64_t)q * cap + lo;

    uint32_t ubound = 0xFFFFFFFFu;   // keep keys whose distance bits are <= ubound
    uint32_t cnt = 0;                // keys in the list (wave-uniform)
    // Keys are loaded one chunk ahead, unconditionally with the index clamped.
    auto load_chunk = [&](u64 c, u64(&k)[SK_CHUNK]) {
#pragma unroll
        for (int j = 0; j < SK_CHUNK; ++j) {
            const u64 i = c + (u64)j * SK_THREADS + tid;
            k[j] = in[i < n ? i : n - 1];
        }
    };
    auto step = [&](u64 c, u64(&kA)[SK_CHUNK], u64(&kNext)[SK_CHUNK]) {   // wave-uniform c < n
        load_chunk(c + (u64)SK_FIRST, kNext);   // one chunk ahead
        if (c == 0 && n > (u64)topk && (uint32_t)topk < (uint32_t)SK_FIRST) {
            // first chunk: its topk-th smallest distance bounds everything that follows
            const uint32_t n1 = n < (u64)SK_FIRST ? (uint32_t)n : (uint32_t)SK_FIRST;
            uint32_t umin = 0xFFFFFFFFu, umax = 0u;
#pragma unroll
            for (int j = 0; j < SK_CHUNK; ++j) {
                const uint32_t i = j * SK_THREADS + tid;
                const uint32_t u = (uint32_t)(kA[j] >> 32);
                if (i < n1) {
                    U[i] = u;
                    umin = u < umin ? u : umin;
                    umax = u > umax ? u : umax;
                }
            }
            umin = wave_min_u32(umin);
            umax = wave_max_u32(umax);
            __syncthreads();
            if (n1 > (uint32_t)topk) ubound = wave_radix_select(&sh, U, n1, (uint32_t)topk, umin, umax);
        }
        // keep what is at or below the bound (ties at the bound included; the final sort
        // decides); ballot compaction, the list cursor is wave-uniform
#pragma unroll
        for (int j = 0; j < SK_CHUNK; ++j) {
            const u64 i = c + (u64)j * SK_THREADS + tid;
            const bool keep = i < n && (uint32_t)(kA[j] >> 32) <= ubound;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(keep);
            if (keep) list[cnt + __builtin_popcountll(mask & ((1ull << tid) - 1))] = kA[j];
            cnt += (uint32_t)__builtin_popcountll(mask);
        }
        if (cnt > (uint32_t)(listcap - SK_FIRST) && c + SK_FIRST < n) {
            // the next chunk might not fit: cut the list back to topk, tighten the bound
            __syncthreads();
            cnt = wave_cut_list(&sh, list, U, cnt, topk, &ubound);
            if (cnt > (uint32_t)(listcap - SK_FIRST)) {
                // so many ties at the cut that the list is still too full: order by the
                // whole key and keep exactly topk (the ids decide among equal distances)
                for (int i = (int)cnt + tid; i < listcap; i += SK_THREADS) list[i] = KEY_PAD;
                __syncthreads();
                wave_sort(list, listcap, threadIdx.x);
                __syncthreads();
                cnt = (uint32_t)topk;
                ubound = (uint32_t)(list[topk - 1] >> 32);
            }
        }
    };
    if (n > 0) {
        u64 k0[SK_CHUNK], k1[SK_CHUNK];
        load_chunk(0, k0);
        for (u64 c = 0; c < n; c += 2 * (u64)SK_FIRST) {
            step(c, k0, k1);
            if (c + SK_FIRST < n) step(c + SK_FIRST, k1, k0);
        }
    }

    // ---- final order: cut to the topk smallest distances, then sort what is left
    __syncthreads();
    if (cnt > (uint32_t)topk) cnt = wave_cut_list(&sh, list, U, cnt, topk, &ubound);
    int len = 64;
    while (len < (int)cnt) len <<= 1;
    for (int i = (int)cnt + tid; i < len; i += SK_THREADS) list[i] = KEY_PAD;
    __syncthreads();
    wave_sort(list, len, threadIdx.x);
    __syncthreads();
    const int kept = (int)cnt < topk ? (int)cnt : topk;
    uint32_t *oi = out_ids + (int64_t)q * topk;
    float *od = out_dist + (int64_t)q * topk;
    u64 *dst = keys_out + ((int64_t)q * splits + sp) * topk;
    for (int r = tid; r < topk; r += SK_THREADS) {
        if (splits == 1) {
            oi[r] = r < kept ? (uint32_t)list[r] : ICQ_PAD_ID;
            od[r] = r < kept ? unorder_bits((uint32_t)(list[r] >> 32)) : INFINITY;
        } else {
            dst[r] = r < kept ? list[r] : KEY_PAD;
        }
    }
}

// ------------------------------------------------------------------ stage 2 from hit bits
// icq_search with the item-by-item stage 1: stage 1 leaves one hit bit per scan position and query,
// and this kernel turns them into distances and keys.  The positions are cut into chunks of 32768
// (4 KB of hit bits per query, 512 KB of 16-byte item records).  A block belongs to ONE query --
// its tables stay in LDS for the block's whole life -- and walks a window of a few chunks, its
// four wavefronts a chunk at a time each and each on its own (no barrier after the tables are
// in place).  Workgroups go round the 8 XCDs in turn, each XCD has a cache of its own (block x of
// the grid is on XCD x % 8), and they start in the order of their numbers: the blocks are
// numbered window by window, within a window query by query, then XCD -- so the blocks of ALL
// queries of the batch that walk the same window run on the same XCD at about the same time,
// the chip holds the blocks of two windows at once, and that XCD has a few chunks' records in its
// cache at a time.  An item that survives for several queries of the batch -- or shares its cache
// line with one that does -- is then fetched from memory once: with 1 % survivors and 128
// queries that is ten uses per 128-byte line.  Per chunk and wavefront: the query's 256 words of hit
// bits (one 128-bit load per lane, two chunks ahead), a prefix of their popcounts, the set bits
// expanded into a position list in the wavefront's part of LDS, then per position the record
// gather, the K table reads and the key, as in refine_dist_kernel.
// Every 65th chunk is done in a first launch, unfiltered (!FILTER); the select kernel's topk-th
// distance of those keys then bounds what the other chunks add in a second launch (FILTER: keys
// above it are dropped; ties at it are kept, the final select decides).  The final lists are
// unchanged -- at least topk keys at or below the bound are already there -- and the key lists
// shrink to a few per cent.  Survivors are counted from the popcounts.
constexpr int RM_THREADS = 256;
constexpr int RM_WAVES = RM_THREADS / 64;
constexpr uint32_t RM_CHUNK = 32768;                  // positions per chunk; a multiple of the scan kernel's block step
constexpr int RM_WORDS = RM_CHUNK / 32 / 64;          // 32-bit words of hit bits per lane and chunk
constexpr int RM_PER = 4;                             // records a lane gathers together
constexpr int RM_LIST = 512;                          // positions a wavefront expands per round
constexpr int RM_QPB = 1;                             // queries per block (two: 1.39 against 1.25 ms at N = 1e8, 128 queries)
constexpr int RM_SEED_EVERY = 65;                     // odd: the first launch's chunks are spread over all XCDs
static_assert(RM_LIST % (64 * RM_PER) == 0, "a round of the list is whole steps of gathers");
static_assert(RM_CHUNK <= 65536, "the position lists hold 16-bit offsets into the chunk");

// QPB queries per block: their tables sit in LDS side by side and every chunk is worked through for one
// query after the other, so the later ones find the chunk's records in the cache for certain.
// EXACT: the hit bits mark a superset of the survivors (the 16-bit pre-filter of stage 1); an item is a
// survivor when the first Kf terms of its sum -- the crude distance of Eq. 2, the same fp32 additions
// stage 1 makes item by item -- are below thr[q].  Only survivors are counted and get keys.
// The filtered launch is held to the registers of five wavefronts per SIMD (the exact comparison's few
// more would cost the fifth: 1.17 -> 1.29 ms for the stage at N = 1e8).
template <int WORDS, bool FILTER, int QPB, bool EXACT>
__global__ __launch_bounds__(RM_THREADS, FILTER ? 5 : 1) void refine_mask_kernel(
    const uint8_t *__restrict__ items, int K, const float *__restrict__ lut, const uint32_t *__restrict__ masks,
    size_t mask_words, const uint32_t *__restrict__ perm, uint32_t nsel, uint32_t seed_every, int window, int xs_shift, int Q,
    const float *__restrict__ kth_dist, int topk, u64 *__restrict__ keys, uint32_t *__restrict__ key_count,
    int64_t cap, uint32_t *__restrict__ cand_count, const float *__restrict__ thr, int Kf) {
    __shared__ __attribute__((aligned(16))) float T_all[QPB][4 * WORDS * ICQ_LUT_W];
    __shared__ uint16_t cand_all[RM_WAVES][RM_LIST];  // positions inside the chunk (RM_CHUNK <= 65536)
    constexpr int RW = WORDS;
    const int tid = threadIdx.x;
    const uint32_t lane = (uint32_t)tid & 63u;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    uint16_t *cand = cand_all[wave];
    // block -> (window, query group, XCD): chunks i = (win * window + j) * 8 + xcd, j = 0 .. window - 1, of this
    // launch's; wavefront w takes j = w, w + 4, ..  (An index of few chunks is cut 2^xs_shift < 8 ways instead, so
    // that a block still has a window's worth of chunks for the tables it loads.)
    const uint32_t ngroups = ((uint32_t)Q + QPB - 1) / QPB;
    const uint32_t xcd = blockIdx.x & ((1u << xs_shift) - 1u), rest = blockIdx.x >> xs_shift;
    const uint32_t q0 = (rest % ngroups) * QPB, win = rest / ngroups;
    const uint32_t nq = (uint32_t)Q - q0 < (uint32_t)QPB ? (uint32_t)Q - q0 : (uint32_t)QPB;
    auto chunk_of = [&](uint32_t j) -> uint32_t {
        const uint32_t i = ((win * (uint32_t)window + j) << xs_shift) + xcd;
        if (j >= (uint32_t)window || i >= nsel) return 0xFFFFFFFFu;
        return FILTER ? i + i / (seed_every - 1u) + 1u : i * seed_every;   // the others : every seed_every-th
    };
    if (chunk_of(0) == 0xFFFFFFFFu) return;           // block-uniform: nothing for this block
    // Word r of this lane covers the 32 positions from c * RM_CHUNK + (r * 64 + lane) * 32: neighbouring
    // words sit in neighbouring lanes, so a dense stretch of hits is shared out among many lanes.
    // The wavefront's work is the sequence (chunk j, query qq), qq fastest; the next one's hit bits travel
    // while the current one is worked on.
    const uint32_t *mq = masks + (size_t)q0 * mask_words + lane;
    uint32_t j = (uint32_t)wave, qq = 0;
    uint32_t c = chunk_of(j);
    uint32_t nxt[RM_WORDS];
    {
        const uint32_t c0 = c != 0xFFFFFFFFu ? c : 0u;
#pragma unroll
        for (int r = 0; r < RM_WORDS; ++r) nxt[r] = __builtin_nontemporal_load(mq + (size_t)c0 * (RM_CHUNK / 32) + r * 64);
    }
    // the queries' tables -> LDS, one table per record byte, zero beyond K
#pragma unroll
    for (int g = 0; g < QPB; ++g) {
        const uint32_t qg = q0 + ((uint32_t)g < nq ? (uint32_t)g : 0u);
        const float4 *src = reinterpret_cast<const float4 *>(lut + (int64_t)qg * K * ICQ_LUT_W);
        float4 *dst = reinterpret_cast<float4 *>(T_all[g]);
        constexpr int N4 = 4 * WORDS * (ICQ_LUT_W / 4);
        float4 v[N4 / RM_THREADS];
#pragma unroll
        for (int u = 0; u < N4 / RM_THREADS; ++u) {
            const int i = u * RM_THREADS + tid;
            v[u] = i / (ICQ_LUT_W / 4) < K ? src[i] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
        }
#pragma unroll
        for (int u = 0; u < N4 / RM_THREADS; ++u) dst[u * RM_THREADS + tid] = v[u];
    }
    uint32_t bound_all[QPB];
#pragma unroll
    for (int g = 0; g < QPB; ++g) {
        bound_all[g] = 0xFFFFFFFFu;
        if (FILTER) {
            const uint32_t qg = q0 + ((uint32_t)g < nq ? (uint32_t)g : 0u);
            const uint32_t ob = icq_order_bits(kth_dist[(int64_t)qg * topk + topk - 1]);
            if (ob < 0xFF800000u) bound_all[g] = ob;  // a finite topk-th distance; else the list is still open
        }
    }
    __syncthreads();                                  // the only barrier: from here on every wavefront is on its own
    uint32_t survivors[QPB];                          // of this wavefront's chunks (wavefront-uniform)
    uint32_t lane_survivors[QPB];                     // EXACT: counted per lane, summed at the end
#pragma unroll
    for (int g = 0; g < QPB; ++g) survivors[g] = lane_survivors[g] = 0;
    while (c != 0xFFFFFFFFu) {
        uint32_t w[RM_WORDS];
#pragma unroll
        for (int r = 0; r < RM_WORDS; ++r) w[r] = nxt[r];
        // next piece of work: the next query of this chunk, else the wavefront's next chunk
        uint32_t qn = qq + 1, jn = j, cn = c;
        if (qn >= nq) {
            qn = 0;
            jn = j + RM_WAVES;
            cn = chunk_of(jn);
        }
        if (cn != 0xFFFFFFFFu) {
            const uint32_t *mn = mq + (size_t)qn * mask_words + (size_t)cn * (RM_CHUNK / 32);
#pragma unroll
            for (int r = 0; r < RM_WORDS; ++r) nxt[r] = __builtin_nontemporal_load(mn + r * 64);
        }
        const uint32_t q = q0 + qq;
        const float tq = EXACT ? thr[q] : 0.0f;
        const float *T = T_all[QPB == 1 ? 0 : qq];
        uint32_t bound = bound_all[0];
#pragma unroll
        for (int g = 1; g < QPB; ++g) bound = qq == (uint32_t)g ? bound_all[g] : bound;
        u64 *kout = keys + (int64_t)q * cap;
        uint32_t mine = 0;
#pragma unroll
        for (int r = 0; r < RM_WORDS; ++r) mine += (uint32_t)__builtin_popcount(w[r]);
        const uint32_t incl = wave_scan_add(mine);
        const uint32_t total = (uint32_t)__builtin_amdgcn_readlane((int)incl, 63);
        const uint32_t off = incl - mine;
        if (!EXACT) {
#pragma unroll
            for (int g = 0; g < QPB; ++g) survivors[g] += qq == (uint32_t)g ? total : 0u;
        }
        // unfiltered: every survivor of the chunk gets a key, so their slots are reserved at once (the atomic's
        // answer travels while the positions are expanded)
        uint32_t chunk_slot = 0;
        if (!FILTER && !EXACT && total != 0) {
            if (lane == 0) chunk_slot = atomicAdd(&key_count[q], total);
        }
        const uint32_t cbase = c * RM_CHUNK, p0 = lane * 32u;
        for (uint32_t lo = 0; lo < total; lo += RM_LIST) {      // wavefront-uniform; one round unless the chunk is dense
            __builtin_amdgcn_wave_barrier();          // LDS runs a wavefront's accesses in order: the last round's reads are done
            if (off + mine > lo && off < lo + RM_LIST) {
                uint32_t idx = off - lo;              // wraps below the window: fails the test until it is inside
#pragma unroll
                for (int r = 0; r < RM_WORDS; ++r) {
                    uint32_t m = w[r];
                    while (m != 0) {
                        const uint32_t bit = (uint32_t)__builtin_ctz(m);
                        m &= m - 1;
                        if (idx < (uint32_t)RM_LIST) cand[idx] = (uint16_t)(p0 + (uint32_t)r * 2048u + bit);
                        ++idx;
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
            const uint32_t n = total - lo < (uint32_t)RM_LIST ? total - lo : (uint32_t)RM_LIST;
            for (uint32_t base = 0; base < n; base += 64 * RM_PER) {
                uint32_t id[RM_PER], rec[RM_PER][RW];
#pragma unroll
                for (int u = 0; u < RM_PER; ++u) {
                    const uint32_t i = base + (uint32_t)u * 64u + lane;
                    id[u] = cbase + cand[i < n ? i : n - 1];
                }
#pragma unroll
                for (int u = 0; u < RM_PER; ++u) {
                    const uint32_t *p = reinterpret_cast<const uint32_t *>(items + (size_t)id[u] * (RW * 4));
                    if (RW == 1) {
                        rec[u][0] = p[0];
                    } else if (RW == 2) {
                        const uint2 v = *reinterpret_cast<const uint2 *>(p);
                        rec[u][0] = v.x;
                        rec[u][1 % RW] = v.y;
                    } else {
                        const uint4 v = *reinterpret_cast<const uint4 *>(p);
                        rec[u][0] = v.x;
                        rec[u][1 % RW] = v.y;
                        rec[u][2 % RW] = v.z;
                        rec[u][3 % RW] = v.w;
                    }
                }
                u64 key[RM_PER];
                uint64_t mk[RM_PER];
                uint32_t mycnt = 0;
#pragma unroll
                for (int u = 0; u < RM_PER; ++u) {
                    // all table reads of the record first (a read waited for before the next is asked for is a
                    // chain of 4 * WORDS LDS round trips), then the sum: k ascending like every other kernel, the
                    // first term standing for 0 + itself (no table holds -0)
                    float tv[4 * WORDS];
#pragma unroll
                    for (int x = 0; x < WORDS; ++x) {
#pragma unroll
                        for (int b = 0; b < 4; ++b) tv[x * 4 + b] = T[(x * 4 + b) * ICQ_LUT_W + ((rec[u][x] >> (8 * b)) & 0xffu)];
                    }
                    __builtin_amdgcn_sched_barrier(0);
                    float d = tv[0];
                    float crude = d;                  // the sum after its first Kf terms (Kf <= 4: inside the first word)
#pragma unroll
                    for (int i = 1; i < 4 * WORDS; ++i) {
                        d += tv[i];
                        if (EXACT && i < 4) crude = i < Kf ? d : crude;
                    }
                    const uint32_t ob = icq_order_bits(d);
                    bool keep = base + (uint32_t)u * 64u + lane < n;
                    if (EXACT) {
                        keep = keep && crude < tq;
#pragma unroll
                        for (int g = 0; g < QPB; ++g) lane_survivors[g] += (qq == (uint32_t)g && keep) ? 1u : 0u;
                    }
                    keep = keep && ob <= bound;
                    mk[u] = __builtin_amdgcn_ballot_w64(keep);
                    mycnt += (uint32_t)__builtin_popcountll(mk[u]);
                    key[u] = (u64)ob << 32;
                }
                if (mycnt == 0) continue;             // wavefront-uniform
                uint32_t slot0 = 0;
                if (FILTER || EXACT) {
                    if (lane == 0) slot0 = atomicAdd(&key_count[q], mycnt);
                    slot0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)slot0);
                } else {
                    slot0 = (uint32_t)__builtin_amdgcn_readfirstlane((int)chunk_slot) + lo + base;
                }
#pragma unroll
                for (int u = 0; u < RM_PER; ++u) {
                    if ((mk[u] >> lane) & 1ull) {
                        const uint64_t slot = (uint64_t)__builtin_amdgcn_mbcnt_hi(
                            (uint32_t)(mk[u] >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)mk[u], slot0));
                        if (slot < (uint64_t)cap) kout[slot] = key[u] | (perm ? perm[id[u]] : id[u]);
                    }
                    slot0 += (uint32_t)__builtin_popcountll(mk[u]);
                }
            }
        }
        qq = qn;
        j = jn;
        c = cn;
    }
    if (EXACT) {
#pragma unroll
        for (int g = 0; g < QPB; ++g)
            survivors[g] = (uint32_t)__builtin_amdgcn_readlane((int)wave_scan_add(lane_survivors[g]), 63);
    }
#pragma unroll
    for (int g = 0; g < QPB; ++g)
        if (lane == 0 && (uint32_t)g < nq && survivors[g] != 0) atomicAdd(&cand_count[q0 + g], survivors[g]);
}

}  // namespace

// Item records of at most 16 bytes take the bounded-stream kernel; wider records
// (K > 16) the generic streaming kernel.
static bool use_select(const icq_index *ix, int topk) { return ix->item_stride <= 16 && topk <= 512; }

// keys: [Q][splits][topk] keys (bits of D, id), KEY_PAD where a list is short; splits * topk <= 4096.
// ascending: every list is sorted (pads last) and no key occurs twice.
int icq_launch_merge(const unsigned long long *keys, int Q, int splits, int topk, bool ascending,
                     uint32_t *out_ids, float *out_dist, hipStream_t s) {
    if (ascending) {
        merge_sorted_kernel<<<Q, RF_THREADS, sizeof(u64) * splits * topk, s>>>(keys, splits, topk, out_ids, out_dist);
        return icq_check_launch();
    }
    int len = 2;
    while (len < splits * topk) len <<= 1;
    merge_kernel<<<Q, RF_THREADS, sizeof(u64) * len, s>>>(keys, splits, topk, len, out_ids, out_dist);
    return icq_check_launch();
}

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
                      const float *cand_part, int list_kind,
                      const uint32_t *cand_count, int64_t cap, int topk, int splits, u64 *keys,
                      uint32_t *out_ids, float *out_dist, hipStream_t s) {
    if (Q == 0 || list_kind == ICQ_LIST_DONE) return ICQ_OK;
    const uint8_t *items = list_kind == ICQ_LIST_POSITIONS ? ix->items_grouped : ix->items;
    const uint32_t *perm = list_kind == ICQ_LIST_POSITIONS ? ix->perm : nullptr;
    const unsigned grid = (unsigned)Q * (unsigned)splits;
    const size_t tab = sizeof(float) * (size_t)(cand_part ? ix->Ks : ix->K) * ICQ_LUT_W;
    if (use_select(ix, topk)) {
        // distances for every candidate (flat), then the per-query select over the keys
        u64 *cand_keys = icq_cand_keys(keys, Q, splits, topk);   // [Q][cap], behind the slice lists
        int64_t len = cap < ix->N ? cap : ix->N;
        const int bpq = len > 0 ? (int)((len + RD_BLOCK - 1) / RD_BLOCK) : 1;
        const unsigned dgrid = (unsigned)Q * (unsigned)bpq;
        if (list_kind != ICQ_LIST_KEYS) {
#define ICQ_RD_LAUNCH(W)                                                                          \
    refine_dist_kernel<W><<<dgrid, RF_THREADS, 0, s>>>(items, ix->K, ix->Kf, lut, cand_ids,       \
                                                       cand_part, cand_count, cap, bpq, cand_keys)
        switch (ix->item_stride) {
            case 4: ICQ_RD_LAUNCH(1); break;
            case 8: ICQ_RD_LAUNCH(2); break;
            default: ICQ_RD_LAUNCH(4); break;
        }
#undef ICQ_RD_LAUNCH
        if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
        }
        const int listcap = 1024;   // register sort and cut handle up to 1024 keys: topk <= 512 here
        select_keys_kernel<<<grid, SK_THREADS, (sizeof(u64) + sizeof(uint32_t)) * listcap, s>>>(
            cand_keys, cand_count, cap, topk, listcap, splits, keys, out_ids, out_dist);
    } else {
        const int bufn = bufn_for(topk);
        const size_t lds = sizeof(u64) * bufn + tab;
        ICQ_HIP_TRY(icq_allow_lds(reinterpret_cast<const void *>(&refine_kernel), 98304));
        refine_kernel<<<grid, RF_THREADS, lds, s>>>(items, ix->item_stride, ix->K, ix->Kf, lut,
                                                    cand_ids, cand_part, perm, cand_count, cap, topk,
                                                    bufn, splits, keys, out_ids, out_dist);
    }
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    if (splits > 1) return icq_launch_merge(keys, Q, splits, topk, false, out_ids, out_dist, s);
    return ICQ_OK;
}

ICQ_EXPORT int icq_refine(const icq_index *ix, const float *lut, int Q, const uint32_t *cand_ids,
                          const float *cand_part, const uint32_t *cand_count, int64_t cap, int topk,
                          uint32_t *out_ids, float *out_dist, void *workspace,
                          size_t workspace_bytes, void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK)
        return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if (!lut || !cand_ids || !cand_count || !out_ids || !out_dist) return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    icq_ws_layout L = icq_layout(ix, Q, cap, topk, false, false);
    if (L.total > 0 &&
        (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < L.total))
        return ICQ_ERR_WORKSPACE;
    u64 *keys = reinterpret_cast<u64 *>(static_cast<char *>(workspace) + L.keys_off);
    return icq_launch_refine(ix, lut, Q, cand_ids, cand_part, ICQ_LIST_IDS, cand_count, cap, topk,
                             L.splits, keys, out_ids, out_dist, (hipStream_t)stream);
}

// From about four million items on: below that the item records stay in the caches whatever the
// order of the gathers, and candidate lists with the flat distance kernel are quicker (N = 1e6,
// K = 16, 1000 queries: 0.15 against 0.24 ms for stage 2).
bool icq_masks_usable(const icq_index *ix, int Q, int topk) {
    // from 2^22 items on; with the 16-bit pre-filter (eight queries per pass of stage 1) and enough queries to
    // fill the chunk walk already from 2^19 (1000 queries, K = 16: lists are ahead up to 3e5 items, hit bits from 6e5)
    const bool large = ix->N >= (1ll << 22) || (ix->N >= (1ll << 19) && Q >= 32 && icq_scan_q16_usable(ix, Q));
    return ix->Kf <= 4 && !icq_group_usable(ix, Q) && use_select(ix, topk) && large &&
           ix->N + 16ll * 65536 < (1ll << 31);
}

int64_t icq_mask_scan_end(const icq_index *ix) {
    const int64_t npos = icq_g2_usable(ix) ? ix->g2_npos : ix->N;
    return (npos + RM_CHUNK - 1) / RM_CHUNK * RM_CHUNK;
}

int icq_launch_refine_masks(const icq_index *ix, const float *lut, int Q, const uint16_t *masks, size_t mask_stride,
                            int64_t scan_end, int64_t cap, int topk, int splits, u64 *keys, uint32_t *key_count,
                            uint32_t *cand_count, const float *thr, uint32_t *out_ids, float *out_dist, hipStream_t s) {
    if (Q == 0) return ICQ_OK;
    const bool g2 = icq_g2_usable(ix);
    const uint8_t *items = g2 ? ix->items_grouped : ix->items;
    const uint32_t *perm = g2 ? ix->perm : nullptr;
    u64 *cand_keys = icq_cand_keys(keys, Q, splits, topk);     // [Q][cap], behind the slice lists
    const uint32_t chunks = (uint32_t)(scan_end / RM_CHUNK);
    // few chunks: one unfiltered launch over all of them (a bound would save less than its second launch costs)
    const uint32_t seed_every = chunks < 2 * RM_SEED_EVERY ? 1u : (uint32_t)RM_SEED_EVERY;
    const uint32_t nseed = (chunks + seed_every - 1) / seed_every, nmain = chunks - nseed;
    const unsigned grid_sel = (unsigned)Q * (unsigned)splits;
    const int listcap = 1024;
    auto select = [&]() -> int {
        select_keys_kernel<<<grid_sel, SK_THREADS, (sizeof(u64) + sizeof(uint32_t)) * listcap, s>>>(
            cand_keys, key_count, cap, topk, listcap, splits, keys, out_ids, out_dist);
        if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
        // every slice comes out of the selection ascending, and a position -- hence an id -- has one key
        if (splits > 1) return icq_launch_merge(keys, Q, splits, topk, true, out_ids, out_dist, s);
        return ICQ_OK;
    };
    // Chunks per block: few, so that the blocks in flight (two windows' worth when the queries fill the
    // chip) keep to a few chunks per XCD; more when there are so few queries that the table load would weigh.
    // An unfiltered launch with little work for the chip (the first part of a large index: one chunk per
    // wavefront is all the parallelism there is) is spread over as many blocks as possible; one that is the
    // whole stage (a small index, many queries) takes full windows, and the chunks are cut fewer than 8
    // ways when 8 windows' worth do not exist: 16 MB of records stay in the caches wherever the blocks run.
    auto plan_for = [&](uint32_t nsel, bool filtered, int *xs_shift) -> int {
        int w = Q >= 8 ? (g2 ? 12 : 8) : 16;          // at N = 1e8, 128 queries, pair ordering: 16 / 12 / 8 / 6 / 4: 1.105 / 1.090 / 1.109 / 1.18 / 1.31 ms
        if (!filtered && Q >= 8) w = (uint64_t)nsel * (uint64_t)Q <= 16384u ? 4 : 16;
        // (with thousands of queries a window's blocks no longer run at the same time, and the 8-way cut that
        // keeps a chunk's records in ONE L2 is worth more than the longer windows: 1e4 queries, 1e6 items,
        // 8-byte records: 0.80 ms with it, 0.83 without)
        int shift = 3;
        while (Q <= 2048 && shift > 0 && ((uint32_t)w << shift) > nsel) --shift;
        *xs_shift = shift;
        const int most = (int)((nsel + (1u << shift) - 1) >> shift);
        return w < most ? w : (most > 0 ? most : 1);
    };
    const size_t mask_words = mask_stride / 2;
    const uint32_t *m32 = reinterpret_cast<const uint32_t *>(masks);
#define ICQ_RM_LAUNCH(W, FILTER, NSEL)                                                                       \
    do {                                                                                                     \
        int xs_shift = 3;                                                                                    \
        const int window = plan_for(NSEL, FILTER, &xs_shift);                                                \
        const unsigned per_win = (unsigned)window << xs_shift;                                               \
        const unsigned nwin = ((NSEL) + per_win - 1) / per_win;                                              \
        const unsigned ngroups = ((unsigned)Q + RM_QPB - 1) / RM_QPB;                                        \
        if (thr)                                                                                             \
            refine_mask_kernel<W, FILTER, RM_QPB, true><<<(nwin * ngroups) << xs_shift, RM_THREADS, 0, s>>>(           \
                items, ix->K, lut, m32, mask_words, perm, (NSEL), seed_every, window, xs_shift, Q, out_dist, topk,     \
                cand_keys, key_count, cap, cand_count, thr, ix->Kf);                                         \
        else                                                                                                 \
            refine_mask_kernel<W, FILTER, RM_QPB, false><<<(nwin * ngroups) << xs_shift, RM_THREADS, 0, s>>>(          \
                items, ix->K, lut, m32, mask_words, perm, (NSEL), seed_every, window, xs_shift, Q, out_dist, topk,     \
                cand_keys, key_count, cap, cand_count, nullptr, ix->Kf);                                     \
    } while (0)
    switch (ix->item_stride) {
        case 4: ICQ_RM_LAUNCH(1, false, nseed); break;
        case 8: ICQ_RM_LAUNCH(2, false, nseed); break;
        default: ICQ_RM_LAUNCH(4, false, nseed); break;
    }
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    if (nmain == 0) return select();
    int rc = select();
    if (rc != ICQ_OK) return rc;
    switch (ix->item_stride) {
        case 4: ICQ_RM_LAUNCH(1, true, nmain); break;
        case 8: ICQ_RM_LAUNCH(2, true, nmain); break;
        default: ICQ_RM_LAUNCH(4, true, nmain); break;
    }
#undef ICQ_RM_LAUNCH
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    return select();
}
