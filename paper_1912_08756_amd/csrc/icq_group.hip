// Grouped form of stage 1 (arxiv 1912.08756, Eq. 2).  The crude distance
//   P[q][i] = sum_{k<Kf} lut[q][k][code_k(i)]
// depends on item i only through its Kf fast sub-codes.  With Kf <= 2 there are
// at most 65536 different tuples, so for N >> 256^Kf the index keeps the items
// grouped by tuple (a counting sort: positions, a position -> id map and the
// item records in grouped order) and a query evaluates P once per tuple; every
// item of a tuple below the threshold survives.  Values and survivor sets are
// the ones the item-by-item scan produces.
#include "icq_internal.h"

#include <math.h>

namespace {

__device__ __forceinline__ uint32_t lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}

__device__ __forceinline__ uint32_t group_of(const uint8_t *__restrict__ fast, int64_t Npad, int Kf,
                                              int64_t i) {
    uint32_t g = fast[i];
    if (Kf == 2) g = g * 256u + fast[Npad + i];
    return g;
}

// ---- index build: counting sort by tuple
__global__ void group_count_kernel(const uint8_t *__restrict__ fast, int64_t Npad, int Kf, int64_t N,
                                   uint32_t *__restrict__ cursor) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) atomicAdd(&cursor[group_of(fast, Npad, Kf, i)], 1u);
}

// Exclusive scan of cursor[0..G) into start[0..G], one block of 1024 threads; cursor
// is left equal to start (the scatter pass advances it).
__global__ __launch_bounds__(1024) void group_offsets_kernel(uint32_t *__restrict__ cursor, int G,
                                                             uint32_t *__restrict__ start) {
    __shared__ uint32_t part[1024];
    const int tid = threadIdx.x;
    const int per = (G + 1023) / 1024;
    uint32_t sum = 0;
    for (int j = 0; j < per; ++j) {
        const int g = tid * per + j;
        if (g < G) sum += cursor[g];
    }
    part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {     // Hillis-Steele inclusive scan
        uint32_t v = tid >= d ? part[tid - d] : 0u;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    uint32_t run = part[tid] - sum;
    for (int j = 0; j < per; ++j) {
        const int g = tid * per + j;
        if (g < G) {
            const uint32_t c = cursor[g];
            start[g] = run;
            cursor[g] = run;
            run += c;
        }
    }
    if (tid == 1023) start[G] = part[1023];
}

__global__ void group_scatter_kernel(const uint8_t *__restrict__ fast, int64_t Npad, int Kf, int64_t N,
                                     uint32_t *__restrict__ cursor, const uint8_t *__restrict__ items,
                                     int stride, uint32_t *__restrict__ perm,
                                     uint8_t *__restrict__ items_grouped) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const uint32_t pos = atomicAdd(&cursor[group_of(fast, Npad, Kf, i)], 1u);
    perm[pos] = (uint32_t)i;
    // grouped record: the item's sub-codes, then its id, padded to twice the record size
    const int W = stride / 4;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(items + (size_t)i * stride);
    uint32_t *dst = reinterpret_cast<uint32_t *>(items_grouped + (size_t)pos * (2 * stride));
    for (int w = 0; w < W; ++w) dst[w] = src[w];
    dst[W] = (uint32_t)i;
    for (int w = W + 1; w < 2 * W; ++w) dst[w] = 0u;
}

__global__ void group_zero_kernel(uint32_t *__restrict__ p, int n) {
    const int i = blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = 0u;
}

// ---- query time
constexpr int GS_THREADS = 256;
constexpr int GS_HITS = 8192;     // LDS buffer of tuples below the threshold
constexpr int GS_ROWS = 16;       // rows (of 256 tuples) between two looks at the buffer

// grid (parts, Q): a block evaluates the tuples (c0, c1) with c0 in its part's row
// range for one query; thread t owns column c1 = t (Kf == 2) or tuple c0 = t (Kf == 1).
// Tuples below the threshold are buffered in LDS (typically all of a query's fit, so
// there is one expansion at the end); each wavefront then takes 64 of them at a
// time, reserves list space for all their items with one atomic and writes the
// items' positions (or ids) with coalesced stores.
template <int KF>
__global__ __launch_bounds__(GS_THREADS) void group_scan_kernel(
    const float *__restrict__ lut, int K, const float *__restrict__ thr,
    const uint32_t *__restrict__ start, const uint32_t *__restrict__ perm,
    uint32_t *__restrict__ out, uint32_t *__restrict__ count, int64_t cap, int rows_per_block) {
    __shared__ float t0[ICQ_LUT_W];
    __shared__ uint32_t hits[GS_HITS];
    __shared__ uint32_t s_nh;
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = tid >> 6;
    const int q = blockIdx.y;
    const float *T = lut + (int64_t)q * K * ICQ_LUT_W;
    const float t = thr[q];
    uint32_t *my_out = out + (int64_t)q * cap;

    t0[tid] = T[tid];
    const float t1 = KF == 2 ? T[ICQ_LUT_W + tid] : 0.0f;
    if (tid == 0) s_nh = 0;
    __syncthreads();

    auto expand = [&](uint32_t nh) {   // every thread calls; nh is block-uniform
        for (uint32_t h0 = wave * 64; h0 < nh; h0 += (GS_THREADS / 64) * 64) {
            const uint32_t h = h0 + lane;
            uint32_t s = 0, n = 0;
            if (h < nh) {
                const uint32_t g = hits[h];
                s = start[g];
                n = start[g + 1] - s;
            }
            uint32_t incl = n;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t o = __shfl_up(incl, d, 64);
                if ((int)lane >= d) incl += o;
            }
            const uint32_t tot = __builtin_amdgcn_readlane(incl, 63);
            if (tot == 0) continue;
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&count[q], tot);
            base = __builtin_amdgcn_readfirstlane(base);
            const uint32_t excl = incl - n;
            uint64_t live = __builtin_amdgcn_ballot_w64(n != 0);
            while (live != 0) {
                const int l = __builtin_ctzll(live);
                live &= live - 1;
                const uint32_t sl = __builtin_amdgcn_readlane(s, l);
                const uint32_t nl = __builtin_amdgcn_readlane(n, l);
                const uint64_t ol = (uint64_t)base + __builtin_amdgcn_readlane(excl, l);
                for (uint32_t j = lane; j < nl; j += 64) {
                    const uint64_t slot = ol + j;
                    if (slot < (uint64_t)cap) my_out[slot] = perm ? perm[sl + j] : sl + j;
                }
            }
        }
    };

    const int row_begin = KF == 2 ? blockIdx.x * rows_per_block : 0;
    const int row_end = KF == 2 ? (row_begin + rows_per_block < 256 ? row_begin + rows_per_block : 256) : 1;
    for (int r0 = row_begin; r0 < row_end; r0 += GS_ROWS) {
        const int r1 = r0 + GS_ROWS < row_end ? r0 + GS_ROWS : row_end;
        for (int c0 = r0; c0 < r1; ++c0) {
            // same additions as the item-by-item scan: lut[0][c0] (+ lut[1][c1])
            const float P = KF == 2 ? t0[c0] + t1 : t0[tid];
            const bool hit = P < t;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
            if (mask != 0) {
                uint32_t base = 0;
                const int leader = __builtin_ctzll(mask);
                if ((int)lane == leader) base = atomicAdd(&s_nh, (uint32_t)__builtin_popcountll(mask));
                base = __builtin_amdgcn_readlane(base, leader);
                if (hit)
                    hits[base + __builtin_popcountll(mask & ((1ull << lane) - 1))] =
                        KF == 2 ? (uint32_t)c0 * 256u + (uint32_t)tid : (uint32_t)tid;
            }
        }
        if (r1 < row_end) {
            // room for another GS_ROWS rows?  (uniform decision: read between two barriers)
            __syncthreads();
            const uint32_t nh = s_nh;
            __syncthreads();
            if (nh > (uint32_t)(GS_HITS - GS_ROWS * 256)) {
                expand(nh);
                __syncthreads();
                if (tid == 0) s_nh = 0;
                __syncthreads();
            }
        }
    }
    __syncthreads();
    expand(s_nh);
}

// ---- grouped stage 1 fused with the stage-2 distances
constexpr int GD_HITS = 2048;     // tuples below the threshold buffered per block
constexpr int GD_POS = 1024;      // survivor positions buffered per wavefront

// grid (parts, Q) like group_scan_kernel, but instead of listing the survivors the
// block finishes them: a wavefront expands 64 surviving tuples into a flat buffer of
// grouped positions in LDS, then all 64 lanes walk that buffer -- grouped records are
// contiguous per tuple, so the 16/32-byte record reads coalesce -- add up the K table
// entries (all K tables of the query in LDS, k ascending, one table per record byte,
// zero tables beyond K) and write the 64-bit key (order-preserving bits of D, item id)
// to the query's key list.  No position list is written or read back.
template <int KF, int WORDS>
__global__ __launch_bounds__(GS_THREADS) void group_keys_kernel(
    const float *__restrict__ lut, int K, const float *__restrict__ thr,
    const uint32_t *__restrict__ start, const uint8_t *__restrict__ items_grouped,
    unsigned long long *__restrict__ keys_out, uint32_t *__restrict__ count, int64_t cap,
    int rows_per_block) {
    __shared__ float t0[ICQ_LUT_W];
    __shared__ float T[4 * WORDS * ICQ_LUT_W];
    __shared__ uint32_t hits[GD_HITS];
    __shared__ uint32_t posbuf[GS_THREADS / 64][GD_POS];
    __shared__ uint32_t s_nh;
    constexpr int RW = 2 * WORDS;
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = tid >> 6;
    const int q = blockIdx.y;
    const float *Tq = lut + (int64_t)q * K * ICQ_LUT_W;
    const float t = thr[q];
    unsigned long long *my_out = keys_out + (int64_t)q * cap;

    t0[tid] = Tq[tid];
    const float t1 = KF == 2 ? Tq[ICQ_LUT_W + tid] : 0.0f;
    for (int i = tid; i < 4 * WORDS * ICQ_LUT_W; i += GS_THREADS) T[i] = i < K * ICQ_LUT_W ? Tq[i] : 0.0f;
    if (tid == 0) s_nh = 0;
    __syncthreads();

    auto finish = [&](uint32_t nh) {   // every thread calls; nh is block-uniform
        uint32_t *pb = posbuf[wave];
        for (uint32_t h0 = wave * 64; h0 < nh; h0 += (GS_THREADS / 64) * 64) {
            const uint32_t h = h0 + lane;
            uint32_t s = 0, n = 0;
            if (h < nh) {
                const uint32_t g = hits[h];
                s = start[g];
                n = start[g + 1] - s;
            }
            uint32_t incl = n;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const uint32_t o = __shfl_up(incl, d, 64);
                if ((int)lane >= d) incl += o;
            }
            const uint32_t tot = __builtin_amdgcn_readlane(incl, 63);
            if (tot == 0) continue;
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(&count[q], tot);
            base = __builtin_amdgcn_readfirstlane(base);
            const uint32_t excl = incl - n;
            for (uint32_t c0 = 0; c0 < tot; c0 += GD_POS) {
                // positions [c0, c0 + GD_POS) of this batch -> LDS
                uint64_t live = __builtin_amdgcn_ballot_w64(n != 0 && excl < c0 + GD_POS && excl + n > c0);
                while (live != 0) {
                    const int l = __builtin_ctzll(live);
                    live &= live - 1;
                    const uint32_t sl = __builtin_amdgcn_readlane(s, l);
                    const uint32_t nl = __builtin_amdgcn_readlane(n, l);
                    const uint32_t ol = __builtin_amdgcn_readlane(excl, l);
                    const uint32_t lo = ol > c0 ? ol : c0;
                    const uint32_t hi = ol + nl < c0 + GD_POS ? ol + nl : c0 + GD_POS;
                    for (uint32_t j = lo + lane; j < hi; j += 64) pb[j - c0] = sl + (j - ol);
                }
                __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
                __builtin_amdgcn_wave_barrier();
                __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
                const uint32_t clen = tot - c0 < (uint32_t)GD_POS ? tot - c0 : (uint32_t)GD_POS;
                for (uint32_t i0 = 0; i0 < clen; i0 += 64 * 4) {
                    uint32_t rec[4][RW];
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        const uint32_t idx = i0 + u * 64 + lane;
                        const uint32_t pos = pb[idx < clen ? idx : clen - 1];
                        const uint32_t *p = reinterpret_cast<const uint32_t *>(items_grouped + (size_t)pos * (RW * 4));
                        if (RW == 2) {
                            const uint2 v = *reinterpret_cast<const uint2 *>(p);
                            rec[u][0] = v.x;
                            rec[u][1 % RW] = v.y;
                        } else {
#pragma unroll
                            for (int w4 = 0; w4 < RW / 4; ++w4) {
                                const uint4 v = reinterpret_cast<const uint4 *>(p)[w4];
                                rec[u][(4 * w4) % RW] = v.x;
                                rec[u][(4 * w4 + 1) % RW] = v.y;
                                rec[u][(4 * w4 + 2) % RW] = v.z;
                                rec[u][(4 * w4 + 3) % RW] = v.w;
                            }
                        }
                    }
#pragma unroll
                    for (int u = 0; u < 4; ++u) {
                        float d = 0.0f;
#pragma unroll
                        for (int w = 0; w < WORDS; ++w) {
#pragma unroll
                            for (int b = 0; b < 4; ++b)
                                d += T[(w * 4 + b) * ICQ_LUT_W + ((rec[u][w] >> (8 * b)) & 0xffu)];
                        }
                        const uint32_t idx = i0 + u * 64 + lane;
                        const uint64_t slot = (uint64_t)base + c0 + idx;
                        if (idx < clen && slot < (uint64_t)cap)
                            my_out[slot] = ((unsigned long long)icq_order_bits(d) << 32) | rec[u][WORDS % RW];
                    }
                }
                __builtin_amdgcn_wave_barrier();
            }
        }
    };

    const int row_begin = KF == 2 ? blockIdx.x * rows_per_block : 0;
    const int row_end = KF == 2 ? (row_begin + rows_per_block < 256 ? row_begin + rows_per_block : 256) : 1;
    constexpr int ROWS = GD_HITS / 256 / 2;   // rows between two looks at the buffer (half of it)
    for (int r0 = row_begin; r0 < row_end; r0 += ROWS) {
        const int r1 = r0 + ROWS < row_end ? r0 + ROWS : row_end;
        for (int c0 = r0; c0 < r1; ++c0) {
            // same additions as the item-by-item scan: lut[0][c0] (+ lut[1][c1])
            const float P = KF == 2 ? t0[c0] + t1 : t0[tid];
            const bool hit = P < t;
            const uint64_t mask = __builtin_amdgcn_ballot_w64(hit);
            if (mask != 0) {
                uint32_t base = 0;
                const int leader = __builtin_ctzll(mask);
                if ((int)lane == leader) base = atomicAdd(&s_nh, (uint32_t)__builtin_popcountll(mask));
                base = __builtin_amdgcn_readlane(base, leader);
                if (hit)
                    hits[base + __builtin_popcountll(mask & ((1ull << lane) - 1))] =
                        KF == 2 ? (uint32_t)c0 * 256u + (uint32_t)tid : (uint32_t)tid;
            }
        }
        if (r1 < row_end) {
            __syncthreads();
            const uint32_t nh = s_nh;
            __syncthreads();
            if (nh > (uint32_t)(GD_HITS - ROWS * 256)) {
                finish(nh);
                __syncthreads();
                if (tid == 0) s_nh = 0;
                __syncthreads();
            }
        }
    }
    __syncthreads();
    finish(s_nh);
}

}  // namespace

int icq_group_build(icq_index *ix, hipStream_t s) {
    ix->groups = 0;
    ix->group_start = nullptr;
    ix->group_cursor = nullptr;
    ix->perm = nullptr;
    ix->items_grouped = nullptr;
    if (ix->Kf > 2 || ix->N == 0) return ICQ_OK;
    const int G = ix->Kf == 1 ? 256 : 65536;
    bool ok = hipMalloc(&ix->group_start, sizeof(uint32_t) * (G + 1)) == hipSuccess &&
              hipMalloc(&ix->group_cursor, sizeof(uint32_t) * G) == hipSuccess &&
              hipMalloc(&ix->perm, sizeof(uint32_t) * (size_t)ix->N) == hipSuccess &&
              hipMalloc(&ix->items_grouped, (size_t)ix->N * ix->item_stride * 2) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        return ICQ_ERR_HIP;   // the caller destroys the index, which frees whatever was allocated
    }
    const int T = 256;
    const unsigned nb = (unsigned)((ix->N + T - 1) / T);
    group_zero_kernel<<<(G + T - 1) / T, T, 0, s>>>(ix->group_cursor, G);
    group_count_kernel<<<nb, T, 0, s>>>(ix->fast, ix->Npad, ix->Kf, ix->N, ix->group_cursor);
    group_offsets_kernel<<<1, 1024, 0, s>>>(ix->group_cursor, G, ix->group_start);
    group_scatter_kernel<<<nb, T, 0, s>>>(ix->fast, ix->Npad, ix->Kf, ix->N, ix->group_cursor, ix->items,
                                          ix->item_stride, ix->perm, ix->items_grouped);
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    ix->groups = G;
    return ICQ_OK;
}

bool icq_group_usable(const icq_index *ix, int Q) {
    if (ix->groups == 0 || ix->scan_mode == ICQ_SCAN_STREAMED) return false;
    if (ix->scan_mode == ICQ_SCAN_GROUPED) return true;
    // automatic: the grouped form costs 256^Kf evaluations per query whatever N is
    return Q > 4 && ix->N >= (int64_t)ix->groups / 2;
}

int icq_launch_group_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                          uint32_t *cand_ids, bool as_positions, uint32_t *cand_count, int64_t cap,
                          hipStream_t s) {
    // cand_count has been zeroed by the caller (icq_launch_scan)
    int parts = 1;
    if (ix->Kf == 2) {
        parts = (2 * ix->num_cu + Q - 1) / Q;
        if (parts > 16) parts = 16;
        if (parts < 1) parts = 1;
    }
    const int rows = (256 + parts - 1) / parts;
    for (int q0 = 0; q0 < Q; q0 += 65535) {
        const int nq = Q - q0 < 65535 ? Q - q0 : 65535;
        dim3 grid((unsigned)parts, (unsigned)nq);
        if (ix->Kf == 1)
            group_scan_kernel<1><<<grid, GS_THREADS, 0, s>>>(
                lut + (int64_t)q0 * ix->K * ICQ_LUT_W, ix->K, thr + q0, ix->group_start,
                as_positions ? nullptr : ix->perm, cand_ids + (int64_t)q0 * cap, cand_count + q0, cap, rows);
        else
            group_scan_kernel<2><<<grid, GS_THREADS, 0, s>>>(
                lut + (int64_t)q0 * ix->K * ICQ_LUT_W, ix->K, thr + q0, ix->group_start,
                as_positions ? nullptr : ix->perm, cand_ids + (int64_t)q0 * cap, cand_count + q0, cap, rows);
    }
    return icq_check_launch();
}

int icq_launch_group_keys(const icq_index *ix, const float *lut, int Q, const float *thr,
                          unsigned long long *cand_keys, uint32_t *cand_count, int64_t cap,
                          hipStream_t s) {
    // cand_count has been zeroed by the caller (icq_launch_scan); item_stride <= 16 here
    int parts = 1;
    if (ix->Kf == 2) {
        parts = (2 * ix->num_cu + Q - 1) / Q;
        if (parts > 16) parts = 16;
        if (parts < 1) parts = 1;
    }
    const int rows = (256 + parts - 1) / parts;
    for (int q0 = 0; q0 < Q; q0 += 65535) {
        const int nq = Q - q0 < 65535 ? Q - q0 : 65535;
        dim3 grid((unsigned)parts, (unsigned)nq);
        const float *l = lut + (int64_t)q0 * ix->K * ICQ_LUT_W;
        unsigned long long *ko = cand_keys + (int64_t)q0 * cap;
#define ICQ_GK(KF, W)                                                                                \
    group_keys_kernel<KF, W><<<grid, GS_THREADS, 0, s>>>(l, ix->K, thr + q0, ix->group_start,         \
                                                         ix->items_grouped, ko, cand_count + q0, cap, \
                                                         rows)
        const int W = ix->item_stride / 4;
        if (ix->Kf == 1) {
            if (W == 1) ICQ_GK(1, 1); else if (W == 2) ICQ_GK(1, 2); else ICQ_GK(1, 4);
        } else {
            if (W == 1) ICQ_GK(2, 1); else if (W == 2) ICQ_GK(2, 2); else ICQ_GK(2, 4);
        }
#undef ICQ_GK
    }
    return icq_check_launch();
}

ICQ_EXPORT int icq_index_set_scan_mode(icq_index *ix, int mode) {
    if (!ix || mode < ICQ_SCAN_AUTO || mode > ICQ_SCAN_GROUPED) return ICQ_ERR_ARG;
    ix->scan_mode = mode;
    return ICQ_OK;
}
