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
constexpr int GD_HITS = 2048;     // tuples below the threshold handled per pass
constexpr int GD_PER = GD_HITS / GS_THREADS;
constexpr int GD_LINEAR = 12;     // up to this many tuple boundaries in a row of 64 survivors: count them one by one
static_assert(GD_HITS <= 2048 && GD_HITS % GS_THREADS == 0, "tuple search covers 64 x 32 entries");

// Inclusive scan of two counters over the block (GS_THREADS threads); returns the
// exclusive prefixes through ex_a / ex_b and the block totals through tot_a / tot_b.
// Contains two barriers; every thread calls it.
__device__ __forceinline__ void block_scan2(uint32_t a, uint32_t b, uint32_t (*wsum)[2], uint32_t lane, int wave,
                                            uint32_t &ex_a, uint32_t &ex_b, uint32_t &tot_a, uint32_t &tot_b) {
    uint32_t ia = a, ib = b;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const uint32_t oa = __shfl_up(ia, d, 64);
        const uint32_t ob = __shfl_up(ib, d, 64);
        if ((int)lane >= d) { ia += oa; ib += ob; }
    }
    __syncthreads();                       // earlier readers of wsum are done
    if (lane == 63) { wsum[wave][0] = ia; wsum[wave][1] = ib; }
    __syncthreads();
    uint32_t pa = 0, pb = 0, ta = 0, tb = 0;
#pragma unroll
    for (int w = 0; w < GS_THREADS / 64; ++w) {
        const uint32_t va = wsum[w][0], vb = wsum[w][1];
        if (w < wave) { pa += va; pb += vb; }
        ta += va; tb += vb;
    }
    ex_a = pa + ia - a; ex_b = pb + ib - b;
    tot_a = ta; tot_b = tb;
}

// grid (parts, Q): a block evaluates the tuples (c0, c1) with c0 in its part's row
// range for one query; thread t owns column c1 = t (Kf == 2) or tuple c0 = t (Kf == 1)
// and keeps one bit per row: crude distance below the threshold or not.  The
// surviving tuples are compacted into LDS together with their first grouped
// position and an exclusive prefix of their sizes (empty tuples dropped), which
// turns "all items of all surviving tuples" into a flat range of survivor numbers
// 0 .. tot-1.  The wavefronts then walk that range 64 survivors at a time: a lane
// finds its tuple by counting the tuple boundaries at or below its number, reads
// the item's grouped record (records of one tuple are contiguous, so the loads
// coalesce), adds up the K table entries (all K tables of the query in LDS, k
// ascending, one table per record byte, zero tables beyond K) and writes the
// 64-bit key (order-preserving bits of D, item id) to slot base + number of the
// query's key list.  No list of positions or ids is written or read back.  A block
// that owns its query alone (parts == 1) counts the survivors locally and writes the
// count once; otherwise every pass reserves its slots with one atomic.
template <int KF, int WORDS>
__global__ __launch_bounds__(GS_THREADS) void group_keys_kernel(
    const float *__restrict__ lut, int K, const float *__restrict__ thr,
    const uint32_t *__restrict__ start, const uint8_t *__restrict__ items_grouped,
    unsigned long long *__restrict__ keys_out, uint32_t *__restrict__ count, int64_t cap,
    int rows_per_block) {
    __shared__ float T[4 * WORDS * ICQ_LUT_W];
    __shared__ uint32_t hbuf[GD_HITS];        // tuple ids while compacting, then first positions
    __shared__ uint32_t hx[GD_HITS + 1];      // exclusive prefix of the tuple sizes, hx[nhc] = tot
    __shared__ uint32_t wsum[GS_THREADS / 64][2];
    __shared__ uint32_t s_base;
    constexpr int RW = 2 * WORDS;
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = tid >> 6;
    const int q = blockIdx.y;
    const float *Tq = lut + (int64_t)q * K * ICQ_LUT_W;
    const float t = thr[q];
    unsigned long long *my_out = keys_out + (int64_t)q * cap;
    const bool own_query = gridDim.x == 1;

    for (int i = tid; i < 4 * WORDS * ICQ_LUT_W; i += GS_THREADS) T[i] = i < K * ICQ_LUT_W ? Tq[i] : 0.0f;

    // ---- one bit per (row, column): same additions as the item-by-item scan, lut[0][c0] (+ lut[1][c1])
    const int row_begin = KF == 2 ? blockIdx.x * rows_per_block : 0;
    const int row_end = KF == 2 ? (row_begin + rows_per_block < 256 ? row_begin + rows_per_block : 256) : 1;
    uint32_t m[8];
    uint32_t mine = 0;
    if (KF == 2) {
        const float t1 = Tq[ICQ_LUT_W + tid];
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            uint32_t bits = 0;
            if (w * 32 + 32 > row_begin && w * 32 < row_end) {       // block-uniform
#pragma unroll
                for (int b = 0; b < 32; ++b) bits |= (Tq[w * 32 + b] + t1 < t ? 1u : 0u) << b;
                const int lo = row_begin - w * 32, hi = row_end - w * 32;
                if (lo > 0) bits &= ~0u << lo;
                if (hi < 32) bits &= ~(~0u << hi);
            }
            m[w] = bits;
            mine += __builtin_popcount(bits);
        }
    } else {
#pragma unroll
        for (int w = 0; w < 8; ++w) m[w] = 0;
        m[0] = Tq[tid] < t ? 1u : 0u;
        mine = m[0];
    }
    uint32_t off_all, dummy0, total_hits, dummy1;
    block_scan2(mine, 0u, wsum, lane, wave, off_all, dummy0, total_hits, dummy1);
    // every surviving tuple at once if they fit, else eight rows (at most GD_HITS tuples) per pass
    const bool single = total_hits <= (uint32_t)GD_HITS;
    const int pass_rows = single ? 256 : GD_HITS / 256;
    uint32_t run = 0;                          // survivors so far (block-uniform)

    for (int ra = row_begin; ra < row_end; ra += pass_rows) {
        const int rb = ra + pass_rows < row_end ? ra + pass_rows : row_end;
        // ---- compact the tuples of rows [ra, rb) into hbuf
        uint32_t off, nh;
        if (single) {
            off = off_all;
            nh = total_hits;
        } else {
            uint32_t c = 0;
#pragma unroll
            for (int w = 0; w < 8; ++w) {
                const int lo = ra - w * 32, hi = rb - w * 32;
                if (hi > 0 && lo < 32) {
                    uint32_t bits = m[w];
                    if (lo > 0) bits &= ~0u << lo;
                    if (hi < 32) bits &= ~(~0u << hi);
                    c += __builtin_popcount(bits);
                }
            }
            uint32_t d0, d1;
            block_scan2(c, 0u, wsum, lane, wave, off, d0, nh, d1);
        }
        if (nh == 0) continue;                 // block-uniform
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            const int lo = ra - w * 32, hi = rb - w * 32;
            if (hi > 0 && lo < 32) {
                uint32_t bits = m[w];
                if (lo > 0) bits &= ~0u << lo;
                if (hi < 32) bits &= ~(~0u << hi);
                while (bits != 0) {
                    const int b = __builtin_ctz(bits);
                    bits &= bits - 1;
                    hbuf[off++] = KF == 2 ? (uint32_t)(w * 32 + b) * 256u + (uint32_t)tid : (uint32_t)tid;
                }
            }
        }
        __syncthreads();

        // ---- first position and size of every buffered tuple
        uint32_t s[GD_PER], n[GD_PER];
        uint32_t tn = 0, tc = 0;
#pragma unroll
        for (int u = 0; u < GD_PER; ++u) {
            const uint32_t h = (uint32_t)u * GS_THREADS + tid;
            const uint32_t g = hbuf[h < nh ? h : 0];
            s[u] = start[g];
            n[u] = start[g + 1];
        }
#pragma unroll
        for (int u = 0; u < GD_PER; ++u) {
            const uint32_t h = (uint32_t)u * GS_THREADS + tid;
            n[u] = h < nh ? n[u] - s[u] : 0u;
            tn += n[u];
            tc += n[u] != 0 ? 1u : 0u;
        }
        uint32_t x, c, tot, nhc;
        block_scan2(tn, tc, wsum, lane, wave, x, c, tot, nhc);   // its barriers also order the hbuf reads above
        if (tot == 0) continue;                // block-uniform
#pragma unroll
        for (int u = 0; u < GD_PER; ++u) {
            if (n[u] != 0) {
                hbuf[c] = s[u];
                hx[c] = x;
                ++c;
                x += n[u];
            }
        }
        if (tid == 0) {
            hx[nhc] = tot;
            if (!own_query) s_base = atomicAdd(&count[q], tot);
        }
        __syncthreads();
        const uint32_t base = own_query ? run : s_base;
        run += tot;

        // ---- the survivors, 64 per row; the rows are dealt to the wavefronts in contiguous runs
        const uint32_t nrows = (tot + 63) >> 6;
        const uint32_t rpw = (nrows + GS_THREADS / 64 - 1) / (GS_THREADS / 64);
        uint32_t r = (uint32_t)wave * rpw;
        const uint32_t rend = r + rpw < nrows ? r + rpw : nrows;
        if (r < rend) {
            // tuple holding survivor r * 64: the last one whose prefix is <= it (two 64-way probes)
            uint32_t ha;
            {
                const uint32_t p = r * 64;
                const uint32_t i1 = lane * 32;
                const uint32_t v1 = hx[i1 < nhc ? i1 : nhc];
                const uint32_t c1 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(i1 < nhc && v1 <= p));
                const uint32_t b0 = (c1 - 1) * 32;
                const uint32_t i2 = b0 + lane;
                const uint32_t v2 = hx[i2 < nhc ? i2 : nhc];
                const uint32_t c2 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < 32 && i2 < nhc && v2 <= p));
                ha = b0 + c2 - 1;
            }
            // grouped position of this lane's survivor in row `row`; moves ha to the tuple of the next row
            auto locate = [&](uint32_t row) -> uint32_t {
                const uint32_t pl = row * 64 + 63 < tot ? row * 64 + 63 : tot - 1;
                uint32_t p = row * 64 + lane;
                p = p < pl ? p : pl;
                const uint32_t bi = ha + 1 + lane;
                const uint32_t bnd = hx[bi < nhc ? bi : nhc];      // prefixes of the tuples after ha
                const uint32_t nb = __builtin_popcountll(__builtin_amdgcn_ballot_w64(bnd <= pl));
                uint32_t h = ha;
                if (nb <= (uint32_t)GD_LINEAR) {
                    for (uint32_t j = 0; j < nb; ++j) h += p >= (uint32_t)__builtin_amdgcn_readlane((int)bnd, (int)j) ? 1u : 0u;
                } else {
                    uint32_t lo = ha, hi = ha + nb;                 // hx[lo] <= p, answer in [lo, hi]
                    while (__builtin_amdgcn_ballot_w64(lo < hi) != 0) {
                        const uint32_t mid = (lo + hi + 1) >> 1;
                        const bool le = hx[mid] <= p;
                        if (lo < hi) {
                            if (le) lo = mid; else hi = mid - 1;
                        }
                    }
                    h = lo;
                }
                const uint32_t pos = hbuf[h] + (p - hx[h]);
                ha += __builtin_popcountll(__builtin_amdgcn_ballot_w64(bnd <= pl + 1 && bi < nhc));
                return pos;
            };
            auto fetch = [&](uint32_t r0, uint32_t (*rec)[RW]) {
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    uint32_t pos = 0;
                    if (r0 + u < rend) pos = locate(r0 + u);        // wavefront-uniform
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
            };
            uint32_t cur[4][RW], nxt[4][RW];
            fetch(r, cur);
            for (; r < rend; r += 4) {
                fetch(r + 4, nxt);                                   // rows past rend read record 0, unused
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    float d = 0.0f;
#pragma unroll
                    for (int w = 0; w < WORDS; ++w) {
#pragma unroll
                        for (int b = 0; b < 4; ++b)
                            d += T[(w * 4 + b) * ICQ_LUT_W + ((cur[u][w] >> (8 * b)) & 0xffu)];
                    }
                    const uint32_t num = (r + u) * 64 + lane;
                    const uint64_t slot = (uint64_t)base + num;
                    if (r + u < rend && num < tot && slot < (uint64_t)cap)
                        my_out[slot] = ((unsigned long long)icq_order_bits(d) << 32) | cur[u][WORDS % RW];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u)
#pragma unroll
                    for (int w = 0; w < RW; ++w) cur[u][w] = nxt[u][w];
            }
        }
        __syncthreads();                       // hbuf / hx are rewritten by the next pass
    }
    if (own_query && tid == 0) count[q] = run;
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
