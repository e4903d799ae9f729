// Grouped form of stage 1 (arxiv 1912.08756, Eq. 2).  The crude distance
//   P[q][i] = sum_{k<Kf} lut[q][k][code_k(i)]
// depends on item i only through its Kf fast sub-codes.  With Kf <= 2 there are
// at most 65536 different tuples, so for N >> 256^Kf the index keeps the items
// grouped by tuple (a counting sort: positions, a position -> id map and the
// item records in grouped order) and a query evaluates P once per tuple; every
// item of a tuple below the threshold survives.  Values and survivor sets are
// the ones the item-by-item scan produces.
#include "icq_internal.h"
#include "icq_sort.h"

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
    // the item's record, moved to its grouped position
    const int W = stride / 4;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(items + (size_t)i * stride);
    uint32_t *dst = reinterpret_cast<uint32_t *>(items_grouped + (size_t)pos * stride);
    for (int w = 0; w < W; ++w) dst[w] = src[w];
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
            const uint32_t incl = wave_scan_add(n);
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

// ---- grouped stage 1 fused with stage 2
constexpr int GD_HITS = 768;      // tuples below the threshold handled per pass
constexpr int GD_PER = GD_HITS / GS_THREADS;
constexpr int GD_SEED = 4;        // survivors of a pass's first part, in result lengths
constexpr int GD_ROWS = 2;        // rows of 64 survivors per wavefront and step
constexpr int GD_STEP = GD_ROWS * GS_THREADS;            // most keys one step can add to the list
constexpr int GD_LIST = 1024;     // keys of the block's nearest-neighbour list
constexpr int GD_LPT = GD_LIST / GS_THREADS;             // list entries per thread in a cut
constexpr int GD_SORT = 1024;     // most keys the final register sort takes
constexpr int GD_TOPK = 256;      // longest result the on-chip list serves
constexpr int GD_OWN = 12;        // surviving tuples a thread lists by itself (or four times the average): more are listed by its wavefront together
static_assert(GD_HITS <= 2048 && GD_HITS % GS_THREADS == 0, "tuple search covers 64 x 32 entries");
static_assert(GS_THREADS == 256, "one histogram bin per thread");
static_assert(GD_ROWS % 2 == 0, "a step is two half steps");
static_assert(GD_LIST - GD_STEP >= 2 * GD_TOPK, "room for the longest result plus as many ties between two cuts");
static_assert(GD_LIST <= GD_SORT, "the final list fits the register sort");

struct GdShared {
    IcqKthShared kth;
    uint32_t wtot[2][GS_THREADS / 64];
    uint32_t wsum[GS_THREADS / 64][2];
    uint32_t flag[GS_THREADS / 64][64];    // locate(): stamps of the tuple starts inside a row of survivors
    uint32_t base;
    float tmin[16];                        // smallest entry of each of the query's tables
    float colmin[GS_THREADS / 64];         // smallest second-codebook entry of each wavefront's columns
    uint32_t nlive[GS_THREADS / 64];       // rows that can hold a hit, per wavefront of rows
};

// Inclusive scan of two counters over the block (GS_THREADS threads); returns the
// exclusive prefixes through ex_a / ex_b and the block totals through tot_a / tot_b.
// Contains two barriers; every thread calls it.
__device__ __forceinline__ void block_scan2(uint32_t a, uint32_t b, uint32_t (*wsum)[2], uint32_t lane, int wave,
                                            uint32_t &ex_a, uint32_t &ex_b, uint32_t &tot_a, uint32_t &tot_b) {
    const uint32_t ia = wave_scan_add(a), ib = wave_scan_add(b);
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

// Cut list[0..cnt) (cnt block-uniform, > topk) back to the keys whose distance word is at
// or below a bound that keeps the topk smallest distances (ties at the bound kept; with
// !EXACT the bound is the top of a histogram bin, see block_kth).  Returns the new count,
// *bound = the bound.  Every thread calls.
__device__ __forceinline__ uint32_t block_cut(GdShared &sh, unsigned long long *list, uint32_t cnt, uint32_t topk,
                                              uint32_t *bound, bool EXACT, int tid, uint32_t lane, int wave) {
    unsigned long long e[GD_LPT];
    uint32_t v[GD_LPT], ok = 0;
    __syncthreads();                       // the list is complete
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u) {
        const uint32_t i = (uint32_t)u * GS_THREADS + tid;
        if (i < cnt) ok |= 1u << u;
        e[u] = list[i < cnt ? i : 0];
        v[u] = (uint32_t)(e[u] >> 32);
    }
    const uint32_t cut = block_kth<GD_LPT>(sh.kth, v, ok, topk, EXACT, tid, lane, wave);
    uint32_t c = 0;
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u) c += ((ok >> u) & 1u) && v[u] <= cut ? 1u : 0u;
    uint32_t off, d0, tot, d1;
    block_scan2(c, 0u, sh.wsum, lane, wave, off, d0, tot, d1);
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u)
        if (((ok >> u) & 1u) && v[u] <= cut) list[off++] = e[u];
    __syncthreads();
    *bound = cut;
    return tot;
}

// After an exact cut that left more than topk keys because many share the distance
// `cut`: keep the keys below it and, of those at it, the ones with the smallest item ids
// (the low word of a key is a grouped position; perm maps it to the id), exactly topk in
// all -- the order (distance, id) decides, as in the final list.  Every thread calls.
__device__ __forceinline__ uint32_t block_tie_cut(GdShared &sh, unsigned long long *list, uint32_t cnt, uint32_t topk, uint32_t cut,
                                  const uint32_t *__restrict__ perm, int tid, uint32_t lane, int wave) {
    unsigned long long e[GD_LPT];
    uint32_t w[GD_LPT], lt = 0, eq = 0;
    __syncthreads();
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u) {
        const uint32_t i = (uint32_t)u * GS_THREADS + tid;
        e[u] = list[i < cnt ? i : 0];
        const uint32_t d = (uint32_t)(e[u] >> 32);
        if (i < cnt && d < cut) lt |= 1u << u;
        if (i < cnt && d == cut) eq |= 1u << u;
        w[u] = perm[(uint32_t)e[u]];       // a valid position even where the entry is unused
    }
    uint32_t x0, x1, n_lt, n_eq;
    block_scan2((uint32_t)__builtin_popcount(lt), (uint32_t)__builtin_popcount(eq), sh.wsum, lane, wave, x0, x1,
                n_lt, n_eq);
    const uint32_t need = topk - n_lt;     // >= 1: the topk-th smallest distance is `cut`
    const uint32_t idcut = block_kth<GD_LPT>(sh.kth, w, eq, need, true, tid, lane, wave);
    uint32_t keep = lt;
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u)
        if (((eq >> u) & 1u) && w[u] <= idcut) keep |= 1u << u;
    uint32_t off, d0, tot, d1;
    block_scan2((uint32_t)__builtin_popcount(keep), 0u, sh.wsum, lane, wave, off, d0, tot, d1);
#pragma unroll
    for (int u = 0; u < GD_LPT; ++u)
        if ((keep >> u) & 1u) list[off++] = e[u];
    __syncthreads();
    return tot;
}

// Tuples whose crude distance P has order bits above the returned value cannot hold an item
// that reaches the result: every item's distance is P plus one entry of each remaining table,
// so D >= P + smin (smin = the sum of those tables' smallest entries), and with P above
// dk * (1 + 1e-5) - smin that exceeds dk, the distance behind `bound`.  All tables are
// non-negative where this is used; the 1e-5 covers the roundings of the fp32 sums on both
// sides (7 additions of non-negative terms lose less than 8 * 2^-24 of the sum, the sum of
// the minima and the two operations here as much again: under 3e-6 in all).
__device__ __forceinline__ uint32_t prune_above(uint32_t bound, float smin) {
    if (bound >= 0xFF800000u) return 0xFFFFFFFFu;     // open, infinite or not a number: nothing is pruned
    float tb = icq_unorder_bits(bound) * (1.0f + 1e-5f) - smin;
    if (!(tb > 0.0f)) tb = 0.0f;                      // P >= 0: a tuple at 0 is never pruned
    return icq_order_bits(tb);
}

// grid (parts, Q): a block evaluates tuples (c0, c1) for one query; thread t owns column
// c1 = t (Kf == 2) or tuple c0 = t (Kf == 1) and keeps one bit per row that can hold a hit (see
// the evaluation): crude distance below the threshold or not.  The surviving tuples are compacted into LDS (GD_HITS at a time)
// together with their first grouped position and an exclusive prefix of their sizes (empty
// tuples dropped), which turns "all items of all surviving tuples" into a flat range of
// survivor numbers 0 .. tot-1.  The wavefronts walk that range 64 survivors at a time: a lane
// finds its tuple by counting the tuple boundaries at or below its number, reads the item's
// record in grouped order (records of one tuple are contiguous, so the loads coalesce) and adds
// up the K table entries (all K tables of the query in LDS, k ascending, one table per record
// byte, zero tables beyond K).
//
// FUSED (topk <= GD_TOPK): the nearest-neighbour list of Sec. 3.4 is kept right here.  A key
// (order-preserving bits of D, grouped position) enters the block's list in LDS only if D is at
// or below the running bound; when the list could overflow it is cut back to the topk smallest
// distances, which tightens the bound (one histogram pass, see block_cut).  The bound also
// prunes whole tuples (prune_above: crude distance + the smallest the other tables can add is
// beyond it), and to have one early a pass whose list is still open first takes the tuples with
// the smallest crude distances, a few topk survivors' worth, and then the rest, pruned; the
// result and the survivor count (tuple sizes) are those of visiting everything.  At the end
// positions become item ids and the keys are ranked by (D, id) -- after one counting cut if the
// list is longer than a block's worth of keys.  No candidate list ever reaches memory.  One block per query writes the result rows; with
// several (few queries) every block evaluates and lists all tuples, takes its slice of every
// surviving tuple's items and leaves its topk best as ascending keys in keys_out[q][part][topk]
// for the merge.
//
// !FUSED (topk above GD_TOPK): the blocks of a query split the tuple rows; every survivor's key
// (bits of D, item id) is written to slot base + number of the query's key list for the select
// kernel; each pass reserves its slots with one atomic on the query's counter.
template <int KF, int WORDS, bool FUSED>
__global__ __launch_bounds__(GS_THREADS) __attribute__((amdgpu_waves_per_eu(WORDS == 4 ? 3 : 6, 8))) void group_keys_kernel(
    const float *__restrict__ lut, int K, const float *__restrict__ thr,
    const uint32_t *__restrict__ start, const uint8_t *__restrict__ items_grouped,
    const uint32_t *__restrict__ perm, unsigned long long *__restrict__ keys_out,
    uint32_t *__restrict__ count, int64_t cap, int rows_per_block, int topk,
    uint32_t *__restrict__ out_ids, float *__restrict__ out_dist) {
    __shared__ __attribute__((aligned(16))) float T[4 * WORDS * ICQ_LUT_W];
    __shared__ uint32_t hbuf[GD_HITS];        // tuple ids while compacting, then first positions
    __shared__ __attribute__((aligned(16))) uint32_t hx[GD_HITS + 1];      // exclusive prefix of the tuple sizes, hx[nhc] = tot
    __shared__ uint8_t rowid[256];            // KF == 2: the rows that can hold a hit, ascending
    __shared__ __attribute__((aligned(16))) unsigned long long list[FUSED ? GD_LIST : 2];
    __shared__ GdShared sh;
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);    // wavefront-uniform, and known to be
    const int q = blockIdx.y;
    const float *Tq = lut + (int64_t)q * K * ICQ_LUT_W;
    const float t = thr[q];
    unsigned long long *my_out = FUSED ? nullptr : keys_out + (int64_t)q * cap;

    // the query's tables: loads now, LDS writes after the tuple evaluation below, which hides their latency
    constexpr int T_PER = 4 * WORDS * ICQ_LUT_W / GS_THREADS / 4;
    float4 tv[T_PER];
#pragma unroll
    for (int r = 0; r < T_PER; ++r) {
        const int i4 = r * GS_THREADS + tid;            // float4 index; a table row is 64 of them
        tv[r] = i4 * 4 < K * ICQ_LUT_W ? reinterpret_cast<const float4 *>(Tq)[i4] : make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    }
    uint32_t *flag = sh.flag[wave];
    flag[lane] = 0;
    uint32_t stamp = 0;                        // wavefront-uniform, never 0 when compared

    // ---- one bit per (row, column): same additions as the item-by-item scan, lut[0][c0] (+ lut[1][c1])
    // Several blocks per query: the key-list form splits the tuple rows; the form that keeps the
    // lists on chip evaluates every tuple in every block and splits the surviving tuples evenly
    // (a query's survivors sit in the few rows of its nearest first-codebook codewords).
    const int row_begin = KF == 2 && !FUSED ? blockIdx.x * rows_per_block : 0;
    const int row_end = KF == 2 ? (row_begin + rows_per_block < 256 && !FUSED ? row_begin + rows_per_block : 256) : 1;
    // m: one bit per live row (KF == 2: bit i stands for row rowid[i], see below) or the tuple's own bit (KF == 1)
    uint32_t m[8];
    uint32_t mine = 0;
    uint32_t live_words = 1;                   // words of m that can hold a bit (block-uniform)
    if (KF == 2) {
        // Rows that can hold a hit at all: lut[0][row] + (the smallest lut[1][.]) < t.  Rounding is
        // monotone, so a row that fails this fails with every column.  A query's hits sit in the
        // rows of its few nearest first-codebook codewords: the live rows are numbered 0 .. nlive - 1
        // in row order, their values go to LDS (hx is free until the first pass) and the
        // evaluation walks those only, 32 at a time (padded with +inf).
        const float t1 = Tq[ICQ_LUT_W + tid];
        const float r0v = Tq[tid];                                   // this thread's row, for the liveness test
        const float wmin = wave_min_f32(t1);
        if (lane == 0) sh.colmin[wave] = wmin;
        __syncthreads();
        float cmin = sh.colmin[0];
#pragma unroll
        for (int w = 1; w < GS_THREADS / 64; ++w) cmin = fminf(cmin, sh.colmin[w]);
        const bool live = tid >= row_begin && tid < row_end && r0v + cmin < t;
        const uint64_t lv = __builtin_amdgcn_ballot_w64(live);
        if (lane == 0) sh.nlive[wave] = (uint32_t)__builtin_popcountll(lv);
        __syncthreads();
        uint32_t before = 0, nlive = 0;
#pragma unroll
        for (int w = 0; w < GS_THREADS / 64; ++w) {
            const uint32_t c = (uint32_t)__builtin_amdgcn_readfirstlane((int)sh.nlive[w]);
            if (w < wave) before += c;
            nlive += c;
        }
        float *rowT = reinterpret_cast<float *>(hx);
        if (live) {
            const uint32_t slot = __builtin_amdgcn_mbcnt_hi((uint32_t)(lv >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)lv, before));
            rowT[slot] = r0v;
            rowid[slot] = (uint8_t)tid;
        }
        const uint32_t nlive_pad = (nlive + 31u) & ~31u;
        live_words = nlive_pad >> 5;
        if ((uint32_t)tid >= nlive && (uint32_t)tid < nlive_pad) rowT[tid] = INFINITY;
        __syncthreads();
#pragma unroll
        for (int w = 0; w < 8; ++w) {
            uint32_t bits = 0;
            if ((uint32_t)(w * 32) < nlive) {                        // block-uniform
#pragma unroll
                for (int b4 = 0; b4 < 8; ++b4) {
                    const float4 v = reinterpret_cast<const float4 *>(rowT)[w * 8 + b4];   // one address for all lanes
                    bits |= (v.x + t1 < t ? 1u : 0u) << (b4 * 4);
                    bits |= (v.y + t1 < t ? 1u : 0u) << (b4 * 4 + 1);
                    bits |= (v.z + t1 < t ? 1u : 0u) << (b4 * 4 + 2);
                    bits |= (v.w + t1 < t ? 1u : 0u) << (b4 * 4 + 3);
                }
            }
            m[w] = bits;
            mine += __builtin_popcount(bits);
        }
        // (hx is next written in the first pass, behind the barriers of the scan below)
    } else {
#pragma unroll
        for (int w = 0; w < 8; ++w) m[w] = 0;
        m[0] = Tq[tid] < t ? 1u : 0u;
        mine = m[0];
    }
#pragma unroll
    for (int r = 0; r < T_PER; ++r) reinterpret_cast<float4 *>(T)[r * GS_THREADS + tid] = tv[r];
    if (FUSED) {
        // load r of wavefront w is table 4 r + w, whole: its smallest entry (tables beyond K hold zeros)
#pragma unroll
        for (int r = 0; r < T_PER; ++r) {
            const float v = wave_min_f32(fminf(fminf(tv[r].x, tv[r].y), fminf(tv[r].z, tv[r].w)));
            if (lane == 0) sh.tmin[r * 4 + wave] = v;
        }
    }
    // this thread's surviving tuples are numbers [off_all, off_all + mine) of the block's total_hits
    uint32_t off_all, dummy0, total_hits, dummy1;
    block_scan2(mine, 0u, sh.wsum, lane, wave, off_all, dummy0, total_hits, dummy1);

    // FUSED: the bound of the list also prunes whole tuples (prune_above) -- if no table entry is negative
    float smin = 0.0f;
    bool prune_ok = false;
    if (FUSED) {
        float all = INFINITY;
#pragma unroll
        for (int k = 0; k < 4 * WORDS; ++k) {
            const float v = sh.tmin[k];            // written before the barriers of the scan above
            all = fminf(all, v);
            if (k >= KF) smin += v;
        }
        prune_ok = all >= 0.0f;
    }
    uint32_t run = 0;                          // survivors so far (block-uniform)
    uint32_t cnt = 0;                          // FUSED: keys in the list (block-uniform)
    uint32_t bound = 0xFFFFFFFFu;              // FUSED: keys with distance bits above it cannot reach the result

    // Every block of a query lists all its surviving tuples; with several blocks (lists on chip, few
    // queries) each takes its slice of every tuple's items (see below), so the blocks are balanced
    // whatever the tuple sizes.
    for (uint32_t pass_lo = 0; pass_lo < total_hits; pass_lo += GD_HITS) {
        const uint32_t nh = total_hits - pass_lo < (uint32_t)GD_HITS ? total_hits - pass_lo : (uint32_t)GD_HITS;
        // ---- tuples number pass_lo .. pass_lo + nh - 1 -> hbuf
        // A thread lists its own hits one by one -- unless it has many: the column of the query's
        // nearest second-codebook codeword can hold a hundred, and one lane walking them alone
        // kept its whole block waiting.  Such columns are listed by the wavefront together, 64
        // rows at a time (same numbering: rows ascending).
        {
            // many = far above the average of the block's threads: the walk by one lane costs as many
            // rounds as its wavefront's longest list, the joint listing a fixed amount per column
            const uint32_t own = total_hits / 64 > (uint32_t)GD_OWN ? total_hits / 64 : (uint32_t)GD_OWN;
            const bool heavy = mine > own;
            if (!heavy) {
                uint32_t idx = off_all;
#pragma unroll
                for (int w = 0; w < 8; ++w) {
                    uint32_t bits = (uint32_t)w < live_words ? m[w] : 0u;
                    while (bits != 0) {
                        const int b = __builtin_ctz(bits);
                        bits &= bits - 1;
                        const uint32_t rel = idx - pass_lo;         // wraps below the pass: fails the test
                        if (rel < nh) hbuf[rel] = KF == 2 ? (uint32_t)rowid[w * 32 + b] * 256u + (uint32_t)tid : (uint32_t)tid;
                        ++idx;
                    }
                }
            }
            uint64_t hv = __builtin_amdgcn_ballot_w64(heavy);       // wavefront-uniform
            while (hv != 0) {
                const int src = __builtin_ctzll(hv);
                hv &= hv - 1;
                uint32_t idx = (uint32_t)__builtin_amdgcn_readlane((int)off_all, src);
                const uint32_t col = (uint32_t)wave * 64u + (uint32_t)src;
#pragma unroll
                for (int wp = 0; wp < 4; ++wp) {
                    if ((uint32_t)(2 * wp) >= live_words) break;    // block-uniform
                    const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)m[2 * wp], src);
                    const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)m[2 * wp + 1], src);
                    const uint32_t mybit = ((lane < 32 ? lo : hi) >> (lane & 31)) & 1u;
                    const uint32_t rel = __builtin_amdgcn_mbcnt_hi(hi, __builtin_amdgcn_mbcnt_lo(lo, idx)) - pass_lo;
                    if (mybit != 0 && rel < nh) hbuf[rel] = (uint32_t)rowid[wp * 64 + (int)lane] * 256u + col;
                    idx += (uint32_t)__builtin_popcount(lo) + (uint32_t)__builtin_popcount(hi);
                }
            }
        }
        __syncthreads();

        // ---- first position and size of every buffered tuple
        uint32_t s[GD_PER], n[GD_PER];
        uint32_t pb[GD_PER];                   // FUSED: order bits of the tuple's crude distance
#pragma unroll
        for (int u = 0; u < GD_PER; ++u) {
            const uint32_t h = (uint32_t)u * GS_THREADS + tid;
            const uint32_t g = hbuf[h < nh ? h : 0];
            s[u] = start[g];
            n[u] = start[g + 1];
            // the same sum as in the evaluation above, from the tables in LDS
            if (FUSED) pb[u] = icq_order_bits(KF == 2 ? T[g >> 8] + T[ICQ_LUT_W + (g & 255u)] : T[g]);
        }
#pragma unroll
        for (int u = 0; u < GD_PER; ++u) {
            const uint32_t h = (uint32_t)u * GS_THREADS + tid;
            n[u] = h < nh ? n[u] - s[u] : 0u;
            if (FUSED && gridDim.x > 1) {
                // this block's slice of the tuple's items: part b of p takes n / p of them (+1 for b < n % p)
                const uint32_t per = n[u] / gridDim.x, rem = n[u] % gridDim.x;
                s[u] += blockIdx.x * per + (blockIdx.x < rem ? blockIdx.x : rem);
                n[u] = per + (blockIdx.x < rem ? 1u : 0u);
            }
        }
        // FUSED: the pass runs in two parts while the list has no bound yet -- first the tuples
        // with the smallest crude distances, about GD_SEED * topk survivors, whose topk-th distance
        // then bounds the list and, through prune_above, the tuples of the second part.  Later
        // passes start with the bound of the earlier ones.
        int nsp = 1;
        uint32_t pivot = 0xFFFFFFFFu;
        if (FUSED) {
            uint32_t tn_all = 0, tc_all = 0, okm = 0;
#pragma unroll
            for (int u = 0; u < GD_PER; ++u) {
                tn_all += n[u];
                tc_all += n[u] != 0 ? 1u : 0u;
                okm |= n[u] != 0 ? 1u << u : 0u;
            }
            uint32_t d0, d1, tot_all, nonempty;
            block_scan2(tn_all, tc_all, sh.wsum, lane, wave, d0, d1, tot_all, nonempty);  // its barriers also order the hbuf reads above
            (void)nonempty;
            run += tot_all;
            if (tot_all == 0) continue;        // block-uniform
            if (prune_ok && bound == 0xFFFFFFFFu && tot_all > (uint32_t)(4 * GD_SEED * topk)) {
                // tuples up to the crude distance below which GD_SEED * topk survivors lie (tuple sizes as weights)
                pivot = block_kth_weighted<GD_PER>(sh.kth, pb, n, okm, (uint32_t)(GD_SEED * topk), tid, lane, wave);
                nsp = 2;
            }
        }
#pragma nounroll
        for (int sp = 0; sp < nsp; ++sp) {
            uint32_t sel = 0;                      // this part's tuples among the thread's GD_PER
            uint32_t tn = 0, tc = 0;
            {
                const uint32_t above = FUSED && prune_ok ? prune_above(bound, smin) : 0xFFFFFFFFu;
#pragma unroll
                for (int u = 0; u < GD_PER; ++u) {
                    bool in = n[u] != 0;
                    if (FUSED) in = in && pb[u] <= above && (nsp == 1 || (pb[u] <= pivot) == (sp == 0));
                    sel |= in ? 1u << u : 0u;
                    tn += in ? n[u] : 0u;
                    tc += in ? 1u : 0u;
                }
            }
            uint32_t x, c, tot, nhc;
            block_scan2(tn, tc, sh.wsum, lane, wave, x, c, tot, nhc);   // its barriers also order the hbuf reads above
            if (tot == 0) continue;                // block-uniform
#pragma unroll
            for (int u = 0; u < GD_PER; ++u) {
                if ((sel >> u) & 1u) {
                    hbuf[c] = s[u] - x;            // first position minus prefix (mod 2^32): position = this + survivor number
                    hx[c] = x;
                    ++c;
                    x += n[u];
                }
            }
            if (tid == 0) {
                hx[nhc] = tot;
                if (!FUSED) sh.base = atomicAdd(&count[q], tot);
            }
            __syncthreads();
            const uint32_t base = FUSED ? 0u : sh.base;
            if (!FUSED) run += tot;

            // ---- the survivors, 64 per row; the rows are dealt to the wavefronts in contiguous runs
            const uint32_t nrows = (tot + 63) >> 6;
            const uint32_t rpw = (nrows + GS_THREADS / 64 - 1) / (GS_THREADS / 64);
            const uint32_t r0 = (uint32_t)wave * rpw;
            const uint32_t rend = r0 + rpw < nrows ? r0 + rpw : nrows;        // <= r0: nothing for this wavefront
            const uint32_t steps = (rpw + GD_ROWS - 1) / GD_ROWS;              // block-uniform
            const uint32_t lane4 = (lane + 1) * 4, nhc4 = nhc * 4;
            const uint32_t lim = rend * 64 < tot ? rend * 64 : tot;            // end of this wavefront's survivors
            uint32_t ha = 0;
            if (r0 < rend) {
                // tuple holding survivor r0 * 64: the last one whose prefix is <= it (two 64-way probes)
                const uint32_t p = r0 * 64;
                const uint32_t i1 = lane * 32;
                const uint32_t v1 = hx[i1 < nhc ? i1 : nhc];
                const uint32_t c1 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(i1 < nhc && v1 <= p));
                const uint32_t b0 = (c1 - 1) * 32;
                const uint32_t i2 = b0 + lane;
                const uint32_t v2 = hx[i2 < nhc ? i2 : nhc];
                const uint32_t c2 = __builtin_popcountll(__builtin_amdgcn_ballot_w64(lane < 32 && i2 < nhc && v2 <= p));
                ha = b0 + c2 - 1;
            }
            // Grouped position of this lane's survivor in row `row` (< rend); moves ha to the tuple of
            // the next row.  Tuple ha holds the row's first survivor; every later tuple that starts
            // inside the row raises a flag at the lane of its first survivor (a stamp in the
            // wavefront's 64 LDS words, unique per call, so nothing has to be cleared), and a lane's
            // tuple is ha + the number of flags at or below it.
            auto locate = [&](uint32_t row) -> uint32_t {
                const uint32_t pf = row * 64;
                const uint32_t pl = pf + 63 < tot ? pf + 63 : tot - 1;
                const uint32_t p = pf + lane < pl ? pf + lane : pl;
                // prefixes of the tuples after ha (hx[nhc] = tot > pl), addressed in bytes: add, min, read
                const uint32_t bi4 = ha * 4 + lane4;
                const uint32_t bnd = *reinterpret_cast<const uint32_t *>(reinterpret_cast<const char *>(hx) + (bi4 < nhc4 ? bi4 : nhc4));
                ++stamp;
                if (bnd <= pl) flag[bnd - pf] = stamp;              // pf < bnd: tuple ha holds pf
                __builtin_amdgcn_wave_barrier();                    // LDS runs a wavefront's accesses in order
                const uint64_t marks = __builtin_amdgcn_ballot_w64(flag[lane] == stamp);
                // flags at or below this lane: lane 0 never holds one (a flagged tuple starts after pf), so
                // that is the count below the lane in the flags moved down by one -- two mbcnt, ha added in
                const uint64_t m1 = marks >> 1;
                const uint32_t h = __builtin_amdgcn_mbcnt_hi((uint32_t)(m1 >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m1, ha));
                const uint32_t pos = hbuf[h] + p;
                // Tuples that start at or before the next row's first survivor.  The clamped lanes read tot,
                // which passes only in the pass's last row -- after which ha is not used again.
                ha += (uint32_t)__builtin_popcountll(__builtin_amdgcn_ballot_w64(bnd <= pl + 1));
                return pos;
            };
            // records (and, for the key list, ids) of rows r, r + 1; rows past rend read record 0, unused
            constexpr int HALF = GD_ROWS / 2;
            auto fetch = [&](uint32_t r, uint32_t (*rec)[WORDS], uint32_t *low) {
#pragma unroll
                for (int u = 0; u < HALF; ++u) {
                    uint32_t pos = 0;
                    if (r + u < rend) pos = locate(r + u);          // wavefront-uniform
                    const uint32_t *p = reinterpret_cast<const uint32_t *>(items_grouped + (size_t)pos * (WORDS * 4));
                    if (WORDS == 1) {
                        rec[u][0] = p[0];
                    } else if (WORDS == 2) {
                        const uint2 v = *reinterpret_cast<const uint2 *>(p);
                        rec[u][0] = v.x;
                        rec[u][1 % WORDS] = v.y;
                    } else {
                        const uint4 v = *reinterpret_cast<const uint4 *>(p);
                        rec[u][0] = v.x;
                        rec[u][1 % WORDS] = v.y;
                        rec[u][2 % WORDS] = v.z;
                        rec[u][3 % WORDS] = v.w;
                    }
                    low[u] = FUSED ? pos : perm[pos];
                }
            };
            unsigned long long key[GD_ROWS];
            bool take[GD_ROWS];
            uint64_t mk[GD_ROWS];                  // FUSED: ballot of take (wavefront-uniform)
            // distances and keys of rows r, r + 1 from their records
            auto finish = [&](uint32_t r, const uint32_t (*rec)[WORDS], const uint32_t *low, int slot0) {
#pragma unroll
                for (int u = 0; u < HALF; ++u) {
                    // k ascending like every other kernel; the first term stands for 0 + itself (no table holds -0)
                    float d = T[rec[u][0] & 0xffu];
#pragma unroll
                    for (int w = 0; w < WORDS; ++w) {
#pragma unroll
                        for (int b = w == 0 ? 1 : 0; b < 4; ++b)
                            d += T[(w * 4 + b) * ICQ_LUT_W + ((rec[u][w] >> (8 * b)) & 0xffu)];
                    }
                    const uint32_t ob = icq_order_bits(d);
                    key[slot0 + u] = ((unsigned long long)ob << 32) | low[u];
                    // survivors of this row that exist (wavefront-uniform count: the last row of a pass is ragged)
                    // (one signed comparison against a wavefront-uniform bound: rows at or past `lim` give <= 0)
                    const uint32_t first = (r + u) * 64;
                    const bool exists = (int)lane < (int)(lim - first);
                    if (FUSED) {
                        // the comparisons feed the ballots directly (one instruction each, no select)
                        const bool near = ob <= bound;
                        mk[slot0 + u] = __builtin_amdgcn_ballot_w64(near) & __builtin_amdgcn_ballot_w64(exists);
                        take[slot0 + u] = near && exists;
                    } else {
                        take[slot0 + u] = exists;
                        const uint64_t slot = (uint64_t)base + first + lane;
                        if (exists && slot < (uint64_t)cap) my_out[slot] = key[slot0 + u];
                    }
                }
            };
            // Two half steps in flight: the records of one half are fetched while the other half's
            // distances are formed, each into registers of its own (no copies, so no wait on the
            // loads that were just sent).
            uint32_t recA[HALF][WORDS], recB[HALF][WORDS], lowA[HALF], lowB[HALF];
            fetch(r0, recA, lowA);
            for (uint32_t it = 0; it < steps; ++it) {
                const uint32_t r = r0 + it * GD_ROWS;
                fetch(r + HALF, recB, lowB);
                finish(r, recA, lowA, 0);
                fetch(r + GD_ROWS, recA, lowA);
                finish(r + HALF, recB, lowB, HALF);
                if (FUSED) {
                    uint32_t pre[GD_ROWS], mycnt = 0;
#pragma unroll
                    for (int u = 0; u < GD_ROWS; ++u) {
                        pre[u] = mycnt;
                        mycnt += (uint32_t)__builtin_popcountll(mk[u]);
                    }
                    if (lane == 0) sh.wtot[it & 1][wave] = mycnt;
                    __syncthreads();
                    uint32_t mybase = cnt, all = 0;              // scalar registers: the counts are read once per wavefront
#pragma unroll
                    for (int w = 0; w < GS_THREADS / 64; ++w) {
                        const uint32_t tw = (uint32_t)__builtin_amdgcn_readfirstlane((int)sh.wtot[it & 1][w]);
                        if (w < wave) mybase += tw;
                        all += tw;
                    }
#pragma unroll
                    for (int u = 0; u < GD_ROWS; ++u)
                        if (take[u])
                            list[__builtin_amdgcn_mbcnt_hi((uint32_t)(mk[u] >> 32),
                                                           __builtin_amdgcn_mbcnt_lo((uint32_t)mk[u], mybase + pre[u]))] = key[u];
                    cnt += all;
                    // block-uniform: cut while the next step might not fit -- one counting pass, then
                    // (fat bin) exactly, then (many equal distances) by id
                    for (int lvl = 0; lvl < 3 && cnt > (uint32_t)(GD_LIST - GD_STEP); ++lvl) {
                        if (lvl < 2) cnt = block_cut(sh, list, cnt, (uint32_t)topk, &bound, lvl == 1, tid, lane, wave);
                        else cnt = block_tie_cut(sh, list, cnt, (uint32_t)topk, bound, perm, tid, lane, wave);
                    }
                }
            }
            __syncthreads();                       // hbuf / hx are rewritten by the next part or pass
            // the first part's topk-th distance (upper end of its histogram bin) becomes the bound
            if (FUSED && nsp == 2 && sp == 0 && cnt > (uint32_t)topk)
                cnt = block_cut(sh, list, cnt, (uint32_t)topk, &bound, false, tid, lane, wave);
        }
    }

    if (!FUSED) return;                        // the atomics have counted the survivors
    // Several blocks per query (few queries): each keeps the list of its slices of the tuples
    // and leaves its topk best as keys (bits of D, id) for the merge kernel.
    unsigned long long *part = keys_out ? keys_out + ((int64_t)q * gridDim.x + blockIdx.x) * topk : nullptr;
    if (tid == 0) {
        if (part) atomicAdd(&count[q], run);
        else count[q] = run;
    }
    // ---- final list: exact cut, positions -> ids, order by (D, id)
    // (the ranking below drops what a counting cut leaves beyond topk; the exact cut is for the
    // lists that one counting pass leaves longer than a block's worth of keys)
    if (cnt > (uint32_t)GS_THREADS) cnt = block_cut(sh, list, cnt, (uint32_t)topk, &bound, false, tid, lane, wave);
    if (cnt > (uint32_t)GS_THREADS) {
        cnt = block_cut(sh, list, cnt, (uint32_t)topk, &bound, true, tid, lane, wave);
        if (cnt > (uint32_t)GD_SORT) cnt = block_tie_cut(sh, list, cnt, (uint32_t)topk, bound, perm, tid, lane, wave);
    }
    __syncthreads();
    uint32_t *oi = out_ids + (int64_t)q * topk;
    float *od = out_dist + (int64_t)q * topk;
    const int kept = (int)cnt < topk ? (int)cnt : topk;
    if (cnt <= (uint32_t)GS_THREADS) {
        // one key per thread: its rank among the (distinct) keys is its row
        unsigned long long mine_k = KEY_PAD;
        if (tid < (int)cnt) {
            const unsigned long long k = list[tid];
            mine_k = (k & 0xFFFFFFFF00000000ull) | perm[(uint32_t)k];
        }
        __syncthreads();
        if (tid <= (int)cnt) list[tid] = mine_k;       // list[cnt] = KEY_PAD: the keys are read in pairs
        __syncthreads();
        uint32_t rank = 0;
        for (uint32_t j = 0; j < cnt; j += 2) {
            const uint4 v = *reinterpret_cast<const uint4 *>(&list[j]);   // one address for all lanes
            rank += (((unsigned long long)v.y << 32) | v.x) < mine_k ? 1u : 0u;
            rank += (((unsigned long long)v.w << 32) | v.z) < mine_k ? 1u : 0u;
        }
        if (tid < (int)cnt && rank < (uint32_t)topk) {
            if (part) {
                part[rank] = mine_k;
            } else {
                oi[rank] = (uint32_t)mine_k;
                od[rank] = icq_unorder_bits((uint32_t)(mine_k >> 32));
            }
        }
        for (int r = kept + tid; r < topk; r += GS_THREADS) {
            if (part) {
                part[r] = KEY_PAD;
            } else {
                oi[r] = ICQ_PAD_ID;
                od[r] = INFINITY;
            }
        }
        return;
    }
    // many equal distances at the cut: bitonic sort of up to GD_SORT keys by one wavefront
    int len = 64;
    while (len < (int)cnt) len <<= 1;
    for (int i = tid; i < len; i += GS_THREADS) {
        unsigned long long k = KEY_PAD;
        if (i < (int)cnt) {
            k = list[i];
            k = (k & 0xFFFFFFFF00000000ull) | perm[(uint32_t)k];
        }
        list[i] = k;
    }
    __syncthreads();
    if (wave == 0) wave_sort(list, len, (int)lane);
    __syncthreads();
    for (int r = tid; r < topk; r += GS_THREADS) {
        if (part) {
            part[r] = r < kept ? list[r] : KEY_PAD;
        } else {
            oi[r] = r < kept ? (uint32_t)list[r] : ICQ_PAD_ID;
            od[r] = r < kept ? icq_unorder_bits((uint32_t)(list[r] >> 32)) : INFINITY;
        }
    }
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
              hipMalloc(&ix->items_grouped, (size_t)ix->N * ix->item_stride) == hipSuccess;
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

// Blocks that share one query's tuple rows in the grouped kernels: enough to fill the chip
// when there are few queries.
static int group_parts(const icq_index *ix, int Q) {
    if (ix->Kf != 2) return 1;
    int parts = (2 * ix->num_cu + Q - 1) / Q;
    if (parts > 16) parts = 16;
    if (parts < 1) parts = 1;
    return parts;
}

int icq_launch_group_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                          uint32_t *cand_ids, bool as_positions, uint32_t *cand_count, int64_t cap,
                          hipStream_t s) {
    // cand_count has been zeroed by the caller (icq_launch_scan)
    const int parts = group_parts(ix, Q);
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

bool icq_group_fused(const icq_index *ix, int Q, int topk) {
    return icq_group_usable(ix, Q) && ix->item_stride <= 16 && topk <= GD_TOPK;
}

// Blocks per query in the fused form: one when the queries alone fill the chip; else each block
// takes its slice of every surviving tuple's items and a merge kernel joins the parts' lists (at
// most 8 parts of at most 256 keys).  Every block evaluates and lists all tuples, so more blocks
// pay only where the items weigh more than that: two blocks per CU with about 16 items per tuple
// (N = 1e6), four with 150 (N = 1e7) measured best.
int icq_group_fused_parts(const icq_index *ix, int Q) {
    if (ix->Kf != 2 || Q <= 0) return 1;
    const int per_cu = ix->N >= (int64_t)64 * ix->groups ? 4 : 2;
    int parts = (per_cu * ix->num_cu + Q - 1) / Q;
    if (parts > 8) parts = 8;
    if (parts < 1) parts = 1;
    return parts;
}

int icq_launch_group_keys(const icq_index *ix, const float *lut, int Q, const float *thr,
                          unsigned long long *cand_keys, uint32_t *cand_count, int64_t cap, int topk,
                          uint32_t *out_ids, float *out_dist, hipStream_t s) {
    // cand_count has been zeroed by the caller (icq_launch_scan); item_stride <= 16 here
    const bool fused = out_ids != nullptr && icq_group_fused(ix, Q, topk);
    const int parts = fused ? icq_group_fused_parts(ix, Q) : group_parts(ix, Q);
    // cand_keys: [Q][cap] keys of the survivors, or (fused, several parts) [Q][parts][topk] part lists
    if ((!fused || parts > 1) && !cand_keys) return ICQ_ERR_ARG;
    const int rows = (256 + parts - 1) / parts;
    for (int q0 = 0; q0 < Q; q0 += 65535) {
        const int nq = Q - q0 < 65535 ? Q - q0 : 65535;
        dim3 grid((unsigned)parts, (unsigned)nq);
        const float *l = lut + (int64_t)q0 * ix->K * ICQ_LUT_W;
        unsigned long long *ko = fused ? (parts > 1 ? cand_keys + (int64_t)q0 * parts * topk : nullptr)
                                       : cand_keys + (int64_t)q0 * cap;
        uint32_t *oi = fused ? out_ids + (int64_t)q0 * topk : nullptr;
        float *od = fused ? out_dist + (int64_t)q0 * topk : nullptr;
#define ICQ_GK(KF, W)                                                                                         \
    do {                                                                                                      \
        if (fused)                                                                                            \
            group_keys_kernel<KF, W, true><<<grid, GS_THREADS, 0, s>>>(                                        \
                l, ix->K, thr + q0, ix->group_start, ix->items_grouped, ix->perm, ko, cand_count + q0, cap,    \
                rows, topk, oi, od);                                                                          \
        else                                                                                                  \
            group_keys_kernel<KF, W, false><<<grid, GS_THREADS, 0, s>>>(                                       \
                l, ix->K, thr + q0, ix->group_start, ix->items_grouped, ix->perm, ko, cand_count + q0, cap,    \
                rows, topk, oi, od);                                                                          \
    } while (0)
        const int W = ix->item_stride / 4;
        if (ix->Kf == 1) {
            if (W == 1) ICQ_GK(1, 1); else if (W == 2) ICQ_GK(1, 2); else ICQ_GK(1, 4);
        } else {
            if (W == 1) ICQ_GK(2, 1); else if (W == 2) ICQ_GK(2, 2); else ICQ_GK(2, 4);
        }
#undef ICQ_GK
    }
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    if (fused && parts > 1) return icq_launch_merge(cand_keys, Q, parts, topk, true, out_ids, out_dist, s);
    return ICQ_OK;
}

ICQ_EXPORT int icq_index_set_scan_mode(icq_index *ix, int mode) {
    if (!ix || mode < ICQ_SCAN_AUTO || mode > ICQ_SCAN_GROUPED) return ICQ_ERR_ARG;
    ix->scan_mode = mode;
    return ICQ_OK;
}
