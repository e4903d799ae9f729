// Stage 1 of the two-step search (arxiv 1912.08756, Eq. 2 and Sec. 3.4): the
// crude distance P[q][i] = sum_{k<Kf} lut[q][k][code_k(i)] over the fast
// codebooks only, compared with a per-query threshold; survivors are appended
// to per-query candidate lists for stage 2.
//
// Item-by-item kernels (the form grouped by fast-code tuple lives in icq_group.hip):
//   scan_stream_kernel - lanes = items, up to Kf = 4.  The tables of B = 1, 2 or 4
//       queries sit in LDS replicated so that the lanes the LDS serves in one clock
//       never share a bank; one pass over the fast sub-codes serves B queries.
//   scan_items_kernel  - lanes = items.  Any Kf; the tables of a few queries
//       sit in LDS as [query][k][code], each lane gathers with its own
//       sub-codes held in registers, survivors are compacted with a ballot.
// Both list survivor ids only; crude distances are filled in afterwards for the
// listed ids when the caller wants them.
#include "icq_internal.h"
#include "icq_sort.h"

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

// cand_part[q][s] = sum_{k<Kf} lut[q][k][code_k(id)] for the listed survivors, in
// the same order of additions as the scan (so the value is the one it compared).
__global__ __launch_bounds__(256) void fill_partials_kernel(
    const uint8_t *__restrict__ fast, int64_t Npad, const float *__restrict__ lut, int K, int Kf,
    const uint32_t *__restrict__ cand_ids, const uint32_t *__restrict__ cand_count, int64_t cap,
    int blocks_per_query, float *__restrict__ cand_part) {
    const int q = blockIdx.x / blocks_per_query, bq = blockIdx.x % blocks_per_query;
    uint64_t n = cand_count[q];
    if (n > (uint64_t)cap) n = (uint64_t)cap;
    const float *T = lut + (int64_t)q * K * ICQ_LUT_W;
    for (uint64_t s = (uint64_t)bq * blockDim.x + threadIdx.x; s < n;
         s += (uint64_t)blocks_per_query * blockDim.x) {
        const uint32_t id = cand_ids[(int64_t)q * cap + s];
        float P = T[fast[id]];
        for (int k = 1; k < Kf; ++k) P += T[k * ICQ_LUT_W + fast[(int64_t)k * Npad + id]];
        cand_part[(int64_t)q * cap + s] = P;
    }
}

// ------------------------------------------------------------------ lanes = items, few queries
// Streaming form for one to a few queries per pass: every code byte is read
// from HBM once per B queries, so the kernel is bound by the code stream.  Each
// lane owns 16 consecutive items per step (one 128-bit load per fast row).  The
// B queries' fast tables sit in LDS replicated C = 16 times, entry (k, c) copy r
// at dword ((k*256 + c)*C + r)*B: lane l reads copy l%C, and the 16 lanes the LDS
// serves per clock then always fall into 16 different banks, whatever their
// sub-codes.  The B values of an entry are adjacent, so one 32/64/128-bit read
// serves all B queries -- the LDS takes 16 addresses per clock whatever the
// width, so B = 4 moves three times the table entries per clock of B = 1.  With
// B = 4 and Kf > 2 only C = 8 copies fit (128 KB): two lanes of a 16-lane group
// then share a copy and collide when their sub-codes have the same parity.
// Calls with many queries and Kf = 3, 4 (no grouping, no transposed tables) run
// this form with B = 4, one block column per group of four queries.
// Survivors: a lane collects the hit bits of its 16 items; a wavefront compacts
// them with ballots into its OWN slice of an LDS staging list (its count lives in
// a scalar register: no atomics, nothing to wait for), and every SS_CHECK steps
// the block looks at the 16 counts; when a slice is half full the block moves all
// slices to the query's global list with ONE global atomic -- all blocks add to
// the same counter, and that address only takes ~10^8 atomics per second.  A
// slice that fills up between two checks is moved out by its wavefront alone.
// The code stream is read R - 1 steps ahead into register sets of their own (R
// copies of the step body, no register moves), with loads that are never
// conditional (past the block's range they re-read its first items), so the
// compiler can leave the newer loads in flight while the oldest are consumed;
// the first of them are sent before the tables are even written to LDS.
constexpr int ss_copies(int KF, int B) { return KF * ICQ_LUT_W * 16 * 4 * B <= 131072 ? 16 : 8; }
constexpr int ss_half(int B) { return B == 4 ? 2 : 8; }   // items per lane whose table reads are issued together
constexpr int SS_CHECK = 8;       // steps between block-wide flush checks
constexpr int SS_THREADS = 1024;
constexpr int SS_WAVES = SS_THREADS / 64;

// NT: the code stream is loaded with the non-temporal hint -- for an array far beyond the 256 MB
// last-level cache that is read once per pass anyway, 400 MB then read in 60 instead of 67 us
// (a plain read kernel in this launch shape); an array that fits is better kept.
//
// G2 (index grouped by the first two fast sub-codes, see icq_group2.hip): the scan walks grouped
// positions; `fast` holds the KF = Kf - 2 remaining fast rows in grouped order and info[p / 16]
// names the tuple that positions p .. p + 15 belong to (c0 | c1 << 8 | valid positions << 16).  The
// sum of the tuple's two table entries is formed once per 16 positions from unreplicated copies of
// the first two tables and the streamed rows' entries are added to it in codebook order -- the same
// additions as item by item.  Listed are grouped positions (ids through `perm` when it is given).
//
// MASK (icq_search): no lists at all.  The kernel stores the hit bits themselves, one bit per
// scan position and query (masks[q * mask_stride + p / 16] holds positions p .. p + 15, bit j =
// position p + j), for every position of the block's range -- zeros beyond N -- and stage 2 walks
// those words.  No staging, no compaction, no atomics; whatever the survivors' number or order.
template <int KF, int B, bool NT, bool G2, bool MASK>
__global__ __launch_bounds__(SS_THREADS) void scan_stream_kernel(
    const uint8_t *fast, int64_t Npad, uint32_t N, const float *__restrict__ lut, int K,
    const float *__restrict__ thr, int Q, uint32_t *__restrict__ cand_ids,
    uint32_t *__restrict__ cand_count, int64_t cap, uint32_t items_per_block, uint32_t wave_cap,
    const uint32_t *__restrict__ info, const uint32_t *__restrict__ perm, uint16_t *__restrict__ masks,
    size_t mask_stride, uint32_t scan_end) {
    extern __shared__ __attribute__((aligned(16))) float smem[];
    __shared__ uint32_t s_wcnt[B][SS_WAVES], s_base[B];
    __shared__ float s_tmin[G2 ? KF : 1][G2 ? B : 1][4];   // G2: smallest entry of each streamed table, per wavefront of entries
    constexpr int C = ss_copies(KF, B);
    constexpr int SS_HALF = G2 && B == 4 ? 4 : ss_half(B);
    constexpr int TAB_FLOATS = KF * ICQ_LUT_W * C * B;
    constexpr int T01_FLOATS = G2 ? 2 * ICQ_LUT_W * B : 0;
    constexpr int K0 = G2 ? 2 : 0;                    // codebook of the first streamed row
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qbase = blockIdx.y * B;

    // The tables go to LDS after the first code loads have been sent (see the end of the kernel).
    // Consecutive threads write consecutive 16-byte pieces (conflict-free; writing an entry's C
    // copies from one thread instead puts 16 lanes on the same banks and took 7 us per block);
    // a piece holds 4 / B copies of the entry's B values.  All loads go out before the writes.
    float tmin[KF][B];
    auto fill_tables = [&]() {
        constexpr int NV = TAB_FLOATS / 4 / SS_THREADS;              // 16-byte pieces per thread
        static_assert(TAB_FLOATS % (4 * SS_THREADS) == 0 && C % 4 == 0, "whole pieces, inside one entry");
        const float *row[B];
#pragma unroll
        for (int b = 0; b < B; ++b) {
            const int qb = (qbase + b) < Q ? qbase + b : Q - 1;       // clamped; replaced by +inf below
            row[b] = lut + ((int64_t)qb * K + K0) * ICQ_LUT_W;
        }
        float x[NV][B];
#pragma unroll
        for (int j = 0; j < NV; ++j) {
            const int e = ((j * SS_THREADS + tid) * 4 / B) / C;
#pragma unroll
            for (int b = 0; b < B; ++b) x[j][b] = row[b][e];
        }
#pragma unroll
        for (int j = 0; j < NV; ++j) {
#pragma unroll
            for (int b = 0; b < B; ++b)
                if ((qbase + b) >= Q) x[j][b] = INFINITY;            // block-uniform
            float4 v;
            v.x = x[j][0];
            v.y = x[j][1 % B];
            v.z = x[j][2 % B];
            v.w = x[j][3 % B];
            reinterpret_cast<float4 *>(smem)[j * SS_THREADS + tid] = v;
        }
        if (G2 && tid < T01_FLOATS / 4) {
            // the first two tables, one copy, the B values of an entry adjacent
            float4 v;
            float *vv = reinterpret_cast<float *>(&v);
#pragma unroll
            for (int f = 0; f < 4; ++f) {
                const int idx = tid * 4 + f, e = idx / B, b = idx % B;
                vv[f] = (qbase + b) < Q ? lut[(int64_t)(qbase + b) * K * ICQ_LUT_W + e] : INFINITY;
            }
            reinterpret_cast<float4 *>(smem + TAB_FLOATS)[tid] = v;
        }
        __syncthreads();
        if (G2) {
            // smallest entry of every streamed table (from its first copy): what the streamed rows add at least
            if (tid < ICQ_LUT_W) {
#pragma unroll
                for (int k = 0; k < KF; ++k) {
#pragma unroll
                    for (int b = 0; b < B; ++b) {
                        const float m = wave_min_f32(smem[((k * ICQ_LUT_W + tid) * C) * B + b]);
                        if (lane == 0) s_tmin[k][b][tid >> 6] = m;
                    }
                }
            }
            __syncthreads();
#pragma unroll
            for (int k = 0; k < KF; ++k) {
#pragma unroll
                for (int b = 0; b < B; ++b)
                    tmin[k][b] = fminf(fminf(s_tmin[k][b][0], s_tmin[k][b][1]), fminf(s_tmin[k][b][2], s_tmin[k][b][3]));
            }
        }
    };
    float t[B];
#pragma unroll
    for (int b = 0; b < B; ++b) t[b] = (qbase + b) < Q ? thr[qbase + b] : -INFINITY;
    // staging: [B][SS_WAVES][wave_cap] ids
    uint32_t *stage = reinterpret_cast<uint32_t *>(smem + TAB_FLOATS + T01_FLOATS);
    const float *t01 = smem + TAB_FLOATS;
    uint32_t wc[B];               // ids staged by this wavefront (wavefront-uniform)
#pragma unroll
    for (int b = 0; b < B; ++b) wc[b] = 0;

    const uint32_t begin = blockIdx.x * items_per_block;
    uint32_t end = begin + items_per_block;
    if (end > N || end < begin) end = N;
    // MASK: the steps run to the end of the block's range even past the last item (scan_end is a whole
    // number of block steps and the mask words reach that far)
    uint32_t walk_end = end;
    if (MASK) {
        walk_end = begin + items_per_block;
        if (walk_end > scan_end || walk_end < begin) walk_end = scan_end;
    }
    // byte offset of this lane's copy inside an entry; an entry is C copies of B floats
    constexpr int ENTRY_BYTES = C * 4 * B;
    constexpr int ENTRY_SHIFT = ENTRY_BYTES == 64 ? 6 : ENTRY_BYTES == 128 ? 7 : 8;
    static_assert((1 << ENTRY_SHIFT) == ENTRY_BYTES, "entry size is 64, 128 or 256 bytes");
    const uint32_t copy_off = (lane & (C - 1)) * (4 * B);
    const char *tab_bytes = reinterpret_cast<const char *>(smem);
    constexpr uint32_t step = (uint32_t)SS_WAVES * 1024u;
    const uint32_t nsteps = walk_end > begin ? (walk_end - begin + step - 1) / step : 0;   // same for every wavefront

    // 1024 items at g into w; past the block's range the block's first items are read instead
    // (unused, but in bounds: g < end <= N and the rows are padded by more than 1024 bytes)
    constexpr int R = B == 1 ? 3 : 2;
    static_assert(B == 1 || B == 2 || B == 4, "one 32/64/128-bit table read per lookup");
    uint4 w[R][KF];
    uint32_t ci[R];               // G2: the tuple and valid count of this lane's 16 positions
    auto load = [&](uint32_t g, uint4 (&w)[KF], uint32_t &ci) {
        const uint32_t gs = (g < end && g >= begin) ? g : begin;
        if (G2) ci = info[(gs >> 4) + lane];
#pragma unroll
        for (int k = 0; k < KF; ++k) {
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 *src = reinterpret_cast<const u32x4 *>(fast + (int64_t)k * Npad + gs + lane * 16);
            const u32x4 v = NT ? __builtin_nontemporal_load(src) : *src;
            w[k] = make_uint4(v.x, v.y, v.z, v.w);
        }
    };
    // n staged ids of query b -> the query's list from slot `first` on
    auto move_out = [&](int b, const uint32_t *src, uint32_t n, uint64_t first) {
        uint32_t *dst = cand_ids + (int64_t)(qbase + b) * cap;
        for (uint32_t i = lane; i < n; i += 64) {
            const uint64_t slot = first + i;
            if (slot < (uint64_t)cap) dst[slot] = (G2 && perm) ? perm[src[i]] : src[i];
        }
    };
    // the 1024 items at g held in w: table sums and hit bits.  hm[b] (zero on entry) receives the hit
    // bits of this lane's 16 items for query b, item j in bit 15 - j.
    auto hits = [&](uint32_t g, const uint4 (&w)[KF], uint32_t ci, uint32_t (&hm)[B]) {
        const uint32_t id0 = g + lane * 16;
        float p01[B];
        if (G2) {
            // the tuple's two entries, summed once for the 16 positions
            const float *e0 = t01 + (ci & 0xffu) * B, *e1 = t01 + (ICQ_LUT_W + ((ci >> 8) & 0xffu)) * B;
            if (B == 1) {
                p01[0] = e0[0] + e1[0];
            } else if (B == 2) {
                const float2 a = *reinterpret_cast<const float2 *>(e0), c = *reinterpret_cast<const float2 *>(e1);
                p01[0] = a.x + c.x;
                p01[1 % B] = a.y + c.y;
            } else {
                const float4 a = *reinterpret_cast<const float4 *>(e0), c = *reinterpret_cast<const float4 *>(e1);
                p01[0] = a.x + c.x;
                p01[1 % B] = a.y + c.y;
                p01[2 % B] = a.z + c.z;
                p01[3 % B] = a.w + c.w;
            }
        }
        // G2: a query none of whose 64 x 16 positions can be a hit is left out of this step.  Every
        // position's sum is its pair's sum plus one entry of each streamed table, added in this order;
        // rounding is monotone, so the same additions with the tables' smallest entries bound it from below
        // exactly -- a lane whose bound is not below the threshold has no hit.  (A pair's run is some
        // 1500 positions at N = 1e8, so the wavefront's 1024 positions belong to one or two pairs, and for
        // most queries most pairs are out of reach.)
        bool live[B];
        bool any_live = !G2;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            live[b] = true;
            if (G2) {
                float lb = p01[b] + tmin[0][b];
#pragma unroll
                for (int k = 1; k < KF; ++k) lb += tmin[k][b];
                live[b] = __builtin_amdgcn_ballot_w64(lb < t[b]) != 0;      // wavefront-uniform
                any_live |= live[b];
            }
        }
        if (!any_live) return;
#pragma unroll
        for (int h = 0; h < 16; h += SS_HALF) {
            // phase 1: every table address of the half step
            uint32_t off[SS_HALF][KF];
#pragma unroll
            for (int jj = 0; jj < SS_HALF; ++jj) {
                const int j = h + jj;
#pragma unroll
                for (int k = 0; k < KF; ++k) {
                    const uint32_t word = j < 4 ? w[k].x : j < 8 ? w[k].y : j < 12 ? w[k].z : w[k].w;
                    // extract + shift-add: two instructions per byte.  For the lowest byte the compiler
                    // pulls the shift in front of the mask and needs three, hence the opaque extract.
                    uint32_t code;
                    if ((j & 3) == 0) asm("v_bfe_u32 %0, %1, 0, 8" : "=v"(code) : "v"(word));
                    else code = (word >> (8 * (j & 3))) & 0xffu;
                    off[jj][k] = (code << ENTRY_SHIFT) + copy_off;
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // phase 2: all reads in flight together
            float v[SS_HALF][KF][B];
#pragma unroll
            for (int jj = 0; jj < SS_HALF; ++jj) {
#pragma unroll
                for (int k = 0; k < KF; ++k) {
                    const char *e = tab_bytes + k * (ICQ_LUT_W * ENTRY_BYTES) + off[jj][k];
                    if (B == 1) {
                        v[jj][k][0] = *reinterpret_cast<const float *>(e);
                    } else if (B == 2) {
                        const float2 x = *reinterpret_cast<const float2 *>(e);
                        v[jj][k][0] = x.x;
                        v[jj][k][1 % B] = x.y;
                    } else {
                        const float4 x = *reinterpret_cast<const float4 *>(e);
                        v[jj][k][0] = x.x;
                        v[jj][k][1 % B] = x.y;
                        v[jj][k][2 % B] = x.z;
                        v[jj][k][3 % B] = x.w;
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            // phase 3: sums (k ascending) and hit bits
#pragma unroll
            for (int b = 0; b < B; ++b) {
                if (G2 && !live[b]) continue;             // wavefront-uniform; hm[b] stays zero for the whole step
#pragma unroll
                for (int jj = 0; jj < SS_HALF; ++jj) {
                    float P = G2 ? p01[b] + v[jj][0][b] : v[jj][0][b];
#pragma unroll
                    for (int k = 1; k < KF; ++k) P += v[jj][k][b];
                    icq_hit_shift_in(hm[b], P, t[b]);
                }
            }
        }
        if (id0 + 16 > end || id0 + 16 < id0) {   // ragged tail: drop bits of items at or beyond `end`
            const uint32_t valid = id0 < end ? 0xFFFFu & ~((1u << (16 - (end - id0))) - 1u) : 0u;
#pragma unroll
            for (int b = 0; b < B; ++b) hm[b] &= valid;
        }
        if (G2) {   // the padding behind a tuple's last item
            const uint32_t valid = (0xFFFF0000u >> (ci >> 16)) & 0xFFFFu;
#pragma unroll
            for (int b = 0; b < B; ++b) hm[b] &= valid;
        }
    };
    // With two register sets the hit bits of two consecutive steps share one compaction: the earlier
    // step's bits sit in the upper half of the mask, so one round of ballots serves 2048 items.
    constexpr bool PAIR = R == 2;
    // compaction: each round appends every lane's lowest remaining hit.  Bit p of hm[b] names item
    // id_lo + 15 - p (p < 16) or id_hi + 31 - p.
    auto compact = [&](uint32_t (&hm)[B], uint32_t id_hi, uint32_t id_lo) {
#pragma unroll
        for (int b = 0; b < B; ++b) {
            uint32_t *mine_stage = stage + ((uint32_t)b * SS_WAVES + wave) * wave_cap;
            uint64_t mask = __builtin_amdgcn_ballot_w64(hm[b] != 0);
            while (mask != 0) {
                const uint32_t n = (uint32_t)__builtin_popcountll(mask);
                const uint32_t rank = (uint32_t)__builtin_popcountll(mask & ((1ull << lane) - 1));
                if (wc[b] + n > wave_cap) {   // slice full between two checks: the wavefront moves it out itself
                    uint32_t gb = 0;
                    if (lane == 0) gb = atomicAdd(&cand_count[qbase + b], wc[b]);
                    gb = (uint32_t)__builtin_amdgcn_readfirstlane((int)gb);
                    move_out(b, mine_stage, wc[b], gb);
                    wc[b] = 0;
                }
                if (hm[b] != 0) {
                    const uint32_t p = (uint32_t)__builtin_ctz(hm[b]);
                    mine_stage[wc[b] + rank] = (PAIR && p >= 16 ? id_hi + 31u : id_lo + 15u) - p;
                }
                wc[b] += n;
                hm[b] &= hm[b] - 1;
                mask = __builtin_amdgcn_ballot_w64(hm[b] != 0);
            }
        }
    };
    // block-wide look at the slices; moves them out when one is half full (or at the end)
    auto flush_check = [&](bool last) {
        if (lane == 0) {
#pragma unroll
            for (int b = 0; b < B; ++b) s_wcnt[b][wave] = wc[b];
        }
        __syncthreads();
        uint32_t pre[B], tot[B];
        bool any = false;
#pragma unroll
        for (int b = 0; b < B; ++b) {
            // lane w < 16 takes wavefront w's count; prefix over the 16 lanes
            const uint32_t c = lane < SS_WAVES ? s_wcnt[b][lane] : 0u;
            static_assert(SS_WAVES == 16, "the prefix below covers one DPP row of 16 lanes");
            uint32_t incl = c;
            incl += icq_dpp<0x111, 0xf, 0u>(incl);
            incl += icq_dpp<0x112, 0xf, 0u>(incl);
            incl += icq_dpp<0x114, 0xf, 0u>(incl);
            incl += icq_dpp<0x118, 0xf, 0u>(incl);
            pre[b] = (uint32_t)__builtin_amdgcn_readlane((int)(incl - c), wave);
            tot[b] = (uint32_t)__builtin_amdgcn_readlane((int)incl, SS_WAVES - 1);
            any |= __builtin_amdgcn_ballot_w64(c > wave_cap / 2) != 0;
            any |= last && tot[b] > 0;
        }
        __syncthreads();   // nobody publishes again before every thread has read the counts
        if (!any) return;  // block-uniform
        if (tid < B) s_base[tid] = tot[tid] ? atomicAdd(&cand_count[qbase + tid], tot[tid]) : 0;
        __syncthreads();
#pragma unroll
        for (int b = 0; b < B; ++b) {
            move_out(b, stage + ((uint32_t)b * SS_WAVES + wave) * wave_cap, wc[b], (uint64_t)s_base[b] + pre[b]);
            wc[b] = 0;
        }
        // the next publish of s_wcnt / s_base comes after at least one more barrier pair
    };

    // R register sets of 1024 items per wavefront: R - 1 steps are always in flight
    uint32_t g = begin + wave * 1024u;
#pragma unroll
    for (int r = 0; r < R - 1; ++r) load(g + (uint32_t)r * step, w[r], ci[r]);
    fill_tables();
    static_assert(SS_CHECK % 2 == 0, "a pair of steps never straddles a periodic check");
    uint32_t held[B];        // PAIR: the even step's hit bits, waiting for the odd step's
    uint32_t id_held = 0;
#pragma unroll
    for (int b = 0; b < B; ++b) held[b] = 0;
    for (uint32_t it = 0; it < nsteps; it += R, g += R * step) {
#pragma unroll
        for (int u = 0; u < R; ++u) {
            load(g + (uint32_t)(u + R - 1) * step, w[(u + R - 1) % R], ci[(u + R - 1) % R]);     // never conditional
            const uint32_t gu = g + (uint32_t)u * step, itu = it + u;
            const uint32_t idu = gu + lane * 16;
            const bool check = itu < nsteps && ((itu % SS_CHECK) == SS_CHECK - 1 || itu == nsteps - 1);   // block-uniform
            uint32_t hm[B];
#pragma unroll
            for (int b = 0; b < B; ++b) hm[b] = 0;
            if (gu < end && gu >= begin) hits(gu, w[u], ci[u], hm);
            if (MASK) {
                // the 16 hit bits of this lane's positions, first position in bit 0
                if (itu < nsteps) {
#pragma unroll
                    for (int b = 0; b < B; ++b)
                        if (qbase + b < Q)
                            masks[(size_t)(qbase + b) * mask_stride + (gu >> 4) + lane] = (uint16_t)(__builtin_bitreverse32(hm[b]) >> 16);
                }
                continue;
            }
            if (PAIR && u % 2 == 0) {
#pragma unroll
                for (int b = 0; b < B; ++b) held[b] = hm[b] << 16;
                id_held = idu;
                if (check) compact(held, id_held, id_held);   // the last step of the range (leaves held zero)
            } else if (PAIR) {
#pragma unroll
                for (int b = 0; b < B; ++b) held[b] |= hm[b];
                compact(held, id_held, idu);
            } else {
                compact(hm, idu, idu);
            }
            if (check) flush_check(itu == nsteps - 1);
        }
    }
}

// masks == nullptr: the queries' lists cand_ids [Q][cap] (item ids); else one hit bit per scan position
// and query, mask_stride 16-bit words per query, for the positions below scan_end (whole block steps).
template <int KF, int B, bool NT, bool G2, bool MASK>
int launch_stream_as(const icq_index *ix, const float *lut, int Q, const float *thr, uint32_t *cand_ids,
                     uint32_t *cand_count, int64_t cap, uint16_t *masks, size_t mask_stride, int64_t scan_end,
                     hipStream_t s) {
    const size_t tab = sizeof(float) * (KF * ICQ_LUT_W * ss_copies(KF, B) * B + (G2 ? 2 * ICQ_LUT_W * B : 0));
    const int threads = SS_THREADS;
    // ids one wavefront stages per query: 512 (32 KB per query) when the tables leave that much LDS
    uint32_t wave_cap = 512;
    while (tab + sizeof(uint32_t) * B * SS_WAVES * wave_cap > 163840 - 1024) wave_cap -= 8;   // 1024: the static arrays
    const size_t lds = MASK ? tab : tab + sizeof(uint32_t) * B * SS_WAVES * wave_cap;
    ICQ_HIP_TRY(icq_allow_lds(reinterpret_cast<const void *>(&scan_stream_kernel<KF, B, NT, G2, MASK>), 163840 - 1024));
    const int groups = (Q + B - 1) / B;
    const uint32_t step = (uint32_t)(threads / 64) * 1024u;
    const int64_t nitems = G2 ? ix->g2_npos : ix->N;          // scan positions that can hold an item
    const int64_t npos = MASK ? scan_end : nitems;            // positions to walk
    // one wave of equally loaded blocks: the chip is filled once and every block streams a long run
    int64_t chunks = ((int64_t)ix->num_cu + groups - 1) / groups;
    int64_t max_chunks = (npos + step - 1) / step;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    uint32_t per = (uint32_t)(((npos + chunks - 1) / chunks + step - 1) / step * step);
    chunks = (npos + per - 1) / per;
    // query groups along grid.y, at most 65535 per launch
    for (int g0 = 0; g0 < groups; g0 += 65535) {
        const int ng = groups - g0 < 65535 ? groups - g0 : 65535;
        const int q0 = g0 * B, nq = (Q - q0) < ng * B ? (Q - q0) : ng * B;
        dim3 grid((unsigned)chunks, (unsigned)ng);
        scan_stream_kernel<KF, B, NT, G2, MASK><<<grid, threads, lds, s>>>(
            G2 ? ix->g2_rows : ix->fast, G2 ? ix->g2_npad : ix->Npad, (uint32_t)nitems,
            lut + (int64_t)q0 * ix->K * ICQ_LUT_W, ix->K, thr + q0, nq, MASK ? nullptr : cand_ids + (int64_t)q0 * cap,
            cand_count + q0, cap, per, wave_cap, G2 ? ix->g2_info : nullptr, G2 ? ix->perm : nullptr,
            MASK ? masks + (size_t)q0 * mask_stride : nullptr, mask_stride, (uint32_t)scan_end);
    }
    return icq_check_launch();
}

// One or two queries per pass over a code array that cannot stay in the 256 MB last-level cache:
// the memory-bound case, where the non-temporal stream pays.  (Four queries per pass are bound by
// the table lookups, and a smaller array is re-read from the cache by the next pass or call.)
template <int KF, int B, bool G2>
int launch_stream(const icq_index *ix, const float *lut, int Q, const float *thr, uint32_t *cand_ids,
                  uint32_t *cand_count, int64_t cap, uint16_t *masks, size_t mask_stride, int64_t scan_end,
                  hipStream_t s) {
    constexpr int64_t NT_BYTES = 256ll << 20;
    const int64_t bytes = G2 ? (int64_t)KF * ix->g2_npad : (int64_t)KF * ix->Npad;
    const bool nt = B <= 2 && bytes > NT_BYTES;
    if (masks) {
        if (nt) return launch_stream_as<KF, B, (B <= 2), G2, true>(ix, lut, Q, thr, cand_ids, cand_count, cap, masks, mask_stride, scan_end, s);
        return launch_stream_as<KF, B, false, G2, true>(ix, lut, Q, thr, cand_ids, cand_count, cap, masks, mask_stride, scan_end, s);
    }
    if (nt) return launch_stream_as<KF, B, (B <= 2), G2, false>(ix, lut, Q, thr, cand_ids, cand_count, cap, masks, mask_stride, scan_end, s);
    return launch_stream_as<KF, B, false, G2, false>(ix, lut, Q, thr, cand_ids, cand_count, cap, masks, mask_stride, scan_end, s);
}

// Item-by-item stage 1 for Kf <= 4: one pass over the fast sub-codes per group of B queries, B = 1 or 2
// for one or two queries, else 4.  An index that also keeps the items grouped by their first two
// fast sub-codes streams only the remaining Kf - 2 rows.
int launch_stream_any(const icq_index *ix, const float *lut, int Q, const float *thr, uint32_t *cand_ids,
                      uint32_t *cand_count, int64_t cap, uint16_t *masks, size_t mask_stride, int64_t scan_end,
                      hipStream_t s) {
    const int bsel = Q >= 3 ? 2 : Q >= 2 ? 1 : 0;
#define ICQ_SS(KF, B, G2) launch_stream<KF, B, G2>(ix, lut, Q, thr, cand_ids, cand_count, cap, masks, mask_stride, scan_end, s)
    if (icq_g2_usable(ix)) {
        switch ((ix->Kf - 2) * 3 + bsel) {
            case 3: return ICQ_SS(1, 1, true);
            case 4: return ICQ_SS(1, 2, true);
            case 5: return ICQ_SS(1, 4, true);
            case 6: return ICQ_SS(2, 1, true);
            case 7: return ICQ_SS(2, 2, true);
            default: return ICQ_SS(2, 4, true);
        }
    }
    switch (ix->Kf * 3 + bsel) {
        case 3: return ICQ_SS(1, 1, false);
        case 4: return ICQ_SS(1, 2, false);
        case 5: return ICQ_SS(1, 4, false);
        case 6: return ICQ_SS(2, 1, false);
        case 7: return ICQ_SS(2, 2, false);
        case 8: return ICQ_SS(2, 4, false);
        case 9: return ICQ_SS(3, 1, false);
        case 10: return ICQ_SS(3, 2, false);
        case 11: return ICQ_SS(3, 4, false);
        case 12: return ICQ_SS(4, 1, false);
        case 13: return ICQ_SS(4, 2, false);
        default: return ICQ_SS(4, 4, false);
    }
#undef ICQ_SS
}

// ------------------------------------------------------------------ lanes = items
constexpr int SI_THREADS = 256;

// Block (x = query group of up to `nb` queries, y = item chunk).  LDS holds
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
    const int qbase = blockIdx.x * nb;
    const int nq = (Q - qbase) < nb ? (Q - qbase) : nb;

    for (int i = tid; i < nq * Kf * ICQ_LUT_W; i += SI_THREADS) {
        int b = i / (Kf * ICQ_LUT_W), r = i % (Kf * ICQ_LUT_W);
        smem[i] = lut[((int64_t)(qbase + b) * K) * ICQ_LUT_W + r];
    }
    __syncthreads();

    const uint32_t begin = blockIdx.y * items_per_block;
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
                            if (cand_part) cand_part[row + slot] = P;
                        }
                    }
                }
            }
        }
    }
}

}  // namespace

int icq_launch_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                    uint32_t *cand_ids, float *cand_part, unsigned long long *cand_keys, int *list_kind, uint32_t *cand_count, int64_t cap,
                    int topk, uint32_t *out_ids, float *out_dist, hipEvent_t after_fill, hipStream_t s) {
    if (list_kind) *list_kind = ICQ_LIST_IDS;
    if (Q == 0) return ICQ_OK;
    zero_counts_kernel<<<(Q + 255) / 256, 256, 0, s>>>(cand_count, Q);
    if (after_fill) ICQ_HIP_TRY(hipEventRecord(after_fill, s));
    if (ix->N == 0) return icq_check_launch();

    const int bpq_fill = (int)((cap + 255) / 256 < 32 ? (cap + 255) / 256 : 32);
    if (icq_group_usable(ix, Q) && list_kind && !cand_part && ix->item_stride <= 16 &&
        (cand_keys || (out_ids && icq_group_fused(ix, Q, topk)))) {
        // the caller only wants the final lists: finish the distances (and, where one block
        // owns a query, the lists) right here
        *list_kind = out_ids && icq_group_fused(ix, Q, topk) ? ICQ_LIST_DONE : ICQ_LIST_KEYS;
        return icq_launch_group_keys(ix, lut, Q, thr, cand_keys, cand_count, cap, topk, out_ids, out_dist, s);
    }
    if (icq_group_usable(ix, Q)) {
        // positions only when the caller can take them and needs no crude distances
        const bool as_positions = list_kind != nullptr && cand_part == nullptr;
        int rc = icq_launch_group_scan(ix, lut, Q, thr, cand_ids, as_positions, cand_count, cap, s);
        if (rc != ICQ_OK) return rc;
        if (as_positions) *list_kind = ICQ_LIST_POSITIONS;
        if (!cand_part) return ICQ_OK;
        fill_partials_kernel<<<(unsigned)Q * (unsigned)bpq_fill, 256, 0, s>>>(
            ix->fast, ix->Npad, lut, ix->K, ix->Kf, cand_ids, cand_count, cap, bpq_fill, cand_part);
        return icq_check_launch();
    }

    if (ix->Kf <= 4) {
        // lanes = items, one pass over the fast sub-codes per group of B queries: B = 1 or 2 for one or
        // two queries, B = 4 for every larger call that has neither grouping nor transposed tables
        const int rc = launch_stream_any(ix, lut, Q, thr, cand_ids, cand_count, cap, nullptr, 0, 0, s);
        if (rc != ICQ_OK || !cand_part) return rc;
        const int bpq = (int)((cap + 255) / 256 < 256 ? (cap + 255) / 256 : 256);
        fill_partials_kernel<<<(unsigned)Q * (unsigned)bpq, 256, 0, s>>>(
            ix->fast, ix->Npad, lut, ix->K, ix->Kf, cand_ids, cand_count, cap, bpq, cand_part);
        return icq_check_launch();
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
    dim3 grid((unsigned)groups, (unsigned)chunks);
#define ICQ_SI_LAUNCH(KFM)                                                                          \
    do {                                                                                            \
        ICQ_HIP_TRY(icq_allow_lds(reinterpret_cast<const void *>(&scan_items_kernel<KFM>), 65536)); \
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

// *superset: the bits written mark a superset of the survivors (the 16-bit pre-filter); stage 2 then
// applies the exact comparison itself.
int icq_launch_scan_masks(const icq_index *ix, const float *lut, int Q, const float *thr, uint16_t *masks,
                          size_t mask_stride, int64_t scan_end, uint32_t *cand_count, uint32_t *key_count,
                          hipEvent_t after_fill, bool *superset, hipStream_t s) {
    *superset = false;
    if (Q == 0) return ICQ_OK;
    zero_counts_kernel<<<(Q + 255) / 256, 256, 0, s>>>(cand_count, Q);
    zero_counts_kernel<<<(Q + 255) / 256, 256, 0, s>>>(key_count, Q);
    if (after_fill) ICQ_HIP_TRY(hipEventRecord(after_fill, s));
    if (icq_scan_q16_usable(ix, Q)) {
        *superset = true;
        return icq_launch_scan_masks_q16(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
    }
    return launch_stream_any(ix, lut, Q, thr, nullptr, cand_count, 0, masks, mask_stride, scan_end, s);
}

ICQ_EXPORT int icq_scan_fast(const icq_index *ix, const float *lut, int Q, const float *thresholds,
                             uint32_t *cand_ids, float *cand_part, uint32_t *cand_count,
                             int64_t cap, void *workspace, size_t workspace_bytes, void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || cap < 1) return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if (!lut || !thresholds || !cand_ids || !cand_count) return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    icq_ws_layout L = icq_layout(ix, Q, cap, 1, false, false);
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < L.total)
        return ICQ_ERR_WORKSPACE;
    // stage timing: [0] entry .. [1] after the counter fill .. [2] after the scan (.. [3] = [2])
    icq_stage_timer *tm = ix->timer;
    hipEvent_t *ev = nullptr;
    hipStream_t s = (hipStream_t)stream;
    if (tm) {
        if (tm->batches < 1) tm->batches = 1;
        ev = tm->ev[tm->calls % ICQ_TIMED_CALLS];
        ICQ_HIP_TRY(hipEventRecord(ev[0], s));
    }
    const int rc = icq_launch_scan(ix, lut, Q, thresholds, cand_ids, cand_part, nullptr, nullptr, cand_count, cap,
                                   0, nullptr, nullptr, ev ? ev[1] : nullptr, s);
    if (rc != ICQ_OK) return rc;
    if (ev) {
        ICQ_HIP_TRY(hipEventRecord(ev[2], s));
        ICQ_HIP_TRY(hipEventRecord(ev[3], s));
        tm->calls += 1;           // counted once all four events of the call are recorded
    }
    return ICQ_OK;
}
