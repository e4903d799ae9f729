// Stage 1 of the two-step search (arxiv 1912.08756, Eq. 2) as a conservative pre-filter in 16-bit
// integers, for icq_search when it keeps hit bits: over the index ordered by the first two fast
// sub-codes (G2: the pair's part of the sum once per 16 positions, Kf - 2 rows streamed) or over the
// items in id order (all Kf rows streamed).
//
// The crude comparison P = sum_{k<Kf} T_k[code_k] < t is decided exactly where the item's record
// is in hand anyway -- by the kernel that forms the exact distance, from the same fp32 additions.
// What this kernel leaves is a SUPERSET of the survivors, found with a quarter of the work per
// (query, position): every fast table is replaced by
//     q_k[c] = min(8000, max(0, floor((T_k[c] - min T_k) / s) - 1))   (16-bit, never above the true quotient)
// with one scale s per query chosen so that the threshold falls at 7500 units, and an item passes
// when  q_0 + q_1 + q_2 (+ q_3) <= floor((t - sum_k min T_k) / s) + 1.  Rounding down every term
// and up the right side cannot lose a survivor (the slack of one unit per term also covers the
// rounding of the fp32 sum the exact test uses, which s >= |t| * 2^-18 keeps below a sixteenth of a
// unit); what it lets through beyond the survivors are items within a few units -- a few
// ten-thousandths of the threshold's distance from the tables' minimum -- of the threshold.
// Eight queries' 16-bit entries make one 16-byte LDS read, and two queries share every 32-bit
// instruction: entries stop at 8000 units and the first table carries 32768 - (threshold units + 1),
// so a sum of up to four entries stays inside its 16 bits -- the two halves of a word are added by
// ONE plain 32-bit addition with no carry between them -- and bit 15 of a half is clear exactly when
// the sum is at or below the threshold's units (an entry stopped at 8000 units is beyond the threshold
// by itself).  The miss bits of two positions are collected by one byte permute, one shift and one
// bit-field insert.  The byte extraction and table address of a position serve eight queries.
#include "icq_internal.h"
#include "icq_sort.h"

#include <math.h>

namespace {


typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int QS_THREADS = 1024;
constexpr int QS_WAVES = QS_THREADS / 64;
constexpr int QS_B = 8;                  // queries per pass
// copies of a streamed table's entry (lane l reads copy l % C): 16 while the tables fit, else 8 -- two
// lanes of a 16-lane group then share a copy and collide when their sub-codes have the same parity
constexpr int qs_copies(int KF) { return KF <= 2 ? 16 : 8; }
// positions whose table reads are issued together: 8 with one or two streamed rows (4: 3 % slower; 16 spills),
// fewer with more rows -- the reads of a phase are 16 bytes per row and position, all held in registers
constexpr int qs_half(int KF) { return KF <= 2 ? 8 : KF == 3 ? 4 : 2; }   // even: positions come in pairs (j, j + 8)
constexpr float QS_UNITS = 7500.0f;      // where the threshold falls on the 16-bit scale
constexpr float QS_CAP = 8000.0f;        // entries stop here (above the threshold): bias + four entries < 65536
constexpr int QS_BIAS = 32768;           // the first table carries QS_BIAS - (threshold units + 1): bit 15 clear = passes
static_assert(QS_UNITS + 1.0f < QS_CAP && QS_BIAS + 1 + 4 * (int)QS_CAP < 65536, "sums stay inside 16 bits");

__device__ __forceinline__ uint32_t lane_id() {
    return __builtin_amdgcn_mbcnt_hi(~0u, __builtin_amdgcn_mbcnt_lo(~0u, 0u));
}
// never above the true quotient (x - base) / s: floor, minus one unit for the rounding of the product
__device__ __forceinline__ int quantise(float x, float base, float inv_s) {
    const float v = floorf((x - base) * inv_s) - 1.0f;
    return (int)fminf(fmaxf(v, 0.0f), QS_CAP);            // a NaN (inf * 0) ends as 0
}

// KF streamed rows: Kf - 2 (G2: `rows` = the grouped rows, `info` the pairs' labels) or Kf (`rows` =
// the fast rows in id order).  Grid: x = ranges of scan positions, y = groups of eight queries.
// masks (rows for ceil(Q / 8) * 8 queries) [q * mask_stride + p / 16] receives the hit bits of positions p .. p + 15 (bit j = position
// p + j) for every position of the block's range below scan_end, zeros beyond the last item.
template <int KF, bool G2>
__global__ __launch_bounds__(QS_THREADS) void scan_pairs_q16_kernel(
    const uint8_t *rows, int64_t npad, uint32_t N, const float *__restrict__ lut, int K, const float *__restrict__ thr,
    int Q, uint32_t items_per_block, const uint32_t *__restrict__ info, uint16_t *__restrict__ masks, size_t mask_stride,
    uint32_t scan_end) {
    // The streamed tables sit at LDS address 0 (no static arrays in this kernel; the launcher checks that the
    // kernel's static LDS size is zero): the table addresses the inner loop assembles from bytes are then the
    // LDS addresses themselves, and the reads take them as such -- nothing to add, not even a zero.
    extern __shared__ __attribute__((aligned(16))) uint4 qs_smem[];
    constexpr int QS_C = qs_copies(KF);
    constexpr int QS_HALF = qs_half(KF);
    constexpr int KFAST = G2 ? KF + 2 : KF;                 // fast codebooks
    constexpr int K0 = G2 ? 2 : 0;                          // codebook of the first streamed row
    uint4 *tab = qs_smem;                                   // [KF][256][QS_C]
    uint4 *t01 = qs_smem + KF * ICQ_LUT_W * QS_C;           // G2: [2][256]
    float (*s_min)[QS_B] = reinterpret_cast<float (*)[QS_B]>(t01 + (G2 ? 2 * ICQ_LUT_W : 0));     // [KFAST][QS_B]
    float *s_inv = &s_min[KFAST][0];                        // [QS_B]
    int *s_thr = reinterpret_cast<int *>(s_inv + QS_B);     // [QS_B]
    const int tid = threadIdx.x;
    const uint32_t lane = lane_id();
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int qbase = blockIdx.y * QS_B;

    const uint32_t begin = blockIdx.x * items_per_block;
    uint32_t end = begin + items_per_block;
    if (end > N || end < begin) end = N;
    uint32_t walk_end = begin + items_per_block;
    if (walk_end > scan_end || walk_end < begin) walk_end = scan_end;
    constexpr uint32_t step = (uint32_t)QS_WAVES * 1024u;
    const uint32_t nsteps = walk_end > begin ? (walk_end - begin + step - 1) / step : 0;

    uint4 w[2][KF];
    uint32_t ci[2];
    // 1024 positions at g; past the block's range the block's first positions are read instead
    // (unused, in bounds: the rows are padded by more than a block step)
    auto load = [&](uint32_t g, uint4 (&w)[KF], uint32_t &ci) {
        const uint32_t gs = (g < end && g >= begin) ? g : begin;
        ci = G2 ? info[(gs >> 4) + lane] : 0u;
#pragma unroll
        for (int k = 0; k < KF; ++k) w[k] = *reinterpret_cast<const uint4 *>(rows + (int64_t)k * npad + gs + lane * 16);
    };
    uint32_t g = begin + wave * 1024u;
    load(g, w[0], ci[0]);                                   // in flight while the tables are prepared

    auto row_of = [&](int b, int k) -> const float * {
        const int qb = qbase + b < Q ? qbase + b : Q - 1;   // a slot past the last query: clamped, and never stored
        return lut + ((int64_t)qb * K + k) * ICQ_LUT_W;
    };
    // smallest entry of every fast table of every query: 8 * Kf combinations over 16 wavefronts
    for (int combo = wave; combo < QS_B * KFAST; combo += QS_WAVES) {
        const int b = combo % QS_B, k = combo / QS_B;
        const float *r = row_of(b, k);
        float m = fminf(fminf(r[lane], r[lane + 64]), fminf(r[lane + 128], r[lane + 192]));
        m = wave_min_f32(m);
        if (lane == 0) s_min[k][b] = m;
    }
    __syncthreads();
    if (tid < QS_B) {
        const float t = qbase + tid < Q ? thr[qbase + tid] : -INFINITY;
        float L = s_min[0][tid];                            // the order of the additions of Eq. 2
#pragma unroll
        for (int k = 1; k < KFAST; ++k) L += s_min[k][tid];
        float inv = 0.0f;
        int units = -2;                                     // nothing can pass: t <= L, t = -inf or NaN
        if (t == INFINITY) {
            units = (int)QS_UNITS;                          // everything passes (all quotients are 0)
        } else if (t > L) {
            const float s = fmaxf(fmaxf((t - L) / QS_UNITS, fabsf(t) * 3.814697265625e-6f), 1e-30f);
            inv = 1.0f / s;
            units = (int)fminf(floorf((t - L) * inv) + 1.0f, QS_UNITS);
        }
        s_inv[tid] = inv;
        s_thr[tid] = units;
    }
    __syncthreads();
    // the streamed tables, 16 copies of every entry, eight queries' values side by side; consecutive
    // threads write consecutive 16-byte pieces
    auto entry = [&](int k, int c, bool first) -> uint4 {
        uint32_t h[QS_B];
#pragma unroll
        for (int b = 0; b < QS_B; ++b) {
            int v = quantise(row_of(b, k)[c], s_min[k][b], s_inv[b]);
            if (first) v += QS_BIAS - (s_thr[b] + 1);       // the threshold rides on the first table: a sum below 32768 passes
            h[b] = (uint32_t)v & 0xFFFFu;
        }
        return make_uint4(h[0] | (h[1] << 16), h[2] | (h[3] << 16), h[4] | (h[5] << 16), h[6] | (h[7] << 16));
    };
#pragma unroll
    for (int j = 0; j < KF * ICQ_LUT_W * QS_C / QS_THREADS; ++j) {
        const int p = j * QS_THREADS + tid, e = p / QS_C;
        const int k = K0 + e / ICQ_LUT_W;
        tab[p] = entry(k, e % ICQ_LUT_W, k == 0);
    }
    if (G2 && tid < 2 * ICQ_LUT_W) t01[tid] = entry(tid / ICQ_LUT_W, tid % ICQ_LUT_W, tid < ICQ_LUT_W);
    __syncthreads();

    // 16 copies: a table address is assembled from bytes by one instruction: byte 0 = this lane's copy
    // (times 16), byte 1 = the sub-code (an entry is 16 copies of 16 bytes), byte 2 = the streamed table.
    // 8 copies (entries of 128 bytes): sub-code * 128 + (copy * 16 + table * 32768), the bracket per lane.
    const uint32_t lane_bytes = (lane & (QS_C - 1)) * 16u | 0x100u;      // byte 1 = 1: the source of "table 1"
    uint32_t lane_off[KF];
#pragma unroll
    for (int k = 0; k < KF; ++k) lane_off[k] = (lane & (QS_C - 1)) * 16u + (uint32_t)k * (ICQ_LUT_W * QS_C * 16);
    // hit bits of the 1024 positions at g: hm[d] = queries 2d (low half) and 2d + 1, position j in bit j
    auto hits = [&](uint32_t g, const uint4 (&w)[KF], uint32_t ci, uint32_t (&hm)[QS_B / 2]) {
        uint32_t p01[QS_B / 2];
        bool live[QS_B / 2], any_live = !G2;
#pragma unroll
        for (int d = 0; d < QS_B / 2; ++d) {
            p01[d] = 0;
            live[d] = true;
        }
        if (G2) {
            const uint4 a = t01[ci & 0xffu], c = t01[ICQ_LUT_W + ((ci >> 8) & 0xffu)];
            p01[0] = a.x + c.x;
            p01[1] = a.y + c.y;
            p01[2] = a.z + c.z;
            p01[3] = a.w + c.w;
            // the streamed tables add at least 0: a pair of queries whose two sums have reached 32768 in every
            // lane has no hit among the wavefront's 1024 positions
#pragma unroll
            for (int d = 0; d < QS_B / 2; ++d) {
                live[d] = __builtin_amdgcn_ballot_w64((~p01[d] & 0x80008000u) != 0u) != 0;  // wavefront-uniform
                any_live |= live[d];
            }
        }
        if (!any_live) return;
        // MISS bits, positions j and j + 8 together: one byte permute brings the top bytes of their two sums (two
        // queries each) side by side -- low query: bytes 0 (j) and 1 (j + 8), high query: bytes 2 and 3 -- and every
        // such step shifts the collecting word right and takes bit 7 of each byte from them (a bit-field insert:
        // what the shift moved into those bits from the byte above is replaced).  After the eight steps j = 0 .. 7
        // position p sits in bit p (and 16 + p).  A pair of queries that is skipped keeps all ones.
        uint32_t acc[QS_B / 2];
#pragma unroll
        for (int d = 0; d < QS_B / 2; ++d) acc[d] = 0xFFFFFFFFu;
        uint32_t top_bits;                                   // in a register: an instruction with a literal issues slower
        asm volatile("v_mov_b32 %0, 0x80808080" : "=v"(top_bits));
#pragma unroll
        for (int h = 0; h < 16; h += QS_HALF) {
            // the phase's positions: j = h / 2 .. h / 2 + QS_HALF / 2 - 1 (even jj) and their partners j + 8 (odd jj)
            uint32_t off[QS_HALF][KF];
#pragma unroll
            for (int jj = 0; jj < QS_HALF; ++jj) {
                const int j = h / 2 + (jj >> 1) + 8 * (jj & 1);
#pragma unroll
                for (int k = 0; k < KF; ++k) {
                    const uint32_t word = j < 4 ? w[k].x : j < 8 ? w[k].y : j < 12 ? w[k].z : w[k].w;
                    if (QS_C == 16) {
                        // selector bytes: 0 = lane_bytes byte 0, 4 + n = byte n of the code word, 1 = lane_bytes byte 1, 0x0c = zero
                        const uint32_t sel = 0x0c000000u | (k == 0 ? 0x000c0000u : 0x00010000u) | ((4u + (j & 3)) << 8);
                        off[jj][k] = __builtin_amdgcn_perm(word, lane_bytes, sel);
                    } else {
                        uint32_t code;
                        if ((j & 3) == 0) asm("v_bfe_u32 %0, %1, 0, 8" : "=v"(code) : "v"(word));
                        else code = (word >> (8 * (j & 3))) & 0xffu;
                        off[jj][k] = (code << 7) + lane_off[k];
                    }
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            uint4 v[QS_HALF][KF];
#pragma unroll
            for (int jj = 0; jj < QS_HALF; ++jj)
#pragma unroll
                for (int k = 0; k < KF; ++k)
                {
                    const u32x4 e = *(const __attribute__((address_space(3))) u32x4 *)(uintptr_t)off[jj][k];   // LDS address = table offset
                    v[jj][k] = make_uint4(e.x, e.y, e.z, e.w);
                }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int d = 0; d < QS_B / 2; ++d) {
                if (!live[d]) continue;                      // wavefront-uniform
#pragma unroll
                for (int jj = 0; jj < QS_HALF; jj += 2) {
                    uint32_t x[2];
#pragma unroll
                    for (int u = 0; u < 2; ++u) {
                        x[u] = p01[d];
#pragma unroll
                        for (int k = 0; k < KF; ++k) {
                            const uint4 &t = v[jj + u][k];
                            const uint32_t e = d == 0 ? t.x : d == 1 ? t.y : d == 2 ? t.z : t.w;
                            x[u] = (!G2 && k == 0) ? e : x[u] + e;       // id order: the first table carries the threshold
                        }
                    }
                    // bytes 1 and 3 of both sums: x[0] (position j) to bytes 0 and 2, x[1] (position j + 8) to bytes 1 and 3
                    const uint32_t tops = __builtin_amdgcn_perm(x[1], x[0], 0x07030501u);
                    // two instructions per step (left to itself the compiler regroups the chain into more)
                    asm("v_lshrrev_b32 %0, 1, %0\n\tv_bfi_b32 %0, %2, %1, %0" : "+v"(acc[d]) : "v"(tops), "v"(top_bits));
                }
            }
        }
        // the padding behind a pair's last item, and positions at or beyond the end
        uint32_t valid = G2 ? (1u << (ci >> 16)) - 1u : 0xFFFFu;      // the label's count is at most 16
        const uint32_t id0 = g + lane * 16;
        if (id0 + 16 > end || id0 + 16 < id0) valid &= id0 < end ? (1u << (end - id0)) - 1u : 0u;
        valid |= valid << 16;
#pragma unroll
        for (int d = 0; d < QS_B / 2; ++d) hm[d] = ~acc[d] & valid;
    };

    for (uint32_t it = 0; it < nsteps; it += 2, g += 2 * step) {
#pragma unroll
        for (int u = 0; u < 2; ++u) {
            load(g + (uint32_t)(u + 1) * step, w[(u + 1) % 2], ci[(u + 1) % 2]);        // never conditional
            const uint32_t gu = g + (uint32_t)u * step;
            uint32_t hm[QS_B / 2];
#pragma unroll
            for (int d = 0; d < QS_B / 2; ++d) hm[d] = 0;
            if (gu < end && gu >= begin) hits(gu, w[u], ci[u], hm);
            if (it + u < nsteps) {
#pragma unroll
                for (int d = 0; d < QS_B / 2; ++d) {
                    // the wavefront's row piece (uniform), lane l's word behind it.  Slots past the last query have
                    // rows too (the caller sizes the bits for whole groups of eight) and get zeros: no conditions.
                    uint16_t *row = masks + (size_t)(qbase + 2 * d) * mask_stride + (gu >> 4);
                    // written once, read once by stage 2: kept out of the caches the code rows are re-read from
                    __builtin_nontemporal_store((uint16_t)hm[d], row + lane);
                    __builtin_nontemporal_store((uint16_t)(hm[d] >> 16), row + mask_stride + lane);
                }
            }
        }
    }
}

template <int KF, bool G2>
int launch_q16(const icq_index *ix, const float *lut, int Q, const float *thr, uint16_t *masks, size_t mask_stride,
               int64_t scan_end, hipStream_t s) {
    const size_t lds = sizeof(uint4) * (size_t)(KF * ICQ_LUT_W * qs_copies(KF) + (G2 ? 2 * ICQ_LUT_W : 0)) +
                       sizeof(float) * ((G2 ? KF + 2 : KF) + 2) * QS_B;
    // the kernel reads its tables at absolute LDS addresses: its dynamic LDS must start at 0 (no static LDS)
    ICQ_HIP_TRY(icq_allow_lds(reinterpret_cast<const void *>(&scan_pairs_q16_kernel<KF, G2>), lds, true));
    const int groups = (Q + QS_B - 1) / QS_B;
    const uint32_t step = (uint32_t)QS_WAVES * 1024u;
    // one wave of equally loaded blocks: the chip is filled once and every block streams a long run
    int64_t chunks = ((int64_t)ix->num_cu + groups - 1) / groups;
    const int64_t max_chunks = (scan_end + step - 1) / step;
    if (chunks > max_chunks) chunks = max_chunks;
    if (chunks < 1) chunks = 1;
    const uint32_t per = (uint32_t)(((scan_end + chunks - 1) / chunks + step - 1) / step * step);
    chunks = (scan_end + per - 1) / per;
    for (int g0 = 0; g0 < groups; g0 += 65535) {
        const int ng = groups - g0 < 65535 ? groups - g0 : 65535;
        const int q0 = g0 * QS_B, nq = (Q - q0) < ng * QS_B ? (Q - q0) : ng * QS_B;
        dim3 grid((unsigned)chunks, (unsigned)ng);
        scan_pairs_q16_kernel<KF, G2><<<grid, QS_THREADS, lds, s>>>(
            G2 ? ix->g2_rows : ix->fast, G2 ? ix->g2_npad : ix->Npad, (uint32_t)(G2 ? ix->g2_npos : ix->N),
            lut + (int64_t)q0 * ix->K * ICQ_LUT_W, ix->K, thr + q0, nq, per, G2 ? ix->g2_info : nullptr,
            masks + (size_t)q0 * mask_stride, mask_stride, (uint32_t)scan_end);
    }
    return icq_check_launch();
}

}  // namespace

// Calls with at least this many queries take the 16-bit pre-filter (below, a pass of eight would be mostly empty
// slots); Kf <= 4 (the caller keeps hit bits only then).
bool icq_scan_q16_usable(const icq_index *ix, int Q) { return ix->Kf <= 4 && Q >= 6; }

// Hit bits of a superset of the survivors; the caller's stage 2 applies the exact comparison.
int icq_launch_scan_masks_q16(const icq_index *ix, const float *lut, int Q, const float *thr, uint16_t *masks,
                              size_t mask_stride, int64_t scan_end, hipStream_t s) {
    if (icq_g2_usable(ix)) {
        if (ix->Kf == 3) return launch_q16<1, true>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
        return launch_q16<2, true>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
    }
    switch (ix->Kf) {
        case 1: return launch_q16<1, false>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
        case 2: return launch_q16<2, false>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
        case 3: return launch_q16<3, false>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
        default: return launch_q16<4, false>(ix, lut, Q, thr, masks, mask_stride, scan_end, s);
    }
}
