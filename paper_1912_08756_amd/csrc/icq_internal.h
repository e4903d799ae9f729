// Internal declarations shared by the HIP translation units of libicq.
// Not installed; the public contract is include/icq.h.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "icq.h"

#define ICQ_EXPORT extern "C" __attribute__((visibility("default")))
#define ICQ_LUT_W 256          // table row width (entries j >= m hold +inf)
#define ICQ_WAVE 64            // gfx950 wavefront
#define ICQ_ALIGN 256          // workspace sub-buffer alignment

// Events around the stages of the latest icq_search (icq_index_set_stage_timing).
struct icq_stage_timer {
    hipEvent_t ev[ICQ_TIMED_CALLS][4];
    long long calls;           // searches recorded since the last read (slot = call % ICQ_TIMED_CALLS)
    int batches;               // most sub-batches among them
};

struct icq_index {
    int K, m, d, Kf, Ks;       // Ks = K - Kf slow codebooks
    int d_pad;                 // d rounded up to a multiple of 16 (zero filled)
    int item_stride;           // bytes per item record in `items`
    int device;
    int num_cu;
    int64_t N, Npad;           // Npad: N rounded up to a multiple of 4096
    float *cb;                 // [K*256][d_pad] codewords, rows j >= m are zero
    float *cnorm;              // [K*256] squared codeword norms, +inf for j >= m
    uint8_t *fast;             // [Kf][Npad] fast sub-codes, zero padded
    uint8_t *items;            // [N][item_stride] all K sub-codes of an item, item-major
    // Grouping by fast-code tuple (Kf <= 2): items with the same fast sub-codes share their
    // crude distance, so batch-mode stage 1 evaluates each tuple once.
    int groups;                // 256^Kf, or 0 when the index is not grouped
    int scan_mode;             // ICQ_SCAN_AUTO / ICQ_SCAN_STREAMED / ICQ_SCAN_GROUPED
    uint32_t *group_start;     // [groups + 1] first grouped position of each tuple
    uint32_t *group_cursor;    // [groups] scratch of the build
    uint32_t *perm;            // [N] grouped position -> item id
    uint8_t *items_grouped;    // [N][item_stride] the item records in grouped order
    // Grouping by the first two fast sub-codes (Kf = 3, 4 and N large enough, icq_group2.hip): the
    // items ordered by that pair -- the pairs themselves in a scattered order, so that any stretch of
    // positions holds unrelated pairs -- every pair's run padded to whole 16 positions.  Stage 1 then
    // streams only the remaining Kf - 2 fast rows and forms the pair's table sum once per 16
    // positions.  Uses group_start [65537], perm [g2_npad] (ICQ_PAD_ID in the padding) and
    // items_grouped [g2_npad][item_stride] as the Kf <= 2 grouping does.
    int g2;                    // 1 when this grouping exists
    int64_t g2_npos;           // positions stage 1 walks: an upper bound of the padded total, whole block steps
    int64_t g2_npad;           // row stride of g2_rows = length of perm / items_grouped (g2_npos + read-ahead spare)
    uint8_t *g2_rows;          // [Kf - 2][g2_npad] the remaining fast sub-codes in grouped order
    uint32_t *g2_info;         // [g2_npad / 16] c0 | c1 << 8 | valid positions << 16 of each 16 positions
    icq_stage_timer *timer;    // nullptr unless stage timing is on
};

// Position of pair (c0, c1) in the grouped order and back: multiplication by an odd constant is a
// bijection on 16 bits that sends neighbouring pairs far apart.
#define ICQ_G2_MUL 0x9E37u
#define ICQ_G2_INV 0x7787u     // ICQ_G2_MUL * ICQ_G2_INV == 1 (mod 65536)
static inline __host__ __device__ uint32_t icq_g2_slot_of_pair(uint32_t pair) { return (pair * ICQ_G2_INV) & 0xFFFFu; }
static inline __host__ __device__ uint32_t icq_g2_pair_of_slot(uint32_t slot) { return (slot * ICQ_G2_MUL) & 0xFFFFu; }
// automatic: when a pair's run averages 64 items or more, so that the padding to 16 weighs little
static inline bool icq_g2_usable(const icq_index *ix) {
    if (!ix->g2 || ix->scan_mode == ICQ_SCAN_STREAMED) return false;
    return ix->scan_mode == ICQ_SCAN_GROUPED || ix->N >= 64ll * 65536;
}
int icq_group2_build(icq_index *ix, hipStream_t s);
int icq_group2_export(const icq_index *ix, uint8_t *codes_out, hipStream_t s);

// hipFuncSetAttribute(fn, MaxDynamicSharedMemorySize, bytes), once per (device, kernel); thread-safe.
// no_static_lds: also refuse (hipErrorInvalidValue) a kernel whose code object holds static LDS.
hipError_t icq_allow_lds(const void *fn, int bytes, bool no_static_lds = false);

// What a candidate list holds.
enum icq_list_kind {
    ICQ_LIST_IDS = 0,          // item ids
    ICQ_LIST_POSITIONS = 1,    // grouped positions (ids through perm, records from items_grouped)
    ICQ_LIST_KEYS = 2,         // stage 1 already wrote one 64-bit key (bits of D, id) per survivor
    ICQ_LIST_DONE = 3          // stage 1 kept the nearest-neighbour lists itself and wrote the results
};

// hm = 2 * hm + (P < t): the comparison's carry shifted in with one add (the compiler's own
// form is a select and an or per item).  After n calls the first comparison sits in bit n - 1, the last in bit 0.
// (Tried: the sign of P - t funnel-shifted in -- v_sub_f32 + v_alignbit_b32 issue in 6.3 clocks per item
// against 10.2 for this pair in isolation -- and the table address as shift + v_and_or_b32; both exact,
// neither shortened the scans, which wait on the LDS and on each other's phases rather than on issue slots.)
__device__ __forceinline__ void icq_hit_shift_in(uint32_t &hm, float P, float t) {
    // the two wait states are the ones the compiler itself puts between a vector instruction that
    // writes VCC and one that reads it (it does not look inside an asm statement)
    // (t is wavefront-uniform where this is used and may stay in a scalar register: first source of the compare)
    asm("v_cmp_gt_f32 vcc, %2, %1\n\ts_nop 1\n\tv_addc_co_u32 %0, vcc, %0, %0, vcc" : "+v"(hm) : "v"(P), "s"(t) : "vcc");
}

// Order-preserving bits of a float: u(a) < u(b) <=> a < b.
__device__ __forceinline__ uint32_t icq_order_bits(float x) {
    // negative: all bits flipped; else the sign bit set -- as an arithmetic shift and one xor-or
    const uint32_t b = __float_as_uint(x);
    return b ^ ((uint32_t)((int32_t)b >> 31) | 0x80000000u);
}

// Sub-buffers carved out of the caller's workspace for one query batch.
struct icq_ws_layout {
    size_t lut_off, ids_off, count_off, keys_off, total;
    int splits;                // stage-2 blocks per query
    // icq_search with the item-by-item stage 1: hit bits instead of candidate lists (ids_off holds them)
    bool masked;
    size_t keycount_off;       // [Q] keys written per query
    size_t mask_stride;        // 16-bit words of hit bits per query
    int64_t scan_end;          // scan positions the hit bits cover (whole chunks)
};

static inline size_t icq_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Layout for `Q` queries processed together.  with_lut / with_cands select the
// parts a call needs (icq_scan_fast and icq_refine get their tables and lists
// from the caller).
icq_ws_layout icq_layout(const icq_index *ix, int Q, int64_t cap, int topk, bool with_lut,
                         bool with_cands);
int icq_refine_splits(const icq_index *ix, int Q, int64_t cap, int topk);
// icq_search with the item-by-item stage 1 hands the survivors to stage 2 as one hit bit per scan
// position and query instead of lists.
bool icq_masks_usable(const icq_index *ix, int Q, int topk);
int64_t icq_mask_scan_end(const icq_index *ix);              // positions the hit bits cover: whole stage-2 chunks
// Stage 1 into hit bits (zeroes cand_count and key_count first; after_fill as in icq_launch_scan).
// icq_search's body; lut_ext (device, [Q][K][256]) replaces the table build when not null.
int icq_search_impl(const icq_index *ix, const float *queries, const float *lut_ext, int Q, const float *thresholds,
                    int64_t cap, int topk, uint32_t *out_ids, float *out_dist, uint32_t *out_survivors,
                    void *workspace, size_t workspace_bytes, void *stream);
int icq_launch_scan_masks(const icq_index *ix, const float *lut, int Q, const float *thr, uint16_t *masks,
                          size_t mask_stride, int64_t scan_end, uint32_t *cand_count, uint32_t *key_count,
                          hipEvent_t after_fill, bool *superset, hipStream_t s);
// The 16-bit pre-filter over the pair ordering (icq_scan16.hip): hit bits of a superset of the survivors.
bool icq_scan_q16_usable(const icq_index *ix, int Q);
int icq_launch_scan_masks_q16(const icq_index *ix, const float *lut, int Q, const float *thr, uint16_t *masks,
                              size_t mask_stride, int64_t scan_end, hipStream_t s);
// Stage 2 from hit bits; keys [Q][cap] (+ slice lists in front, see icq_cand_keys); adds the survivors to cand_count.
// thr != nullptr: the bits mark a superset of the survivors, and an item counts only if its crude distance
// (the first Kf terms of the sum, the additions of Eq. 2) is below thr[q].
int icq_launch_refine_masks(const icq_index *ix, const float *lut, int Q, const uint16_t *masks, size_t mask_stride,
                            int64_t scan_end, int64_t cap, int topk, int splits, unsigned long long *keys,
                            uint32_t *key_count, uint32_t *cand_count, const float *thr, uint32_t *out_ids,
                            float *out_dist, hipStream_t s);

// Kernel launchers (each checks nothing; the extern "C" entry points validate).
int icq_launch_build_lut(const icq_index *ix, const float *queries, int Q, float *lut,
                         hipStream_t s);
// cand_part == nullptr: the crude distances are not materialised (the fused path
// recomputes the full sum in stage 2 from the item records).
// list_kind == nullptr: the list must hold item ids (public contract).  Otherwise the
// scan picks the cheapest representation for stage 2 and reports it: finished keys in
// cand_keys ([Q][cap], may be nullptr), grouped positions, or plain ids.
// topk / out_ids / out_dist (may be nullptr): where the scan may write the final lists
// itself (ICQ_LIST_DONE) when its grouped form covers stage 2 as well.
// after_fill (may be nullptr): event recorded once the survivor counters are zeroed.
int icq_launch_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                    uint32_t *cand_ids, float *cand_part, unsigned long long *cand_keys, int *list_kind,
                    uint32_t *cand_count, int64_t cap, int topk, uint32_t *out_ids, float *out_dist,
                    hipEvent_t after_fill, hipStream_t s);
// Grouped stage 1 fused with stage 2: the final lists when icq_group_fused() holds and
// out_ids is given, else one 64-bit key per survivor in cand_keys.
bool icq_group_fused(const icq_index *ix, int Q, int topk);
int icq_launch_group_keys(const icq_index *ix, const float *lut, int Q, const float *thr,
                          unsigned long long *cand_keys, uint32_t *cand_count, int64_t cap, int topk,
                          uint32_t *out_ids, float *out_dist, hipStream_t s);
// Where the per-candidate keys live inside the key area of the workspace.
static inline unsigned long long *icq_cand_keys(unsigned long long *keys, int Q, int splits, int topk) {
    return keys + (splits > 1 ? (size_t)Q * splits * topk : 0);
}
// Grouped stage 1 (icq_group.hip); as_positions: list grouped positions instead of ids.
bool icq_group_usable(const icq_index *ix, int Q);
int icq_group_fused_parts(const icq_index *ix, int Q);
int icq_launch_merge(const unsigned long long *keys, int Q, int splits, int topk, bool ascending,
                     uint32_t *out_ids, float *out_dist, hipStream_t s);
int icq_launch_group_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                          uint32_t *cand_ids, bool as_positions, uint32_t *cand_count, int64_t cap,
                          hipStream_t s);
int icq_group_build(icq_index *ix, hipStream_t s);
// cand_part == nullptr: D is the full K-term sum; else D = cand_part + slow terms.
// list_kind says what cand_ids holds, see icq_list_kind.
int icq_launch_refine(const icq_index *ix, const float *lut, int Q, const uint32_t *cand_ids,
                      const float *cand_part, int list_kind,
                      const uint32_t *cand_count, int64_t cap, int topk, int splits,
                      unsigned long long *keys, uint32_t *out_ids, float *out_dist, hipStream_t s);

#define ICQ_HIP_TRY(expr)                      \
    do {                                       \
        hipError_t e__ = (expr);               \
        if (e__ != hipSuccess) return ICQ_ERR_HIP; \
    } while (0)

static inline int icq_check_launch() {
    return hipGetLastError() == hipSuccess ? ICQ_OK : ICQ_ERR_HIP;
}
