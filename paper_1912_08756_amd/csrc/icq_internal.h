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
};

// Sub-buffers carved out of the caller's workspace for one query batch.
struct icq_ws_layout {
    size_t lut_off, lutT_off, ids_off, rec_off, count_off, keys_off, total;
    int splits;                // stage-2 blocks per query
};

static inline size_t icq_align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

// Layout for `Q` queries processed together.  with_lut / with_cands select the
// parts a call needs (icq_scan_fast and icq_refine get their tables and lists
// from the caller).
icq_ws_layout icq_layout(const icq_index *ix, int Q, int64_t cap, int topk, bool with_lut,
                         bool with_cands);
int icq_refine_splits(const icq_index *ix, int Q, int64_t cap, int topk);

// Kernel launchers (each checks nothing; the extern "C" entry points validate).
int icq_launch_build_lut(const icq_index *ix, const float *queries, int Q, float *lut,
                         hipStream_t s);
// cand_part == nullptr: the crude distances are not materialised (the fused path
// recomputes the full sum in stage 2 from the item records).
// cand_rec != nullptr: the scan may also write each survivor's item record next
// to its id ([Q][cap][item_stride/4] words) and says so through *rec_written.
int icq_launch_scan(const icq_index *ix, const float *lut, int Q, const float *thr,
                    uint32_t *cand_ids, float *cand_part, uint32_t *cand_rec, bool *rec_written,
                    uint32_t *cand_count, int64_t cap, float *lutT, hipStream_t s);
// cand_part == nullptr: D is the full K-term sum; else D = cand_part + slow terms.
// cand_rec != nullptr: item records come from the candidate list instead of a gather.
int icq_launch_refine(const icq_index *ix, const float *lut, int Q, const uint32_t *cand_ids,
                      const float *cand_part, const uint32_t *cand_rec, const uint32_t *cand_count,
                      int64_t cap, int topk, int splits, unsigned long long *keys, uint32_t *out_ids,
                      float *out_dist, hipStream_t s);

#define ICQ_HIP_TRY(expr)                      \
    do {                                       \
        hipError_t e__ = (expr);               \
        if (e__ != hipSuccess) return ICQ_ERR_HIP; \
    } while (0)

static inline int icq_check_launch() {
    return hipGetLastError() == hipSuccess ? ICQ_OK : ICQ_ERR_HIP;
}
