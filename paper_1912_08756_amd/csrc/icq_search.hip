// The whole query-time path of arxiv 1912.08756 (Sec. 3.4) for a batch of
// queries: table precompute, crude comparison over the fast codebooks (Eq. 2),
// exact comparison for the survivors (Eq. 1), nearest-neighbour list.  Host
// side only: workspace carving and kernel sequencing on one stream.
#include "icq_internal.h"

#include <mutex>

icq_ws_layout icq_layout(const icq_index *ix, int Q, int64_t cap, int topk, bool with_lut,
                         bool with_cands) {
    icq_ws_layout L = {};
    size_t off = 0;
    L.lut_off = off;
    if (with_lut) off = icq_align_up(off + sizeof(float) * (size_t)Q * ix->K * ICQ_LUT_W, ICQ_ALIGN);
    // icq_search with the grouped stage 1 keeping the lists on chip: no candidate lists in the
    // workspace, only (few queries, several blocks per query) the parts' lists for the merge
    const bool on_chip = with_cands && icq_group_fused(ix, Q, topk);
    L.masked = with_cands && !on_chip && icq_masks_usable(ix, Q, topk);
    L.splits = icq_refine_splits(ix, Q, cap, topk);
    L.ids_off = off;
    if (L.masked) {
        L.scan_end = icq_mask_scan_end(ix);
        L.mask_stride = (size_t)(L.scan_end / 16);
        // rows for whole groups of eight queries: the pre-filter kernel stores all eight slots of its last group
        off = icq_align_up(off + sizeof(uint16_t) * (size_t)((Q + 7) / 8 * 8) * L.mask_stride, ICQ_ALIGN);
        L.keycount_off = off;
        off = icq_align_up(off + sizeof(uint32_t) * (size_t)Q, ICQ_ALIGN);
    } else if (with_cands && !on_chip) {
        off = icq_align_up(off + sizeof(uint32_t) * (size_t)Q * (size_t)cap, ICQ_ALIGN);
    }
    L.count_off = off;
    if (with_cands) off = icq_align_up(off + sizeof(uint32_t) * (size_t)Q, ICQ_ALIGN);
    L.keys_off = off;
    // slice lists [Q][splits][topk] (when sliced), then one 64-bit key per candidate [Q][cap]
    if (on_chip) {
        const int parts = icq_group_fused_parts(ix, Q);
        if (parts > 1) off = icq_align_up(off + sizeof(unsigned long long) * (size_t)Q * parts * topk, ICQ_ALIGN);
    } else {
        if (L.splits > 1)
            off = icq_align_up(off + sizeof(unsigned long long) * (size_t)Q * L.splits * topk, 8);
        if (ix->item_stride <= 16)
            off = icq_align_up(off + sizeof(unsigned long long) * (size_t)Q * (size_t)cap, ICQ_ALIGN);
    }
    L.total = off;
    return L;
}

// Most queries icq_search takes through the kernels at once.
constexpr int SEARCH_MAX_BATCH = 32768;

ICQ_EXPORT int icq_workspace_bytes(const icq_index *ix, int Q, int64_t cap, int topk, size_t *out) {
    if (!ix || !out || Q < 0 || Q > ICQ_MAX_Q || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK)
        return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    // the largest of what icq_search and the staged calls (which take lists from the caller) carve
    // out, whichever stage-1 strategy is selected when they run
    size_t need = ICQ_ALIGN;
    const int Qs = Q < SEARCH_MAX_BATCH ? Q : SEARCH_MAX_BATCH;
    for (int mode = ICQ_SCAN_AUTO; mode <= ICQ_SCAN_GROUPED; ++mode) {
        icq_index view = *ix;
        view.scan_mode = mode;
        const size_t a = icq_layout(&view, Qs, cap, topk, true, true).total;
        const size_t b = icq_layout(&view, Q, cap, topk, false, false).total;
        if (a > need) need = a;
        if (b > need) need = b;
    }
    *out = need;
    return ICQ_OK;
}

// lut_ext: the queries' tables when the caller has built them already (queries is not read then).
int icq_search_impl(const icq_index *ix, const float *queries, const float *lut_ext, int Q, const float *thresholds,
                    int64_t cap, int topk, uint32_t *out_ids, float *out_dist,
                    uint32_t *out_survivors, void *workspace, size_t workspace_bytes,
                    void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK)
        return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if ((!queries && !lut_ext) || !thresholds || !out_ids || !out_dist) return ICQ_ERR_ARG;
    const bool own_lut = lut_ext == nullptr;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0) return ICQ_ERR_WORKSPACE;

    // Largest sub-batch (all of Q, else a multiple of 64 queries) that fits the workspace.
    int Qb = Q < SEARCH_MAX_BATCH ? Q : SEARCH_MAX_BATCH;
    while (icq_layout(ix, Qb, cap, topk, own_lut, true).total > workspace_bytes) {
        if (Qb <= 64) return ICQ_ERR_WORKSPACE;
        Qb = ((Qb / 2) + 63) / 64 * 64;
    }
    if (Q % Qb != 0 && icq_layout(ix, Q % Qb, cap, topk, own_lut, true).total > workspace_bytes)
        return ICQ_ERR_WORKSPACE;
    hipStream_t s = (hipStream_t)stream;
    char *ws = static_cast<char *>(workspace);
    icq_stage_timer *tm = ix->timer;
    hipEvent_t *ev = nullptr;
    if (tm) {
        const int nb = (Q + Qb - 1) / Qb;
        if (nb > tm->batches) tm->batches = nb;
        ev = tm->ev[tm->calls % ICQ_TIMED_CALLS];
    }
    for (int q0 = 0; q0 < Q; q0 += Qb) {
        const bool timed = tm && q0 == 0;
        const int nq = (Q - q0) < Qb ? (Q - q0) : Qb;
        const icq_ws_layout L = icq_layout(ix, nq, cap, topk, own_lut, true);
        const float *lut = own_lut ? reinterpret_cast<float *>(ws + L.lut_off)
                                   : lut_ext + (int64_t)q0 * ix->K * ICQ_LUT_W;
        uint32_t *ids = reinterpret_cast<uint32_t *>(ws + L.ids_off);
        uint32_t *cnt = out_survivors ? out_survivors + q0 : reinterpret_cast<uint32_t *>(ws + L.count_off);
        unsigned long long *keys = reinterpret_cast<unsigned long long *>(ws + L.keys_off);
        if (timed) ICQ_HIP_TRY(hipEventRecord(ev[0], s));
        int rc = ICQ_OK;
        if (own_lut) rc = icq_launch_build_lut(ix, queries + (int64_t)q0 * ix->d, nq, reinterpret_cast<float *>(ws + L.lut_off), s);
        if (rc != ICQ_OK) return rc;
        if (L.masked) {
            // item-by-item stage 1 into hit bits, stage 2 chunk by chunk from them
            uint16_t *masks = reinterpret_cast<uint16_t *>(ws + L.ids_off);
            uint32_t *key_count = reinterpret_cast<uint32_t *>(ws + L.keycount_off);
            bool superset = false;
            rc = icq_launch_scan_masks(ix, lut, nq, thresholds + q0, masks, L.mask_stride, L.scan_end, cnt, key_count,
                                       timed ? ev[1] : nullptr, &superset, s);
            if (rc != ICQ_OK) return rc;
            if (timed) ICQ_HIP_TRY(hipEventRecord(ev[2], s));
            rc = icq_launch_refine_masks(ix, lut, nq, masks, L.mask_stride, L.scan_end, cap, topk, L.splits, keys,
                                         key_count, cnt, superset ? thresholds + q0 : nullptr,
                                         out_ids + (int64_t)q0 * topk, out_dist + (int64_t)q0 * topk, s);
            if (rc != ICQ_OK) return rc;
            if (timed) ICQ_HIP_TRY(hipEventRecord(ev[3], s));
            continue;
        }
        int list_kind = ICQ_LIST_IDS;
        // keys of the survivors behind the slice lists, or (on-chip lists) the parts' lists
        unsigned long long *cand_keys = icq_group_fused(ix, nq, topk) ? keys
                                        : (ix->item_stride <= 16 && topk <= 512) ? icq_cand_keys(keys, nq, L.splits, topk)
                                                                                 : nullptr;
        rc = icq_launch_scan(ix, lut, nq, thresholds + q0, ids, nullptr, cand_keys, &list_kind, cnt,
                             cap, topk, out_ids + (int64_t)q0 * topk, out_dist + (int64_t)q0 * topk,
                             timed ? ev[1] : nullptr, s);
        if (rc != ICQ_OK) return rc;
        if (timed) ICQ_HIP_TRY(hipEventRecord(ev[2], s));
        rc = icq_launch_refine(ix, lut, nq, ids, nullptr, list_kind, cnt, cap, topk, L.splits, keys,
                               out_ids + (int64_t)q0 * topk, out_dist + (int64_t)q0 * topk, s);
        if (rc != ICQ_OK) return rc;
        if (timed) ICQ_HIP_TRY(hipEventRecord(ev[3], s));
    }
    if (tm) tm->calls += 1;       // counted once every launch and event of the call is enqueued
    return ICQ_OK;
}

ICQ_EXPORT int icq_search(const icq_index *ix, const float *queries, int Q, const float *thresholds,
                          int64_t cap, int topk, uint32_t *out_ids, float *out_dist,
                          uint32_t *out_survivors, void *workspace, size_t workspace_bytes,
                          void *stream) {
    return icq_search_impl(ix, queries, nullptr, Q, thresholds, cap, topk, out_ids, out_dist, out_survivors, workspace,
                           workspace_bytes, stream);
}

// ---- icq_search for callers that cannot allocate: the workspace is a fixed array in the
// library's own device image.  Every GPU holds its own copy of the array at its own address;
// host code never uses the array's name as an address, only the pointer that
// hipGetSymbolAddress returned for the device in question.
static __device__ __align__(256) unsigned char scratch[ICQ_STATIC_SCRATCH_BYTES];

namespace {
constexpr int MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
void *g_scratch_ptr[MAX_DEVICES];      // per device, nullptr until its first call
}  // namespace

// Device address of `scratch` on the current device (looked up once per device).
static int scratch_address(void **out) {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= MAX_DEVICES) return ICQ_ERR_HIP;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void *p = nullptr;
        if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
            (void)hipGetLastError();
            return ICQ_ERR_HIP;
        }
        g_scratch_ptr[dev] = p;
    }
    *out = g_scratch_ptr[dev];
    return ICQ_OK;
}

ICQ_EXPORT int icq_search_static(const icq_index *ix, const float *queries, int Q, const float *thresholds,
                                 int64_t cap, int topk, uint32_t *out_ids, float *out_dist,
                                 uint32_t *out_survivors, void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK) return ICQ_ERR_ARG;
    if (Q == 0) return ICQ_OK;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess) return ICQ_ERR_HIP;
    if (dev != ix->device) return ICQ_ERR_ARG;          // the array used is the current device's
    // the whole call must fit at once: no silent split into sub-batches here
    if (icq_layout(ix, Q, cap, topk, true, true).total > (size_t)ICQ_STATIC_SCRATCH_BYTES) return ICQ_ERR_SCRATCH;
    void *ws = nullptr;
    const int rc = scratch_address(&ws);
    if (rc != ICQ_OK) return rc;
    return icq_search_impl(ix, queries, nullptr, Q, thresholds, cap, topk, out_ids, out_dist, out_survivors, ws,
                       (size_t)ICQ_STATIC_SCRATCH_BYTES, stream);
}
