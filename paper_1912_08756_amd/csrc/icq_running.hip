// The search loop of arxiv 1912.08756, Sec. 3.4, with its running threshold refreshed per tile of
// items.  The paper visits the items one by one and compares an item's crude distance (Eq. 2) with
// that of the furthest element f of the nearest-neighbour list plus the margin sigma; a machine that
// scans many items at once cannot refresh f per item, but it can per tile: the index is given as R
// tiles (indexes over consecutive ranges of item ids, same codebooks), and tile r is searched with
//     t_q = P(f) + sigma_q,   f = the furthest element of the list after tiles 0 .. r-1
// (+inf while the list is not full: every item of the tile then gets the exact comparison), its
// survivors' exact distances (Eq. 1) are merged into the list, and the threshold is refreshed.
// Tiles of one item are the paper's loop; one tile is the exhaustive search.
// Host side: table build once, then per tile the ordinary two-step search and one merge kernel.
#include "icq_internal.h"

namespace {

constexpr int RM_T = 256;

__global__ void running_init_kernel(uint32_t *__restrict__ ids, float *__restrict__ dist, int64_t n, float *__restrict__ thr,
                                    uint32_t *__restrict__ refined, int Q) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) {
        ids[i] = ICQ_PAD_ID;
        dist[i] = __builtin_inff();
    }
    if (i < Q) {
        thr[i] = __builtin_inff();
        refined[i] = 0u;
    }
}

__device__ __forceinline__ unsigned long long list_key(float d, uint32_t id) {
    const uint32_t b = __float_as_uint(d);
    const uint32_t ob = b ^ ((b >> 31) ? 0xFFFFFFFFu : 0x80000000u);       // order-preserving bits
    return ((unsigned long long)ob << 32) | id;
}

// One block per query.  The running list (ids, distances, crude distances; ascending by (D, id),
// padded with (0xFFFFFFFF, +inf)) and the tile's list (local ids) are both sorted, so an element's
// place in their union is its own index plus a binary search in the other list.  Ids of different
// tiles differ, so only paddings tie; the running list's paddings go first among them.
__global__ __launch_bounds__(RM_T) void running_merge_kernel(
    uint32_t *__restrict__ ids, float *__restrict__ dist, float *__restrict__ crude, const uint32_t *__restrict__ tile_ids,
    const float *__restrict__ tile_dist, const uint32_t *__restrict__ tile_surv, uint32_t id_base,
    const uint8_t *__restrict__ items, int stride, int K, int Kf, const float *__restrict__ lut,
    const float *__restrict__ sigma, int topk, float *__restrict__ thr, uint32_t *__restrict__ refined) {
    extern __shared__ __attribute__((aligned(16))) unsigned char rm_smem[];
    unsigned long long *key = reinterpret_cast<unsigned long long *>(rm_smem);     // [2 * topk]: list, then tile
    float *pc = reinterpret_cast<float *>(key + 2 * topk);                         // [2 * topk] crude distances
    const int q = blockIdx.x;
    const float *Tq = lut + (int64_t)q * K * ICQ_LUT_W;
    for (int e = threadIdx.x; e < topk; e += RM_T) {
        const int64_t o = (int64_t)q * topk + e;
        key[e] = list_key(dist[o], ids[o]);
        pc[e] = crude[o];
        const uint32_t lid = tile_ids[o];
        float p = 0.0f;
        uint32_t gid = ICQ_PAD_ID;
        if (lid != ICQ_PAD_ID) {
            gid = id_base + lid;
            const uint8_t *rec = items + (size_t)lid * stride;
            for (int k = 0; k < Kf; ++k) p += Tq[k * ICQ_LUT_W + rec[k]];        // Eq. 2, k ascending, fp32
        }
        key[topk + e] = list_key(tile_dist[o], gid);
        pc[topk + e] = p;
    }
    __syncthreads();
    for (int e = threadIdx.x; e < 2 * topk; e += RM_T) {
        const bool from_tile = e >= topk;
        const unsigned long long mine = key[e];
        const unsigned long long *other = from_tile ? key : key + topk;
        // elements of the other list before mine: strictly smaller, and (for a tile element) equal ones too
        int lo = 0, hi = topk;
        while (lo < hi) {
            const int mid = (lo + hi) >> 1;
            const bool before = from_tile ? other[mid] <= mine : other[mid] < mine;
            if (before) lo = mid + 1; else hi = mid;
        }
        const int rank = (from_tile ? e - topk : e) + lo;
        if (rank < topk) {
            const int64_t o = (int64_t)q * topk + rank;
            const uint32_t id = (uint32_t)mine;
            const uint32_t ob = (uint32_t)(mine >> 32);
            ids[o] = id;
            dist[o] = __uint_as_float(ob ^ ((ob >> 31) ? 0x80000000u : 0xFFFFFFFFu));
            crude[o] = pc[e];
            if (rank == topk - 1)      // the furthest element: the next tile's right side of Eq. 2
                thr[q] = id != ICQ_PAD_ID ? pc[e] + (sigma ? sigma[q] : 0.0f) : __builtin_inff();
        }
    }
    if (threadIdx.x == 0) refined[q] += tile_surv[q];
}

struct running_layout {
    size_t lut_off, thr_off, tids_off, tdist_off, tsurv_off, crude_off, inner_off, inner_bytes, total;
};

int running_plan(const icq_index *const *tiles, int R, int Q, int64_t cap, int topk, running_layout *L) {
    if (!tiles || R < 1 || Q < 0 || Q > ICQ_MAX_Q || cap < 1 || topk < 1 || topk > ICQ_MAX_TOPK) return ICQ_ERR_ARG;
    if ((double)Q * (double)cap >= 1099511627776.0) return ICQ_ERR_ARG;
    int64_t total = 0;
    for (int r = 0; r < R; ++r) {
        const icq_index *t = tiles[r];
        if (!t || t->K != tiles[0]->K || t->Kf != tiles[0]->Kf || t->d != tiles[0]->d || t->m != tiles[0]->m ||
            t->device != tiles[0]->device)
            return ICQ_ERR_ARG;
        total += t->N;
    }
    if (total > ICQ_MAX_N) return ICQ_ERR_ARG;
    const icq_index *t0 = tiles[0];
    size_t off = 0;
    L->lut_off = off;   off = icq_align_up(off + sizeof(float) * (size_t)Q * t0->K * ICQ_LUT_W, ICQ_ALIGN);
    L->thr_off = off;   off = icq_align_up(off + sizeof(float) * (size_t)Q, ICQ_ALIGN);
    L->tids_off = off;  off = icq_align_up(off + sizeof(uint32_t) * (size_t)Q * topk, ICQ_ALIGN);
    L->tdist_off = off; off = icq_align_up(off + sizeof(float) * (size_t)Q * topk, ICQ_ALIGN);
    L->tsurv_off = off; off = icq_align_up(off + sizeof(uint32_t) * (size_t)Q, ICQ_ALIGN);
    L->crude_off = off; off = icq_align_up(off + sizeof(float) * (size_t)Q * topk, ICQ_ALIGN);
    L->inner_off = off;
    size_t inner = ICQ_ALIGN;
    for (int r = 0; r < R; ++r) {
        // a tile needs room for at most its own items as candidates
        const int64_t c = cap < tiles[r]->N ? cap : tiles[r]->N;
        const size_t b = icq_layout(tiles[r], Q, c, topk, false, true).total;
        if (b > inner) inner = b;
    }
    L->inner_bytes = inner;
    L->total = off + inner;
    return ICQ_OK;
}

}  // namespace

ICQ_EXPORT int icq_running_workspace_bytes(const icq_index *const *tiles, int R, int Q, int64_t cap, int topk,
                                           size_t *out) {
    running_layout L;
    if (!out) return ICQ_ERR_ARG;
    const int rc = running_plan(tiles, R, Q, cap, topk, &L);
    if (rc != ICQ_OK) return rc;
    *out = L.total;
    return ICQ_OK;
}

ICQ_EXPORT int icq_search_running(const icq_index *const *tiles, const uint32_t *id_base, int R, const float *queries,
                                  int Q, const float *sigma, int64_t cap, int topk, uint32_t *out_ids, float *out_dist,
                                  uint32_t *out_refined, void *workspace, size_t workspace_bytes, void *stream) {
    running_layout L;
    int rc = running_plan(tiles, R, Q, cap, topk, &L);
    if (rc != ICQ_OK) return rc;
    if (Q == 0) return ICQ_OK;
    if (!id_base || !queries || !out_ids || !out_dist || !out_refined) return ICQ_ERR_ARG;
    if (!workspace || ((uintptr_t)workspace % ICQ_ALIGN) != 0 || workspace_bytes < L.total) return ICQ_ERR_WORKSPACE;
    for (int r = 0; r < R; ++r)
        if ((int64_t)id_base[r] + tiles[r]->N > ICQ_MAX_N) return ICQ_ERR_ARG;
    const size_t lds = (size_t)2 * topk * (sizeof(unsigned long long) + sizeof(float));
    hipStream_t s = (hipStream_t)stream;
    char *ws = static_cast<char *>(workspace);
    float *lut = reinterpret_cast<float *>(ws + L.lut_off);
    float *thr = reinterpret_cast<float *>(ws + L.thr_off);
    uint32_t *tids = reinterpret_cast<uint32_t *>(ws + L.tids_off);
    float *tdist = reinterpret_cast<float *>(ws + L.tdist_off);
    uint32_t *tsurv = reinterpret_cast<uint32_t *>(ws + L.tsurv_off);
    float *crude = reinterpret_cast<float *>(ws + L.crude_off);
    rc = icq_launch_build_lut(tiles[0], queries, Q, lut, s);
    if (rc != ICQ_OK) return rc;
    const int64_t n = (int64_t)Q * topk;
    running_init_kernel<<<(unsigned)((n + 255) / 256), 256, 0, s>>>(out_ids, out_dist, n, thr, out_refined, Q);
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    for (int r = 0; r < R; ++r) {
        const icq_index *t = tiles[r];
        const int64_t c = cap < t->N ? cap : t->N;
        rc = icq_search_impl(t, nullptr, lut, Q, thr, c, topk, tids, tdist, tsurv, ws + L.inner_off, L.inner_bytes, stream);
        if (rc != ICQ_OK) return rc;
        running_merge_kernel<<<Q, RM_T, lds, s>>>(out_ids, out_dist, crude, tids, tdist, tsurv, id_base[r], t->items,
                                                  t->item_stride, t->K, t->Kf, lut, sigma, topk, thr, out_refined);
        if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    }
    return ICQ_OK;
}
