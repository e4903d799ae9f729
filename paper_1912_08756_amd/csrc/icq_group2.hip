// Grouping by the first two fast sub-codes, for Kf = 3 and 4 (arxiv 1912.08756, Eq. 2).  The crude
// distance is a sum of Kf table entries in codebook order; with the items ordered by their pair
// (code_0, code_1), the first two entries are the same for a whole run of items, so stage 1 forms
// their sum once per 16 positions and looks up only the remaining Kf - 2 entries per item: half the
// table reads and half the code bytes of the item-by-item scan at Kf = 4, identical sums.
//
// Layout (built once by a counting sort): the 65536 pairs in the scattered order of
// icq_g2_pair_of_slot, every pair's run padded to whole 16 positions; per position the item id (perm),
// the item's record (items_grouped) and its remaining fast sub-codes as rows of their own (g2_rows);
// per 16 positions the pair and the number of real items (g2_info).
#include "icq_internal.h"

namespace {

constexpr int G2_PAIRS = 65536;

__device__ __forceinline__ uint32_t slot_of_item(const uint8_t *__restrict__ fast, int64_t Npad, int64_t i) {
    return icq_g2_slot_of_pair((uint32_t)fast[i] | ((uint32_t)fast[Npad + i] << 8));
}

__global__ void g2_count_kernel(const uint8_t *__restrict__ fast, int64_t Npad, int64_t N,
                                uint32_t *__restrict__ cursor) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) atomicAdd(&cursor[slot_of_item(fast, Npad, i)], 1u);
}

// start[s] = sum over the slots before s of their counts rounded up to 16; cursor is left equal to
// start (the scatter advances it); start[G2_PAIRS] = the padded total.  One block of 1024 threads.
__global__ __launch_bounds__(1024) void g2_offsets_kernel(uint32_t *__restrict__ cursor, uint32_t *__restrict__ start) {
    __shared__ uint32_t part[1024];
    const int tid = threadIdx.x;
    constexpr int PER = G2_PAIRS / 1024;
    uint32_t sum = 0;
    for (int j = 0; j < PER; ++j) sum += (cursor[tid * PER + j] + 15u) & ~15u;
    part[tid] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {     // Hillis-Steele inclusive scan
        const uint32_t v = tid >= d ? part[tid - d] : 0u;
        __syncthreads();
        part[tid] += v;
        __syncthreads();
    }
    uint32_t run = part[tid] - sum;
    for (int j = 0; j < PER; ++j) {
        const int g = tid * PER + j;
        const uint32_t c = (cursor[g] + 15u) & ~15u;
        start[g] = run;
        cursor[g] = run;
        run += c;
    }
    if (tid == 1023) start[G2_PAIRS] = part[1023];
}

__global__ void g2_scatter_kernel(const uint8_t *__restrict__ fast, int64_t Npad, int Kf, int64_t N,
                                  uint32_t *__restrict__ cursor, const uint8_t *__restrict__ items, int stride,
                                  uint32_t *__restrict__ perm, uint8_t *__restrict__ items_grouped,
                                  uint8_t *__restrict__ rows, int64_t g2_npad) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= N) return;
    const uint32_t pos = atomicAdd(&cursor[slot_of_item(fast, Npad, i)], 1u);
    perm[pos] = (uint32_t)i;
    for (int r = 0; r < Kf - 2; ++r) rows[(int64_t)r * g2_npad + pos] = fast[(int64_t)(r + 2) * Npad + i];
    const int W = stride / 4;
    const uint32_t *src = reinterpret_cast<const uint32_t *>(items + (size_t)i * stride);
    uint32_t *dst = reinterpret_cast<uint32_t *>(items_grouped + (size_t)pos * stride);
    for (int w = 0; w < W; ++w) dst[w] = src[w];
}

// One thread per slot: the info word of each of its groups of 16 positions (cursor = start + count now).
__global__ void g2_info_kernel(const uint32_t *__restrict__ start, const uint32_t *__restrict__ cursor,
                               uint32_t *__restrict__ info) {
    const int s = blockIdx.x * blockDim.x + threadIdx.x;
    if (s >= G2_PAIRS) return;
    const uint32_t pair = icq_g2_pair_of_slot((uint32_t)s);
    const uint32_t b = start[s];
    uint32_t left = cursor[s] - b;
    for (uint32_t j = b >> 4; left > 0; ++j) {
        const uint32_t n = left < 16u ? left : 16u;
        info[j] = pair | (n << 16);
        left -= n;
    }
}

__global__ void g2_fill_kernel(uint32_t *__restrict__ p, size_t n, uint32_t v) {
    const size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}

// codes_out[k][perm[pos]] from the grouped layout alone: rows 0, 1 from the pair of the position's
// group of 16, rows 2 .. Kf-1 from the streamed rows, the rest from the grouped item records.
__global__ void g2_export_kernel(const uint32_t *__restrict__ info, const uint8_t *__restrict__ rows, int64_t g2_npad,
                                 const uint8_t *__restrict__ items_grouped, const uint32_t *__restrict__ perm,
                                 int64_t npos, int64_t N, int Kf, int stride, uint8_t *__restrict__ out) {
    const int k = blockIdx.y;
    const int64_t pos = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (pos >= npos) return;
    const uint32_t id = perm[pos];
    if (id == ICQ_PAD_ID) return;
    uint8_t v;
    if (k < 2) v = (uint8_t)(info[pos >> 4] >> (8 * k));
    else if (k < Kf) v = rows[(int64_t)(k - 2) * g2_npad + pos];
    else v = items_grouped[pos * stride + k];
    out[(int64_t)k * N + id] = v;
}

}  // namespace

int icq_group2_build(icq_index *ix, hipStream_t s) {
    ix->g2 = 0;
    if (ix->Kf < 3 || ix->Kf > 4 || ix->N == 0 || ix->N + 16ll * G2_PAIRS >= (1ll << 31)) return ICQ_OK;
    bool ok = hipMalloc(&ix->group_start, sizeof(uint32_t) * (G2_PAIRS + 1)) == hipSuccess &&
              hipMalloc(&ix->group_cursor, sizeof(uint32_t) * G2_PAIRS) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        return ICQ_ERR_HIP;       // the caller destroys the index, which frees whatever was allocated
    }
    const int T = 256;
    const unsigned nb = (unsigned)((ix->N + T - 1) / T);
    g2_fill_kernel<<<G2_PAIRS / T, T, 0, s>>>(ix->group_cursor, G2_PAIRS, 0u);
    g2_count_kernel<<<nb, T, 0, s>>>(ix->fast, ix->Npad, ix->N, ix->group_cursor);
    g2_offsets_kernel<<<1, 1024, 0, s>>>(ix->group_cursor, ix->group_start);
    uint32_t total = 0;
    if (icq_check_launch() != ICQ_OK ||
        hipMemcpyAsync(&total, ix->group_start + G2_PAIRS, sizeof(uint32_t), hipMemcpyDeviceToHost, s) != hipSuccess ||
        hipStreamSynchronize(s) != hipSuccess) {
        (void)hipGetLastError();
        return ICQ_ERR_HIP;
    }
    // whole block steps of the scan kernel, plus a spare step: its read-ahead never checks bounds
    ix->g2_npos = ((int64_t)total + 16383) / 16384 * 16384;
    ix->g2_npad = ix->g2_npos + 16384;
    const size_t np = (size_t)ix->g2_npad;
    ok = hipMalloc(&ix->g2_rows, (size_t)(ix->Kf - 2) * np) == hipSuccess &&
         hipMalloc(&ix->g2_info, sizeof(uint32_t) * (np / 16)) == hipSuccess &&
         hipMalloc(&ix->perm, sizeof(uint32_t) * np) == hipSuccess &&
         hipMalloc(&ix->items_grouped, np * ix->item_stride) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        return ICQ_ERR_HIP;
    }
    auto fill = [&](void *p, size_t bytes, uint32_t v) {
        const size_t n = bytes / 4;
        g2_fill_kernel<<<(unsigned)((n + T - 1) / T), T, 0, s>>>(static_cast<uint32_t *>(p), n, v);
    };
    fill(ix->g2_rows, (size_t)(ix->Kf - 2) * np, 0u);
    fill(ix->g2_info, sizeof(uint32_t) * (np / 16), 0u);
    fill(ix->perm, sizeof(uint32_t) * np, ICQ_PAD_ID);
    fill(ix->items_grouped, np * ix->item_stride, 0u);
    g2_scatter_kernel<<<nb, T, 0, s>>>(ix->fast, ix->Npad, ix->Kf, ix->N, ix->group_cursor, ix->items, ix->item_stride,
                                       ix->perm, ix->items_grouped, ix->g2_rows, ix->g2_npad);
    g2_info_kernel<<<G2_PAIRS / T, T, 0, s>>>(ix->group_start, ix->group_cursor, ix->g2_info);
    if (icq_check_launch() != ICQ_OK) return ICQ_ERR_HIP;
    ix->g2 = 1;
    return ICQ_OK;
}

int icq_group2_export(const icq_index *ix, uint8_t *codes_out, hipStream_t s) {
    const int T = 256;
    dim3 g((unsigned)((ix->g2_npos + T - 1) / T), (unsigned)ix->K);
    g2_export_kernel<<<g, T, 0, s>>>(ix->g2_info, ix->g2_rows, ix->g2_npad, ix->items_grouped, ix->perm, ix->g2_npos,
                                     ix->N, ix->Kf, ix->item_stride, codes_out);
    return icq_check_launch();
}
