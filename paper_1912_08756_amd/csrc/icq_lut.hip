// Lookup-table precompute (arxiv 1912.08756, Sec. 1, text after Eq. 1): for
// every query the squared distance to every codeword of every codebook,
//   lut[q][k][j] = ||q||^2 - 2<q, c_{k,j}> + ||c_{k,j}||^2.
// The inner products are one [Q x d] . [d x K*256] contraction and run on the
// fp32 matrix cores (v_mfma_f32_32x32x2_f32); norms are added in the epilogue.
#include "icq_internal.h"
#include "icq_sort.h"

namespace {

typedef float float16v __attribute__((ext_vector_type(16)));

constexpr int BM = 64;   // queries per block
constexpr int BN = 64;   // table entries per block and column block of a wavefront row (NB of them side by side)
constexpr int BK = 16;   // reduction slice staged in LDS
constexpr int LD = 65;   // LDS row stride (floats): k-major tiles, +1 to spread the transposing writes

// Block = 4 wavefronts in a 2x2 arrangement, each owning NB 32x32 output blocks side by side
// (NB = 2: the query fragment of a step serves two matrix instructions, and a slice's two
// barriers are spread over twice the arithmetic).
// MFMA 32x32x2 operand layout: lane l supplies A[l%32][l/32] and B[l/32][l%32];
// accumulator register v of lane l is C[(v%4) + 4*(l/32) + 8*(v/4)][l%32].
template <int NB>
__global__ __launch_bounds__(256) void build_lut_kernel(const float *__restrict__ queries, int Q,
                                                        int d, const float *__restrict__ cb,
                                                        int d_pad, const float *__restrict__ cnorm,
                                                        int ncols, float *__restrict__ lut) {
    __shared__ float As[BK][LD];
    __shared__ float Bs[BK][NB * BN + 1];
    __shared__ float qn_s[BM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int n0 = blockIdx.x * (NB * BN);
    const int q0 = blockIdx.y * BM;

    const int le = tid & 15;    // position along the reduction axis for the loads
    const int lr = tid >> 4;    // row (0..15), +16 per pass

    float16v acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    float qn[4] = {0.0f, 0.0f, 0.0f, 0.0f};   // this thread's share of ||q||^2 of its four staged rows

    // Rows past Q read the last query instead (their results are never stored) and columns past d
    // read column d - 1 (the codebook copy is zero there, so the product vanishes): no load
    // depends on a condition, so all eight of a slice are in flight together.
    const float *qrow[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int q = q0 + lr + 16 * p;
        qrow[p] = queries + (int64_t)(q < Q ? q : Q - 1) * d;
    }
    for (int k0 = 0; k0 < d_pad; k0 += BK) {
        float a[4], b[4 * NB];
        const int e = k0 + le;
        const int ec = e < d ? e : d - 1;
#pragma unroll
        for (int p = 0; p < 4; ++p) a[p] = qrow[p][ec];
#pragma unroll
        for (int p = 0; p < 4 * NB; ++p) b[p] = cb[(int64_t)(n0 + lr + 16 * p) * d_pad + e];
        if (e < d) {
#pragma unroll
            for (int p = 0; p < 4; ++p) qn[p] = fmaf(a[p], a[p], qn[p]);
        }
        __syncthreads();   // previous slice fully consumed
#pragma unroll
        for (int p = 0; p < 4; ++p) As[le][lr + 16 * p] = a[p];
#pragma unroll
        for (int p = 0; p < 4 * NB; ++p) Bs[le][lr + 16 * p] = b[p];
        __syncthreads();
#pragma unroll
        for (int s = 0; s < BK / 2; ++s) {
            const float av = As[2 * s + (lane >> 5)][wm * 32 + (lane & 31)];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const float bv = Bs[2 * s + (lane >> 5)][(wn * NB + j) * 32 + (lane & 31)];
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av, bv, acc[j], 0, 0, 0);
            }
        }
    }
    // the 16 threads of a staged row are 16 consecutive lanes: sum their shares (lane 15 of the row ends with the total)
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        float x = qn[p];
        x += __uint_as_float(icq_dpp<0x111, 0xf, 0u>(__float_as_uint(x)));
        x += __uint_as_float(icq_dpp<0x112, 0xf, 0u>(__float_as_uint(x)));
        x += __uint_as_float(icq_dpp<0x114, 0xf, 0u>(__float_as_uint(x)));
        x += __uint_as_float(icq_dpp<0x118, 0xf, 0u>(__float_as_uint(x)));
        if (le == 15) qn_s[lr + 16 * p] = x;
    }
    __syncthreads();

#pragma unroll
    for (int j = 0; j < NB; ++j) {
        const int col = n0 + (wn * NB + j) * 32 + (lane & 31);
        const float cn = cnorm[col];
        // all 16 values first, then the stores back to back: a store inside a branch of its own is
        // followed by a wait for everything outstanding, the previous store included
        float r[16];
#pragma unroll
        for (int v = 0; v < 16; ++v) {
            const int i = (v & 3) + 4 * (lane >> 5) + 8 * (v >> 2);
            r[v] = (qn_s[wm * 32 + i] + cn) - 2.0f * acc[j][v];
        }
        float *out = lut + (int64_t)(q0 + wm * 32 + 4 * (lane >> 5)) * ncols + col;
        if (q0 + wm * 32 + 32 <= Q) {            // wavefront-uniform: every row of the 32 exists
#pragma unroll
            for (int v = 0; v < 16; ++v) out[(int64_t)((v & 3) + 8 * (v >> 2)) * ncols] = r[v];
        } else {
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int i = (v & 3) + 4 * (lane >> 5) + 8 * (v >> 2);
                if (q0 + wm * 32 + i < Q) out[(int64_t)((v & 3) + 8 * (v >> 2)) * ncols] = r[v];
            }
        }
    }
}

}  // namespace

int icq_launch_build_lut(const icq_index *ix, const float *queries, int Q, float *lut,
                         hipStream_t s) {
    if (Q == 0) return ICQ_OK;
    const int ncols = ix->K * ICQ_LUT_W;
    // two column blocks per wavefront: 5 % faster than one at C1 and C2; four are slower at d = 960 and for few queries
    constexpr int NB = 2;
    // query blocks along grid.y, at most 65535 per launch
    constexpr int SLICE = 65535 * BM;
    for (int q0 = 0; q0 < Q; q0 += SLICE) {
        const int nq = Q - q0 < SLICE ? Q - q0 : SLICE;
        dim3 grid((unsigned)(ncols / (NB * BN)), (unsigned)((nq + BM - 1) / BM));   // ncols = K * 256
        build_lut_kernel<NB><<<grid, 256, 0, s>>>(queries + (int64_t)q0 * ix->d, nq, ix->d, ix->cb, ix->d_pad,
                                                      ix->cnorm, ncols, lut + (int64_t)q0 * ncols);
    }
    return icq_check_launch();
}

ICQ_EXPORT int icq_build_lut(const icq_index *ix, const float *queries, int Q, float *lut,
                             void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || (Q > 0 && (!queries || !lut))) return ICQ_ERR_ARG;
    return icq_launch_build_lut(ix, queries, Q, lut, (hipStream_t)stream);
}
