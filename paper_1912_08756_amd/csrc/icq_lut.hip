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
constexpr int LD = 20;   // LDS row stride (floats): a row holds its 16 slice values; 20 = 4 * 5 spreads 16 rows' 16-byte pieces over all banks

typedef float float4v __attribute__((ext_vector_type(4)));

// Block = 4 wavefronts in a 2x2 arrangement, each owning NB 32x32 output blocks side by side
// (NB = 2: the query fragment of a step serves two matrix instructions, and a slice's two
// barriers are spread over twice the arithmetic).
// MFMA 32x32x2 operand layout: lane l supplies A[l%32][l/32] and B[l/32][l%32];
// accumulator register v of lane l is C[(v%4) + 4*(l/32) + 8*(v/4)][l%32].
// A slice of 16 reduction indices is staged row-major ([row][16]), moved in 16-byte pieces all the
// way: a thread loads four consecutive values of a row, writes them with one LDS store, and a
// lane's eight operands of a slice (one per matrix instruction) are eight consecutive values of
// its row, two 16-byte LDS reads.  Which reduction index meets which instruction does not matter
// as long as both operands agree: step s multiplies index s (lower half of the lanes) and 8 + s
// (upper half).
template <int NB, bool VEC, bool AHEAD>
__global__ __launch_bounds__(256) void build_lut_kernel(const float *queries, int Q,
                                                        int d, const float *cb,
                                                        int d_pad, const float *__restrict__ cnorm,
                                                        int ncols, float *__restrict__ lut) {
    __shared__ __attribute__((aligned(16))) float As[BM][LD];
    __shared__ __attribute__((aligned(16))) float Bs[NB * BN][LD];
    __shared__ float qn_s[BM];

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wave = tid >> 6;
    const int wm = wave >> 1, wn = wave & 1;
    const int n0 = blockIdx.x * (NB * BN);
    const int q0 = blockIdx.y * BM;

    const int lq = tid & 3;     // which four of the slice's 16 values this thread moves
    const int lr = tid >> 2;    // row (0..63), +64 per pass for the table side

    float16v acc[NB];
#pragma unroll
    for (int j = 0; j < NB; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    float qn = 0.0f;            // this thread's share of ||q||^2 of its staged row

    // A row past Q reads the last query instead (its results are never stored) and values past d
    // read in-range ones (the codebook copy is zero there, so the product vanishes): no load
    // depends on a condition, so all of a slice's are in flight together.
    const int qr = q0 + lr;
    const float *qrow = queries + (int64_t)(qr < Q ? qr : Q - 1) * d;
    const float *brow = cb + (int64_t)(n0 + lr) * d_pad + 4 * lq;
    const int half = lane >> 5, l32 = lane & 31;
    float4v a, b[NB];
    auto load_slice = [&](int k0) {
        const int e = k0 + 4 * lq;
        if (VEC) {              // d is a multiple of 4 and the rows are 16-byte aligned: e < d means e + 3 < d
            a = *reinterpret_cast<const float4v *>(qrow + (e < d ? e : d - 4));
        } else {
#pragma unroll
            for (int i = 0; i < 4; ++i) a[i] = qrow[e + i < d ? e + i : d - 1];
        }
#pragma unroll
        for (int p = 0; p < NB; ++p) b[p] = *reinterpret_cast<const float4v *>(brow + (int64_t)(64 * p) * d_pad + k0);
    };
    if (AHEAD) load_slice(0);
    for (int k0 = 0; k0 < d_pad; k0 += BK) {
        if (!AHEAD) load_slice(k0);
        const int e = k0 + 4 * lq;
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (e + i < d) qn = fmaf(a[i], a[i], qn);
        __syncthreads();   // previous slice fully consumed
        *reinterpret_cast<float4v *>(&As[lr][4 * lq]) = a;
#pragma unroll
        for (int p = 0; p < NB; ++p) *reinterpret_cast<float4v *>(&Bs[lr + 64 * p][4 * lq]) = b[p];
        __syncthreads();
        // AHEAD: the next slice's values are requested before this slice's matrix instructions (the
        // last slice asks for itself again: no condition on a load)
        if (AHEAD) {
            load_slice(k0 + BK < d_pad ? k0 + BK : k0);
            __builtin_amdgcn_sched_barrier(0);
        }
        float av[8], bv[NB][8];
#pragma unroll
        for (int h = 0; h < 2; ++h) {
            const float4v t = *reinterpret_cast<const float4v *>(&As[wm * 32 + l32][8 * half + 4 * h]);
#pragma unroll
            for (int i = 0; i < 4; ++i) av[4 * h + i] = t[i];
#pragma unroll
            for (int j = 0; j < NB; ++j) {
                const float4v u = *reinterpret_cast<const float4v *>(&Bs[(wn * NB + j) * 32 + l32][8 * half + 4 * h]);
#pragma unroll
                for (int i = 0; i < 4; ++i) bv[j][4 * h + i] = u[i];
            }
        }
#pragma unroll
        for (int s = 0; s < BK / 2; ++s) {
#pragma unroll
            for (int j = 0; j < NB; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(av[s], bv[j][s], acc[j], 0, 0, 0);
        }
    }
    // the 4 threads of a staged row are 4 consecutive lanes: sum their shares (the last of them ends with the total)
    {
        float x = qn;
        x += __uint_as_float(icq_dpp<0x111, 0xf, 0u>(__float_as_uint(x)));
        x += __uint_as_float(icq_dpp<0x112, 0xf, 0u>(__float_as_uint(x)));
        if (lq == 3) qn_s[lr] = x;
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
    // two column blocks per wavefront: four are slower everywhere, one is within 3 % either way
    constexpr int NB = 2;
    // query blocks along grid.y, at most 65535 per launch
    constexpr int SLICE = 65535 * BM;
    for (int q0 = 0; q0 < Q; q0 += SLICE) {
        const int nq = Q - q0 < SLICE ? Q - q0 : SLICE;
        dim3 grid((unsigned)(ncols / (NB * BN)), (unsigned)((nq + BM - 1) / BM));   // ncols = K * 256
        const float *qs = queries + (int64_t)q0 * ix->d;
        float *out = lut + (int64_t)q0 * ncols;
        // 16-byte query loads need whole pieces inside a row and aligned rows
        const bool vec = ix->d % 4 == 0 && ((uintptr_t)qs & 15) == 0;
        // With fewer than four blocks per compute unit nothing else covers a slice's load latency, so
        // the loads run a slice ahead (d = 960, 1000 queries: 89 -> 84 us); with more, the other blocks
        // cover it (d = 128, 10^4 queries: no gain).  Tried without effect on either shape: the LDS in
        // two buffers with one barrier per slice, the barrier and the next slice's operand reads in the
        // middle of a slice's matrix instructions, one to eight wavefronts per SIMD by register limit.
        // Slower: the entries as rows of the matrix instruction (16-byte stores of 32-byte pieces in 32
        // rows instead of 4-byte stores of whole 128-byte lines).
        const bool ahead = (int64_t)grid.x * grid.y < 4 * 256;
        auto launch = [&](auto kernel) {
            kernel<<<grid, 256, 0, s>>>(qs, nq, ix->d, ix->cb, ix->d_pad, ix->cnorm, ncols, out);
        };
        if (vec) { if (ahead) launch(build_lut_kernel<NB, true, true>); else launch(build_lut_kernel<NB, true, false>); }
        else     { if (ahead) launch(build_lut_kernel<NB, false, true>); else launch(build_lut_kernel<NB, false, false>); }
    }
    return icq_check_launch();
}

ICQ_EXPORT int icq_build_lut(const icq_index *ix, const float *queries, int Q, float *lut,
                             void *stream) {
    if (!ix || Q < 0 || Q > ICQ_MAX_Q || (Q > 0 && (!queries || !lut)) || ((uintptr_t)lut & 15) != 0) return ICQ_ERR_ARG;
    return icq_launch_build_lut(ix, queries, Q, lut, (hipStream_t)stream);
}
