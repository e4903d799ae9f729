// Machine-limit probes: a few plain kernels that show what one MI355X delivers for the access
// patterns the search kernels are made of -- a streaming read, LDS table reads of 4, 8 and 16
// bytes, plain vector arithmetic, the single-precision matrix instruction, atomics on one address.  The rooflines of the search kernels are
// judged against these figures next to the published peaks.  A measurement aid; nothing on the
// search path calls it.
#include "icq_internal.h"

namespace {

constexpr int PB_THREADS = 1024;

// Contiguous block ranges, U 128-bit loads in flight per thread, never conditional.
template <int U, bool NT>
__global__ __launch_bounds__(PB_THREADS) void probe_read_kernel(const uint4 *__restrict__ p, size_t n, uint32_t *out) {
    const size_t per = (n + gridDim.x - 1) / gridDim.x;
    const size_t b = blockIdx.x * per, e = b + per < n ? b + per : n;
    uint32_t acc = 0;
    for (size_t i = b + threadIdx.x; i < e; i += (size_t)blockDim.x * U) {
        uint4 v[U];
#pragma unroll
        for (int u = 0; u < U; ++u) {
            const size_t j = i + (size_t)u * blockDim.x;
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 *src = reinterpret_cast<const u32x4 *>(p + (j < e ? j : b));
            const u32x4 t = NT ? __builtin_nontemporal_load(src) : *src;
            v[u] = make_uint4(t.x, t.y, t.z, t.w);
        }
#pragma unroll
        for (int u = 0; u < U; ++u) acc += v[u].x ^ v[u].y ^ v[u].z ^ v[u].w;
    }
    if (acc == 0x12345678u) out[0] = acc;       // keeps the loads alive
}

// Every lane reads WIDTH dwords from a pseudo-random row of a table laid out so that the 64 lanes of
// a read fall into consecutive words (no bank conflicts): the rate the LDS serves table reads at best.
template <int WIDTH>
__global__ __launch_bounds__(PB_THREADS, 1) void probe_lds_kernel(float *out, int iters) {
    __shared__ __attribute__((aligned(16))) float smem[128 * 64 * 4];       // 128 KB
    constexpr int ROWS = 128 * 4 / WIDTH;
    for (int i = threadIdx.x; i < 128 * 64 * 4; i += blockDim.x) smem[i] = (float)(i & 7);
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    float a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    uint32_t r = wave * 7 + 1;
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
            r += 0x9E3779B1u;
            const uint32_t row = (r >> 16) & (uint32_t)(ROWS - 1);
            if (WIDTH == 1) {
                const float v = smem[row * 64 + lane];
                if (u & 1) a0 += v; else a1 += v;
            } else if (WIDTH == 2) {
                const float2 v = reinterpret_cast<const float2 *>(smem)[row * 64 + lane];
                a0 += v.x; a1 += v.y;
            } else {
                const float4 v = reinterpret_cast<const float4 *>(smem)[row * 64 + lane];
                a0 += v.x; a1 += v.y; a2 += v.z; a3 += v.w;
            }
        }
    }
    out[blockIdx.x * blockDim.x + threadIdx.x] = a0 + a1 + a2 + a3;
}

// Eight independent chains of plain (not packed) vector additions per lane.
__global__ __launch_bounds__(PB_THREADS, 1) void probe_valu_kernel(float *out, int iters) {
    float a[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a[j] = (float)(threadIdx.x + j);
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 16; ++u) {
#pragma unroll
            for (int j = 0; j < 8; ++j) asm volatile("v_add_f32 %0, 1.0, %0" : "+v"(a[j]));
        }
    }
    float s = 0;
#pragma unroll
    for (int j = 0; j < 8; ++j) s += a[j];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// Four independent accumulators of the single-precision 32x32x2 matrix instruction per wavefront,
// operands in registers: the rate the matrix cores sustain for the table build's instruction.
// RANDOM: the operands are 32 different pseudo-random values per lane, full mantissas (what real
// data looks like to the multipliers); otherwise two small integers.
template <bool RANDOM>
__global__ __launch_bounds__(256) void probe_mfma_kernel(float *out, int iters) {
    typedef float float16v __attribute__((ext_vector_type(16)));
    float16v acc[4];
#pragma unroll
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) acc[j][v] = 0.0f;
    float a[16], b[16];
    uint32_t r = (blockIdx.x * blockDim.x + threadIdx.x) * 2654435761u + 12345u;
#pragma unroll
    for (int u = 0; u < 16; ++u) {
        if (RANDOM) {
            r = r * 1664525u + 1013904223u;
            a[u] = __uint_as_float(0x3F800000u | (r >> 9)) - 1.5f;      // uniform in [-0.5, 0.5)
            r = r * 1664525u + 1013904223u;
            b[u] = __uint_as_float(0x3F800000u | (r >> 9)) - 1.5f;
        } else {
            a[u] = (float)(threadIdx.x & 7);
            b[u] = (float)(threadIdx.x & 3);
        }
    }
    for (int it = 0; it < iters; ++it) {
#pragma unroll
        for (int u = 0; u < 4; ++u) {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                acc[j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[4 * u + j], b[4 * u + j], acc[j], 0, 0, 0);
        }
    }
    float s = 0;
#pragma unroll
    for (int j = 0; j < 4; ++j)
        for (int v = 0; v < 16; ++v) s += acc[j][v];
    out[blockIdx.x * blockDim.x + threadIdx.x] = s;
}

// One atomic per wavefront and iteration, all on the same word.
__global__ __launch_bounds__(PB_THREADS) void probe_atomic_kernel(uint32_t *counter, int iters) {
    if ((threadIdx.x & 63) != 0) return;
    for (int it = 0; it < iters; ++it) atomicAdd(counter, 1u);
}

}  // namespace

ICQ_EXPORT int icq_machine_probe(int kind, void *buffer, size_t bytes, int reps, double *ms_out, double *units_out,
                                 void *stream) {
    if (kind < ICQ_PROBE_READ || kind > ICQ_PROBE_MFMA_F32_RANDOM || !buffer || bytes < (1u << 22) || reps < 1 || !ms_out ||
        !units_out || ((uintptr_t)buffer % 16) != 0)
        return ICQ_ERR_ARG;
    hipStream_t s = (hipStream_t)stream;
    int dev = 0;
    hipDeviceProp_t prop;
    if (hipGetDevice(&dev) != hipSuccess || hipGetDeviceProperties(&prop, dev) != hipSuccess) return ICQ_ERR_HIP;
    const int cus = prop.multiProcessorCount > 0 ? prop.multiProcessorCount : 256;
    const int iters = 2000;
    double units = 0.0;
    auto launch = [&]() {
        switch (kind) {
            case ICQ_PROBE_READ:
            case ICQ_PROBE_READ_NT: {
                const size_t n = bytes / 16;
                if (kind == ICQ_PROBE_READ)
                    probe_read_kernel<4, false><<<cus, PB_THREADS, 0, s>>>(static_cast<const uint4 *>(buffer), n,
                                                                          static_cast<uint32_t *>(buffer));
                else
                    probe_read_kernel<4, true><<<cus, PB_THREADS, 0, s>>>(static_cast<const uint4 *>(buffer), n,
                                                                         static_cast<uint32_t *>(buffer));
                units = (double)n * 16.0;                               // bytes read
                break;
            }
            case ICQ_PROBE_LDS_B32:
                probe_lds_kernel<1><<<cus, PB_THREADS, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * PB_THREADS * iters * 16.0;        // lane reads (addresses)
                break;
            case ICQ_PROBE_LDS_B64:
                probe_lds_kernel<2><<<cus, PB_THREADS, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * PB_THREADS * iters * 16.0;
                break;
            case ICQ_PROBE_LDS_B128:
                probe_lds_kernel<4><<<cus, PB_THREADS, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * PB_THREADS * iters * 16.0;
                break;
            case ICQ_PROBE_VALU:
                probe_valu_kernel<<<cus, PB_THREADS, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * PB_THREADS * iters * 16.0 * 8.0;  // lane operations
                break;
            case ICQ_PROBE_MFMA_F32:
                // 8 blocks of 4 wavefronts per CU; 32*32*2 multiply-adds per instruction
                probe_mfma_kernel<false><<<cus * 8, 256, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * 8 * 4 * iters * 16.0 * 4096.0;   // floating-point operations
                break;
            case ICQ_PROBE_MFMA_F32_RANDOM:
                probe_mfma_kernel<true><<<cus * 8, 256, 0, s>>>(static_cast<float *>(buffer), iters);
                units = (double)cus * 8 * 4 * iters * 16.0 * 4096.0;
                break;
            default:
                probe_atomic_kernel<<<cus, PB_THREADS, 0, s>>>(static_cast<uint32_t *>(buffer), 64);
                units = (double)cus * (PB_THREADS / 64) * 64.0;         // atomics
                break;
        }
    };
    hipEvent_t a, b;
    if (hipEventCreate(&a) != hipSuccess) return ICQ_ERR_HIP;
    if (hipEventCreate(&b) != hipSuccess) {
        (void)hipEventDestroy(a);
        return ICQ_ERR_HIP;
    }
    launch();                                                           // warm-up
    int rc = ICQ_OK;
    float ms = 0.0f;
    if (hipEventRecord(a, s) != hipSuccess) rc = ICQ_ERR_HIP;
    for (int i = 0; i < reps && rc == ICQ_OK; ++i) launch();
    if (rc == ICQ_OK && (hipEventRecord(b, s) != hipSuccess || hipEventSynchronize(b) != hipSuccess ||
                         hipEventElapsedTime(&ms, a, b) != hipSuccess || hipGetLastError() != hipSuccess))
        rc = ICQ_ERR_HIP;
    (void)hipEventDestroy(a);
    (void)hipEventDestroy(b);
    if (rc != ICQ_OK) return rc;
    *ms_out = (double)ms / reps;
    *units_out = units;
    return ICQ_OK;
}
