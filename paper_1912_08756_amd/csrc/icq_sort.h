// Register-resident sort of up to 1024 64-bit keys by one wavefront, and the key
// helpers shared by the kernels that keep nearest-neighbour lists (Sec. 3.4 of
// arxiv 1912.08756: the list of the nearest neighbours found so far).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

typedef unsigned long long u64;
constexpr u64 KEY_PAD = ~0ull;     // sorts behind every real key

// Inverse of icq_order_bits.
__device__ __forceinline__ float icq_unorder_bits(uint32_t u) {
    return __uint_as_float((u & 0x80000000u) ? (u & 0x7fffffffu) : ~u);
}

constexpr int ICQ_SORT_THREADS = 256;   // block size block_sort is written for

// Wavefront scans and reductions on the data-parallel-primitive path of the vector unit: a lane
// reads its neighbour's register directly (row shifts inside the rows of 16 lanes, then lane 15 and
// lane 31 broadcast to the rows after them), so a step is two vector instructions and nothing goes
// through the LDS crossbar -- a shuffle there is a round trip that a dependent chain of six waits
// for six times.  FILL is what a lane without a source adds (the identity of the operation).
template <int CTRL, int ROW_MASK, uint32_t FILL>
__device__ __forceinline__ uint32_t icq_dpp(uint32_t x) {
    return (uint32_t)__builtin_amdgcn_update_dpp((int)FILL, (int)x, CTRL, ROW_MASK, 0xf, false);
}
// inclusive prefix sum over the 64 lanes
__device__ __forceinline__ uint32_t wave_scan_add(uint32_t x) {
    x += icq_dpp<0x111, 0xf, 0u>(x);       // row_shr:1
    x += icq_dpp<0x112, 0xf, 0u>(x);       // row_shr:2
    x += icq_dpp<0x114, 0xf, 0u>(x);       // row_shr:4
    x += icq_dpp<0x118, 0xf, 0u>(x);       // row_shr:8
    x += icq_dpp<0x142, 0xa, 0u>(x);       // row_bcast:15 into rows 1 and 3
    x += icq_dpp<0x143, 0xc, 0u>(x);       // row_bcast:31 into rows 2 and 3
    return x;
}
// minimum over the 64 lanes (wavefront-uniform result); a NaN loses against any number
__device__ __forceinline__ float wave_min_f32(float x) {
    constexpr uint32_t INF = 0x7F800000u;
    x = fminf(x, __uint_as_float(icq_dpp<0x111, 0xf, INF>(__float_as_uint(x))));
    x = fminf(x, __uint_as_float(icq_dpp<0x112, 0xf, INF>(__float_as_uint(x))));
    x = fminf(x, __uint_as_float(icq_dpp<0x114, 0xf, INF>(__float_as_uint(x))));
    x = fminf(x, __uint_as_float(icq_dpp<0x118, 0xf, INF>(__float_as_uint(x))));
    x = fminf(x, __uint_as_float(icq_dpp<0x142, 0xa, INF>(__float_as_uint(x))));
    x = fminf(x, __uint_as_float(icq_dpp<0x143, 0xc, INF>(__float_as_uint(x))));
    return __uint_as_float((uint32_t)__builtin_amdgcn_readlane((int)__float_as_uint(x), 63));
}
// minimum / maximum over the 64 lanes, in every lane
__device__ __forceinline__ uint32_t wave_min_u32(uint32_t x) {
    uint32_t y;
    y = icq_dpp<0x111, 0xf, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    y = icq_dpp<0x112, 0xf, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    y = icq_dpp<0x114, 0xf, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    y = icq_dpp<0x118, 0xf, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    y = icq_dpp<0x142, 0xa, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    y = icq_dpp<0x143, 0xc, 0xFFFFFFFFu>(x); x = y < x ? y : x;
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}
__device__ __forceinline__ uint32_t wave_max_u32(uint32_t x) {
    uint32_t y;
    y = icq_dpp<0x111, 0xf, 0u>(x); x = y > x ? y : x;
    y = icq_dpp<0x112, 0xf, 0u>(x); x = y > x ? y : x;
    y = icq_dpp<0x114, 0xf, 0u>(x); x = y > x ? y : x;
    y = icq_dpp<0x118, 0xf, 0u>(x); x = y > x ? y : x;
    y = icq_dpp<0x142, 0xa, 0u>(x); x = y > x ? y : x;
    y = icq_dpp<0x143, 0xc, 0u>(x); x = y > x ? y : x;
    return (uint32_t)__builtin_amdgcn_readlane((int)x, 63);
}

// Compare-exchange steps j = jmax, jmax/2, .., 1 of bitonic stage k on the element
// a lane holds, against lanes lane^j of its own wavefront (no LDS, no barrier).
__device__ __forceinline__ u64 wave_bitonic_steps(u64 x, int e, int k, int jmax) {
    const int lane = threadIdx.x & 63;
    for (int j = jmax; j > 0; j >>= 1) {
        const u64 y = __shfl_xor(x, j, 64);
        const bool up = (e & k) == 0;            // this run sorts ascending
        const bool low = (lane & j) == 0;        // this lane holds the lower index of the pair
        const bool take_min = up == low;
        x = take_min ? (x < y ? x : y) : (x > y ? x : y);
    }
    return x;
}

// Ascending bitonic sort of keys[0..len), len a power of two >= 2, whole block
// (ICQ_SORT_THREADS threads).  Element e lives on lane e % 64, so every exchange at
// distance < 64 stays inside a wavefront and is done with shuffles; only the
// exchanges at distance >= 64 go through LDS with a barrier.
__device__ inline void block_sort(u64 *keys, int len) {
    const int tid = threadIdx.x;
    // stages k <= 64: entirely inside 64-element groups
    for (int base = 0; base < len; base += ICQ_SORT_THREADS) {
        const int e = base + tid;
        if ((e & ~63) < len) {                   // wavefront-uniform
            u64 x = e < len ? keys[e] : KEY_PAD;
            for (int k = 2; k <= 64 && k <= len; k <<= 1) x = wave_bitonic_steps(x, e, k, k >> 1);
            if (e < len) keys[e] = x;
        }
    }
    __syncthreads();
    for (int k = 128; k <= len; k <<= 1) {
        for (int j = k >> 1; j >= 64; j >>= 1) {
            for (int i = tid; i < len / 2; i += ICQ_SORT_THREADS) {
                const int a = ((i / j) * 2 * j) + (i % j);
                const int b = a + j;
                const bool up = (a & k) == 0;
                const u64 x = keys[a], y = keys[b];
                if ((x > y) == up) {
                    keys[a] = y;
                    keys[b] = x;
                }
            }
            __syncthreads();
        }
        for (int base = 0; base < len; base += ICQ_SORT_THREADS) {
            const int e = base + tid;            // len >= 128 here: every wavefront of the pass is full
            if (e < len) keys[e] = wave_bitonic_steps(keys[e], e, k, 32);
        }
        __syncthreads();
    }
}

// Compare-exchange of the register pairs (r, r | M) of a lane: elements 64*M apart.
template <int M>
__device__ __forceinline__ void reg_exchange(u64 (&x)[16], int E, int k, int lane) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
        if ((r & M) == 0 && (r | M) < E) {
            const bool up = (((r * 64 + lane) & k) == 0);
            const u64 a = x[r], b = x[r | M];
            const bool sw = (a > b) == up;
            x[r] = sw ? b : a;
            x[r | M] = sw ? a : b;
        }
    }
}

// Ascending bitonic sort of keys[0..len) by ONE wavefront, len a power of two, 64 <= len
// <= 1024, entirely in registers: element e sits in register e/64 of lane e%64, so an
// exchange at distance >= 64 pairs two registers of a lane and one at distance < 64 is
// a shuffle; the len/64 elements of a lane are independent, which keeps the shuffles
// pipelined.  keys[len..) is not touched; keys must hold len valid or padding entries.
// No barrier inside: the caller orders the LDS traffic around the call.
__device__ inline void wave_sort(u64 *keys, int len, int lane) {
    const int E = len >> 6;
    u64 x[16];
#pragma unroll
    for (int r = 0; r < 16; ++r) x[r] = r < E ? keys[r * 64 + lane] : KEY_PAD;
    for (int k = 2; k <= len; k <<= 1) {
        for (int j = k >> 1; j >= 64; j >>= 1) {
            switch (j >> 6) {
                case 1: reg_exchange<1>(x, E, k, lane); break;
                case 2: reg_exchange<2>(x, E, k, lane); break;
                case 4: reg_exchange<4>(x, E, k, lane); break;
                default: reg_exchange<8>(x, E, k, lane); break;
            }
        }
        for (int j = (k >> 1) < 32 ? (k >> 1) : 32; j > 0; j >>= 1) {
            const bool low = (lane & j) == 0;
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                if (r < E) {
                    const u64 y = __shfl_xor(x[r], j, 64);
                    const bool up = (((r * 64 + lane) & k) == 0);
                    const bool take_min = up == low;
                    x[r] = take_min ? (x[r] < y ? x[r] : y) : (x[r] > y ? x[r] : y);
                }
            }
        }
    }
#pragma unroll
    for (int r = 0; r < 16; ++r)
        if (r < E) keys[r * 64 + lane] = x[r];
}

// LDS scratch of block_kth.
struct IcqKthShared {
    uint32_t hist[256];
    uint32_t wred[ICQ_SORT_THREADS / 64][2];
};

// The kr-th smallest (1-based) of the values v[u] whose bit u is set in `ok`, taken over
// the whole block of ICQ_SORT_THREADS threads (LPT <= 32 values per thread); at least kr values are flagged.  EXACT: that value (radix select, 8-bit
// digits over the occupied range).  Otherwise a single counting pass over the top 8 bits
// of the occupied range; the result is the largest value of the bin that holds the kr-th
// smallest, i.e. an upper bound that keeps the bin whole.  Every thread calls (barriers).
// WEIGHTED: value v[u] counts wgt[u] times (kr at most the flagged weights' sum, which fits 32 bits).
template <int LPT, bool WEIGHTED>
__device__ __forceinline__ uint32_t block_kth_impl(IcqKthShared &sh, const uint32_t (&v)[LPT], const uint32_t (&wgt)[LPT],
                                                   uint32_t ok, uint32_t kr, bool EXACT, int tid, uint32_t lane, int wave) {
    uint32_t vmin = 0xFFFFFFFFu, vmax = 0u;
#pragma unroll
    for (int u = 0; u < LPT; ++u) {
        if ((ok >> u) & 1u) {
            vmin = v[u] < vmin ? v[u] : vmin;
            vmax = v[u] > vmax ? v[u] : vmax;
        }
    }
    vmin = wave_min_u32(vmin);
    vmax = wave_max_u32(vmax);
    __syncthreads();                       // earlier readers of wred / hist are done
    if (lane == 0) { sh.wred[wave][0] = vmin; sh.wred[wave][1] = vmax; }
    __syncthreads();
#pragma unroll
    for (int w = 0; w < ICQ_SORT_THREADS / 64; ++w) {
        const uint32_t a = sh.wred[w][0], b = sh.wred[w][1];
        vmin = a < vmin ? a : vmin;
        vmax = b > vmax ? b : vmax;
    }
    const uint32_t range = vmax - vmin;
    const int bits = range == 0 ? 0 : 32 - __builtin_clz(range);
    if (bits == 0) return vmin;
    int shift = bits > 8 ? bits - 8 : 0;
    int width = bits < 8 ? bits : 8;
    uint32_t prefix = 0;       // chosen high digits of (value - vmin)
    int fixed_from = 32;       // bits [fixed_from, 32) of (value - vmin) are decided
    for (;;) {
        sh.hist[tid] = 0;
        __syncthreads();
        const uint32_t dmask = (1u << width) - 1u;
#pragma unroll
        for (int u = 0; u < LPT; ++u) {
            if ((ok >> u) & 1u) {
                const uint32_t y = v[u] - vmin;
                const bool match = fixed_from >= 32 ? true : (y >> fixed_from) == prefix;
                if (match) atomicAdd(&sh.hist[(y >> shift) & dmask], WEIGHTED ? wgt[u] : 1u);
            }
        }
        __syncthreads();
        // every wavefront locates the bin by itself (4 bins per lane)
        uint32_t h[4], mine = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            h[r] = sh.hist[lane * 4 + r];
            mine += h[r];
        }
        const uint32_t incl = wave_scan_add(mine);
        const int L = __builtin_ctzll(__builtin_amdgcn_ballot_w64(incl >= kr));
        uint32_t run = incl - mine, my_bin = 0, my_below = 0;
#pragma unroll
        for (int r = 0; r < 4; ++r) {
            if (run < kr && run + h[r] >= kr) {
                my_bin = lane * 4 + r;
                my_below = run;
            }
            run += h[r];
        }
        const uint32_t bin = (uint32_t)__builtin_amdgcn_readlane((int)my_bin, L);
        const uint32_t below = (uint32_t)__builtin_amdgcn_readlane((int)my_below, L);
        kr -= below;
        prefix = (prefix << width) | bin;
        fixed_from = shift;
        if (!EXACT || shift == 0) break;
        const int ns = shift > 8 ? shift - 8 : 0;
        width = shift - ns;
        shift = ns;
        __syncthreads();                   // every wavefront has read the histogram
    }
    if (shift == 0) return vmin + prefix;
    const unsigned long long top = (unsigned long long)vmin + ((((unsigned long long)prefix + 1ull) << shift) - 1ull);
    return top < (unsigned long long)vmax ? (uint32_t)top : vmax;
}
template <int LPT>
__device__ __forceinline__ uint32_t block_kth(IcqKthShared &sh, const uint32_t (&v)[LPT], uint32_t ok, uint32_t kr,
                                              bool EXACT, int tid, uint32_t lane, int wave) {
    return block_kth_impl<LPT, false>(sh, v, v, ok, kr, EXACT, tid, lane, wave);
}
// One counting pass with weights: the top of the first bin at which the weights of the flagged
// values at or below it add up to kr or more.
template <int LPT>
__device__ __forceinline__ uint32_t block_kth_weighted(IcqKthShared &sh, const uint32_t (&v)[LPT], const uint32_t (&wgt)[LPT],
                                                       uint32_t ok, uint32_t kr, int tid, uint32_t lane, int wave) {
    return block_kth_impl<LPT, true>(sh, v, wgt, ok, kr, false, tid, lane, wave);
}

