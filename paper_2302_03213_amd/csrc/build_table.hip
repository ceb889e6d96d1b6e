// Offline table construction (arXiv 2302.03213, Eq. 3) and symmetric INT8 scalar quantisation of the
// table (Sec. 3.3) for gfx950.  Offline for inference, but training rebuilds the table from the
// updated centroids in every forward pass (Sec. 3.1), so it is kept to two passes over the table:
// max |T|, then quantise and write both layouts.  No workspace - each pass recomputes the fp32
// entry (V fused multiply-adds) instead of storing it.  Grids are (column block, codebook x
// centroid) so that no thread divides.
//
//   T[c][k][m] = sum_v P[c][k][v] * W[cV+v][m]          fp32, v ascending, one fma per term
//   s = max|T| / 127 (1 if the table is all zero),  q = clamp(rint(T / s), -127, 127)
//   INT4 (n = 4 in the same formula): 7 in place of 127, two entries per byte.
#include <algorithm>

#include "lutnn_kernels.h"

namespace lutnn {
namespace {

constexpr int kThreads = 256;

__device__ __forceinline__ float table_entry(const float* __restrict__ P,
                                             const float* __restrict__ W, int64_t ldw, int K, int V,
                                             int c, int k, int m) {
    const float* p = P + ((size_t)c * K + k) * V;
    const float* w = W + (size_t)c * V * ldw + m;
    float acc = 0.f;
    for (int v = 0; v < V; ++v) acc = __fmaf_rn(p[v], w[(size_t)v * ldw], acc);
    return acc;
}

// qmax = 2^(n-1) - 1: 127 for INT8, 7 for INT4.
__device__ __forceinline__ float quantise(float t, float s, float qmax) {
    float r = rintf(__fdiv_rn(t, s));  // IEEE division, round half to even
    r = fminf(fmaxf(r, -qmax), qmax);
    return r;
}

__device__ __forceinline__ float scale_from_amax(float amax, float qmax) {
    return amax == 0.f ? 1.f : __fdiv_rn(amax, qmax);
}

// Grid for the per-entry kernels: blockIdx.x = c*K + k (one table row), blockIdx.y = block of 256
// columns.  The row index is wave-uniform, so its division is scalar work done once.
__global__ __launch_bounds__(kThreads) void table_f32_kernel(const float* __restrict__ P,
                                                             const float* __restrict__ W, int64_t ldw, int K,
                                                             int V, int M, float* __restrict__ T) {
    const int m = blockIdx.y * kThreads + threadIdx.x;
    if (m >= M) return;
    const int c = blockIdx.x / K, k = blockIdx.x % K;
    T[(size_t)blockIdx.x * M + m] = table_entry(P, W, ldw, K, V, c, k, m);
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

// max |T| over the layer.  Non-negative floats order like their bit patterns, so the running
// maximum is kept with an integer atomicMax on the bits of *amax_bits.  One thread owns (c, block of
// 16 centroids, column m), like the quantising pass below: the 16 centroids of a codebook share the
// V weights of the column.  A wavefront issues its atomic only when its value exceeds the maximum
// it can see (a stale, smaller reading costs an unnecessary atomic, never a missed one): tens of
// thousands of atomics on one address would take longer than the arithmetic.
// grid: blockIdx.x = c*Kb + kb, blockIdx.y = block of 256 columns.
__global__ __launch_bounds__(kThreads) void table_amax_kernel(const float* __restrict__ P,
                                                              const float* __restrict__ W, int64_t ldw, int K,
                                                              int V, int M, int Kb, uint32_t* amax_bits) {
    const int m = blockIdx.y * kThreads + threadIdx.x;
    const int c = blockIdx.x / Kb, kb = blockIdx.x % Kb;
    float a = 0.f;
    if (m < M) {
        for (int kk = 0; kk < 16; ++kk) {
            const int k = kb * 16 + kk;
            if (k >= K) break;
            a = fmaxf(a, fabsf(table_entry(P, W, ldw, K, V, c, k, m)));
        }
    }
    for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
    if ((threadIdx.x & 63) == 0) {
        const uint32_t mine = __float_as_uint(a);
        if (mine > __atomic_load_n(amax_bits, __ATOMIC_RELAXED)) atomicMax(amax_bits, mine);
    }
}

// INT8: quantises and writes both layouts in one pass.  One thread owns (c, block of 16 centroids,
// column m): its 16 codes are the 16 bytes of packed[(c*Kb + kb)][m][0..15] (zero where k >= K or
// m >= M) and one byte in each of 16 rows of T[c][k][m]; neighbouring threads are neighbouring
// columns, so every one of those row writes is contiguous across the wavefront.
// grid: blockIdx.x = c*Kb + kb, blockIdx.y = block of 256 columns of the padded width Mp.
__global__ __launch_bounds__(kThreads) void table_quant_pack_kernel(
    const float* __restrict__ P, const float* __restrict__ W, int64_t ldw, int K, int V, int M, int Mp,
    int Kb, const float* __restrict__ amax, int8_t* __restrict__ T, uint4* __restrict__ packed) {
    const int m = blockIdx.y * kThreads + threadIdx.x;
    if (m >= Mp) return;
    const int c = blockIdx.x / Kb, kb = blockIdx.x % Kb;
    const float s = scale_from_amax(*amax, 127.f);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (m < M) {
        for (int kk = 0; kk < 16; ++kk) {
            const int k = kb * 16 + kk;
            if (k >= K) break;
            const int q = (int)quantise(table_entry(P, W, ldw, K, V, c, k, m), s, 127.f);
            T[((size_t)c * K + k) * M + m] = (int8_t)q;
            w[kk >> 2] |= (uint32_t)(q & 0xff) << (8 * (kk & 3));
        }
    }
    if (packed) packed[(size_t)blockIdx.x * Mp + m] = make_uint4(w[0], w[1], w[2], w[3]);
}

// INT4 storage: byte j of row (c, k) holds columns 2j (low nibble) and 2j+1 (high nibble, 0 past M).
// grid: blockIdx.x = c*K + k, blockIdx.y = block of 256 bytes.
__global__ __launch_bounds__(kThreads) void table_quant_i4_kernel(
    const float* __restrict__ P, const float* __restrict__ W, int64_t ldw, int K, int V, int M,
    const float* __restrict__ amax, uint8_t* __restrict__ T) {
    const int Mb = (M + 1) / 2;
    const int j = blockIdx.y * kThreads + threadIdx.x;
    if (j >= Mb) return;
    const int c = blockIdx.x / K, k = blockIdx.x % K;
    const float s = scale_from_amax(*amax, 7.f);
    const int lo = (int)quantise(table_entry(P, W, ldw, K, V, c, k, 2 * j), s, 7.f);
    const int hi = 2 * j + 1 < M ? (int)quantise(table_entry(P, W, ldw, K, V, c, k, 2 * j + 1), s, 7.f) : 0;
    T[(size_t)blockIdx.x * Mb + j] = (uint8_t)((lo & 0xf) | ((hi & 0xf) << 4));
}

// MFMA operand copy alone (INT4 tables, whose T has its own layout):
// packed[(c*Kb + kb)][m][kk] = q[c][16*kb + kk][m], zero where k >= K or m >= M.
// grid as table_quant_pack_kernel.
__global__ __launch_bounds__(kThreads) void table_pack_kernel(const float* __restrict__ P,
                                                              const float* __restrict__ W, int64_t ldw, int K,
                                                              int V, int M, int Mp, int Kb,
                                                              const float* __restrict__ amax, float qmax,
                                                              uint4* __restrict__ packed) {
    const int m = blockIdx.y * kThreads + threadIdx.x;
    if (m >= Mp) return;
    const int c = blockIdx.x / Kb, kb = blockIdx.x % Kb;
    const float s = scale_from_amax(*amax, qmax);
    uint32_t w[4] = {0u, 0u, 0u, 0u};
    if (m < M) {
        for (int kk = 0; kk < 16; ++kk) {
            const int k = kb * 16 + kk;
            if (k >= K) break;
            const int q = (int)quantise(table_entry(P, W, ldw, K, V, c, k, m), s, qmax);
            w[kk >> 2] |= (uint32_t)(q & 0xff) << (8 * (kk & 3));
        }
    }
    packed[(size_t)blockIdx.x * Mp + m] = make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ void scale_finalise_kernel(float* scale, float qmax) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *scale = scale_from_amax(*scale, qmax);
}

inline unsigned col_blocks(int64_t cols) { return (unsigned)((cols + kThreads - 1) / kThreads); }

}  // namespace

// Callers guarantee C*K < 2^31 (grid.x) and M <= 2^24 (grid.y <= 65536).
hipError_t launch_build_table_f32(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                  int M, float* T, hipStream_t s) {
    hipLaunchKernelGGL(table_f32_kernel, dim3((unsigned)C * K, col_blocks(M)), dim3(kThreads), 0, s, P, W,
                       ldw, K, V, M, T);
    return hipGetLastError();
}

hipError_t launch_build_table_i8(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                 int M, int8_t* T, int8_t* packed, float* scale, int bits,
                                 hipStream_t s) {
    const float qmax = bits == 4 ? 7.f : 127.f;
    const int Kb = kblocks(K);
    const int Mp = (int)packed_cols(M);
    // *scale holds max|T| (as float bits) between the passes and becomes s in the last one.
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(scale), 0u);
    hipLaunchKernelGGL(table_amax_kernel, dim3((unsigned)C * Kb, col_blocks(M)), dim3(kThreads), 0, s, P, W,
                       ldw, K, V, M, Kb, reinterpret_cast<uint32_t*>(scale));
    if (bits == 4) {
        hipLaunchKernelGGL(table_quant_i4_kernel, dim3((unsigned)C * K, col_blocks((M + 1) / 2)),
                           dim3(kThreads), 0, s, P, W, ldw, K, V, M, scale, reinterpret_cast<uint8_t*>(T));
        if (packed)
            hipLaunchKernelGGL(table_pack_kernel, dim3((unsigned)C * Kb, col_blocks(Mp)), dim3(kThreads), 0, s,
                               P, W, ldw, K, V, M, Mp, Kb, scale, qmax, reinterpret_cast<uint4*>(packed));
    } else {
        // without a packed copy only the M real columns need threads
        hipLaunchKernelGGL(table_quant_pack_kernel, dim3((unsigned)C * Kb, col_blocks(packed ? Mp : M)),
                           dim3(kThreads), 0, s, P, W, ldw, K, V, M, Mp, Kb, scale, T,
                           reinterpret_cast<uint4*>(packed));
    }
    hipLaunchKernelGGL(scale_finalise_kernel, dim3(1), dim3(64), 0, s, scale, qmax);
    return hipGetLastError();
}

}  // namespace lutnn
