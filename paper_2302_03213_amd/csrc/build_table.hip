// Offline table construction (arXiv 2302.03213, Eq. 3) and symmetric INT8 scalar quantisation of the
// table (Sec. 3.3) for gfx950.  Not on the timed path: clarity over speed, and no workspace - the
// INT8 path recomputes the fp32 entry (V fused multiply-adds) in each pass instead of storing it.
//
//   T[c][k][m] = sum_v P[c][k][v] * W[cV+v][m]          fp32, v ascending, one fma per term
//   s = max|T| / 127 (1 if the table is all zero),  q = clamp(rint(T / s), -127, 127)
//   INT4 (n = 4 in the same formula): 7 in place of 127, two entries per byte.
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

__global__ void table_f32_kernel(const float* __restrict__ P, const float* __restrict__ W, int64_t ldw,
                                 int C, int K, int V, int M, float* __restrict__ T) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)C * K * M) return;
    const int m = (int)(i % M);
    const int k = (int)((i / M) % K);
    const int c = (int)(i / ((int64_t)M * K));
    T[i] = table_entry(P, W, ldw, K, V, c, k, m);
}

__global__ void fill_u32_kernel(uint32_t* p, uint32_t v) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *p = v;
}

// max |T| over the layer.  Non-negative floats order like their bit patterns, so the running
// maximum is kept with an integer atomicMax on the bits of *amax_bits.
__global__ void table_amax_kernel(const float* __restrict__ P, const float* __restrict__ W, int64_t ldw,
                                  int C, int K, int V, int M, uint32_t* amax_bits) {
    const int64_t total = (int64_t)C * K * M;
    float a = 0.f;
    for (int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x; i < total;
         i += (int64_t)gridDim.x * kThreads) {
        const int m = (int)(i % M);
        const int k = (int)((i / M) % K);
        const int c = (int)(i / ((int64_t)M * K));
        a = fmaxf(a, fabsf(table_entry(P, W, ldw, K, V, c, k, m)));
    }
    for (int off = 32; off > 0; off >>= 1) a = fmaxf(a, __shfl_xor(a, off));
    if ((threadIdx.x & 63) == 0) atomicMax(amax_bits, __float_as_uint(a));
}

__global__ void table_quant_kernel(const float* __restrict__ P, const float* __restrict__ W,
                                   int64_t ldw, int C, int K, int V, int M,
                                   const float* __restrict__ amax, int8_t* __restrict__ T) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)C * K * M) return;
    const int m = (int)(i % M);
    const int k = (int)((i / M) % K);
    const int c = (int)(i / ((int64_t)M * K));
    const float s = scale_from_amax(*amax, 127.f);
    T[i] = (int8_t)quantise(table_entry(P, W, ldw, K, V, c, k, m), s, 127.f);
}

// INT4 storage: byte j of row (c, k) holds columns 2j (low nibble) and 2j+1 (high nibble, 0 past M).
__global__ void table_quant_i4_kernel(const float* __restrict__ P, const float* __restrict__ W,
                                      int64_t ldw, int C, int K, int V, int M,
                                      const float* __restrict__ amax, uint8_t* __restrict__ T) {
    const int Mb = (M + 1) / 2;
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)C * K * Mb) return;
    const int j = (int)(i % Mb);
    const int k = (int)((i / Mb) % K);
    const int c = (int)(i / ((int64_t)Mb * K));
    const float s = scale_from_amax(*amax, 7.f);
    const int lo = (int)quantise(table_entry(P, W, ldw, K, V, c, k, 2 * j), s, 7.f);
    const int hi = 2 * j + 1 < M ? (int)quantise(table_entry(P, W, ldw, K, V, c, k, 2 * j + 1), s, 7.f) : 0;
    T[i] = (uint8_t)((lo & 0xf) | ((hi & 0xf) << 4));
}

// MFMA operand copy: packed[(c*Kb + kb)][m][kk] = q[c][16*kb + kk][m], zero where k >= K or m >= M.
// One thread writes the 16 bytes of one (c, kb, m).
__global__ void table_pack_kernel(const float* __restrict__ P, const float* __restrict__ W,
                                  int64_t ldw, int C, int K, int V, int M, int Mp, int Kb,
                                  const float* __restrict__ amax, float qmax,
                                  uint4* __restrict__ packed) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= (int64_t)C * Kb * Mp) return;
    const int m = (int)(i % Mp);
    const int kb = (int)((i / Mp) % Kb);
    const int c = (int)(i / ((int64_t)Mp * Kb));
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
    packed[i] = make_uint4(w[0], w[1], w[2], w[3]);
}

__global__ void scale_finalise_kernel(float* scale, float qmax) {
    if (threadIdx.x == 0 && blockIdx.x == 0) *scale = scale_from_amax(*scale, qmax);
}

inline unsigned blocks_for(int64_t total) { return (unsigned)((total + kThreads - 1) / kThreads); }

}  // namespace

hipError_t launch_build_table_f32(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                  int M, float* T, hipStream_t s) {
    const int64_t total = (int64_t)C * K * M;
    hipLaunchKernelGGL(table_f32_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, s, P, W, ldw, C, K,
                       V, M, T);
    return hipGetLastError();
}

hipError_t launch_build_table_i8(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                 int M, int8_t* T, int8_t* packed, float* scale, int bits,
                                 hipStream_t s) {
    const int64_t total = (int64_t)C * K * M;
    const float qmax = bits == 4 ? 7.f : 127.f;
    // *scale holds max|T| (as float bits) between the passes and becomes s in the last one.
    hipLaunchKernelGGL(fill_u32_kernel, dim3(1), dim3(64), 0, s, reinterpret_cast<uint32_t*>(scale), 0u);
    const unsigned amax_blocks = (unsigned)std::min<int64_t>(blocks_for(total), 4096);
    hipLaunchKernelGGL(table_amax_kernel, dim3(amax_blocks), dim3(kThreads), 0, s, P, W, ldw, C, K, V,
                       M, reinterpret_cast<uint32_t*>(scale));
    if (bits == 4)
        hipLaunchKernelGGL(table_quant_i4_kernel, dim3(blocks_for((int64_t)C * K * ((M + 1) / 2))),
                           dim3(kThreads), 0, s, P, W, ldw, C, K, V, M, scale,
                           reinterpret_cast<uint8_t*>(T));
    else
        hipLaunchKernelGGL(table_quant_kernel, dim3(blocks_for(total)), dim3(kThreads), 0, s, P, W, ldw,
                           C, K, V, M, scale, T);
    if (packed) {
        const int Kb = kblocks(K);
        const int Mp = (int)packed_cols(M);
        const int64_t ptotal = (int64_t)C * Kb * Mp;
        hipLaunchKernelGGL(table_pack_kernel, dim3(blocks_for(ptotal)), dim3(kThreads), 0, s, P, W, ldw,
                           C, K, V, M, Mp, Kb, scale, qmax, reinterpret_cast<uint4*>(packed));
    }
    hipLaunchKernelGGL(scale_finalise_kernel, dim3(1), dim3(64), 0, s, scale, qmax);
    return hipGetLastError();
}

}  // namespace lutnn
