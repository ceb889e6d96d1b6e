// Table read and accumulation (arXiv 2302.03213, Eq. 4) with 16-bit indices: the lookup behind the
// hash encoder's deep trees (Sec. 2, Sec. 7: up to 12 levels, K = 4096 buckets per codebook).
//
// With thousands of table rows per codebook nothing of the table can be staged or turned into a
// matrix operand: a (row, codebook) pair selects one of K rows of M entries, which is read straight
// from global memory.  One wavefront owns one input row and a run of 256 output columns; the
// index is wave-uniform (a scalar load), each lane reads four consecutive columns of the selected
// table row (the wavefront's loads are contiguous) and adds them to its accumulators, codebooks in
// ascending order: exact int32 for INT8 tables, fp32 in a fixed order for fp32 tables.  Four
// codebooks are in flight at once.
#include <type_traits>

#include "lutnn_kernels.h"

namespace lutnn {
namespace {

constexpr int kWideThreads = 256;  // 4 wavefronts = 4 (row, column chunk) pairs
constexpr int kWideCols = 256;     // columns per wavefront

__device__ __forceinline__ void add4(int32_t (&acc)[4], uint32_t v) {
    acc[0] += (int32_t)(int8_t)(v & 0xff);
    acc[1] += (int32_t)(int8_t)((v >> 8) & 0xff);
    acc[2] += (int32_t)(int8_t)((v >> 16) & 0xff);
    acc[3] += (int32_t)(int8_t)(v >> 24);
}
__device__ __forceinline__ void add4(float (&acc)[4], float4 v) {
    acc[0] += v.x;
    acc[1] += v.y;
    acc[2] += v.z;
    acc[3] += v.w;
}

// VEC: M % 4 == 0 and the table aligned for a four-column load; otherwise column by column.
template <typename TT, bool VEC>
__global__ __launch_bounds__(kWideThreads) void lookup_wide_kernel(
    const TT* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias, int C,
    int K, int M, const uint16_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy,
    int col_chunks) {
    constexpr bool I8 = sizeof(TT) == 1;
    typedef typename std::conditional<I8, int32_t, float>::type Acc;
    typedef typename std::conditional<I8, uint32_t, float4>::type Vec;
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t unit = (int64_t)blockIdx.x * (kWideThreads / 64) + w;  // wave-uniform
    if (unit >= N * col_chunks) return;
    const int64_t n = unit / col_chunks;
    const int m0 = (int)(unit % col_chunks) * kWideCols + 4 * lane;
    const uint16_t* __restrict__ row_idx = idx + n * C;

    Acc acc[4] = {0, 0, 0, 0};
    auto table_row = [&](int c) {
        int k = row_idx[c];  // wave-uniform
        k = k < K ? k : K - 1;
        return T + ((size_t)c * K + k) * M;
    };
    auto add_row = [&](const TT* __restrict__ r) {
        if constexpr (VEC) {
            if (m0 < M) add4(acc, *reinterpret_cast<const Vec*>(r + m0));
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j)
                if (m0 + j < M) acc[j] += (Acc)r[m0 + j];
        }
    };
    int c = 0;
    for (; c + 4 <= C; c += 4) {  // four independent loads before the first add
        const TT* r0 = table_row(c);
        const TT* r1 = table_row(c + 1);
        const TT* r2 = table_row(c + 2);
        const TT* r3 = table_row(c + 3);
        if constexpr (VEC) {
            if (m0 < M) {
                const Vec v0 = *reinterpret_cast<const Vec*>(r0 + m0);
                const Vec v1 = *reinterpret_cast<const Vec*>(r1 + m0);
                const Vec v2 = *reinterpret_cast<const Vec*>(r2 + m0);
                const Vec v3 = *reinterpret_cast<const Vec*>(r3 + m0);
                add4(acc, v0);
                add4(acc, v1);
                add4(acc, v2);
                add4(acc, v3);
            }
        } else {
            add_row(r0);
            add_row(r1);
            add_row(r2);
            add_row(r3);
        }
    }
    for (; c < C; ++c) add_row(table_row(c));

    float* __restrict__ y = Y + n * ldy;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        const int m = m0 + j;
        if (m >= M) continue;
        if constexpr (I8)
            y[m] = bias ? __fmaf_rn((float)acc[j], *scale, bias[m]) : __fmul_rn((float)acc[j], *scale);
        else
            y[m] = bias ? acc[j] + bias[m] : acc[j];
    }
}

template <typename TT>
hipError_t launch_wide(const TT* T, const float* scale, const float* bias, int C, int K, int M,
                       const uint16_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    const int col_chunks = (M + kWideCols - 1) / kWideCols;
    const int64_t units = N * col_chunks;
    const int64_t blocks = (units + kWideThreads / 64 - 1) / (kWideThreads / 64);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool vec = M % 4 == 0 && (reinterpret_cast<uintptr_t>(T) & (4 * sizeof(TT) - 1)) == 0;
    if (vec)
        hipLaunchKernelGGL((lookup_wide_kernel<TT, true>), dim3((unsigned)blocks), dim3(kWideThreads), 0, s, T,
                           scale, bias, C, K, M, idx, N, Y, ldy, col_chunks);
    else
        hipLaunchKernelGGL((lookup_wide_kernel<TT, false>), dim3((unsigned)blocks), dim3(kWideThreads), 0, s, T,
                           scale, bias, C, K, M, idx, N, Y, ldy, col_chunks);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_lookup_wide_i8(const int8_t* T, const float* scale, const float* bias, int C, int K, int M,
                                 const uint16_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    return launch_wide<int8_t>(T, scale, bias, C, K, M, idx, N, Y, ldy, s);
}

hipError_t launch_lookup_wide_f32(const float* T, const float* bias, int C, int K, int M, const uint16_t* idx,
                                  int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    return launch_wide<float>(T, nullptr, bias, C, K, M, idx, N, Y, ldy, s);
}

}  // namespace lutnn
