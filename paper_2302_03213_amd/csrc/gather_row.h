// One output row's share of the table read and accumulation (arXiv 2302.03213, Eq. 4) when the
// table rows are read straight from global memory: a lane owns four consecutive columns and adds
// the selected row of every codebook, in codebook order, sixteen loads in flight at a time.
// Shared by the stand-alone gather kernel and the one-launch kernel for small problems.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include <type_traits>

namespace lutnn {

//   T       table, fp32 or int8, [C][K][M]; M % 4 == 0 and T aligned for a four-column load
//   irow    this row's C index bytes (global memory or LDS); IDX_DWORD: 4-byte aligned, read
//           four codebooks at a time
//   m       first of the lane's four columns (< M)
//   yrow    &Y[row][0]
//   UNIFORM the whole wavefront works on the same row: index words are made wave-uniform
template <typename TT, bool IDX_DWORD, bool UNIFORM>
__device__ __forceinline__ void gather_row(const TT* __restrict__ T, const float* __restrict__ scale,
                                           const float* __restrict__ bias, int C, int K, int M,
                                           const uint8_t* __restrict__ irow, int m, float* __restrict__ yrow) {
    constexpr bool I8 = sizeof(TT) == 1;
    typedef typename std::conditional<I8, uint32_t, float4>::type Vec;  // four columns
    auto uni = [](uint32_t x) { return UNIFORM ? (uint32_t)__builtin_amdgcn_readfirstlane(x) : x; };
    const TT* __restrict__ tcol = T + m;

    float fa[4] = {0.f, 0.f, 0.f, 0.f};
    int32_t ia[4] = {0, 0, 0, 0};
    auto accumulate = [&](const Vec& v) {
        if constexpr (I8) {
            ia[0] += (int32_t)(int8_t)(v & 0xffu);
            ia[1] += (int32_t)(int8_t)((v >> 8) & 0xffu);
            ia[2] += (int32_t)(int8_t)((v >> 16) & 0xffu);
            ia[3] += (int32_t)v >> 24;
        } else {
            fa[0] += v.x;
            fa[1] += v.y;
            fa[2] += v.z;
            fa[3] += v.w;
        }
    };
    auto add = [&](int c, int k) {
        k = k < K ? k : K - 1;
        accumulate(*reinterpret_cast<const Vec*>(tcol + ((size_t)c * K + k) * M));
    };
    int c = 0;
    if (IDX_DWORD) {
        // sixteen table rows in flight at a time (added in codebook order all the same)
        for (; c + 16 <= C; c += 16) {
            uint32_t word[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) word[q] = uni(*reinterpret_cast<const uint32_t*>(irow + c + 4 * q));
            Vec v[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                int k = (int)((word[b >> 2] >> (8 * (b & 3))) & 0xffu);
                k = k < K ? k : K - 1;
                v[b] = *reinterpret_cast<const Vec*>(tcol + ((size_t)(c + b) * K + k) * M);
            }
#pragma unroll
            for (int b = 0; b < 16; ++b) accumulate(v[b]);
        }
        for (; c + 4 <= C; c += 4) {
            const uint32_t word = uni(*reinterpret_cast<const uint32_t*>(irow + c));
#pragma unroll
            for (int b = 0; b < 4; ++b) add(c + b, (int)((word >> (8 * b)) & 0xffu));
        }
    }
    for (; c < C; ++c) add(c, (int)uni((uint32_t)irow[c]));

    float* __restrict__ y = yrow + m;
    float4 out;
    if constexpr (I8) {
        const float s = *scale;
        if (bias) {
            out = make_float4(__fmaf_rn((float)ia[0], s, bias[m]), __fmaf_rn((float)ia[1], s, bias[m + 1]),
                              __fmaf_rn((float)ia[2], s, bias[m + 2]), __fmaf_rn((float)ia[3], s, bias[m + 3]));
        } else {
            out = make_float4(__fmul_rn((float)ia[0], s), __fmul_rn((float)ia[1], s),
                              __fmul_rn((float)ia[2], s), __fmul_rn((float)ia[3], s));
        }
    } else {
        out = bias ? make_float4(fa[0] + bias[m], fa[1] + bias[m + 1], fa[2] + bias[m + 2], fa[3] + bias[m + 3])
                   : make_float4(fa[0], fa[1], fa[2], fa[3]);
    }
    y[0] = out.x;
    y[1] = out.y;
    y[2] = out.z;
    y[3] = out.w;
}

// The same for a handful of rows: the SPLIT wavefronts of a workgroup share one (row, 256 columns)
// and take a contiguous range of `per_wave` codebooks each (a multiple of 4); the partial sums meet
// in LDS and wavefront 0 adds them in range order (exact for integer tables, a fixed order for fp32
// ones).  Every thread of the workgroup must call it (it holds a barrier); m may lie past M.
template <typename TT, bool IDX_DWORD, int SPLIT>
__device__ __forceinline__ void gather_row_split(const TT* __restrict__ T, const float* __restrict__ scale,
                                                 const float* __restrict__ bias, int C, int K, int M,
                                                 const uint8_t* __restrict__ irow, int m,
                                                 float* __restrict__ yrow, int per_wave) {
    constexpr bool I8 = sizeof(TT) == 1;
    typedef typename std::conditional<I8, uint32_t, float4>::type Vec;  // four columns
    typedef typename std::conditional<I8, int32_t, float>::type Acc;
    __shared__ Acc part[SPLIT][4][64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const bool col_ok = m < M;  // M % 4 == 0: a lane's four columns are all inside or all outside
    const TT* __restrict__ tcol = T + (col_ok ? m : 0);

    Acc a[4] = {0, 0, 0, 0};
    auto accumulate = [&](const Vec& v) {
        if constexpr (I8) {
            a[0] += (int32_t)(int8_t)(v & 0xffu);
            a[1] += (int32_t)(int8_t)((v >> 8) & 0xffu);
            a[2] += (int32_t)(int8_t)((v >> 16) & 0xffu);
            a[3] += (int32_t)v >> 24;
        } else {
            a[0] += v.x;
            a[1] += v.y;
            a[2] += v.z;
            a[3] += v.w;
        }
    };
    auto add = [&](int c, int k) {
        k = k < K ? k : K - 1;
        accumulate(*reinterpret_cast<const Vec*>(tcol + ((size_t)c * K + k) * M));
    };
    // codebooks [c, c_end) of this wavefront; per_wave is a multiple of 4, so dword index loads stay aligned
    int c = w * per_wave;
    const int c_end = min(C, c + per_wave);
    if (IDX_DWORD) {
        // sixteen table rows in flight at a time: with so few wavefronts the loop is a latency chain,
        // and a wait per group of four codebooks would be most of the kernel
        for (; c + 16 <= c_end; c += 16) {
            uint32_t word[4];
#pragma unroll
            for (int q = 0; q < 4; ++q)
                word[q] = (uint32_t)__builtin_amdgcn_readfirstlane(*reinterpret_cast<const uint32_t*>(irow + c + 4 * q));
            Vec v[16];
#pragma unroll
            for (int b = 0; b < 16; ++b) {
                int k = (int)((word[b >> 2] >> (8 * (b & 3))) & 0xffu);
                k = k < K ? k : K - 1;
                v[b] = *reinterpret_cast<const Vec*>(tcol + ((size_t)(c + b) * K + k) * M);
            }
#pragma unroll
            for (int b = 0; b < 16; ++b) accumulate(v[b]);
        }
        for (; c + 4 <= c_end; c += 4) {
            const uint32_t word =
                (uint32_t)__builtin_amdgcn_readfirstlane(*reinterpret_cast<const uint32_t*>(irow + c));
#pragma unroll
            for (int b = 0; b < 4; ++b) add(c + b, (int)((word >> (8 * b)) & 0xffu));
        }
    }
    for (; c < c_end; ++c) add(c, (int)__builtin_amdgcn_readfirstlane((uint32_t)irow[c]));
#pragma unroll
    for (int j = 0; j < 4; ++j) part[w][j][lane] = a[j];
    __syncthreads();
    if (w != 0 || !col_ok) return;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
        Acc sum = part[0][j][lane];
        for (int ww = 1; ww < SPLIT; ++ww) sum += part[ww][j][lane];
        a[j] = sum;
    }
    float* __restrict__ y = yrow + m;
    if constexpr (I8) {
        const float s = *scale;
#pragma unroll
        for (int j = 0; j < 4; ++j)
            y[j] = bias ? __fmaf_rn((float)a[j], s, bias[m + j]) : __fmul_rn((float)a[j], s);
    } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) y[j] = bias ? a[j] + bias[m + j] : a[j];
    }
}

}  // namespace lutnn
