// Table read and accumulation (arXiv 2302.03213, Eq. 4 and Sec. 5.2), LDS gather variant for many
// rows, gfx950.
//
//   Y[n][m] = epilogue( sum_c T[c][idx[n][c]][m] )
//
// Lane = row.  A workgroup owns 256 rows x MT columns: every lane keeps the MT accumulators of its
// own row in registers, and the K x MT slabs of CC codebooks at a time are staged in LDS, where
// 256 rows share them.  For one codebook a lane reads the table row its own index selects, 16
// bytes at a time.  Rows of the slab are padded by 16 bytes, so that the K (<= 16) rows start in
// different banks: lanes with different indices hit different banks, lanes with the same index
// the same address - the gather is nearly conflict free although every lane goes its own way
// (measured: a quarter of the LDS-active cycles are conflicts, while the VALU sets the pace).  This is the closest CDNA form of the paper's table read: there the index vector shuffles
// a 16-entry register table (pshufb / tbl), here it picks one of 16 LDS rows per lane.
//
// INT8 / INT4 entries are added into 32-bit accumulators one byte lane at a time (the compiler
// uses the sub-dword operand selects, one instruction per entry, sign extension included), so
// unlike the paper's 16-bit partial sums nothing has to be widened or biased.
#include <algorithm>

#include "lutnn_kernels.h"

namespace lutnn {
namespace {

constexpr int kRowsThreads = 256;  // = rows per workgroup
constexpr int kRowsMaxCC = 16;     // codebooks per stage at most (their indices sit in four dwords)
constexpr int kRowsLdsBudget = 40 * 1024;

template <int MT_DWORDS>
struct RowsTile {
    static constexpr int SROW = MT_DWORDS + 4;  // dwords per staged table row, 16 bytes of padding
};

// The lane's CC index bytes of this stage, four to a dword; codebooks past C read as index 0 (their
// slab is staged as zeros).  IDX_DWORD: C % 4 == 0 and idx 4-byte aligned.
template <bool IDX_DWORD>
__device__ __forceinline__ void load_stage_indices(const uint8_t* __restrict__ irow, int C, int c0, int CC,
                                                   uint32_t (&iw)[kRowsMaxCC / 4]) {
#pragma unroll
    for (int q = 0; q < kRowsMaxCC / 4; ++q) {
        iw[q] = 0;
        if (4 * q < CC) {
            const int c = c0 + 4 * q;
            if (IDX_DWORD && (CC & 3) == 0) {
                if (c < C) iw[q] = *reinterpret_cast<const uint32_t*>(irow + c);
            } else {
                for (int b = 0; b < 4; ++b)
                    if (4 * q + b < CC && c + b < C) iw[q] |= (uint32_t)irow[c + b] << (8 * b);
            }
        }
    }
}

// ------------------------------------------------------------------------------------------ INT8
constexpr int kRowsColsI8 = 128;

// BITS = 8: T[C][K][M] int8.  BITS = 4: T[C][K][ceil(M/2)] bytes, two 4-bit entries each (even
// column in the low nibble), widened to bytes while being staged.
template <bool IDX_DWORD, int BITS>
__global__ __launch_bounds__(kRowsThreads) void lookup_rows_i8_kernel(
    const int8_t* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias, int C,
    int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy, int CC,
    int col_tiles, int table_vec16, int y_vec4) {
    constexpr int MT = kRowsColsI8;
    constexpr int SROW = RowsTile<MT / 4>::SROW;
    extern __shared__ uint32_t lds[];  // [CC][K][SROW]
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)(blockIdx.x / col_tiles) * kRowsThreads + tid;
    const int n0 = (int)(blockIdx.x % col_tiles) * MT;
    const bool row_ok = row < N;
    const uint8_t* __restrict__ irow = idx + (row_ok ? row : N - 1) * C;  // always a valid row

    int32_t acc[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[j] = 0;

    for (int c0 = 0; c0 < C; c0 += CC) {
        __syncthreads();  // previous stage fully consumed
        // ---- stage [CC][K] rows of MT bytes as 16-byte chunks; bytes outside the table become 0
        const int chunks = CC * K * (MT / 16);
        for (int i = tid; i < chunks; i += kRowsThreads) {
            const int rowid = i / (MT / 16), ch = i % (MT / 16);
            const int cl = rowid / K, k = rowid - cl * K;
            const int c = c0 + cl;
            const int m = n0 + ch * 16;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (c < C && BITS == 4 && table_vec16 && m + 16 <= M) {
                // eight bytes = sixteen entries: split the nibbles, interleave them back into column
                // order, and sign-extend each 4-bit value in its byte
                const uint2 w2 = *reinterpret_cast<const uint2*>(
                    reinterpret_cast<const uint8_t*>(T) + ((size_t)c * K + k) * (size_t)(M / 2) + m / 2);
                const uint32_t ws[2] = {w2.x, w2.y};
                uint32_t t[4];
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const uint32_t lo = ws[q] & 0x0f0f0f0fu, hi = (ws[q] >> 4) & 0x0f0f0f0fu;
                    const uint32_t a = __builtin_amdgcn_perm(hi, lo, 0x05010400u);  // lo0 hi0 lo1 hi1
                    const uint32_t b = __builtin_amdgcn_perm(hi, lo, 0x07030602u);  // lo2 hi2 lo3 hi3
                    t[2 * q + 0] = a | (((a >> 3) & 0x01010101u) * 0xf0u);
                    t[2 * q + 1] = b | (((b >> 3) & 0x01010101u) * 0xf0u);
                }
                v = make_uint4(t[0], t[1], t[2], t[3]);
            } else if (c < C && BITS == 4) {
                const uint8_t* src =
                    reinterpret_cast<const uint8_t*>(T) + ((size_t)c * K + k) * ((M + 1) / 2) + m / 2;
                uint32_t t[4] = {0u, 0u, 0u, 0u};
                for (int b = 0; b < 16; b += 2) {  // m is even: byte b/2 holds columns m+b, m+b+1
                    if (m + b >= M) break;
                    const uint32_t two = src[b >> 1];
                    const uint32_t lo = ((two & 0xfu) ^ 8u) - 8u, hi = ((two >> 4) ^ 8u) - 8u;  // sign extend
                    t[b >> 2] |= (lo & 0xffu) << (8 * (b & 3));
                    if (m + b + 1 < M) t[b >> 2] |= (hi & 0xffu) << (8 * ((b + 1) & 3));
                }
                v = make_uint4(t[0], t[1], t[2], t[3]);
            } else if (c < C) {
                const int8_t* src = T + ((size_t)c * K + k) * M + m;
                if (table_vec16 && m + 16 <= M) {
                    v = *reinterpret_cast<const uint4*>(src);
                } else {
                    uint32_t t[4] = {0u, 0u, 0u, 0u};
                    for (int b = 0; b < 16; ++b)
                        if (m + b < M) t[b >> 2] |= (uint32_t)(uint8_t)src[b] << (8 * (b & 3));
                    v = make_uint4(t[0], t[1], t[2], t[3]);
                }
            }
            *reinterpret_cast<uint4*>(lds + (size_t)rowid * SROW + ch * 4) = v;
        }
        uint32_t iw[kRowsMaxCC / 4];
        load_stage_indices<IDX_DWORD>(irow, C, c0, CC, iw);
        __syncthreads();

        for (int cl = 0; cl < CC; ++cl) {
            int k = (iw[cl >> 2] >> (8 * (cl & 3))) & 0xff;
            k = k < K ? k : K - 1;  // out-of-range indices must not read out of bounds
            const uint4* __restrict__ trow = reinterpret_cast<const uint4*>(lds + (size_t)(cl * K + k) * SROW);
#pragma unroll
            for (int j = 0; j < MT / 16; ++j) {
                const uint4 x = trow[j];
                const uint32_t xs[4] = {x.x, x.y, x.z, x.w};
#pragma unroll
                for (int d = 0; d < 4; ++d)
#pragma unroll
                    for (int b = 0; b < 4; ++b) acc[16 * j + 4 * d + b] += (int32_t)(int8_t)(xs[d] >> (8 * b));
            }
        }
    }

    // ---- epilogue: dequantise (r = s*q, Sec. 3.3), add the layer bias; the lane writes its row
    if (!row_ok) return;
    const float s = *scale;
    float* __restrict__ y = Y + row * ldy + n0;
#pragma unroll
    for (int j = 0; j < MT / 4; ++j) {
        const int col = n0 + 4 * j;
        if (col >= M) break;
        float o[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) {
            const float a = (float)acc[4 * j + b];
            o[b] = (bias && col + b < M) ? __fmaf_rn(a, s, bias[col + b]) : __fmul_rn(a, s);
        }
        if (y_vec4 && col + 4 <= M) {
            *reinterpret_cast<float4*>(y + 4 * j) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (col + b < M) y[4 * j + b] = o[b];
        }
    }
}

// ------------------------------------------------------------------------------------------ FP32
constexpr int kRowsColsF32 = 64;

template <bool IDX_DWORD>
__global__ __launch_bounds__(kRowsThreads) void lookup_rows_f32_kernel(
    const float* __restrict__ T, const float* __restrict__ bias, int C, int K, int M,
    const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy, int CC, int col_tiles,
    int table_vec4, int y_vec4) {
    constexpr int MT = kRowsColsF32;
    constexpr int SROW = RowsTile<MT>::SROW;
    extern __shared__ uint32_t lds[];
    float* tab = reinterpret_cast<float*>(lds);  // [CC][K][SROW]
    const int tid = threadIdx.x;
    const int64_t row = (int64_t)(blockIdx.x / col_tiles) * kRowsThreads + tid;
    const int n0 = (int)(blockIdx.x % col_tiles) * MT;
    const bool row_ok = row < N;
    const uint8_t* __restrict__ irow = idx + (row_ok ? row : N - 1) * C;

    float acc[MT];
#pragma unroll
    for (int j = 0; j < MT; ++j) acc[j] = 0.f;

    for (int c0 = 0; c0 < C; c0 += CC) {
        __syncthreads();
        const int chunks = CC * K * (MT / 4);  // 16-byte chunks of four columns
        for (int i = tid; i < chunks; i += kRowsThreads) {
            const int rowid = i / (MT / 4), ch = i % (MT / 4);
            const int cl = rowid / K, k = rowid - cl * K;
            const int c = c0 + cl;
            const int m = n0 + ch * 4;
            float4 v = make_float4(0.f, 0.f, 0.f, 0.f);
            if (c < C) {
                const float* src = T + ((size_t)c * K + k) * M + m;
                if (table_vec4 && m + 4 <= M) {
                    v = *reinterpret_cast<const float4*>(src);
                } else {
                    if (m < M) v.x = src[0];
                    if (m + 1 < M) v.y = src[1];
                    if (m + 2 < M) v.z = src[2];
                    if (m + 3 < M) v.w = src[3];
                }
            }
            *reinterpret_cast<float4*>(tab + (size_t)rowid * SROW + ch * 4) = v;
        }
        uint32_t iw[kRowsMaxCC / 4];
        load_stage_indices<IDX_DWORD>(irow, C, c0, CC, iw);
        __syncthreads();

        for (int cl = 0; cl < CC; ++cl) {
            int k = (iw[cl >> 2] >> (8 * (cl & 3))) & 0xff;
            k = k < K ? k : K - 1;
            const float4* __restrict__ trow = reinterpret_cast<const float4*>(tab + (size_t)(cl * K + k) * SROW);
#pragma unroll
            for (int j = 0; j < MT / 4; ++j) {
                const float4 x = trow[j];  // codebooks past C were staged as zeros
                acc[4 * j + 0] += x.x;
                acc[4 * j + 1] += x.y;
                acc[4 * j + 2] += x.z;
                acc[4 * j + 3] += x.w;
            }
        }
    }

    if (!row_ok) return;
    float* __restrict__ y = Y + row * ldy + n0;
#pragma unroll
    for (int j = 0; j < MT / 4; ++j) {
        const int col = n0 + 4 * j;
        if (col >= M) break;
        float o[4];
#pragma unroll
        for (int b = 0; b < 4; ++b) o[b] = (bias && col + b < M) ? acc[4 * j + b] + bias[col + b] : acc[4 * j + b];
        if (y_vec4 && col + 4 <= M) {
            *reinterpret_cast<float4*>(y + 4 * j) = make_float4(o[0], o[1], o[2], o[3]);
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (col + b < M) y[4 * j + b] = o[b];
        }
    }
}

inline bool idx_dword_ok(const uint8_t* idx, int C) {
    return (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
}
inline int y_vec4_ok(const float* Y, int64_t ldy) {
    return (ldy % 4 == 0) && ((reinterpret_cast<uintptr_t>(Y) & 15) == 0);
}

// Codebooks per stage: as many as fit the LDS budget, a multiple of 4 up to 16 when possible.
inline int stage_codebooks(size_t bytes_per_codebook) {
    int cc = (int)(kRowsLdsBudget / bytes_per_codebook);
    if (cc >= 4) cc &= ~3;
    return std::max(1, std::min(cc, kRowsMaxCC));
}

}  // namespace

// The lane = row kernels pay when a workgroup's 256 rows are real rows and the grid still covers
// the chip; below that the 64-row staged kernels (or the direct gather) are the better shape.
bool rows_kernel_preferred(int64_t N, int M, int K, bool f32) {
    const int mt = f32 ? kRowsColsF32 : kRowsColsI8;
    const size_t per_codebook = (size_t)K * (mt * (f32 ? 4 : 1) + 16);
    if (per_codebook > (size_t)kRowsLdsBudget) return false;
    const int64_t blocks = ((N + kRowsThreads - 1) / kRowsThreads) * ((M + mt - 1) / mt);
    // one workgroup per compute unit at least (measured on BERT- and conv-size layers: at 96
    // workgroups the 64-row kernel is 2.4x faster, from 288 on this one is 1.6x faster)
    return N >= 4 * kRowsThreads && blocks >= 256;
}

// bits = 8: T is [C][K][M] int8; bits = 4: [C][K][ceil(M/2)] nibble pairs.
hipError_t launch_lookup_rows_i8(const void* T, int bits, const float* scale, const float* bias, int C,
                                 int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                 hipStream_t s) {
    constexpr int SROW = RowsTile<kRowsColsI8 / 4>::SROW;
    const size_t per_codebook = (size_t)K * SROW * 4;
    const int CC = stage_codebooks(per_codebook);
    const int col_tiles = (M + kRowsColsI8 - 1) / kRowsColsI8;
    const int64_t blocks = ((N + kRowsThreads - 1) / kRowsThreads) * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    // 16-entry chunks as one vector load: 16 bytes of an INT8 row, 8 bytes of an INT4 row
    const int vec16 = bits == 8 ? (M % 16 == 0) && ((reinterpret_cast<uintptr_t>(T) & 15) == 0)
                                : (M % 16 == 0) && ((reinterpret_cast<uintptr_t>(T) & 7) == 0);
    const size_t shmem = (size_t)CC * per_codebook;
    const int8_t* Tb = static_cast<const int8_t*>(T);
    const dim3 grid((unsigned)blocks), block(kRowsThreads);
    const bool dw = idx_dword_ok(idx, C);
#define LUTNN_LAUNCH_ROWS_I8(DW, BITS)                                                                    \
    hipLaunchKernelGGL((lookup_rows_i8_kernel<DW, BITS>), grid, block, shmem, s, Tb, scale, bias, C, K, M, \
                       idx, N, Y, ldy, CC, col_tiles, vec16, y_vec4_ok(Y, ldy))
    if (bits == 4) {
        if (dw) LUTNN_LAUNCH_ROWS_I8(true, 4); else LUTNN_LAUNCH_ROWS_I8(false, 4);
    } else {
        if (dw) LUTNN_LAUNCH_ROWS_I8(true, 8); else LUTNN_LAUNCH_ROWS_I8(false, 8);
    }
#undef LUTNN_LAUNCH_ROWS_I8
    return hipGetLastError();
}

hipError_t launch_lookup_rows_f32(const float* T, const float* bias, int C, int K, int M,
                                  const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    constexpr int SROW = RowsTile<kRowsColsF32>::SROW;
    const size_t per_codebook = (size_t)K * SROW * 4;
    const int CC = stage_codebooks(per_codebook);
    const int col_tiles = (M + kRowsColsF32 - 1) / kRowsColsF32;
    const int64_t blocks = ((N + kRowsThreads - 1) / kRowsThreads) * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int vec4 = (M % 4 == 0) && ((reinterpret_cast<uintptr_t>(T) & 15) == 0);
    const size_t shmem = (size_t)CC * per_codebook;
    const dim3 grid((unsigned)blocks), block(kRowsThreads);
    if (idx_dword_ok(idx, C))
        hipLaunchKernelGGL((lookup_rows_f32_kernel<true>), grid, block, shmem, s, T, bias, C, K, M, idx, N, Y,
                           ldy, CC, col_tiles, vec4, y_vec4_ok(Y, ldy));
    else
        hipLaunchKernelGGL((lookup_rows_f32_kernel<false>), grid, block, shmem, s, T, bias, C, K, M, idx, N,
                           Y, ldy, CC, col_tiles, vec4, y_vec4_ok(Y, ldy));
    return hipGetLastError();
}

}  // namespace lutnn
