// Fused LUT-NN linear operator (arXiv 2302.03213, Fig. 5: closest centroid search followed by
// table read and accumulation) in one kernel for gfx950.  The index matrix never leaves the chip.
//
// A workgroup owns 64 rows.  Phase 1 encodes ALL C codebooks of those rows (Eq. 2; same tile code
// as the stand-alone encoder) into an LDS index array [64][C].  Phase 2 runs the lookup (Eq. 4)
// for the workgroup's share of the column tiles with the indices read from LDS: the one-hot INT8
// MFMA contraction for INT8 tables, an LDS gather for fp32 tables.  Keeping the whole index row
// block on chip means the encode is done once per row block (or once per column group when the
// launch splits the columns over several workgroups to fill the chip), not once per column tile.
#include "encode_tile.h"
#include "lutnn_kernels.h"
#include "mfma_tile.h"

namespace lutnn {
namespace {

constexpr int kLdsMax = 160 * 1024;  // LDS per compute unit on gfx950

// LDS index array: row stride in dwords, odd so that lane = row reads are conflict free.
inline int idx_stride_dwords(int Cpad) { return Cpad / 4 + 1; }

template <int V, int K_T>
__device__ __forceinline__ void fused_encode_phase(const float* __restrict__ X, int64_t ldx,
                                                   const float* __restrict__ P, int C, int K, int64_t N,
                                                   int64_t row0, float* xs, uint32_t* is, int IS,
                                                   int vec4) {
    constexpr int CT = enc_tile_codebooks(V);
    using E = EncTile<V, CT>;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    for (int c0 = 0; c0 < C; c0 += CT) {
        __syncthreads();  // xs free again
        stage_x<V, CT>(X, ldx, N, C * V, row0, c0, xs, vec4, tid);
        __syncthreads();
        uint32_t packed[E::PW];
        encode_codebooks<V, K_T, CT>(xs, P, C, K, c0, w, lane, packed);
        store_index_bytes<V, CT>(is + lane * IS, c0 + w * E::CPW, packed);
    }
    __syncthreads();
}

// ------------------------------------------------------------------------------------------ INT8
template <int V, int K_T>
__global__ __launch_bounds__(kMfmaThreads) void linear_fused_i8_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ P,
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int K_rt, int M, int Mp, int64_t N, float* __restrict__ Y, int64_t ldy, int Cpad,
    int col_groups, int vec4) {
    extern __shared__ uint4 smem[];
    // [0, 64 KiB): B stage buffers of phase 2, reused as the X staging tile in phase 1
    float* xs = reinterpret_cast<float*>(smem);
    uint4* lut = smem + 2 * kMfmaStageVecs;
    uint32_t* is = reinterpret_cast<uint32_t*>(lut + kOnehotLutVecs);
    const int IS = Cpad / 4 + 1;
    const int K = K_T ? K_T : K_rt;

    const int64_t row0 = (int64_t)(blockIdx.x / col_groups) * kEncRows;
    const int g = (int)(blockIdx.x % col_groups);

    init_onehot_lut(lut);
    fused_encode_phase<V, K_T>(X, ldx, P, C, K, N, row0, xs, is, IS, vec4);

    const int lane = threadIdx.x & 63;
    const int wm = threadIdx.x >> 7;
    const int l32 = lane & 31;
    const uint32_t* my_idx = is + (wm * 32 + l32) * IS;
    auto idx_word = [&](int, int cbase) -> uint32_t { return my_idx[cbase >> 2]; };

    const float s = *scale;
    const int col_tiles = Mp / kMfmaBN;
    for (int ct = g; ct < col_tiles; ct += col_groups) {
        v16i acc[1][4];
        mfma_lookup_tile<1>(packed, C, Mp, ct * kMfmaBN, smem, lut, idx_word, acc);
        mfma_store_tile<1>(acc, s, bias, M, N, row0 + wm * 32,
                           ct * kMfmaBN + ((threadIdx.x >> 6) & 1) * 128, Y, ldy);
    }
}

// ------------------------------------------------------------------------------------------ FP32
constexpr int kColsF32 = 128;  // 64 lanes x 2 columns

template <int V, int K_T>
__global__ __launch_bounds__(kEncThreads) void linear_fused_f32_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ P, const float* __restrict__ T,
    const float* __restrict__ bias, int C, int K_rt, int M, int64_t N, float* __restrict__ Y,
    int64_t ldy, int Cpad, int col_groups, int CC, int region_a_bytes, int vec4) {
    extern __shared__ uint4 smem[];
    float* xs = reinterpret_cast<float*>(smem);    // phase 1
    float2* tab = reinterpret_cast<float2*>(smem);  // phase 2: [CC][K][64] float2
    uint32_t* is = reinterpret_cast<uint32_t*>(reinterpret_cast<char*>(smem) + region_a_bytes);
    const int IS = Cpad / 4 + 1;
    const int K = K_T ? K_T : K_rt;

    const int64_t row0 = (int64_t)(blockIdx.x / col_groups) * kEncRows;
    const int g = (int)(blockIdx.x % col_groups);

    fused_encode_phase<V, K_T>(X, ldx, P, C, K, N, row0, xs, is, IS, vec4);

    constexpr int RW = 16;  // rows per wavefront
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col_tiles = (M + kColsF32 - 1) / kColsF32;
    for (int ct = g; ct < col_tiles; ct += col_groups) {
        const int n0 = ct * kColsF32;
        float2 acc[RW];
#pragma unroll
        for (int r = 0; r < RW; ++r) acc[r] = make_float2(0.f, 0.f);
        for (int c0 = 0; c0 < C; c0 += CC) {
            __syncthreads();
            const int elems = CC * K * 64;
            for (int i = tid; i < elems; i += kEncThreads) {
                const int rowid = i >> 6, j = i & 63;
                const int cl = rowid / K, k = rowid - cl * K;
                const int c = c0 + cl;
                const int m = n0 + 2 * j;
                float2 v = make_float2(0.f, 0.f);
                if (c < C) {
                    const float* src = T + ((size_t)c * K + k) * M + m;
                    if (m < M) v.x = src[0];
                    if (m + 1 < M) v.y = src[1];
                }
                tab[i] = v;
            }
            __syncthreads();
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                const uint32_t* row_idx = is + (w * RW + r) * IS;
                for (int cl4 = 0; cl4 < CC; cl4 += 4) {
                    // c0 + cl4 < Cpad always: Cpad is a multiple of 16 and CC of 4
                    const uint32_t word =
                        (c0 + cl4 < Cpad) ? __builtin_amdgcn_readfirstlane(row_idx[(c0 + cl4) >> 2]) : 0u;
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        int k = (word >> (8 * b)) & 0xff;
                        k = k < K ? k : K - 1;
                        const float2 x = tab[((cl4 + b) * K + k) * 64 + lane];
                        acc[r].x += x.x;  // codebooks past C were staged as zeros
                        acc[r].y += x.y;
                    }
                }
            }
        }
        const int col = n0 + lane * 2;
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const int64_t row = row0 + w * RW + r;
            if (row >= N) continue;
            float* y = Y + row * ldy + col;
            if (col < M) y[0] = bias ? acc[r].x + bias[col] : acc[r].x;
            if (col + 1 < M) y[1] = bias ? acc[r].y + bias[col + 1] : acc[r].y;
        }
    }
}

int pick_col_groups(int64_t row_tiles, int col_tiles) {
    // enough workgroups to fill 256 compute units twice over, but never more than the column tiles
    int64_t g = (512 + row_tiles - 1) / row_tiles;
    if (g < 1) g = 1;
    if (g > col_tiles) g = col_tiles;
    return (int)g;
}

template <typename Kern>
hipError_t allow_lds(Kern kern, size_t bytes) {
    if (bytes <= 64 * 1024) return hipSuccess;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(kern),
                               hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
}

template <int V>
hipError_t launch_i8(const float* P, const uint4* packed, const float* scale, const float* bias, int C,
                     int K, int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                     hipStream_t s) {
    constexpr int CT = enc_tile_codebooks(V);
    const int Cpad = (C + CT - 1) / CT * CT;
    const int Mp = (int)packed_cols(M);
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const int col_groups = pick_col_groups(row_tiles, Mp / kMfmaBN);
    const int64_t blocks = row_tiles * col_groups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t shmem = (size_t)2 * kMfmaStageVecs * 16 + kOnehotLutVecs * 16 +
                         (size_t)kEncRows * idx_stride_dwords(Cpad) * 4;
    const int vec4 = enc_vec4_ok(X, ldx, C, V);
    hipError_t e;
    if (K == 16) {
        if ((e = allow_lds(linear_fused_i8_kernel<V, 16>, shmem)) != hipSuccess) return e;
        hipLaunchKernelGGL((linear_fused_i8_kernel<V, 16>), dim3((unsigned)blocks), dim3(kMfmaThreads),
                           shmem, s, X, ldx, P, packed, scale, bias, C, K, M, Mp, N, Y, ldy, Cpad,
                           col_groups, vec4);
    } else {
        if ((e = allow_lds(linear_fused_i8_kernel<V, 0>, shmem)) != hipSuccess) return e;
        hipLaunchKernelGGL((linear_fused_i8_kernel<V, 0>), dim3((unsigned)blocks), dim3(kMfmaThreads),
                           shmem, s, X, ldx, P, packed, scale, bias, C, K, M, Mp, N, Y, ldy, Cpad,
                           col_groups, vec4);
    }
    return hipGetLastError();
}

template <int V>
hipError_t launch_f32(const float* P, const float* T, const float* bias, int C, int K, int M,
                      const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
    constexpr int CT = enc_tile_codebooks(V);
    using E = EncTile<V, CT>;
    const int Cpad = (C + CT - 1) / CT * CT;
    const int CC = 4;
    size_t region_a = (size_t)CC * K * 64 * sizeof(float2);
    if (region_a < (size_t)E::kLdsFloats * 4) region_a = (size_t)E::kLdsFloats * 4;
    region_a = (region_a + 15) & ~(size_t)15;
    const size_t shmem = region_a + (size_t)kEncRows * idx_stride_dwords(Cpad) * 4;
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const int col_groups = pick_col_groups(row_tiles, (M + kColsF32 - 1) / kColsF32);
    const int64_t blocks = row_tiles * col_groups;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int vec4 = enc_vec4_ok(X, ldx, C, V);
    hipError_t e;
    if (K == 16) {
        if ((e = allow_lds(linear_fused_f32_kernel<V, 16>, shmem)) != hipSuccess) return e;
        hipLaunchKernelGGL((linear_fused_f32_kernel<V, 16>), dim3((unsigned)blocks), dim3(kEncThreads),
                           shmem, s, X, ldx, P, T, bias, C, K, M, N, Y, ldy, Cpad, col_groups, CC,
                           (int)region_a, vec4);
    } else {
        if ((e = allow_lds(linear_fused_f32_kernel<V, 0>, shmem)) != hipSuccess) return e;
        hipLaunchKernelGGL((linear_fused_f32_kernel<V, 0>), dim3((unsigned)blocks), dim3(kEncThreads),
                           shmem, s, X, ldx, P, T, bias, C, K, M, N, Y, ldy, Cpad, col_groups, CC,
                           (int)region_a, vec4);
    }
    return hipGetLastError();
}

}  // namespace

bool fused_supported(int C, int K, int V, int M, int dtype) {
    (void)M;
    const int CT = enc_tile_codebooks(V);
    if (!CT || K > 16) return false;
    const int Cpad = (C + CT - 1) / CT * CT;
    const size_t idx_bytes = (size_t)kEncRows * idx_stride_dwords(Cpad) * 4;
    const size_t region_a = 64 * 1024 + kOnehotLutVecs * 16;  // both dtypes stay within this for staging
    (void)dtype;
    return region_a + idx_bytes <= (size_t)kLdsMax;
}

#define LUTNN_DISPATCH_V(V, CALL)            \
    switch (V) {                             \
        case 1: return CALL(1);              \
        case 2: return CALL(2);              \
        case 3: return CALL(3);              \
        case 4: return CALL(4);              \
        case 8: return CALL(8);              \
        case 9: return CALL(9);              \
        case 16: return CALL(16);            \
        case 32: return CALL(32);            \
        default: return hipErrorInvalidValue; \
    }

hipError_t launch_linear_fused_i8(const float* P, const int8_t* packed, const float* scale,
                                  const float* bias, int C, int K, int V, int M, const float* X,
                                  int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
#define CALL_I8(VV) \
    launch_i8<VV>(P, reinterpret_cast<const uint4*>(packed), scale, bias, C, K, M, X, N, ldx, Y, ldy, s)
    LUTNN_DISPATCH_V(V, CALL_I8)
#undef CALL_I8
}

hipError_t launch_linear_fused_f32(const float* P, const float* T, const float* bias, int C, int K,
                                   int V, int M, const float* X, int64_t N, int64_t ldx, float* Y,
                                   int64_t ldy, hipStream_t s) {
#define CALL_F32(VV) launch_f32<VV>(P, T, bias, C, K, M, X, N, ldx, Y, ldy, s)
    LUTNN_DISPATCH_V(V, CALL_F32)
#undef CALL_F32
}

}  // namespace lutnn
