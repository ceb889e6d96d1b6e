// Table read and accumulation (arXiv 2302.03213, Eq. 4 and Sec. 5.2), LDS gather variant, gfx950.
//
//   Y[n][m] = epilogue( sum_c T[c][idx[n][c]][m] )
//
// A workgroup owns an (R rows x MT columns) output tile and walks the codebooks in stages: the
// K x MT slab of each of CC codebooks is staged in LDS as [codebook][k][MT] (m fastest), then
// every wavefront handles its own rows one at a time.  For one (row, codebook) the index is
// wave-uniform: it is fetched with a scalar load, four codebooks per dword, and the 64 lanes read
// 64 consecutive dwords of the selected table row - consecutive banks, conflict free by
// construction.  The paper's byte-shuffle table read (16 lookups per 128-bit shuffle) has no
// CDNA counterpart; a wave-wide LDS row read is the equivalent "one instruction, many lookups".
//
// INT8 accumulation follows the paper's mixed-precision idea (16-bit partial sums, then 32-bit):
// table bytes are stored in LDS with a +128 bias so they are unsigned, one dword carries four
// columns, and the even/odd bytes are added as two packed 16-bit lanes with plain 32-bit adds.
// 256 biased bytes cannot overflow 16 bits (256*255 < 65536); the partial sums are widened to
// int32 at least that often and the bias (128 per codebook) is removed in the epilogue, so the
// result is the exact integer sum.
#include <type_traits>

#include "gather_row.h"
#include "lutnn_kernels.h"

namespace lutnn {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = 4;

// ------------------------------------------------------------------------------------------ INT8
constexpr int kColsI8 = 256;  // MT: 64 lanes x 4 columns
constexpr int kRowsPerWaveI8 = 16;

// BITS = 8: T[C][K][M] int8.  BITS = 4: T[C][K][ceil(M/2)] bytes, two 4-bit entries each (even
// column in the low nibble); they are widened to bytes while being staged, the rest is the same.
template <bool IDX_DWORD, int BITS = 8>
__global__ __launch_bounds__(kThreads) void lookup_lds_i8_kernel(
    const int8_t* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int CC, int col_tiles, int table_vec16) {
    extern __shared__ uint32_t lds[];  // [CC][K][64] dwords = 4 biased bytes each
    constexpr int RW = kRowsPerWaveI8;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row_tile = blockIdx.x / col_tiles;
    const int n0 = (int)(blockIdx.x % col_tiles) * kColsI8;
    const int64_t row0 = row_tile * (RW * kWaves) + (int64_t)w * RW;

    uint32_t lo[RW], hi[RW];
    int32_t acc[RW][4];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        lo[r] = hi[r] = 0;
        acc[r][0] = acc[r][1] = acc[r][2] = acc[r][3] = 0;
    }
    int pending = 0;  // codebooks accumulated in lo/hi since the last widening
    int slots = 0;    // codebook slots accumulated in total (each carries a +128 bias)

    for (int c0 = 0; c0 < C; c0 += CC) {
        __syncthreads();  // previous stage fully consumed
        // ---- stage [CC][K][256 B]; bytes outside the table become 0 (biased: 0x80)
        const int chunks = CC * K * 16;  // 16-byte chunks
        for (int i = tid; i < chunks; i += kThreads) {
            const int rowid = i >> 4, ch = i & 15;
            const int cl = rowid / K, k = rowid - cl * K;
            const int c = c0 + cl;
            const int m = n0 + ch * 16;
            uint4 v = make_uint4(0u, 0u, 0u, 0u);
            if (c < C && BITS == 4) {
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
            v.x ^= 0x80808080u;
            v.y ^= 0x80808080u;
            v.z ^= 0x80808080u;
            v.w ^= 0x80808080u;
            *reinterpret_cast<uint4*>(lds + (size_t)rowid * 64 + ch * 4) = v;
        }
        __syncthreads();

        if (pending + CC > 256) {  // widen before 16-bit lanes could overflow
#pragma unroll
            for (int r = 0; r < RW; ++r) {
                acc[r][0] += lo[r] & 0xffff;
                acc[r][2] += lo[r] >> 16;
                acc[r][1] += hi[r] & 0xffff;
                acc[r][3] += hi[r] >> 16;
                lo[r] = hi[r] = 0;
            }
            pending = 0;
        }
#pragma unroll
        for (int r = 0; r < RW; ++r) {
            const int64_t row = row0 + r;
            if (row < N) {
                for (int cl4 = 0; cl4 < CC; cl4 += 4) {
                    uint32_t word;
                    if (IDX_DWORD) {  // C % 4 == 0, 4-byte aligned: in range whenever c0+cl4 < C
                        word = (c0 + cl4 < C)
                                   ? *reinterpret_cast<const uint32_t*>(idx + row * C + c0 + cl4)
                                   : 0u;
                    } else {
                        word = 0;
                        for (int b = 0; b < 4; ++b)
                            if (c0 + cl4 + b < C)
                                word |= (uint32_t)idx[row * C + c0 + cl4 + b] << (8 * b);
                    }
                    word = __builtin_amdgcn_readfirstlane(word);
#pragma unroll
                    for (int b = 0; b < 4; ++b) {
                        int k = (word >> (8 * b)) & 0xff;
                        k = k < K ? k : K - 1;  // out-of-range indices must not read out of bounds
                        const uint32_t x = lds[((cl4 + b) * K + k) * 64 + lane];
                        lo[r] += x & 0x00ff00ffu;
                        hi[r] += (x >> 8) & 0x00ff00ffu;
                    }
                }
            }
        }
        pending += CC;
        slots += CC;
    }

    // ---- epilogue: widen, remove the bias, dequantise (r = s*q, Sec. 3.3), add the layer bias
    const float s = *scale;
    const int col = n0 + lane * 4;
    float bv[4] = {0.f, 0.f, 0.f, 0.f};
    if (bias)
        for (int j = 0; j < 4; ++j)
            if (col + j < M) bv[j] = bias[col + j];
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row0 + r;
        if (row >= N) continue;
        int32_t a[4];
        a[0] = acc[r][0] + (int32_t)(lo[r] & 0xffff) - 128 * slots;
        a[2] = acc[r][2] + (int32_t)(lo[r] >> 16) - 128 * slots;
        a[1] = acc[r][1] + (int32_t)(hi[r] & 0xffff) - 128 * slots;
        a[3] = acc[r][3] + (int32_t)(hi[r] >> 16) - 128 * slots;
        float* y = Y + row * ldy + col;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            if (col + j < M)
                y[j] = bias ? __fmaf_rn((float)a[j], s, bv[j]) : __fmul_rn((float)a[j], s);
        }
    }
}

// ------------------------------------------------------------------------------------------ FP32
constexpr int kColsF32 = 128;  // MT: 64 lanes x 2 columns
constexpr int kRowsPerWaveF32 = 8;

template <bool IDX_DWORD>
__global__ __launch_bounds__(kThreads) void lookup_lds_f32_kernel(
    const float* __restrict__ T, const float* __restrict__ bias, int C, int K, int M,
    const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy, int CC,
    int col_tiles) {
    extern __shared__ uint32_t lds[];
    float2* tab = reinterpret_cast<float2*>(lds);  // [CC][K][64] float2
    constexpr int RW = kRowsPerWaveF32;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t row_tile = blockIdx.x / col_tiles;
    const int n0 = (int)(blockIdx.x % col_tiles) * kColsF32;
    const int64_t row0 = row_tile * (RW * kWaves) + (int64_t)w * RW;

    float2 acc[RW];
#pragma unroll
    for (int r = 0; r < RW; ++r) acc[r] = make_float2(0.f, 0.f);

    for (int c0 = 0; c0 < C; c0 += CC) {
        __syncthreads();
        const int elems = CC * K * 64;  // float2 elements
        for (int i = tid; i < elems; i += kThreads) {
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
            const int64_t row = row0 + r;
            if (row < N) {
                for (int cl4 = 0; cl4 < CC; cl4 += 4) {
                    uint32_t word;
                    if (IDX_DWORD) {
                        word = (c0 + cl4 < C)
                                   ? *reinterpret_cast<const uint32_t*>(idx + row * C + c0 + cl4)
                                   : 0u;
                    } else {
                        word = 0;
                        for (int b = 0; b < 4; ++b)
                            if (c0 + cl4 + b < C)
                                word |= (uint32_t)idx[row * C + c0 + cl4 + b] << (8 * b);
                    }
                    word = __builtin_amdgcn_readfirstlane(word);
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
    }

    const int col = n0 + lane * 2;
#pragma unroll
    for (int r = 0; r < RW; ++r) {
        const int64_t row = row0 + r;
        if (row >= N) continue;
        float* y = Y + row * ldy + col;
        if (col < M) y[0] = bias ? acc[r].x + bias[col] : acc[r].x;
        if (col + 1 < M) y[1] = bias ? acc[r].y + bias[col + 1] : acc[r].y;
    }
}

// ------------------------------------------------------------------------------- any K: no LDS
// One thread per (row, column); the table is read straight from global memory (L2).  Used when a
// codebook's K x MT slab does not fit the LDS staging buffer.
template <typename TT>
__global__ __launch_bounds__(kThreads) void lookup_global_kernel(
    const TT* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias, int C,
    int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= N * (int64_t)M) return;
    const int64_t n = i / M;
    const int m = (int)(i % M);
    if constexpr (sizeof(TT) == 1) {
        int32_t acc = 0;
        for (int c = 0; c < C; ++c) {
            int k = idx[n * C + c];
            k = k < K ? k : K - 1;
            acc += (int32_t)T[((size_t)c * K + k) * M + m];
        }
        const float s = *scale;
        Y[n * ldy + m] = bias ? __fmaf_rn((float)acc, s, bias[m]) : __fmul_rn((float)acc, s);
    } else {
        float acc = 0.f;
        for (int c = 0; c < C; ++c) {
            int k = idx[n * C + c];
            k = k < K ? k : K - 1;
            acc += T[((size_t)c * K + k) * M + m];
        }
        Y[n * ldy + m] = bias ? acc + bias[m] : acc;
    }
}

// ------------------------------------------------------------------------- few rows: no staging
// Staging a K x MT slab per codebook pays off when many rows of a workgroup read it.  With few
// rows (a batch of a few hundred) the staged grid cannot even fill the chip, and the slab is read
// from L2 by every row tile anyway.  Here one wavefront owns one row and a run of 256 columns,
// each lane four consecutive columns, and reads the selected table row straight from global
// memory (one 4- or 16-byte load per lane and codebook, the wave's loads are contiguous).  The
// index is wave-uniform (scalar load, four codebooks per dword) and the loads of several
// codebooks are in flight at once.  Sums run over the codebooks in order, as in the staged
// kernels.  Needs M % 4 == 0 and a table aligned for the vector load.
constexpr int kGatherCols = 256;

// UNIFORM: a wavefront works on one row (M >= 256: scalar index loads).  Otherwise rows are
// narrower than a wavefront: `lpr` lanes per row, 64 / lpr rows per wavefront, per-lane index loads.
template <typename TT, bool IDX_DWORD, bool UNIFORM>
__global__ __launch_bounds__(kThreads) void lookup_gather_kernel(
    const TT* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias, int C,
    int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy,
    int col_chunks, int lpr) {
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gw = (int64_t)blockIdx.x * kWaves + w;
    int64_t row;
    int m;
    if (UNIFORM) {
        row = gw / col_chunks;
        m = (int)(gw % col_chunks) * kGatherCols + lane * 4;
    } else {
        const int sub = lane / lpr;
        if (sub >= 64 / lpr) return;
        row = gw * (64 / lpr) + sub;
        m = (lane - sub * lpr) * 4;
    }
    if (row >= N) return;
    if (m >= M) return;  // M % 4 == 0: a lane's four columns are all inside or all outside
    gather_row<TT, IDX_DWORD, UNIFORM>(T, scale, bias, C, K, M, idx + row * C, m, Y + row * ldy);
}

// The same gather for a handful of rows (batch-1 inference, the paper's own setting): with so few
// wavefronts the per-row chain of C loads and additions is pure latency, so the SPLIT wavefronts of
// a workgroup share one (row, 256 columns) and take a contiguous range of codebooks each; the
// partial sums meet in LDS and wavefront 0 adds them in range order (exact for integer tables, a
// fixed order for fp32 ones).  M % 4 == 0, table aligned for the vector load, M >= 256.
template <typename TT, bool IDX_DWORD, int SPLIT>
__global__ __launch_bounds__(64 * SPLIT) void lookup_gather_split_kernel(
    const TT* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias, int C,
    int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y, int64_t ldy,
    int col_chunks, int per_wave) {
    const int lane = threadIdx.x & 63;
    const int64_t row = blockIdx.x / col_chunks;  // < N by construction of the grid
    const int m = (int)(blockIdx.x % col_chunks) * kGatherCols + lane * 4;
    gather_row_split<TT, IDX_DWORD, SPLIT>(T, scale, bias, C, K, M, idx + row * C, m, Y + row * ldy, per_wave);
}

// Fewer (row, 256-column chunk) pairs than this and at least this many codebooks: the split form
// (measured at C = 1024, M = 4096: faster than one wavefront per pair up to about 160 rows).
constexpr int64_t kSplitMaxWaves = 2049;
constexpr int kSplitMinCodebooks = 64;

// The staged kernels need at least this many workgroups to be worth their staging.
constexpr int64_t kMinStagedBlocks = 512;

template <typename TT>
bool gather_ok(const TT* T, int M, int64_t staged_blocks) {
    return staged_blocks < kMinStagedBlocks && M % 4 == 0 &&
           (reinterpret_cast<uintptr_t>(T) & (4 * sizeof(TT) - 1)) == 0;
}

inline bool gather_i4_ok(const uint8_t* T, int M, int64_t staged_blocks) {
    return staged_blocks < kMinStagedBlocks && M % 8 == 0 && (reinterpret_cast<uintptr_t>(T) & 3) == 0;
}

template <typename TT>
hipError_t launch_gather(const TT* T, const float* scale, const float* bias, int C, int K, int M,
                         const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    const bool idx_dword = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    const int lpr = M / 4;  // lanes per row when a row is narrower than a wavefront
    if (lpr >= 64) {
        const int col_chunks = (M + kGatherCols - 1) / kGatherCols;
        if (N * col_chunks < kSplitMaxWaves && C >= kSplitMinCodebooks) {
            const dim3 grid((unsigned)(N * col_chunks));
#define LUTNN_LAUNCH_SPLIT(DW, SPLIT)                                                                        \
    hipLaunchKernelGGL((lookup_gather_split_kernel<TT, DW, SPLIT>), grid, dim3(64 * SPLIT), 0, s, T, scale,  \
                       bias, C, K, M, idx, N, Y, ldy, col_chunks, ((C + SPLIT - 1) / SPLIT + 3) & ~3)
            if (C >= 512) {
                if (idx_dword) LUTNN_LAUNCH_SPLIT(true, 16); else LUTNN_LAUNCH_SPLIT(false, 16);
            } else {
                if (idx_dword) LUTNN_LAUNCH_SPLIT(true, 4); else LUTNN_LAUNCH_SPLIT(false, 4);
            }
#undef LUTNN_LAUNCH_SPLIT
            return hipGetLastError();
        }
        const int64_t blocks = (N * col_chunks + kWaves - 1) / kWaves;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        if (idx_dword)
            hipLaunchKernelGGL((lookup_gather_kernel<TT, true, true>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, col_chunks, lpr);
        else
            hipLaunchKernelGGL((lookup_gather_kernel<TT, false, true>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, col_chunks, lpr);
    } else {
        const int64_t rows_per_block = (int64_t)(64 / lpr) * kWaves;
        const int64_t blocks = (N + rows_per_block - 1) / rows_per_block;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        if (idx_dword)
            hipLaunchKernelGGL((lookup_gather_kernel<TT, true, false>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, 1, lpr);
        else
            hipLaunchKernelGGL((lookup_gather_kernel<TT, false, false>), dim3((unsigned)blocks),
                               dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, 1, lpr);
    }
    return hipGetLastError();
}

// 4-bit table, any K, any M: one thread per (row, column), nibbles read from global memory.
__global__ __launch_bounds__(kThreads) void lookup_global_i4_kernel(
    const uint8_t* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy) {
    const int64_t i = (int64_t)blockIdx.x * kThreads + threadIdx.x;
    if (i >= N * (int64_t)M) return;
    const int64_t n = i / M;
    const int m = (int)(i % M);
    const int Mb = (M + 1) / 2;
    int32_t acc = 0;
    for (int c = 0; c < C; ++c) {
        int k = idx[n * C + c];
        k = k < K ? k : K - 1;
        const uint32_t two = T[((size_t)c * K + k) * Mb + (m >> 1)];
        const uint32_t nib = (m & 1) ? two >> 4 : two & 0xfu;
        acc += (int32_t)((nib ^ 8u) - 8u);
    }
    const float s = *scale;
    Y[n * ldy + m] = bias ? __fmaf_rn((float)acc, s, bias[m]) : __fmul_rn((float)acc, s);
}

// 4-bit table, few rows: as lookup_gather_kernel, a lane takes eight columns (one dword of the
// table row), a wavefront 512.  Needs M % 8 == 0 and a 4-byte aligned table.
constexpr int kGatherColsI4 = 512;

template <bool IDX_DWORD, bool UNIFORM>
__global__ __launch_bounds__(kThreads) void lookup_gather_i4_kernel(
    const uint8_t* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int K, int M, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int col_chunks, int lpr) {
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t gw = (int64_t)blockIdx.x * kWaves + w;
    int64_t row;
    int m;
    if (UNIFORM) {
        row = gw / col_chunks;
        m = (int)(gw % col_chunks) * kGatherColsI4 + lane * 8;
    } else {  // rows narrower than a wavefront: lpr lanes per row
        const int sub = lane / lpr;
        if (sub >= 64 / lpr) return;
        row = gw * (64 / lpr) + sub;
        m = (lane - sub * lpr) * 8;
    }
    if (row >= N) return;
    if (m >= M) return;  // M % 8 == 0: a lane's eight columns are all inside or all outside
    auto uni = [](uint32_t x) { return UNIFORM ? (uint32_t)__builtin_amdgcn_readfirstlane(x) : x; };
    const uint8_t* __restrict__ irow = idx + row * C;
    const uint8_t* __restrict__ tcol = T + m / 2;
    const size_t Mb = (size_t)M / 2;
    int32_t a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    auto add = [&](int c, int k) {
        k = k < K ? k : K - 1;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(tcol + ((size_t)c * K + k) * Mb);
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] += (int32_t)(v << (28 - 4 * j)) >> 28;  // nibble j, sign extended
    };
    int c = 0;
    if (IDX_DWORD) {
        for (; c + 4 <= C; c += 4) {
            const uint32_t word = uni(*reinterpret_cast<const uint32_t*>(irow + c));
#pragma unroll
            for (int b = 0; b < 4; ++b) add(c + b, (int)((word >> (8 * b)) & 0xffu));
        }
    }
    for (; c < C; ++c) add(c, (int)uni((uint32_t)irow[c]));
    const float s = *scale;
    float* __restrict__ y = Y + row * ldy + m;
#pragma unroll
    for (int j = 0; j < 8; ++j)
        y[j] = bias ? __fmaf_rn((float)a[j], s, bias[m + j]) : __fmul_rn((float)a[j], s);
}

// The split form of the 4-bit gather for a handful of rows (see lookup_gather_split_kernel): one
// (row, 512 columns) per workgroup, its wavefronts each a range of the codebooks.  M % 8 == 0, M >= 512.
template <bool IDX_DWORD, int SPLIT>
__global__ __launch_bounds__(64 * SPLIT) void lookup_gather_i4_split_kernel(
    const uint8_t* __restrict__ T, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int K, int M, const uint8_t* __restrict__ idx, float* __restrict__ Y, int64_t ldy,
    int col_chunks, int per_wave) {
    __shared__ int32_t part[SPLIT][8][64];
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int64_t row = blockIdx.x / col_chunks;  // < N by construction of the grid
    const int m = (int)(blockIdx.x % col_chunks) * kGatherColsI4 + lane * 8;
    const bool col_ok = m < M;  // M % 8 == 0: a lane's eight columns are all inside or all outside
    const uint8_t* __restrict__ irow = idx + row * C;
    const uint8_t* __restrict__ tcol = T + (col_ok ? m / 2 : 0);
    const size_t Mb = (size_t)M / 2;
    int32_t a[8] = {0, 0, 0, 0, 0, 0, 0, 0};
    auto add = [&](int c, int k) {
        k = k < K ? k : K - 1;
        const uint32_t v = *reinterpret_cast<const uint32_t*>(tcol + ((size_t)c * K + k) * Mb);
#pragma unroll
        for (int j = 0; j < 8; ++j) a[j] += (int32_t)(v << (28 - 4 * j)) >> 28;  // nibble j, sign extended
    };
    int c = w * per_wave;  // per_wave is a multiple of 4: dword index loads stay aligned
    const int c_end = min(C, c + per_wave);
    if (IDX_DWORD) {
        for (; c + 4 <= c_end; c += 4) {
            const uint32_t word =
                (uint32_t)__builtin_amdgcn_readfirstlane(*reinterpret_cast<const uint32_t*>(irow + c));
#pragma unroll
            for (int b = 0; b < 4; ++b) add(c + b, (int)((word >> (8 * b)) & 0xffu));
        }
    }
    for (; c < c_end; ++c) add(c, (int)__builtin_amdgcn_readfirstlane((uint32_t)irow[c]));
#pragma unroll
    for (int j = 0; j < 8; ++j) part[w][j][lane] = a[j];
    __syncthreads();
    if (w != 0 || !col_ok) return;
    const float s = *scale;
    float* __restrict__ y = Y + row * ldy + m;
#pragma unroll
    for (int j = 0; j < 8; ++j) {
        int32_t sum = part[0][j][lane];
        for (int ww = 1; ww < SPLIT; ++ww) sum += part[ww][j][lane];
        y[j] = bias ? __fmaf_rn((float)sum, s, bias[m + j]) : __fmul_rn((float)sum, s);
    }
}

constexpr int kLdsBudget = 64 * 1024;

inline bool idx_dword_ok(const uint8_t* idx, int C) {
    return (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
}

}  // namespace

// True when the gather variant would read the table straight from L2 (no staging) and the whole
// problem is small enough for that to beat the matrix-core kernels, whose tiles and pipeline fill
// are wasted on it (measured cross-over: about 3e7 table entries) ...
bool gather_preferred(const void* T, int table_kind, int C, int M, int64_t N, bool sparse_ok) {
    if (!T) return false;
    const bool f32 = table_kind == 0;
    const int64_t rows_per_block = f32 ? kRowsPerWaveF32 * kWaves : kRowsPerWaveI8 * kWaves;
    const int cols_per_block = f32 ? kColsF32 : kColsI8;
    const int64_t staged_blocks =
        ((N + rows_per_block - 1) / rows_per_block) * ((M + cols_per_block - 1) / cols_per_block);
    const bool direct = table_kind == 0   ? gather_ok(static_cast<const float*>(T), M, staged_blocks)
                        : table_kind == 1 ? gather_ok(static_cast<const int8_t*>(T), M, staged_blocks)
                                          : gather_i4_ok(static_cast<const uint8_t*>(T), M, staged_blocks);
    if (!direct) return false;
    // a few rows: the split gather reads N rows' worth of table entries, the matrix cores the whole
    // table; measured cross-over at config 5's width between 32 and 48 rows (K = 16)
    const int chunk = table_kind == 2 ? kGatherColsI4 : kGatherCols;  // columns per wavefront
    const int64_t col_chunks = (M + chunk - 1) / chunk;
    if (M >= chunk && C >= kSplitMinCodebooks && N <= 32 && N * col_chunks < kSplitMaxWaves) return true;
    // Otherwise price both (ms per call, fitted to sweeps of 32-2048 rows over seventeen layer
    // shapes; the rule picks the faster form or ties on all of them).  The gather costs its
    // N*C*M entry reads; a matrix-core launch costs its pipeline fill and the serial walk over the
    // codebooks - far longer per codebook on the dense kernel, which runs where the sparse one
    // cannot (C % 32 != 0 or unaligned indices).  From 512 codebooks on the sparse kernel shares
    // the codebooks of a tile out over workgroups and its time stops growing with C: there the
    // gather only wins below ~5.6e7 entries.
    const double entries = (double)N * C * M;
    if (C >= 512 && sparse_ok) return entries <= 5.6e7;
    const double t_gather = 0.0038 + 8.9e-11 * entries;
    const double t_matrix = sparse_ok ? 0.0065 + 1.6e-5 * C : 0.0062 + 1.2e-4 * C;
    return t_gather < t_matrix;
}

hipError_t launch_lookup_lds_i8(const int8_t* T, const float* scale, const float* bias, int C, int K,
                                int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                hipStream_t s) {
    if (rows_kernel_preferred(N, M, K, false))
        return launch_lookup_rows_i8(T, 8, scale, bias, C, K, M, idx, N, Y, ldy, s);
    const int per_codebook = K * kColsI8;  // LDS bytes per staged codebook
    if (4 * per_codebook > kLdsBudget) {
        const int64_t blocks = (N * (int64_t)M + kThreads - 1) / kThreads;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL((lookup_global_kernel<int8_t>), dim3((unsigned)blocks), dim3(kThreads), 0, s,
                           T, scale, bias, C, K, M, idx, N, Y, ldy);
        return hipGetLastError();
    }
    int CC = (kLdsBudget / 2 / per_codebook) & ~3;  // aim for 32 KiB so two workgroups share a CU
    if (CC < 4) CC = 4;
    if (CC > 16) CC = 16;
    const int col_tiles = (M + kColsI8 - 1) / kColsI8;
    const int64_t row_tiles = (N + kRowsPerWaveI8 * kWaves - 1) / (kRowsPerWaveI8 * kWaves);
    const int64_t blocks = row_tiles * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (gather_ok(T, M, blocks)) return launch_gather(T, scale, bias, C, K, M, idx, N, Y, ldy, s);
    const int vec16 = (M % 16 == 0) && ((reinterpret_cast<uintptr_t>(T) & 15) == 0);
    const size_t shmem = (size_t)CC * per_codebook;
    if (idx_dword_ok(idx, C))
        hipLaunchKernelGGL((lookup_lds_i8_kernel<true>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, T, scale, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles, vec16);
    else
        hipLaunchKernelGGL((lookup_lds_i8_kernel<false>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, T, scale, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles, vec16);
    return hipGetLastError();
}

hipError_t launch_lookup_lds_i4(const uint8_t* T, const float* scale, const float* bias, int C, int K,
                                int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                hipStream_t s) {
    if (rows_kernel_preferred(N, M, K, false))
        return launch_lookup_rows_i8(T, 4, scale, bias, C, K, M, idx, N, Y, ldy, s);
    const int per_codebook = K * kColsI8;  // LDS bytes per staged codebook (entries widened to bytes)
    if (4 * per_codebook > kLdsBudget) {
        const int64_t blocks = (N * (int64_t)M + kThreads - 1) / kThreads;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL(lookup_global_i4_kernel, dim3((unsigned)blocks), dim3(kThreads), 0, s, T, scale,
                           bias, C, K, M, idx, N, Y, ldy);
        return hipGetLastError();
    }
    int CC = (kLdsBudget / 2 / per_codebook) & ~3;
    if (CC < 4) CC = 4;
    if (CC > 16) CC = 16;
    const int col_tiles = (M + kColsI8 - 1) / kColsI8;
    const int64_t row_tiles = (N + kRowsPerWaveI8 * kWaves - 1) / (kRowsPerWaveI8 * kWaves);
    const int64_t blocks = row_tiles * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool idx_dword = idx_dword_ok(idx, C);
    if (gather_i4_ok(T, M, blocks)) {
        const int lpr = M / 8;
        if (lpr >= 64) {
            const int col_chunks = (M + kGatherColsI4 - 1) / kGatherColsI4;
            if (N * col_chunks < kSplitMaxWaves && C >= kSplitMinCodebooks) {
                const dim3 grid((unsigned)(N * col_chunks));
#define LUTNN_LAUNCH_SPLIT_I4(DW, SPLIT)                                                                      \
    hipLaunchKernelGGL((lookup_gather_i4_split_kernel<DW, SPLIT>), grid, dim3(64 * SPLIT), 0, s, T, scale, bias, \
                       C, K, M, idx, Y, ldy, col_chunks, ((C + SPLIT - 1) / SPLIT + 3) & ~3)
                if (C >= 512) {
                    if (idx_dword) LUTNN_LAUNCH_SPLIT_I4(true, 16); else LUTNN_LAUNCH_SPLIT_I4(false, 16);
                } else {
                    if (idx_dword) LUTNN_LAUNCH_SPLIT_I4(true, 4); else LUTNN_LAUNCH_SPLIT_I4(false, 4);
                }
#undef LUTNN_LAUNCH_SPLIT_I4
                return hipGetLastError();
            }
            const int64_t gblocks = (N * col_chunks + kWaves - 1) / kWaves;
            if (gblocks > 0x7fffffffLL) return hipErrorInvalidValue;
            if (idx_dword)
                hipLaunchKernelGGL((lookup_gather_i4_kernel<true, true>), dim3((unsigned)gblocks),
                                   dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, col_chunks, lpr);
            else
                hipLaunchKernelGGL((lookup_gather_i4_kernel<false, true>), dim3((unsigned)gblocks),
                                   dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, col_chunks, lpr);
        } else {
            const int64_t rows_per_block = (int64_t)(64 / lpr) * kWaves;
            const int64_t gblocks = (N + rows_per_block - 1) / rows_per_block;
            if (gblocks > 0x7fffffffLL) return hipErrorInvalidValue;
            if (idx_dword)
                hipLaunchKernelGGL((lookup_gather_i4_kernel<true, false>), dim3((unsigned)gblocks),
                                   dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, 1, lpr);
            else
                hipLaunchKernelGGL((lookup_gather_i4_kernel<false, false>), dim3((unsigned)gblocks),
                                   dim3(kThreads), 0, s, T, scale, bias, C, K, M, idx, N, Y, ldy, 1, lpr);
        }
        return hipGetLastError();
    }
    const size_t shmem = (size_t)CC * per_codebook;
    const int8_t* Tb = reinterpret_cast<const int8_t*>(T);
    if (idx_dword)
        hipLaunchKernelGGL((lookup_lds_i8_kernel<true, 4>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, Tb, scale, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles, 0);
    else
        hipLaunchKernelGGL((lookup_lds_i8_kernel<false, 4>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, Tb, scale, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles, 0);
    return hipGetLastError();
}

hipError_t launch_lookup_lds_f32(const float* T, const float* bias, int C, int K, int M,
                                 const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    if (rows_kernel_preferred(N, M, K, true)) return launch_lookup_rows_f32(T, bias, C, K, M, idx, N, Y, ldy, s);
    const int per_codebook = K * kColsF32 * 4;
    if (4 * per_codebook > kLdsBudget) {
        const int64_t blocks = (N * (int64_t)M + kThreads - 1) / kThreads;
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        hipLaunchKernelGGL((lookup_global_kernel<float>), dim3((unsigned)blocks), dim3(kThreads), 0, s, T,
                           (const float*)nullptr, bias, C, K, M, idx, N, Y, ldy);
        return hipGetLastError();
    }
    int CC = (kLdsBudget / 2 / per_codebook) & ~3;
    if (CC < 4) CC = 4;
    if (CC > 16) CC = 16;
    const int col_tiles = (M + kColsF32 - 1) / kColsF32;
    const int64_t row_tiles = (N + kRowsPerWaveF32 * kWaves - 1) / (kRowsPerWaveF32 * kWaves);
    const int64_t blocks = row_tiles * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    if (gather_ok(T, M, blocks))
        return launch_gather(T, (const float*)nullptr, bias, C, K, M, idx, N, Y, ldy, s);
    const size_t shmem = (size_t)CC * per_codebook;
    if (idx_dword_ok(idx, C))
        hipLaunchKernelGGL((lookup_lds_f32_kernel<true>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, T, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles);
    else
        hipLaunchKernelGGL((lookup_lds_f32_kernel<false>), dim3((unsigned)blocks), dim3(kThreads), shmem,
                           s, T, bias, C, K, M, idx, N, Y, ldy, CC, col_tiles);
    return hipGetLastError();
}

}  // namespace lutnn
