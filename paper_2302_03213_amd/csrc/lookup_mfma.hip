// Table read and accumulation (arXiv 2302.03213, Eq. 4) as a dense INT8 MFMA contraction, gfx950:
// stand-alone kernel reading the index matrix idx[N][C] from global memory.  The contraction
// itself is in mfma_tile.h.  Accumulation is exact int32; the epilogue dequantises with the layer
// scale (Sec. 3.3) and adds the bias.  15 of every 16 multiplies are by zero; that is the price
// of running the gather on the matrix cores.
//
// Workgroup tile 128 rows x 256 columns (wave tile 64 x 128, 128 accumulator registers per lane).
#include "lutnn_kernels.h"
#include "mfma_tile.h"

namespace lutnn {
namespace {

constexpr int BM = 128;  // rows per workgroup
static_assert(kMfmaBN == kPackedColPad, "packed column padding must match the column tile");

template <bool IDX_DWORD>
__global__ __launch_bounds__(kMfmaThreads, 2) void lookup_mfma_i8_kernel(
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int M, int Mp, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int row_tiles, int64_t tiles) {
    __shared__ uint4 lds[2 * kMfmaStageVecs];

    // XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them, each with
    // its own L2), so give every XCD a contiguous range of tiles; tiles are ordered column-block
    // major, so the workgroups resident on one XCD walk the same slab of the table.
    const int64_t per_xcd = (tiles + 7) / 8;
    const int64_t t = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= tiles) return;
    const int n0 = (int)(t / row_tiles) * kMfmaBN;
    const int64_t m0 = (t % row_tiles) * BM;

    const int lane = threadIdx.x & 63;
    const int wm = threadIdx.x >> 7;
    const int l32 = lane & 31;
    const int64_t row_base = m0 + wm * 64;

    auto idx_word = [&](int i, int cbase) -> uint32_t {
        const int64_t row = row_base + i * 32 + l32;
        uint32_t word = 0;
        if (row < N) {
            if (IDX_DWORD) {  // C % 4 == 0 and aligned: the dword is in range iff cbase < C
                if (cbase < C) word = *reinterpret_cast<const uint32_t*>(idx + row * C + cbase);
            } else {
                for (int b = 0; b < 4; ++b)
                    if (cbase + b < C) word |= (uint32_t)idx[row * C + cbase + b] << (8 * b);
            }
        }
        return word;
    };

    v16i acc[2][4];
    mfma_lookup_tile<2>(packed, C, Mp, n0, lds, idx_word, acc);
    mfma_store_tile<2>(acc, *scale, bias, M, N, row_base, n0, Y, ldy);
}

}  // namespace

hipError_t launch_lookup_mfma_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                 int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                 hipStream_t s) {
    if (K > 16) return hipErrorInvalidValue;  // one 16-wide k block per codebook
    const int Mp = (int)packed_cols(M);
    const int64_t row_tiles = (N + BM - 1) / BM;
    const int64_t col_tiles = Mp / kMfmaBN;
    const int64_t tiles = row_tiles * col_tiles;
    const int64_t blocks = (tiles + 7) / 8 * 8;
    if (blocks > 0x7fffffffLL || row_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    const bool dw = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    if (dw)
        hipLaunchKernelGGL((lookup_mfma_i8_kernel<true>), dim3((unsigned)blocks), dim3(kMfmaThreads), 0, s,
                           reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y, ldy,
                           (int)row_tiles, tiles);
    else
        hipLaunchKernelGGL((lookup_mfma_i8_kernel<false>), dim3((unsigned)blocks), dim3(kMfmaThreads), 0,
                           s, reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y,
                           ldy, (int)row_tiles, tiles);
    return hipGetLastError();
}

}  // namespace lutnn
