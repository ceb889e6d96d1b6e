// Encoding / closest centroid search (arXiv 2302.03213, Eq. 2 and Sec. 5.1) for gfx950.
//
//   idx[n][c] = argmin_k sum_v (X[n][cV+v] - P[c][k][v])^2      fp32, v ascending,
//                                                                one fma per term, lowest k on ties
//
// Mapping.  The paper's "centroid-stationary" scheme keeps a codebook's K centroids in registers
// while the rows stream past.  On CDNA that becomes: a wavefront works on ONE codebook at a time
// with lane = row, so the centroid values are wave-uniform and live in scalar registers (scalar
// loads, no vector memory or LDS traffic for them), and every VALU op takes the centroid as an
// SGPR operand.  The X tile (64 rows x CT codebooks) is read from HBM exactly once with coalesced
// row-segment loads, turned through LDS (padded row stride, conflict-free for lane = row), and
// the chosen indices go back through LDS so that each row's CT index bytes leave as one segment.
// The paper's second optimisation (splitting the arg-min compare chain for ILP) is unnecessary
// here: 64 rows per wave already give independent chains.
#include "encode_tile.h"
#include "lutnn_kernels.h"

namespace lutnn {
namespace {

// CONV != 0: X is an NCHW image batch and the tile is gathered through `geom` (implicit im2col);
// CONV > 0 is the number of filter taps when known at compile time, -1 any filter.
template <int V, int K_T, int CT, int CONV = 0>
__global__ __launch_bounds__(kEncThreads) void encode_tile_kernel(const float* __restrict__ X,
                                                                  int64_t ldx,
                                                                  const float* __restrict__ P,
                                                                  uint8_t* __restrict__ idx,
                                                                  int64_t N, int C, int K_rt, int vec4,
                                                                  int idx_dword_ok, ConvGeom geom) {
    using E = EncTile<V, CT>;
    __shared__ float xs[E::kLdsFloats];
    __shared__ uint32_t is[kEncRows * (CT / 4)];

    const int K = K_T ? K_T : K_rt;
    const int col_tiles = (C + CT - 1) / CT;
    const int64_t row0 = (int64_t)(blockIdx.x / col_tiles) * kEncRows;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int tid = threadIdx.x;

    if constexpr (CONV > 0)
        stage_x_conv_taps<V, CT, CONV>(X, geom, N, C * V, row0, c0, xs, tid);
    else if constexpr (CONV < 0)
        stage_x_conv<V, CT>(X, geom, N, C * V, row0, c0, xs, tid);
    else
        stage_x<V, CT>(X, ldx, N, C * V, row0, c0, xs, vec4, tid);
    __syncthreads();

    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    uint32_t packed[E::PW];
    encode_codebooks<V, K_T, CT>(xs, P, C, K, c0, w, lane, packed);
    store_index_bytes<V, CT>(is + lane * (CT / 4), w * E::CPW, packed);
    __syncthreads();

    // each row's CT index bytes are contiguous in idx[N][C]
    for (int i = tid; i < kEncRows * (CT / 4); i += kEncThreads) {
        const int r = i / (CT / 4), j = i % (CT / 4);
        const int c = c0 + 4 * j;
        if (row0 + r >= N || c >= C) continue;
        const uint32_t wv = is[i];
        uint8_t* dst = idx + (row0 + r) * (int64_t)C + c;
        if (idx_dword_ok) {  // C % 4 == 0 and idx 4-byte aligned -> the whole dword is in range
            *reinterpret_cast<uint32_t*>(dst) = wv;
        } else {
#pragma unroll
            for (int b = 0; b < 4; ++b)
                if (c + b < C) dst[b] = (uint8_t)(wv >> (8 * b));
        }
    }
}

// Any V, any K: one thread per sub-vector, everything from global memory.  Slow path for
// sub-vector lengths outside the tiled kernel's instantiations.
__global__ __launch_bounds__(kEncThreads) void encode_generic_kernel(const float* __restrict__ X,
                                                                     int64_t ldx,
                                                                     const float* __restrict__ P,
                                                                     uint8_t* __restrict__ idx,
                                                                     int64_t N, int C, int K, int V) {
    const int64_t i = (int64_t)blockIdx.x * kEncThreads + threadIdx.x;
    if (i >= N * (int64_t)C) return;
    const int64_t n = i / C;
    const int c = (int)(i % C);
    const float* x = X + n * ldx + (int64_t)c * V;
    const float* pc = P + (size_t)c * K * V;
    uint32_t best = 0;
    float best_d = 0.f;
    for (int k = 0; k < K; ++k) {
        float d = 0.f;
        for (int v = 0; v < V; ++v) {
            const float t = x[v] - pc[k * V + v];
            d = __fmaf_rn(t, t, d);
        }
        if (k == 0) {
            best_d = d;
        } else if (d < best_d) {
            best_d = d;
            best = k;
        }
    }
    idx[i] = (uint8_t)best;
}

template <int V, int CT, int CONV = 0>
hipError_t launch_tile_ct(const float* P, int C, int K, const float* X, int64_t N, int64_t ldx,
                          uint8_t* idx, hipStream_t s, const ConvGeom& geom = ConvGeom{}) {
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const int64_t col_tiles = (C + CT - 1) / CT;
    const int64_t blocks = row_tiles * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int vec4 = ((CT * V) % 4 == 0) && (((int64_t)C * V) % 4 == 0) && (ldx % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const int idx_dword_ok = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    dim3 grid((unsigned)blocks), block(kEncThreads);
    if (K == 16)
        hipLaunchKernelGGL((encode_tile_kernel<V, 16, CT, CONV>), grid, block, 0, s, X, ldx, P, idx, N, C,
                           K, vec4, idx_dword_ok, geom);
    else if (K == 8)
        hipLaunchKernelGGL((encode_tile_kernel<V, 8, CT, CONV>), grid, block, 0, s, X, ldx, P, idx, N, C,
                           K, vec4, idx_dword_ok, geom);
    else
        hipLaunchKernelGGL((encode_tile_kernel<V, 0, CT, CONV>), grid, block, 0, s, X, ldx, P, idx, N, C,
                           K, vec4, idx_dword_ok, geom);
    return hipGetLastError();
}

// Tile width.  The full tile (a row of 64-144 floats) amortises the staging best, but a workgroup
// then encodes CT/4 codebooks per wavefront one after the other: with few rows that serial chain
// and the load latency in front of it are the whole run time, and the grid is too small to hide
// them.  Below ~1024 workgroups a quarter-width tile (never under one codebook per wavefront)
// gives four times the workgroups and a quarter of the chain.
template <int V, int CONV = 0>
hipError_t launch_tile(const float* P, int C, int K, const float* X, int64_t N, int64_t ldx,
                       uint8_t* idx, hipStream_t s, const ConvGeom& geom = ConvGeom{}) {
    constexpr int CT = enc_tile_codebooks(V);
    constexpr int CT_SMALL = CT / 4 >= 4 ? CT / 4 : 4;
    const int64_t full_blocks = ((N + kEncRows - 1) / kEncRows) * ((C + CT - 1) / CT);
    if (CT_SMALL < CT && full_blocks < 1024)
        return launch_tile_ct<V, CT_SMALL, CONV>(P, C, K, X, N, ldx, idx, s, geom);
    return launch_tile_ct<V, CT, CONV>(P, C, K, X, N, ldx, idx, s, geom);
}

}  // namespace

// Sub-vector lengths of the convolution settings in the paper (Sec. 6.1: 9 for a 3x3 filter, 4 for
// 1x1) plus the other tiled lengths that divide common Cin * kh * kw.
bool encode_conv_supported(int V) { return V == 1 || V == 2 || V == 3 || V == 4 || V == 8 || V == 9 || V == 16; }

template <int V>
hipError_t launch_conv_v(const float* P, int C, int K, const float* input, int64_t N, const ConvGeom& g,
                         uint8_t* idx, hipStream_t s) {
    const int taps = g.kh * g.kw;
    if (taps == 1) return launch_tile<V, 1>(P, C, K, input, N, 0, idx, s, g);
    if constexpr (V % 9 == 0) {
        if (taps == 9) return launch_tile<V, 9>(P, C, K, input, N, 0, idx, s, g);
    }
    return launch_tile<V, -1>(P, C, K, input, N, 0, idx, s, g);
}

hipError_t launch_encode_conv(const float* P, int C, int K, int V, const float* input, int64_t B,
                              const ConvGeom& g, uint8_t* idx, hipStream_t s) {
    const int64_t N = B * g.Ho * g.Wo;
    switch (V) {
        case 1: return launch_conv_v<1>(P, C, K, input, N, g, idx, s);
        case 2: return launch_conv_v<2>(P, C, K, input, N, g, idx, s);
        case 3: return launch_conv_v<3>(P, C, K, input, N, g, idx, s);
        case 4: return launch_conv_v<4>(P, C, K, input, N, g, idx, s);
        case 8: return launch_conv_v<8>(P, C, K, input, N, g, idx, s);
        case 9: return launch_conv_v<9>(P, C, K, input, N, g, idx, s);
        case 16: return launch_conv_v<16>(P, C, K, input, N, g, idx, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_encode(const float* P, int C, int K, int V, const float* X, int64_t N, int64_t ldx,
                         uint8_t* idx, hipStream_t s) {
    switch (V) {
        case 1: return launch_tile<1>(P, C, K, X, N, ldx, idx, s);
        case 2: return launch_tile<2>(P, C, K, X, N, ldx, idx, s);
        case 3: return launch_tile<3>(P, C, K, X, N, ldx, idx, s);
        case 4: return launch_tile<4>(P, C, K, X, N, ldx, idx, s);
        case 8: return launch_tile<8>(P, C, K, X, N, ldx, idx, s);
        case 9: return launch_tile<9>(P, C, K, X, N, ldx, idx, s);
        case 16: return launch_tile<16>(P, C, K, X, N, ldx, idx, s);
        case 32: return launch_tile<32>(P, C, K, X, N, ldx, idx, s);
        default: break;
    }
    const int64_t total = N * (int64_t)C;
    const int64_t blocks = (total + kEncThreads - 1) / kEncThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(encode_generic_kernel, dim3((unsigned)blocks), dim3(kEncThreads), 0, s, X, ldx, P,
                       idx, N, C, K, V);
    return hipGetLastError();
}

}  // namespace lutnn
