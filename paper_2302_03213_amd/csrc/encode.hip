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
#include <algorithm>

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

// Convolution with a 9-tap filter and V = 9 (a sub-vector is one channel's patch; Sec. 6.1's
// setting for 3x3 filters), staged by INPUT ROWS.  A workgroup owns 64 consecutive output pixels of
// one image and CT channels.  Instead of the 64 x 9 patch values per channel it stages the band of
// input rows those pixels touch - nrows x ncols floats per channel, zero filled outside the image,
// read as contiguous runs - so every input element is loaded once, not once per tap, and the
// arg-min code reads a lane's patch from LDS at (pixel offset) + (tap offset): consecutive lanes
// are consecutive pixels, hence consecutive LDS words.
//   bs_max  floats reserved per channel (the largest band of any tile; computed by the launcher)
template <int K_T, int CT>
__global__ __launch_bounds__(kEncThreads) void encode_conv9_band_kernel(
    const float* __restrict__ input, const float* __restrict__ P, uint8_t* __restrict__ idx, int C,
    int K_rt, ConvGeom g, int pix_tiles, int bs_max, int idx_dword_ok) {
    constexpr int V = 9;
    using E = EncTile<V, CT>;
    extern __shared__ float band[];  // [CT][bs_max], then the index bytes [64][CT/4] dwords
    uint32_t* is = reinterpret_cast<uint32_t*>(band + (size_t)CT * bs_max);

    const int K = K_T ? K_T : K_rt;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int col_tiles = (C + CT - 1) / CT;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int64_t rt = blockIdx.x / col_tiles;
    const int64_t b = rt / pix_tiles;
    const int pix = g.Ho * g.Wo;
    const int p0 = (int)(rt % pix_tiles) * kEncRows;
    const int p1 = min(p0 + kEncRows - 1, pix - 1);

    // the band of this tile (all wave-uniform)
    const int ho0 = p0 / g.Wo, ho1 = p1 / g.Wo;
    const int h_lo = ho0 * g.sh - g.ph;
    const int nrows = (ho1 - ho0) * g.sh + g.kh;
    const bool one_row = ho0 == ho1;
    const int w_lo = one_row ? (p0 - ho0 * g.Wo) * g.sw - g.pw : -g.pw;
    const int ncols = one_row ? (p1 - p0) * g.sw + g.kw : (g.Wo - 1) * g.sw + g.kw;

    // ---- stage: wave w takes channels w*CPW .. of the tile, lanes run along the columns
    for (int j = 0; j < E::CPW; ++j) {
        const int cl = w * E::CPW + j;
        const int ci = c0 + cl;
        const float* __restrict__ src = input + ((b * g.Cin + ci) * (int64_t)g.H) * g.W;
        float* __restrict__ dst = band + (size_t)cl * bs_max;
        for (int rr = 0; rr < nrows; ++rr) {
            const int hi = h_lo + rr;
            const bool row_in = ci < C && (unsigned)hi < (unsigned)g.H;  // uniform
            for (int cc = lane; cc < ncols; cc += 64) {
                const int wi = w_lo + cc;
                float v = 0.f;
                if (row_in && (unsigned)wi < (unsigned)g.W) v = src[(int64_t)hi * g.W + wi];
                dst[rr * ncols + cc] = v;
            }
        }
    }
    __syncthreads();

    // ---- this lane's pixel and the LDS offsets of its nine taps within a channel's band
    const int p = min(p0 + lane, p1);  // lanes past the last pixel repeat it (never stored)
    const int ho = p / g.Wo, wo = p - ho * g.Wo;
    const int base = (ho - ho0) * g.sh * ncols + (wo * g.sw - g.pw - w_lo);
    int toff[V];
    {
        int rk = 0, sk = 0;
#pragma unroll
        for (int t = 0; t < V; ++t) {
            toff[t] = base + rk * ncols + sk;
            if (++sk == g.kw) {
                sk = 0;
                ++rk;
            }
        }
    }
    uint32_t packed[E::PW];
#pragma unroll
    for (int j = 0; j < E::PW; ++j) packed[j] = 0;
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) {
        const int cl = w * E::CPW + j;
        const int c = c0 + cl;  // wave-uniform
        uint32_t best = 0;
        if (c < C) {
            const float* __restrict__ ch = band + (size_t)cl * bs_max;
            float x[V];
#pragma unroll
            for (int t = 0; t < V; ++t) x[t] = ch[toff[t]];
            best = nearest_centroid<V, K_T>(x, P + (size_t)c * K * V, K);
        }
        packed[j / 4] |= index_byte(best, j % 4);
    }
    store_index_bytes<V, CT>(is + lane * (CT / 4), w * E::CPW, packed);
    __syncthreads();

    const int64_t n0 = b * pix + p0;
    const int rows = p1 - p0 + 1;
    for (int i = tid; i < kEncRows * (CT / 4); i += kEncThreads) {
        const int r = i / (CT / 4), j = i % (CT / 4);
        const int c = c0 + 4 * j;
        if (r >= rows || c >= C) continue;
        const uint32_t wv = is[i];
        uint8_t* dst = idx + (n0 + r) * (int64_t)C + c;
        if (idx_dword_ok) {
            *reinterpret_cast<uint32_t*>(dst) = wv;
        } else {
#pragma unroll
            for (int bb = 0; bb < 4; ++bb)
                if (c + bb < C) dst[bb] = (uint8_t)(wv >> (8 * bb));
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
// them.  Below 2048 workgroups (eight per CU, two rounds of the four that fit) a quarter-width tile
// (never under one codebook per wavefront) gives four times the workgroups and a quarter of the
// chain; BERT's FFN-down at 4096 rows (1536 full tiles: one and a half rounds) 0.034 -> 0.029 ms.
template <int V, int CONV = 0>
hipError_t launch_tile(const float* P, int C, int K, const float* X, int64_t N, int64_t ldx,
                       uint8_t* idx, hipStream_t s, const ConvGeom& geom = ConvGeom{}) {
    constexpr int CT = enc_tile_codebooks(V);
    constexpr int CT_SMALL = CT / 4 >= 4 ? CT / 4 : 4;
    const int64_t full_blocks = ((N + kEncRows - 1) / kEncRows) * ((C + CT - 1) / CT);
    if (CT_SMALL < CT && full_blocks < 2048)
        return launch_tile_ct<V, CT_SMALL, CONV>(P, C, K, X, N, ldx, idx, s, geom);
    return launch_tile_ct<V, CT, CONV>(P, C, K, X, N, ldx, idx, s, geom);
}

}  // namespace

// Sub-vector lengths of the convolution settings in the paper (Sec. 6.1: 9 for a 3x3 filter, 4 for
// 1x1) plus the other tiled lengths that divide common Cin * kh * kw.
bool encode_conv_supported(int V) { return V == 1 || V == 2 || V == 3 || V == 4 || V == 8 || V == 9 || V == 16; }

// Largest band (floats per channel) of any 64-pixel tile of this geometry; see the band kernel.
int64_t conv_band_floats(const ConvGeom& g) {
    const int64_t one_row = (int64_t)g.kh * ((int64_t)std::min(kEncRows - 1, g.Wo - 1) * g.sw + g.kw);
    const int64_t span = std::min<int64_t>(g.Ho, (kEncRows - 2 + g.Wo) / g.Wo + 1);  // output rows a tile can touch
    const int64_t many = ((span - 1) * g.sh + g.kh) * ((int64_t)(g.Wo - 1) * g.sw + g.kw);
    return span >= 2 ? std::max(one_row, many) : one_row;
}

template <int CT>
hipError_t launch_conv9_band(const float* P, int C, int K, const float* input, int64_t B,
                             const ConvGeom& g, uint8_t* idx, int64_t bs_max, hipStream_t s) {
    const int64_t pix_tiles = ((int64_t)g.Ho * g.Wo + kEncRows - 1) / kEncRows;
    const int64_t blocks = B * pix_tiles * ((C + CT - 1) / CT);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const size_t shmem = (size_t)CT * bs_max * 4 + (size_t)kEncRows * (CT / 4) * 4;
    const int idx_dword_ok = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    dim3 grid((unsigned)blocks), block(kEncThreads);
    if (K == 16)
        hipLaunchKernelGGL((encode_conv9_band_kernel<16, CT>), grid, block, shmem, s, input, P, idx, C, K, g,
                           (int)pix_tiles, (int)bs_max, idx_dword_ok);
    else if (K == 8)
        hipLaunchKernelGGL((encode_conv9_band_kernel<8, CT>), grid, block, shmem, s, input, P, idx, C, K, g,
                           (int)pix_tiles, (int)bs_max, idx_dword_ok);
    else
        hipLaunchKernelGGL((encode_conv9_band_kernel<0, CT>), grid, block, shmem, s, input, P, idx, C, K, g,
                           (int)pix_tiles, (int)bs_max, idx_dword_ok);
    return hipGetLastError();
}

template <int V>
hipError_t launch_conv_v(const float* P, int C, int K, const float* input, int64_t B, int64_t N,
                         const ConvGeom& g, uint8_t* idx, hipStream_t s) {
    const int taps = g.kh * g.kw;
    if (taps == 1) return launch_tile<V, 1>(P, C, K, input, N, 0, idx, s, g);
    if constexpr (V == 9) {
        if (taps == 9) {
            // rows of the input staged once, if the widest band fits 48 KiB of LDS
            constexpr int CT = enc_tile_codebooks(9), CT_SMALL = 4;
            const int64_t bs = conv_band_floats(g);
            const int64_t pix_tiles = ((int64_t)g.Ho * g.Wo + kEncRows - 1) / kEncRows;
            const bool small_grid = B * pix_tiles * ((C + CT - 1) / CT) < 1024;
            if (small_grid && CT_SMALL * bs * 4 <= 48 * 1024)
                return launch_conv9_band<CT_SMALL>(P, C, K, input, B, g, idx, bs, s);
            if (!small_grid && CT * bs * 4 <= 48 * 1024)
                return launch_conv9_band<CT>(P, C, K, input, B, g, idx, bs, s);
            return launch_tile<V, 9>(P, C, K, input, N, 0, idx, s, g);
        }
    }
    return launch_tile<V, -1>(P, C, K, input, N, 0, idx, s, g);
}

hipError_t launch_encode_conv(const float* P, int C, int K, int V, const float* input, int64_t B,
                              const ConvGeom& g, uint8_t* idx, hipStream_t s) {
    const int64_t N = B * g.Ho * g.Wo;
    switch (V) {
        case 1: return launch_conv_v<1>(P, C, K, input, B, N, g, idx, s);
        case 2: return launch_conv_v<2>(P, C, K, input, B, N, g, idx, s);
        case 3: return launch_conv_v<3>(P, C, K, input, B, N, g, idx, s);
        case 4: return launch_conv_v<4>(P, C, K, input, B, N, g, idx, s);
        case 8: return launch_conv_v<8>(P, C, K, input, B, N, g, idx, s);
        case 9: return launch_conv_v<9>(P, C, K, input, B, N, g, idx, s);
        case 16: return launch_conv_v<16>(P, C, K, input, B, N, g, idx, s);
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
