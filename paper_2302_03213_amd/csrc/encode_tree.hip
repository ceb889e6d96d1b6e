// Hash encoding (arXiv 2302.03213, Sec. 2 "Hashing for acceleration", evaluated in Sec. 7) for gfx950.
//
// In place of the arg-min over K distances, every codebook owns a balanced binary tree with
// `levels` levels; its 2^levels leaves are the buckets.  A sub-vector starts at the root, and at
// each node compares ONE of its V values (the node's split index) with the node's threshold:
//
//   node <- 2*node + 1 + (x[split[node]] > threshold[node])        heap order, root 0
//   idx[n][c] = node - (2^levels - 1) after `levels` steps          leaves counted from the left
//
// The paper found this slower than the distance search on SIMD CPUs because the walk is a chain of
// dependent, data-dependent steps.  With lane = row a wavefront walks 64 trees at once and the
// steps of different codebooks are independent, so the cost per sub-vector is `levels` pairs of
// LDS reads and a handful of VALU operations against ~11*K operations for Eq. 2 with V = 4: the
// kernel is bound by reading X from HBM.
//
// Mapping: the tile machinery of the distance encoder (64 rows x CT codebooks of X staged through
// LDS with coalesced row segments, indices leaving through LDS as contiguous row segments).  The
// tile's nodes are staged as (threshold, split index) pairs so that a step is one 8-byte LDS read
// for the node and one 4-byte LDS read for the value it points at; within a wavefront the node
// reads hit at most 2^level distinct addresses.
#include <algorithm>
#include <type_traits>

#include "encode_tile.h"
#include "lutnn_kernels.h"

namespace lutnn {
namespace {

// Stages the (threshold, split index) pairs of the tile's codebooks; they are contiguous in both
// node arrays.  A split index outside [0, V) is clamped so that no value outside the sub-vector is
// ever read.  Codebooks past C get (threshold 0, index 0) nodes: their walk is harmless and its
// result is dropped.
template <int V, int CT>
__device__ __forceinline__ void stage_nodes(const int32_t* __restrict__ split_dim,
                                            const float* __restrict__ threshold, int C, int c0, int nodes,
                                            uint2* __restrict__ tp, int tid) {
    const int staged = std::min(CT, C - c0) * nodes;
    for (int i = tid; i < CT * nodes; i += kEncThreads) {
        uint2 node = make_uint2(0u, 0u);
        if (i < staged) {
            const size_t g = (size_t)c0 * nodes + i;
            const int d = split_dim[g];
            node = make_uint2(__float_as_uint(threshold[g]), (uint32_t)(d < 0 ? 0 : d >= V ? V - 1 : d));
        }
        tp[i] = node;
    }
}

// Wave `w` walks the trees of its CPW codebooks for row `lane` and leaves the row's index bytes in
// `is`.  The codebooks advance one level at a time: their walks are independent, so the LDS
// latency of one overlaps the others.  L_T: levels when known at compile time (0 = run-time).
template <int V, int CT, int L_T>
__device__ __forceinline__ void walk_trees(const float* __restrict__ xs, const uint2* __restrict__ tp,
                                           int levels, int nodes, int C, int c0, int w, int lane,
                                           uint32_t* __restrict__ is) {
    using E = EncTile<V, CT>;
    int node[E::CPW];
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) node[j] = 0;
    const float* __restrict__ xrow = xs + lane * E::LS + w * E::CPW * V;
    const uint2* __restrict__ tw = tp + (size_t)w * E::CPW * nodes;
    auto step = [&]() {
        uint2 p[E::CPW];
        float x[E::CPW];
#pragma unroll
        for (int j = 0; j < E::CPW; ++j) p[j] = tw[j * nodes + node[j]];
#pragma unroll
        for (int j = 0; j < E::CPW; ++j) x[j] = xrow[j * V + p[j].y];
#pragma unroll
        for (int j = 0; j < E::CPW; ++j) node[j] = 2 * node[j] + 1 + (x[j] > __uint_as_float(p[j].x) ? 1 : 0);
    };
    if constexpr (L_T != 0) {
#pragma unroll
        for (int l = 0; l < L_T; ++l) step();
    } else {
        for (int l = 0; l < levels; ++l) step();
    }
    uint32_t packed[E::PW];
#pragma unroll
    for (int j = 0; j < E::PW; ++j) packed[j] = 0;
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) {
        const uint32_t leaf = (c0 + w * E::CPW + j < C) ? (uint32_t)(node[j] - nodes) : 0u;
        packed[j / 4] |= leaf << (8 * (j % 4));
    }
    store_index_bytes<V, CT>(is + lane * (CT / 4), w * E::CPW, packed);
}

// Each row's CT index bytes are contiguous in idx[N][C]: out as row segments.
template <int CT>
__device__ __forceinline__ void write_index_rows(const uint32_t* __restrict__ is, uint8_t* __restrict__ idx,
                                                 int64_t N, int C, int64_t row0, int c0, int idx_dword_ok,
                                                 int tid) {
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

template <int V, int CT, int L_T>
__global__ __launch_bounds__(kEncThreads) void encode_tree_tile_kernel(
    const float* __restrict__ X, int64_t ldx, const int32_t* __restrict__ split_dim,
    const float* __restrict__ threshold, uint8_t* __restrict__ idx, int64_t N, int C, int levels_rt,
    int vec4, int idx_dword_ok) {
    using E = EncTile<V, CT>;
    __shared__ float xs[E::kLdsFloats];
    __shared__ uint32_t is[kEncRows * (CT / 4)];
    extern __shared__ uint2 tp[];  // [CT][nodes]: .x = threshold bits, .y = split index

    const int levels = L_T ? L_T : levels_rt;
    const int nodes = (1 << levels) - 1;
    const int col_tiles = (C + CT - 1) / CT;
    const int64_t row0 = (int64_t)(blockIdx.x / col_tiles) * kEncRows;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int tid = threadIdx.x;

    stage_nodes<V, CT>(split_dim, threshold, C, c0, nodes, tp, tid);
    stage_x<V, CT>(X, ldx, N, C * V, row0, c0, xs, vec4, tid);
    __syncthreads();
    walk_trees<V, CT, L_T>(xs, tp, levels, nodes, C, c0, __builtin_amdgcn_readfirstlane(tid >> 6), tid & 63, is);
    __syncthreads();
    write_index_rows<CT>(is, idx, N, C, row0, c0, idx_dword_ok, tid);
}

// The same for a convolution read from its NCHW batch (Sec. 4): the tile's rows are gathered through
// the geometry instead of being copied from a matrix.
template <int V, int CT, int L_T>
__global__ __launch_bounds__(kEncThreads) void encode_tree_conv_kernel(
    const float* __restrict__ input, ConvGeom geom, const int32_t* __restrict__ split_dim,
    const float* __restrict__ threshold, uint8_t* __restrict__ idx, int64_t N, int C, int levels_rt,
    int idx_dword_ok) {
    using E = EncTile<V, CT>;
    __shared__ float xs[E::kLdsFloats];
    __shared__ uint32_t is[kEncRows * (CT / 4)];
    extern __shared__ uint2 tp[];

    const int levels = L_T ? L_T : levels_rt;
    const int nodes = (1 << levels) - 1;
    const int col_tiles = (C + CT - 1) / CT;
    const int64_t row0 = (int64_t)(blockIdx.x / col_tiles) * kEncRows;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int tid = threadIdx.x;

    stage_nodes<V, CT>(split_dim, threshold, C, c0, nodes, tp, tid);
    stage_x_conv<V, CT>(input, geom, N, C * V, row0, c0, xs, tid);
    __syncthreads();
    walk_trees<V, CT, L_T>(xs, tp, levels, nodes, C, c0, __builtin_amdgcn_readfirstlane(tid >> 6), tid & 63, is);
    __syncthreads();
    write_index_rows<CT>(is, idx, N, C, row0, c0, idx_dword_ok, tid);
}

// Deep trees (9 to 12 levels; Sec. 7 evaluates 12): 2^levels - 1 nodes per codebook no longer fit
// LDS for a tile's codebooks, so the walks read their nodes from global memory - the upper levels
// are shared by all 64 lanes of a wavefront and by every row tile, so they stay in the caches; the
// lowest levels are one 8-byte pair of loads per lane.  The X tile is staged as above; leaves are
// 16-bit and leave through LDS so that each row's CT indices go out as one segment.
template <int V, int CT>
__global__ __launch_bounds__(kEncThreads) void encode_tree_deep_kernel(
    const float* __restrict__ X, int64_t ldx, const int32_t* __restrict__ split_dim,
    const float* __restrict__ threshold, uint16_t* __restrict__ idx, int64_t N, int C, int levels,
    int vec4) {
    using E = EncTile<V, CT>;
    __shared__ float xs[E::kLdsFloats];
    __shared__ uint16_t is[kEncRows * CT];

    const int nodes = (1 << levels) - 1;
    const int col_tiles = (C + CT - 1) / CT;
    const int64_t row0 = (int64_t)(blockIdx.x / col_tiles) * kEncRows;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);

    stage_x<V, CT>(X, ldx, N, C * V, row0, c0, xs, vec4, tid);
    __syncthreads();
    const float* __restrict__ xrow = xs + lane * E::LS + w * E::CPW * V;
    int node[E::CPW];
    const int32_t* dim[E::CPW];
    const float* thr[E::CPW];
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) {
        // codebooks past C walk the last codebook's tree; their leaves are never written
        const int c = min(c0 + w * E::CPW + j, C - 1);
        node[j] = 0;
        dim[j] = split_dim + (size_t)c * nodes;
        thr[j] = threshold + (size_t)c * nodes;
    }
    for (int l = 0; l < levels; ++l) {  // the codebooks advance together: independent walks
        int d[E::CPW];
        float t[E::CPW];
#pragma unroll
        for (int j = 0; j < E::CPW; ++j) {
            d[j] = dim[j][node[j]];
            t[j] = thr[j][node[j]];
        }
#pragma unroll
        for (int j = 0; j < E::CPW; ++j) {
            const int dd = d[j] < 0 ? 0 : d[j] >= V ? V - 1 : d[j];
            node[j] = 2 * node[j] + 1 + (xrow[j * V + dd] > t[j] ? 1 : 0);
        }
    }
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) is[lane * CT + w * E::CPW + j] = (uint16_t)(node[j] - nodes);
    __syncthreads();
    for (int i = tid; i < kEncRows * CT; i += kEncThreads) {
        const int r = i / CT, c = c0 + i % CT;
        if (row0 + r < N && c < C) idx[(row0 + r) * (int64_t)C + c] = is[i];
    }
}

// Any V: one thread per sub-vector, everything from global memory.
template <typename IdxT>
__global__ __launch_bounds__(kEncThreads) void encode_tree_generic_kernel(
    const float* __restrict__ X, int64_t ldx, const int32_t* __restrict__ split_dim,
    const float* __restrict__ threshold, IdxT* __restrict__ idx, int64_t N, int C, int levels,
    int V) {
    const int64_t i = (int64_t)blockIdx.x * kEncThreads + threadIdx.x;
    if (i >= N * (int64_t)C) return;
    const int64_t n = i / C;
    const int c = (int)(i % C);
    const int nodes = (1 << levels) - 1;
    const float* x = X + n * ldx + (int64_t)c * V;
    const int32_t* dim = split_dim + (size_t)c * nodes;
    const float* thr = threshold + (size_t)c * nodes;
    int node = 0;
    for (int l = 0; l < levels; ++l) {
        const int d = dim[node];
        node = 2 * node + 1 + (x[d < 0 ? 0 : d >= V ? V - 1 : d] > thr[node] ? 1 : 0);
    }
    idx[i] = (IdxT)(node - nodes);
}

template <int V>
hipError_t launch_tree_deep(const int32_t* split_dim, const float* threshold, int C, int levels,
                            const float* X, int64_t N, int64_t ldx, uint16_t* idx, hipStream_t s) {
    // quarter-width tiles: four times the wavefronts to hide the walks' global-memory latency
    constexpr int CTF = enc_tile_codebooks(V);
    constexpr int CT = CTF / 4 >= 4 ? CTF / 4 : 4;
    const int64_t blocks = ((N + kEncRows - 1) / kEncRows) * ((C + CT - 1) / CT);
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int vec4 = ((CT * V) % 4 == 0) && (((int64_t)C * V) % 4 == 0) && (ldx % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    hipLaunchKernelGGL((encode_tree_deep_kernel<V, CT>), dim3((unsigned)blocks), dim3(kEncThreads), 0, s, X, ldx,
                       split_dim, threshold, idx, N, C, levels, vec4);
    return hipGetLastError();
}

template <int V, int CT>
hipError_t launch_tree_ct(const int32_t* split_dim, const float* threshold, int C, int levels,
                          const float* X, int64_t N, int64_t ldx, uint8_t* idx, hipStream_t s) {
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const int64_t col_tiles = (C + CT - 1) / CT;
    const int64_t blocks = row_tiles * col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    const int vec4 = ((CT * V) % 4 == 0) && (((int64_t)C * V) % 4 == 0) && (ldx % 4 == 0) &&
                     ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
    const int idx_dword_ok = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    const size_t node_bytes = (size_t)CT * ((1u << levels) - 1) * sizeof(uint2);
    dim3 block(kEncThreads);
    dim3 grid((unsigned)blocks);
    if (levels == 4)
        hipLaunchKernelGGL((encode_tree_tile_kernel<V, CT, 4>), grid, block, node_bytes, s, X, ldx,
                           split_dim, threshold, idx, N, C, levels, vec4, idx_dword_ok);
    else
        hipLaunchKernelGGL((encode_tree_tile_kernel<V, CT, 0>), grid, block, node_bytes, s, X, ldx,
                           split_dim, threshold, idx, N, C, levels, vec4, idx_dword_ok);
    return hipGetLastError();
}

// Tile width: the full tile unless the grid would be small (as for the distance encoder) or the
// tile's nodes would take more than 24 KiB of LDS (deep trees); then a quarter of it.
template <int V>
hipError_t launch_tree(const int32_t* split_dim, const float* threshold, int C, int levels,
                       const float* X, int64_t N, int64_t ldx, uint8_t* idx, hipStream_t s) {
    constexpr int CT = enc_tile_codebooks(V);
    constexpr int CT_SMALL = CT / 4 >= 4 ? CT / 4 : 4;
    const int64_t full_blocks = ((N + kEncRows - 1) / kEncRows) * ((C + CT - 1) / CT);
    const size_t full_node_bytes = (size_t)CT * ((1u << levels) - 1) * sizeof(uint2);
    if (CT_SMALL < CT && (full_blocks < 1024 || full_node_bytes > 24 * 1024))
        return launch_tree_ct<V, CT_SMALL>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
    return launch_tree_ct<V, CT>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
}

template <int V>
hipError_t launch_tree_conv(const int32_t* split_dim, const float* threshold, int C, int levels,
                            const float* input, int64_t N, const ConvGeom& g, uint8_t* idx, hipStream_t s) {
    // quarter-width tiles when the grid is small or the nodes of a full tile exceed 24 KiB, as above
    constexpr int CTF = enc_tile_codebooks(V);
    constexpr int CTS = CTF / 4 >= 4 ? CTF / 4 : 4;
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const size_t full_node_bytes = (size_t)CTF * ((1u << levels) - 1) * sizeof(uint2);
    const bool small = CTS < CTF && (row_tiles * ((C + CTF - 1) / CTF) < 1024 || full_node_bytes > 24 * 1024);
    const int idx_dword_ok = (C % 4 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 3) == 0);
    auto go = [&](auto ct_c) {
        constexpr int CT = decltype(ct_c)::value;
        const int64_t blocks = row_tiles * ((C + CT - 1) / CT);
        if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
        const size_t node_bytes = (size_t)CT * ((1u << levels) - 1) * sizeof(uint2);
        if (levels == 4)
            hipLaunchKernelGGL((encode_tree_conv_kernel<V, CT, 4>), dim3((unsigned)blocks), dim3(kEncThreads),
                               node_bytes, s, input, g, split_dim, threshold, idx, N, C, levels, idx_dword_ok);
        else
            hipLaunchKernelGGL((encode_tree_conv_kernel<V, CT, 0>), dim3((unsigned)blocks), dim3(kEncThreads),
                               node_bytes, s, input, g, split_dim, threshold, idx, N, C, levels, idx_dword_ok);
        return hipGetLastError();
    };
    return small ? go(std::integral_constant<int, CTS>{}) : go(std::integral_constant<int, CTF>{});
}

}  // namespace

// Sub-vector lengths as for the distance encoder's convolution form.
hipError_t launch_encode_tree_conv(const int32_t* split_dim, const float* threshold, int C, int levels,
                                   int V, const float* input, int64_t B, const ConvGeom& g, uint8_t* idx,
                                   hipStream_t s) {
    const int64_t N = B * g.Ho * g.Wo;
    switch (V) {
        case 1: return launch_tree_conv<1>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 2: return launch_tree_conv<2>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 3: return launch_tree_conv<3>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 4: return launch_tree_conv<4>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 8: return launch_tree_conv<8>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 9: return launch_tree_conv<9>(split_dim, threshold, C, levels, input, N, g, idx, s);
        case 16: return launch_tree_conv<16>(split_dim, threshold, C, levels, input, N, g, idx, s);
        default: return hipErrorInvalidValue;
    }
}

hipError_t launch_encode_tree(const int32_t* split_dim, const float* threshold, int C, int levels,
                              int V, const float* X, int64_t N, int64_t ldx, uint8_t* idx,
                              hipStream_t s) {
    switch (V) {
        case 1: return launch_tree<1>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 2: return launch_tree<2>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 3: return launch_tree<3>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 4: return launch_tree<4>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 8: return launch_tree<8>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 9: return launch_tree<9>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 16: return launch_tree<16>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 32: return launch_tree<32>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        default: break;
    }
    const int64_t total = N * (int64_t)C;
    const int64_t blocks = (total + kEncThreads - 1) / kEncThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(encode_tree_generic_kernel<uint8_t>, dim3((unsigned)blocks), dim3(kEncThreads), 0, s, X, ldx,
                       split_dim, threshold, idx, N, C, levels, V);
    return hipGetLastError();
}

// 16-bit leaves: trees of up to 12 levels (any depth from 1; the 8-bit form is the faster one up to 8).
hipError_t launch_encode_tree16(const int32_t* split_dim, const float* threshold, int C, int levels,
                                int V, const float* X, int64_t N, int64_t ldx, uint16_t* idx,
                                hipStream_t s) {
    switch (V) {
        case 1: return launch_tree_deep<1>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 2: return launch_tree_deep<2>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 3: return launch_tree_deep<3>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 4: return launch_tree_deep<4>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 8: return launch_tree_deep<8>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 9: return launch_tree_deep<9>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 16: return launch_tree_deep<16>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        case 32: return launch_tree_deep<32>(split_dim, threshold, C, levels, X, N, ldx, idx, s);
        default: break;
    }
    const int64_t total = N * (int64_t)C;
    const int64_t blocks = (total + kEncThreads - 1) / kEncThreads;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL(encode_tree_generic_kernel<uint16_t>, dim3((unsigned)blocks), dim3(kEncThreads), 0, s, X,
                       ldx, split_dim, threshold, idx, N, C, levels, V);
    return hipGetLastError();
}

}  // namespace lutnn
