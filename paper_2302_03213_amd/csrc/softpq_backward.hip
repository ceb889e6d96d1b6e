// Soft-PQ backward pass (arXiv 2302.03213, Sec. 3.1-3.2, Eq. 5-6) for gfx950.
//
// Training replaces the one-hot arg-min encoding by a softmax over the same K squared distances
// (Eq. 5) in the backward pass only (Eq. 6: value of the hard output, gradient of the soft one):
//
//   d_k  = sum_v (x_v - P_kv)^2             s = softmax_k(-d_k / t)
//   Ysoft[n][m] = sum_c sum_k s[n][c][k] T[c][k][m],   T = P . W  (Eq. 3, real valued)
//
// With the weights W fixed (the tables are rebuilt from the centroids), every gradient the paper
// learns follows from  Z = dL/dY . W^T  [N][D], the input gradient of the ordinary linear layer,
// which a plain GEMM supplies.  Per row n and codebook c, with z = Z[n][cV..cV+V):
//
//   A_k  = sum_v z_v P_kv                   (= dL/ds_k, because dL/ds_k = sum_m dL/dY_m T[c][k][m])
//   dz_k = s_k (A_k - sum_j s_j A_j)        softmax;  the logit is -d_k / t
//   dd_k = -dz_k / t                        dL/d(d_k)
//   dL/dt      += sum_k dz_k d_k / t^2
//   dL/dx_v     = sum_k 2 dd_k (x_v - P_kv)
//   dL/dP_kv   += s_k z_v - 2 dd_k (x_v - P_kv)        summed over the rows
//
// Mapping.  The encoder's tile (64 rows x CT codebooks, lane = row, one codebook per wavefront at
// a time, centroids wave-uniform in scalar registers) with a second staged tile for Z.  dL/dx
// overwrites the X tile in LDS and leaves as coalesced row segments.  The sums over rows are the
// expensive part: a lane's K*VG contributions (VG = 64/K values of v at a time = 64 numbers) go
// through a reduce-scatter over the 64 lanes (6 exchange steps that halve the vector: 63
// exchanges instead of 64 x 6 for 64 separate butterflies), after which lane l holds element l of
// the group summed over the tile's rows.  A workgroup walks a chunk of row tiles and keeps these
// sums in registers; per chunk they go to a partial buffer that a second kernel adds up in a
// fixed order, so results are reproducible run to run (no floating-point atomics).
#include <algorithm>
#include <type_traits>

#include "encode_tile.h"
#include "lutnn_kernels.h"

namespace lutnn {
namespace {

// Codebooks per tile: half the encoder's, because two tiles (X and Z) are staged.
constexpr int softpq_tile_codebooks(int V) {
    return enc_tile_codebooks(V) == 0 ? 0 : (enc_tile_codebooks(V) / 2 >= 4 ? enc_tile_codebooks(V) / 2 : 4);
}

typedef unsigned uint2v __attribute__((ext_vector_type(2)));

// lo + (lo of the partner lane) where this lane keeps the lower half, hi + (hi of the partner)
// where it keeps the upper half; the partner is lane ^ 32 / lane ^ 16.  The row-swap instructions
// exchange exactly the halves the two lanes have no use for, so no select is needed.
__device__ __forceinline__ float exchange_add_32(float lo, float hi) {
    const uint2v r = __builtin_amdgcn_permlane32_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}
__device__ __forceinline__ float exchange_add_16(float lo, float hi) {
    const uint2v r = __builtin_amdgcn_permlane16_swap(__float_as_uint(lo), __float_as_uint(hi), false, false);
    return __uint_as_float(r.x) + __uint_as_float(r.y);
}
// x + (x of lane ^ 8 | ^ 2 | ^ 1) as one DPP add; lane ^ 4 has no DPP form and goes through the
// LDS crossbar (no memory access).
template <int CTRL>
__device__ __forceinline__ float add_dpp(float x) {
    return x + __uint_as_float(__builtin_amdgcn_update_dpp(0, __float_as_uint(x), CTRL, 0xf, 0xf, false));
}
__device__ __forceinline__ float add_xor4(float x) {
    return x + __uint_as_float(__builtin_amdgcn_ds_swizzle(__float_as_uint(x), 0x101f));  // swap, mask 4
}

// Sum over the 64 lanes of a wavefront of a 64-element vector per lane; lane l returns element l
// (every step halves the vector: the lane whose bit m is clear keeps the lower half).
__device__ __forceinline__ float reduce_scatter_64(float (&v)[64], int lane) {
#pragma unroll
    for (int i = 0; i < 32; ++i) v[i] = exchange_add_32(v[i], v[i + 32]);
#pragma unroll
    for (int i = 0; i < 16; ++i) v[i] = exchange_add_16(v[i], v[i + 16]);
    const bool up8 = (lane & 8) != 0, up4 = (lane & 4) != 0, up2 = (lane & 2) != 0, up1 = (lane & 1) != 0;
#pragma unroll
    for (int i = 0; i < 8; ++i) {  // row_ror:8 pairs lane with lane ^ 8 inside its row of 16
        const float lo = add_dpp<0x128>(v[i]), hi = add_dpp<0x128>(v[i + 8]);
        v[i] = up8 ? hi : lo;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float lo = add_xor4(v[i]), hi = add_xor4(v[i + 4]);
        v[i] = up4 ? hi : lo;
    }
#pragma unroll
    for (int i = 0; i < 2; ++i) {  // quad_perm [2,3,0,1]
        const float lo = add_dpp<0x4E>(v[i]), hi = add_dpp<0x4E>(v[i + 2]);
        v[i] = up2 ? hi : lo;
    }
    const float lo = add_dpp<0xB1>(v[0]), hi = add_dpp<0xB1>(v[1]);  // quad_perm [1,0,3,2]
    return up1 ? hi : lo;
}

template <int V, int K_T>
struct SoftPq {
    static constexpr int CT = softpq_tile_codebooks(V);
    static constexpr int VG = 64 / K_T;             // values of v per reduce group
    static constexpr int NG = (V + VG - 1) / VG;    // groups per codebook
    static constexpr int GROUP_FLOATS = NG * 64;    // partial floats per codebook
};

// grid: chunks * col_tiles workgroups, column tile fastest.
//   partial    [chunks][C][NG*64] sums of the dP contributions over the chunk's rows
//   partial_dt [gridDim.x] one sum of dz_k * d_k per workgroup
template <int V, int K_T>
__global__ __launch_bounds__(kEncThreads) void softpq_backward_kernel(
    const float* __restrict__ X, int64_t ldx, const float* __restrict__ Z, int64_t ldz,
    const float* __restrict__ P, float inv_t, float* __restrict__ dX, int64_t lddx,
    float* __restrict__ partial, float* __restrict__ partial_dt, int64_t N, int C, int tiles_per_chunk,
    int vec4_x, int vec4_z, int vec4_dx) {
    using S = SoftPq<V, K_T>;
    constexpr int CT = S::CT;
    using E = EncTile<V, CT>;
    __shared__ float xs[E::kLdsFloats];
    __shared__ float zs[E::kLdsFloats];
    __shared__ float dt_s[4];

    const int col_tiles = (C + CT - 1) / CT;
    const int chunk = blockIdx.x / col_tiles;
    const int c0 = (int)(blockIdx.x % col_tiles) * CT;
    const int tid = threadIdx.x;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int lane = tid & 63;
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    const int64_t tile_begin = (int64_t)chunk * tiles_per_chunk;
    const int64_t tile_end = std::min<int64_t>(tile_begin + tiles_per_chunk, row_tiles);

    const float inv_t_log2e = inv_t * 1.44269504f;
    float acc[E::CPW][S::NG];
#pragma unroll
    for (int j = 0; j < E::CPW; ++j)
#pragma unroll
        for (int g = 0; g < S::NG; ++g) acc[j][g] = 0.f;
    float dt_acc = 0.f;

    for (int64_t tile = tile_begin; tile < tile_end; ++tile) {
        const int64_t row0 = tile * kEncRows;
        stage_x<V, CT>(X, ldx, N, C * V, row0, c0, xs, vec4_x, tid);
        stage_x<V, CT>(Z, ldz, N, C * V, row0, c0, zs, vec4_z, tid);
        __syncthreads();

        // one codebook at a time (rolled: a codebook's K*V centroid values fill the scalar registers)
#pragma unroll 1
        for (int j = 0; j < E::CPW; ++j) {
            const int cl = w * E::CPW + j;
            const int c = c0 + cl;  // wave-uniform
            if (c >= C) continue;
            const float* __restrict__ pc = P + (size_t)c * K_T * V;
            float* __restrict__ xr = xs + lane * E::LS + cl * V;
            const float* __restrict__ zr = zs + lane * E::LS + cl * V;

            // centroid by centroid, so that only one centroid's V values (one scalar load) are
            // live at a time: value by value, all K*V of them would have to stay in scalar registers
            // through the loop, and what does not fit is spilled into vector lanes
            float xv[V], zv[V];
#pragma unroll
            for (int v = 0; v < V; ++v) xv[v] = xr[v], zv[v] = zr[v];
            float d[K_T], a[K_T];
#pragma unroll
            for (int k = 0; k < K_T; ++k) {
                d[k] = a[k] = 0.f;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    const float p = pc[k * V + v];
                    const float t = xv[v] - p;
                    d[k] = __fmaf_rn(t, t, d[k]);
                    a[k] = __fmaf_rn(zv[v], p, a[k]);
                }
            }
            float dmin = d[0];
#pragma unroll
            for (int k = 1; k < K_T; ++k) dmin = fminf(dmin, d[k]);
            float s[K_T], ssum = 0.f;
#pragma unroll
            for (int k = 0; k < K_T; ++k) {
                s[k] = __builtin_amdgcn_exp2f((dmin - d[k]) * inv_t_log2e);  // exp((dmin - d_k) / t)
                ssum += s[k];
            }
            const float rs = 1.0f / ssum;
            float abar = 0.f;
#pragma unroll
            for (int k = 0; k < K_T; ++k) {
                s[k] *= rs;
                abar = __fmaf_rn(s[k], a[k], abar);
            }
            float e2[K_T];  // 2 * dd_k = -2 dz_k / t
#pragma unroll
            for (int k = 0; k < K_T; ++k) {
                const float dz = s[k] * (a[k] - abar);
                dt_acc = __fmaf_rn(dz, d[k], dt_acc);
                e2[k] = -2.0f * dz * inv_t;
            }
#pragma unroll
            for (int g = 0; g < S::NG; ++g) {
                float contrib[64];
                float dxv[S::VG];
#pragma unroll
                for (int vv = 0; vv < S::VG; ++vv) dxv[vv] = 0.f;
#pragma unroll
                for (int k = 0; k < K_T; ++k) {
#pragma unroll
                    for (int vv = 0; vv < S::VG; ++vv) {
                        const int v = g * S::VG + vv;
                        if (v < V) {
                            const float t = e2[k] * (xv[v] - pc[k * V + v]);  // 2 dd_k (x_v - P_kv)
                            dxv[vv] += t;
                            contrib[k * S::VG + vv] = __fmaf_rn(s[k], zv[v], -t);
                        } else {
                            contrib[k * S::VG + vv] = 0.f;
                        }
                    }
                }
#pragma unroll
                for (int vv = 0; vv < S::VG; ++vv)
                    if (g * S::VG + vv < V) xr[g * S::VG + vv] = dxv[vv];  // this lane's own element: no other lane reads it
                const float r = reduce_scatter_64(contrib, lane);
#pragma unroll
                for (int jj = 0; jj < E::CPW; ++jj)  // j is wave-uniform; acc keeps static indices
                    if (jj == j) acc[jj][g] += r;
            }
        }
        __syncthreads();

        if (dX) {  // the X tile now holds dL/dX: out as coalesced row segments
            if (vec4_dx) {
                constexpr int Q = E::TW / 4;
                for (int i = tid; i < kEncRows * Q; i += kEncThreads) {
                    const int r = i / Q, col = (i % Q) * 4;
                    const int gcol = c0 * V + col;
                    if (row0 + r < N && gcol < C * V) {
                        const float* src = xs + r * E::LS + col;
                        *reinterpret_cast<float4*>(dX + (row0 + r) * lddx + gcol) =
                            make_float4(src[0], src[1], src[2], src[3]);
                    }
                }
            } else {
                for (int i = tid; i < kEncRows * E::TW; i += kEncThreads) {
                    const int r = i / E::TW, col = i % E::TW;
                    const int gcol = c0 * V + col;
                    if (row0 + r < N && gcol < C * V) dX[(row0 + r) * lddx + gcol] = xs[r * E::LS + col];
                }
            }
        }
        __syncthreads();  // the tiles are restaged next
    }

    // per-chunk sums of the centroid gradient: lane l holds element l of each group
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) {
        const int c = c0 + w * E::CPW + j;
        if (c >= C) continue;
        float* dst = partial + ((size_t)chunk * C + c) * S::GROUP_FLOATS;
#pragma unroll
        for (int g = 0; g < S::NG; ++g) dst[g * 64 + lane] = acc[j][g];
    }
    // temperature: wave sum, then the four waves in a fixed order
#pragma unroll
    for (int m = 32; m >= 1; m >>= 1) dt_acc += __shfl_xor(dt_acc, m, 64);
    if (lane == 0) dt_s[w] = dt_acc;
    __syncthreads();
    if (tid == 0) partial_dt[blockIdx.x] = (dt_s[0] + dt_s[1]) + (dt_s[2] + dt_s[3]);
}

// dP[c][k][v] = sum over chunks (ascending) of partial[chunk][c][group of v][k*VG + v % VG];
// block 0 also folds the workgroups' temperature sums, lane-strided then a fixed butterfly.
template <int V, int K_T>
__global__ __launch_bounds__(256) void softpq_reduce_kernel(const float* __restrict__ partial,
                                                            const float* __restrict__ partial_dt,
                                                            int chunks, int n_dt, int C, float inv_t,
                                                            float* __restrict__ dP, float* __restrict__ dt) {
    using S = SoftPq<V, K_T>;
    const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
    const int64_t total = (int64_t)C * K_T * V;
    if (i < total) {
        const int c = (int)(i / (K_T * V));
        const int k = (int)(i / V) % K_T;
        const int v = (int)(i % V);
        const size_t e = (size_t)c * S::GROUP_FLOATS + (v / S::VG) * 64 + k * S::VG + (v % S::VG);
        // loads eight at a time (independent), added in ascending chunk order
        float sum = 0.f;
        const size_t stride = (size_t)C * S::GROUP_FLOATS;
        int ch = 0;
        for (; ch + 8 <= chunks; ch += 8) {
            float t[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) t[u] = partial[(size_t)(ch + u) * stride + e];
#pragma unroll
            for (int u = 0; u < 8; ++u) sum += t[u];
        }
        for (; ch < chunks; ++ch) sum += partial[(size_t)ch * stride + e];
        dP[i] = sum;
    }
    if (dt && blockIdx.x == 0 && threadIdx.x < 64) {
        float sum = 0.f;
        for (int j = threadIdx.x; j < n_dt; j += 64) sum += partial_dt[j];
#pragma unroll
        for (int m = 32; m >= 1; m >>= 1) sum += __shfl_xor(sum, m, 64);
        if (threadIdx.x == 0) *dt = sum * inv_t * inv_t;
    }
}

struct Plan {
    int chunks, tiles_per_chunk, col_tiles;
};

template <int V, int K_T>
Plan make_plan(int C, int64_t N) {
    constexpr int CT = SoftPq<V, K_T>::CT;
    Plan p;
    p.col_tiles = (C + CT - 1) / CT;
    const int64_t row_tiles = (N + kEncRows - 1) / kEncRows;
    // about 2048 workgroups, at most 64 chunks (the partial buffer is chunks * C * K * V floats)
    int64_t chunks = std::min<int64_t>(std::min<int64_t>((2048 + p.col_tiles - 1) / p.col_tiles, 64), row_tiles);
    chunks = std::max<int64_t>(chunks, 1);
    p.tiles_per_chunk = (int)((row_tiles + chunks - 1) / chunks);
    p.chunks = (int)((row_tiles + p.tiles_per_chunk - 1) / p.tiles_per_chunk);
    return p;
}

template <int V, int K_T>
size_t workspace_bytes_for(int C, int64_t N) {
    const Plan p = make_plan<V, K_T>(C, N);
    return ((size_t)p.chunks * C * SoftPq<V, K_T>::GROUP_FLOATS + (size_t)p.chunks * p.col_tiles) * sizeof(float);
}

inline int vec4_ok(const float* A, int64_t ld, int C, int V, int CT) {
    return ((CT * V) % 4 == 0) && (((int64_t)C * V) % 4 == 0) && (ld % 4 == 0) &&
           ((reinterpret_cast<uintptr_t>(A) & 15) == 0);
}

template <int V, int K_T>
hipError_t launch_softpq(const float* P, int C, float t, const float* X, int64_t N, int64_t ldx,
                         const float* Z, int64_t ldz, float* dP, float* dX, int64_t lddx, float* dt,
                         float* workspace, hipStream_t s) {
    constexpr int CT = SoftPq<V, K_T>::CT;
    const float inv_t = 1.0f / t;
    const int64_t total = (int64_t)C * K_T * V;
    if (N == 0) {  // empty sums: the reduction over zero chunks writes the zeros
        hipLaunchKernelGGL((softpq_reduce_kernel<V, K_T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0,
                           s, workspace, workspace, 0, 0, C, inv_t, dP, dt);
        return hipGetLastError();
    }
    const Plan p = make_plan<V, K_T>(C, N);
    const int64_t blocks = (int64_t)p.chunks * p.col_tiles;
    if (blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    float* partial = workspace;
    float* partial_dt = workspace + (size_t)p.chunks * C * SoftPq<V, K_T>::GROUP_FLOATS;
    hipLaunchKernelGGL((softpq_backward_kernel<V, K_T>), dim3((unsigned)blocks), dim3(kEncThreads), 0, s, X,
                       ldx, Z, ldz, P, inv_t, dX, lddx, partial, partial_dt, N, C, p.tiles_per_chunk,
                       vec4_ok(X, ldx, C, V, CT), vec4_ok(Z, ldz, C, V, CT),
                       dX ? vec4_ok(dX, lddx, C, V, CT) : 0);
    if (hipError_t e = hipGetLastError()) return e;
    hipLaunchKernelGGL((softpq_reduce_kernel<V, K_T>), dim3((unsigned)((total + 255) / 256)), dim3(256), 0, s,
                       partial, partial_dt, p.chunks, (int)blocks, C, inv_t, dP, dt);
    return hipGetLastError();
}

template <int K_T, class F>
auto by_v(int V, F&& f) {
    switch (V) {
        case 1: return f(std::integral_constant<int, 1>{});
        case 2: return f(std::integral_constant<int, 2>{});
        case 3: return f(std::integral_constant<int, 3>{});
        case 4: return f(std::integral_constant<int, 4>{});
        case 8: return f(std::integral_constant<int, 8>{});
        case 9: return f(std::integral_constant<int, 9>{});
        case 16: return f(std::integral_constant<int, 16>{});
        default: return f(std::integral_constant<int, 32>{});
    }
}

}  // namespace

// K in {8, 16} and the sub-vector lengths of the tiled encoder: the paper's (K, V) settings.
bool softpq_supported(int K, int V) { return (K == 8 || K == 16) && enc_tile_codebooks(V) != 0; }

size_t softpq_workspace_bytes(int C, int K, int V, int64_t N) {
    if (!softpq_supported(K, V) || C <= 0 || N <= 0) return 0;
    if (K == 16) return by_v<16>(V, [&](auto v) { return workspace_bytes_for<decltype(v)::value, 16>(C, N); });
    return by_v<8>(V, [&](auto v) { return workspace_bytes_for<decltype(v)::value, 8>(C, N); });
}

hipError_t launch_softpq_backward(const float* P, int C, int K, int V, float t, const float* X, int64_t N,
                                  int64_t ldx, const float* Z, int64_t ldz, float* dP, float* dX,
                                  int64_t lddx, float* dt, float* workspace, hipStream_t s) {
    if (!softpq_supported(K, V)) return hipErrorInvalidValue;
    if (K == 16)
        return by_v<16>(V, [&](auto v) {
            return launch_softpq<decltype(v)::value, 16>(P, C, t, X, N, ldx, Z, ldz, dP, dX, lddx, dt, workspace, s);
        });
    return by_v<8>(V, [&](auto v) {
        return launch_softpq<decltype(v)::value, 8>(P, C, t, X, N, ldx, Z, ldz, dP, dX, lddx, dt, workspace, s);
    });
}

}  // namespace lutnn
