// Device-side building blocks of the encoder (arXiv 2302.03213, Eq. 2 and Sec. 5.1), shared by the
// stand-alone encode kernel and the fused encode+lookup kernels.
//
// A tile is 64 rows x CT codebooks.  stage_x() copies its X values into LDS with coalesced row
// segments; encode_codebooks() then lets each of the 4 wavefronts take CT/4 codebooks, one at a
// time, with lane = row: the codebook's centroids are wave-uniform (scalar loads, SGPR operands),
// which is the paper's centroid-stationary scheme in CDNA form.
//
//   d_k = sum_v (x_v - p_kv)^2   fp32, v ascending, one fma per term;  arg-min keeps the lowest k.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lutnn {

constexpr int kEncRows = 64;      // rows per tile = lanes per wavefront
constexpr int kEncThreads = 256;  // 4 wavefronts

template <int V, int CT>
struct EncTile {
    static_assert(CT % 4 == 0, "CT must be a multiple of 4 (one share per wavefront)");
    static constexpr int TW = CT * V;  // floats per tile row
    static constexpr int PAD = (V % 4 == 0) ? 4 : (V % 2 == 0) ? 2 : ((TW % 2 == 0) ? 1 : 0);
    static constexpr int LS = TW + PAD;  // LDS row stride (floats): conflict free for lane = row
    static constexpr int CPW = CT / 4;   // codebooks per wavefront
    static constexpr int PW = (CPW + 3) / 4;  // dwords holding one lane's CPW index bytes
    static constexpr int kLdsFloats = kEncRows * LS;
};

// Codebooks per tile used for each supported sub-vector length (0 = not supported by the tiled
// kernels).  Chosen so that a tile row is 64..144 floats.  V = 16 and 32 are the sub-vector
// lengths the paper uses for BERT (Sec. 6.1, Table 2).
constexpr int enc_tile_codebooks(int V) {
    return V == 1 ? 64 : V == 2 ? 64 : V == 3 ? 32 : V == 4 ? 32 : V == 8 ? 16 : V == 9 ? 16
         : V == 16 ? 8 : V == 32 ? 4 : 0;
}

inline bool enc_vec4_ok(const float* X, int64_t ldx, int C, int V) {
    const int CT = enc_tile_codebooks(V);
    return CT && ((CT * V) % 4 == 0) && (((int64_t)C * V) % 4 == 0) && (ldx % 4 == 0) &&
           ((reinterpret_cast<uintptr_t>(X) & 15) == 0);
}

template <int V, int CT>
__device__ __forceinline__ void stage_x(const float* __restrict__ X, int64_t ldx, int64_t N, int D,
                                        int64_t row0, int c0, float* __restrict__ xs, int vec4,
                                        int tid) {
    using E = EncTile<V, CT>;
    if (vec4) {
        constexpr int Q = E::TW / 4;
        for (int i = tid; i < kEncRows * Q; i += kEncThreads) {
            const int r = i / Q, col = (i % Q) * 4;
            const int gcol = c0 * V + col;
            float4 val = make_float4(0.f, 0.f, 0.f, 0.f);
            if (row0 + r < N && gcol < D)
                val = *reinterpret_cast<const float4*>(X + (row0 + r) * ldx + gcol);
            float* dst = xs + r * E::LS + col;
            dst[0] = val.x;
            dst[1] = val.y;
            dst[2] = val.z;
            dst[3] = val.w;
        }
    } else {
        for (int i = tid; i < kEncRows * E::TW; i += kEncThreads) {
            const int r = i / E::TW, col = i % E::TW;
            const int gcol = c0 * V + col;
            float val = 0.f;
            if (row0 + r < N && gcol < D) val = X[(row0 + r) * ldx + gcol];
            xs[r * E::LS + col] = val;
        }
    }
}

// The same tile for a convolution (Sec. 4: convolution as a matrix product by im2col), gathered
// from the NCHW input instead of a materialised matrix.  Row r of the tile is the thread's lane, so
// the 64 lanes of a wavefront read 64 consecutive output pixels of one (channel, filter tap):
// contiguous input words for stride 1.  The column (channel, tap) is wave-uniform.
//   g      geometry; row n = (b, ho, wo), column j = (ci, r, s)
//   N      rows = B * Ho * Wo;  D = Cin * kh * kw
template <int V, int CT, class Geom>
__device__ __forceinline__ void stage_x_conv(const float* __restrict__ input, const Geom& g, int64_t N,
                                             int D, int64_t row0, int c0, float* __restrict__ xs,
                                             int tid) {
    using E = EncTile<V, CT>;
    const int r = tid & 63;
    const int64_t n = row0 + r;
    const bool row_ok = n < N;
    const int pix = g.Ho * g.Wo;
    const int64_t b = row_ok ? n / pix : 0;
    const int p = row_ok ? (int)(n % pix) : 0;
    const int hi0 = (p / g.Wo) * g.sh - g.ph;
    const int wi0 = (p % g.Wo) * g.sw - g.pw;
    // offset of (b, ci = 0, hi0, wi0); may lie outside the image, only used where in bounds
    const int64_t off0 = ((b * g.Cin) * g.H + hi0) * (int64_t)g.W + wi0;
    const int taps = g.kh * g.kw;
    for (int col = __builtin_amdgcn_readfirstlane(tid >> 6); col < E::TW; col += 4) {
        const int j = c0 * V + col;  // wave-uniform
        float val = 0.f;
        if (j < D) {
            const int ci = j / taps, rs = j - ci * taps;
            const int rk = rs / g.kw, sk = rs - rk * g.kw;
            const int hi = hi0 + rk, wi = wi0 + sk;
            if (row_ok && (unsigned)hi < (unsigned)g.H && (unsigned)wi < (unsigned)g.W)
                val = input[off0 + ((int64_t)ci * g.H + rk) * g.W + sk];
        }
        xs[r * E::LS + col] = val;
    }
}

template <int V, int K_T>
__device__ __forceinline__ uint32_t nearest_centroid(const float (&x)[V], const float* __restrict__ pc,
                                                     int K) {
    uint32_t best = 0;
    float best_d = 0.f;
    if (K_T) {
#pragma unroll
        for (int k = 0; k < K_T; ++k) {
            float d = 0.f;
#pragma unroll
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
    } else {
        for (int k = 0; k < K; ++k) {
            float d = 0.f;
#pragma unroll
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
    }
    return best;
}

// Wave `w` (wave-uniform) encodes codebooks [w*CPW, (w+1)*CPW) of the tile for row `lane`; the
// CPW index bytes come back packed four to a dword, lowest codebook in the lowest byte.
// K_T == 0 means "K is a run-time value".
template <int V, int K_T, int CT>
__device__ __forceinline__ void encode_codebooks(const float* __restrict__ xs,
                                                 const float* __restrict__ P, int C, int K, int c0,
                                                 int w, int lane,
                                                 uint32_t (&packed)[EncTile<V, CT>::PW]) {
    using E = EncTile<V, CT>;
#pragma unroll
    for (int j = 0; j < E::PW; ++j) packed[j] = 0;
#pragma unroll
    for (int j = 0; j < E::CPW; ++j) {
        const int cl = w * E::CPW + j;
        const int c = c0 + cl;  // wave-uniform
        uint32_t best = 0;
        if (c < C) {
            float x[V];
#pragma unroll
            for (int v = 0; v < V; ++v) x[v] = xs[lane * E::LS + cl * V + v];
            best = nearest_centroid<V, K_T>(x, P + (size_t)c * K * V, K);
        }
        packed[j / 4] |= best << (8 * (j % 4));
    }
}

// Puts a lane's CPW index bytes (codebooks first .. first+CPW-1 of its row) into the row's byte
// array in LDS; `row_bytes` is 4-byte aligned and `first` a multiple of CPW.  Shares of fewer than
// four codebooks are written byte by byte: several wavefronts then fill one dword between them.
template <int V, int CT>
__device__ __forceinline__ void store_index_bytes(uint32_t* __restrict__ row_dwords, int first,
                                                  const uint32_t (&packed)[EncTile<V, CT>::PW]) {
    using E = EncTile<V, CT>;
    if constexpr (E::CPW % 4 == 0) {
#pragma unroll
        for (int j = 0; j < E::PW; ++j) row_dwords[first / 4 + j] = packed[j];
    } else {
        uint8_t* __restrict__ row_bytes = reinterpret_cast<uint8_t*>(row_dwords);
#pragma unroll
        for (int b = 0; b < E::CPW; ++b) row_bytes[first + b] = (uint8_t)(packed[0] >> (8 * b));
    }
}

}  // namespace lutnn
