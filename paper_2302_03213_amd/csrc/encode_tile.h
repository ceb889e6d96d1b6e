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

// X is read exactly once per call and is the largest thing the path touches (config 5: 256 MiB per
// step): loaded with the non-temporal hint it streams past the caches instead of displacing the
// table and the index matrix, which the lookup re-reads (config 5: lookup 0.470 -> 0.451 ms and the
// step 0.561 -> 0.536 ms on one machine, 0.461 -> 0.435 and 0.554 -> 0.530 on another, with nothing
// else changed).  A line that is already cached is still served from the cache.
__device__ __forceinline__ float4 load_once(const float* __restrict__ p) {  // 16-byte aligned
    typedef float f32x4 __attribute__((ext_vector_type(4)));
    const f32x4 q = __builtin_nontemporal_load(reinterpret_cast<const f32x4*>(p));
    return make_float4(q[0], q[1], q[2], q[3]);
}

// The two halves of staging a tile with 16-byte loads (X 16-byte aligned, ldx and C*V multiples of
// 4): a thread's ITER loads into registers, and those registers into LDS.  Kept apart so that a
// kernel can issue the loads of its next tile before it works on the current one.
template <int V, int CT>
struct XTileRegs {
    static constexpr int Q = EncTile<V, CT>::TW / 4;
    static constexpr int ITER = (kEncRows * Q + kEncThreads - 1) / kEncThreads;
    float4 val[ITER];
};

template <int V, int CT>
__device__ __forceinline__ void load_x_tile(const float* __restrict__ X, int64_t ldx, int64_t N, int D,
                                            int64_t row0, int c0, int tid, XTileRegs<V, CT>& t) {
    using R = XTileRegs<V, CT>;
#pragma unroll
    for (int it = 0; it < R::ITER; ++it) {
        const int i = tid + it * kEncThreads;
        const int r = i / R::Q, col = (i % R::Q) * 4;
        const int gcol = c0 * V + col;
        t.val[it] = make_float4(0.f, 0.f, 0.f, 0.f);
        if (i < kEncRows * R::Q && row0 + r < N && gcol < D)
            t.val[it] = load_once(X + (row0 + r) * ldx + gcol);
    }
}

template <int V, int CT>
__device__ __forceinline__ void store_x_tile(float* __restrict__ xs, int tid, const XTileRegs<V, CT>& t) {
    using E = EncTile<V, CT>;
    using R = XTileRegs<V, CT>;
#pragma unroll
    for (int it = 0; it < R::ITER; ++it) {
        const int i = tid + it * kEncThreads;
        if (i < kEncRows * R::Q) {
            float* dst = xs + (i / R::Q) * E::LS + (i % R::Q) * 4;
            dst[0] = t.val[it].x;
            dst[1] = t.val[it].y;
            dst[2] = t.val[it].z;
            dst[3] = t.val[it].w;
        }
    }
}

template <int V, int CT>
__device__ __forceinline__ void stage_x(const float* __restrict__ X, int64_t ldx, int64_t N, int D,
                                        int64_t row0, int c0, float* __restrict__ xs, int vec4,
                                        int tid) {
    using E = EncTile<V, CT>;
    // All of a thread's loads are issued before the first LDS write, so that their latencies
    // overlap instead of adding up (a workgroup has nothing else to do until the tile is staged).
    if (vec4) {
        XTileRegs<V, CT> t;
        load_x_tile<V, CT>(X, ldx, N, D, row0, c0, tid, t);
        store_x_tile<V, CT>(xs, tid, t);
    } else {
        constexpr int TOTAL = kEncRows * E::TW;
        constexpr int BATCH = 8;
        for (int i0 = tid; i0 < TOTAL; i0 += BATCH * kEncThreads) {
            float val[BATCH];
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int i = i0 + b * kEncThreads;
                const int r = i / E::TW, col = i % E::TW;
                const int gcol = c0 * V + col;
                val[b] = 0.f;
                if (i < TOTAL && row0 + r < N && gcol < D) val[b] = __builtin_nontemporal_load(X + (row0 + r) * ldx + gcol);
            }
#pragma unroll
            for (int b = 0; b < BATCH; ++b) {
                const int i = i0 + b * kEncThreads;
                if (i < TOTAL) xs[(i / E::TW) * E::LS + i % E::TW] = val[b];
            }
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
    static_assert(E::TW % 4 == 0, "tile rows are walked four columns at a time");
    const int r = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
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
    // Per lane, one bit per filter tap: does the tap fall inside the image for this output pixel?
    // (Filters of more than 32 taps test the coordinates per element instead.)
    const bool use_mask = taps <= 32;  // uniform
    uint32_t ok = 0;
    if (use_mask && row_ok) {
        int t = 0;
        for (int rk = 0; rk < g.kh; ++rk) {
            const bool h_ok = (unsigned)(hi0 + rk) < (unsigned)g.H;
            for (int sk = 0; sk < g.kw; ++sk, ++t)
                if (h_ok && (unsigned)(wi0 + sk) < (unsigned)g.W) ok |= 1u << t;
        }
    }
    // Wave-uniform walk over the tile's columns: wave w takes columns w, w + 4, ...; the
    // (channel, filter row, filter column) of the column advances by additions only.
    int j = c0 * V + w;
    int ci = j / taps;
    int rk = (j - ci * taps) / g.kw;
    int sk = j - ci * taps - rk * g.kw;
    float* __restrict__ dst = xs + r * E::LS + w;
#pragma unroll 4
    for (int it = 0; it < E::TW / 4; ++it) {
        float val = 0.f;
        if (j < D) {
            const bool inside = use_mask ? ((ok >> (rk * g.kw + sk)) & 1u) != 0
                                         : (row_ok && (unsigned)(hi0 + rk) < (unsigned)g.H &&
                                            (unsigned)(wi0 + sk) < (unsigned)g.W);
            if (inside) val = input[off0 + ((int64_t)ci * g.H + rk) * g.W + sk];
        }
        dst[4 * it] = val;
        j += 4;
        sk += 4;
        while (sk >= g.kw) {
            sk -= g.kw;
            ++rk;
        }
        while (rk >= g.kh) {
            rk -= g.kh;
            ++ci;
        }
    }
}

// The same gather when the filter has TAPS = kh * kw taps known at compile time and a sub-vector
// is whole channels' patches or whole pixels (V % TAPS == 0): 3x3 filters with V = 9 and 1x1
// filters, the paper's two convolution settings (Sec. 6.1).  Wave w stages the columns of its own
// codebooks, so (channel, tap) of every column is known when the loop is unrolled: per element
// there remain one bit test, one address add, the load and the LDS write.
template <int V, int CT, int TAPS, class Geom>
__device__ __forceinline__ void stage_x_conv_taps(const float* __restrict__ input, const Geom& g,
                                                  int64_t N, int D, int64_t row0, int c0,
                                                  float* __restrict__ xs, int tid) {
    using E = EncTile<V, CT>;
    static_assert(V % TAPS == 0 && TAPS <= 32, "sub-vectors must be whole patches");
    constexpr int COLS = E::CPW * V;  // columns per wavefront
    const int r = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int64_t n = row0 + r;
    const bool row_ok = n < N;
    const int pix = g.Ho * g.Wo;
    const int64_t b = row_ok ? n / pix : 0;
    const int p = row_ok ? (int)(n % pix) : 0;
    const int hi0 = (p / g.Wo) * g.sh - g.ph;
    const int wi0 = (p % g.Wo) * g.sw - g.pw;
    const int64_t off0 = ((b * g.Cin) * g.H + hi0) * (int64_t)g.W + wi0;
    uint32_t ok = 0;       // per lane: bit t = tap t lies inside the image
    int tapoff[TAPS];      // uniform: offset of tap t from the patch origin
    {
        int rk = 0, sk = 0;
#pragma unroll
        for (int t = 0; t < TAPS; ++t) {
            tapoff[t] = rk * g.W + sk;
            if (row_ok && (unsigned)(hi0 + rk) < (unsigned)g.H && (unsigned)(wi0 + sk) < (unsigned)g.W)
                ok |= 1u << t;
            if (++sk == g.kw) {
                sk = 0;
                ++rk;
            }
        }
    }
    const int j0 = c0 * V + w * COLS;
    const int64_t HW = (int64_t)g.H * g.W;
    const int64_t ch_off = (int64_t)(j0 / TAPS) * HW;  // first channel of this wavefront
    float* __restrict__ dst = xs + r * E::LS + w * COLS;
#pragma unroll
    for (int it = 0; it < COLS; ++it) {
        constexpr int kT = TAPS;
        const int tap = it % kT, chl = it / kT;
        float val = 0.f;
        if (j0 + it < D && (ok & (1u << tap))) val = input[off0 + ch_off + chl * HW + tapoff[tap]];
        dst[it] = val;
    }
}

// Centroids per chunk of the unrolled search: the largest divisor of K with at most 64 values.
// (Sub-vectors of 8 and 9 values are left to the compiler's own placement of the loads: chunks of
// 8 x 9 values made the 3x3-convolution encoder 11 % slower, the scalar registers being too full.)
constexpr int centroid_chunk(int K, int V) {
    if (K * V > 64 && V < 16) return 0;  // 0: no explicit chunks
    int g = 64 / V > 0 ? 64 / V : 1;
    if (g > K) g = K;
    while (K % g) --g;
    return g;
}

template <int V, int K_T>
__device__ __forceinline__ uint32_t nearest_centroid(const float (&x)[V], const float* __restrict__ pc,
                                                     int K) {
    uint32_t best = 0;
    float best_d = 0.f;
    if (K_T) {
        // The centroids are fetched a chunk at a time - scalar loads when pc is wave-uniform - as many
        // whole centroids as fit the scalar registers beside everything else (64 values), all
        // of a chunk's loads issued together: one wait per chunk instead of one per load (config 5,
        // where a codebook is one chunk: 0.091 -> 0.081 ms; V = 16 and 32 at BERT's FFN shapes:
        // 0.018 -> 0.015 and 0.020 -> 0.017 ms).
        constexpr int G0 = centroid_chunk(K_T ? K_T : 1, V);
        constexpr int G = G0 ? G0 : (K_T ? K_T : 1);
#pragma unroll
        for (int k0 = 0; k0 < K_T; k0 += G) {
            float p[G0 ? G * V : 1];
            if constexpr (G0 != 0) {
#pragma unroll
                for (int i = 0; i < G * V; ++i) p[i] = pc[k0 * V + i];
            }
#pragma unroll
            for (int kk = 0; kk < G; ++kk) {
                const int k = k0 + kk;
                float d = 0.f;
#pragma unroll
                for (int v = 0; v < V; ++v) {
                    float pv;
                    if constexpr (G0 != 0) pv = p[kk * V + v]; else pv = pc[k * V + v];
                    const float t = x[v] - pv;
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

// The index of a search, moved to byte `b` of a dword.  The barrier keeps the shift out of the
// search: folded into it, every "best = k" select would carry the constant k << 8b, which is no
// inline constant - one more move instruction per centroid (15 of 208 per sub-vector).
__device__ __forceinline__ uint32_t index_byte(uint32_t best, int b) {
    asm volatile("" : "+v"(best));
    return best << (8 * b);
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
        packed[j / 4] |= index_byte(best, j % 4);
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
