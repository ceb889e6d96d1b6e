// One-hot INT8 MFMA contraction of Eq. 4 (arXiv 2302.03213) for one workgroup tile: the simple
// loop shared by the fallback lookup kernel and the fused encode+lookup kernel (the main lookup
// kernel in lookup_mfma.hip has its own hand-pipelined version of the same contraction).
//
// Eq. 4 writes the lookup as  g^c(a^c) . h^c(b^c)  with g a one-hot vector of length K: stacked
// over the codebooks this is  OneHot[N x C*K] x T[C*K x M].  With K <= 16 the one-hot slice of one
// (row, codebook) is 16 bytes - exactly one lane's A operand of v_mfma_i32_32x32x32_i8 (a lane
// holds 16 consecutive k of one row).  So the A operand is never read from global memory: each
// lane turns one index byte into its 16 bytes with one read of a 256-byte one-hot table in LDS.
// The B operand is the table in the packed layout [codebook][m][16 k], where a lane's 16 bytes
// are again contiguous, so B tiles are copied global -> LDS -> registers without transposition.
//
// Workgroup = 4 wavefronts arranged 2 x 2 over a (2*TM*32 rows) x 256 columns tile; each wave owns
// TM x 4 MFMA tiles of 32 x 32.  The codebook loop runs in stages of 8 codebooks (32 KiB of B),
// double buffered in LDS with register prefetch.  Within a stage, MFMA step j pairs codebook
// 4h + j for lane half h (lanes 0-31 / 32-63); a lane therefore needs the index bytes of four
// consecutive codebooks per stage, i.e. one dword.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lutnn {

typedef int v4i __attribute__((ext_vector_type(4)));
typedef int v16i __attribute__((ext_vector_type(16)));

constexpr int kMfmaThreads = 256;
constexpr int kMfmaBN = 256;  // columns per workgroup tile
constexpr int kMfmaSC = 8;    // codebooks per stage
constexpr int kMfmaStageVecs = kMfmaSC * kMfmaBN;  // uint4 per stage buffer (32 KiB)

// XCD-aware tile order: consecutive workgroup ids land on different XCDs (8 of them, each with its
// own L2), so give every XCD a contiguous range of tiles; tiles are ordered column-block major, so
// the workgroups resident on one XCD walk the same slab of the table.  Returns -1 for padding ids.
__device__ __forceinline__ int64_t xcd_tile(int64_t tiles) {
    const int64_t per_xcd = (tiles + 7) / 8;
    const int64_t t = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    return t < tiles ? t : -1;
}

// LDS byte offset of a __shared__ object (the low 32 bits of its flat address).
__device__ __forceinline__ uint32_t lds_offset(const void* p) {
    return (uint32_t)reinterpret_cast<uintptr_t>(p);
}
// 64 lanes x 16 bytes from global memory straight into LDS at lds_dst + 16 * lane.
//   sbase: wave-uniform global base;  voff: per-lane byte offset from it.
// The compiler does not see the LDS write: completion is awaited with wait_loads<N>() before the
// barrier that publishes the data.  "memory" keeps LDS reads from being folded or moved across.
__device__ __forceinline__ void dma16(uint32_t lds_dst, const void* sbase, uint32_t voff) {
    asm volatile(
        "s_mov_b32 m0, %0\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2"
        :
        : "s"(lds_dst), "v"(voff), "s"(sbase)
        : "memory", "m0");
}
template <int N>
__device__ __forceinline__ void wait_loads() {
    asm volatile("s_waitcnt vmcnt(%0)" : : "n"(N) : "memory");
}

// One-hot look-up table in LDS: entry k (16 bytes) has byte k = 1 and the rest 0.  Building a
// lane's A operand is then one shift/mask and one 16-byte LDS read instead of a dozen VALU ops;
// the 16 entries sit in 64 different banks, so lanes with different k never conflict and lanes
// with equal k are served by broadcast.  Must be followed by a barrier before first use.
constexpr int kOnehotLutVecs = 16;
__device__ __forceinline__ void init_onehot_lut(uint4* lut) {
    const int t = threadIdx.x;
    if (t < 16) {
        const uint32_t bit = 1u << ((t & 3) * 8);
        const int d = t >> 2;
        lut[t] = make_uint4(d == 0 ? bit : 0u, d == 1 ? bit : 0u, d == 2 ? bit : 0u, d == 3 ? bit : 0u);
    }
}

// Accumulates the whole codebook range into acc for this wave's TM x 4 MFMA tiles.
//   packed    table in MFMA layout, [C][Mp] uint4
//   n0        first column of the workgroup tile (multiple of 256, < Mp)
//   lds       2 * kMfmaStageVecs uint4 of LDS, free for use on entry (all threads must have
//             passed a barrier since its last use); on return every thread has passed a final barrier
//   lut       one-hot table written by init_onehot_lut (a barrier has passed since)
//   idx_word  idx_word(i, cbase) -> the index bytes of codebooks cbase..cbase+3 (cbase % 4 == 0)
//             for the row this lane feeds in row block i.  For codebooks >= C any value will do
//             (their table slab is staged as zeros); likewise for rows >= N (never stored).
template <int TM, class IdxWord>
__device__ __forceinline__ void mfma_lookup_tile(const uint4* __restrict__ packed, int C, int Mp, int n0,
                                                 uint4* __restrict__ lds, const uint4* __restrict__ lut,
                                                 IdxWord idx_word, v16i (&acc)[TM][4]) {
    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int wn = (tid >> 6) & 1;
    const int l32 = lane & 31, h = lane >> 5;

#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    const int stages = (C + kMfmaSC - 1) / kMfmaSC;
    const uint4* __restrict__ src = packed + n0 + tid;  // column tid of the tile, codebook 0
    uint4 pre[kMfmaSC];  // next stage's B bytes in flight: thread tid copies column tid of each codebook

    auto fetch = [&](int st) {
        const uint4* __restrict__ p = src + (size_t)st * kMfmaSC * Mp;
        if ((st + 1) * kMfmaSC <= C) {
#pragma unroll
            for (int i = 0; i < kMfmaSC; ++i) pre[i] = p[(size_t)i * Mp];
        } else {
#pragma unroll
            for (int i = 0; i < kMfmaSC; ++i)
                pre[i] = (st * kMfmaSC + i < C) ? p[(size_t)i * Mp] : make_uint4(0u, 0u, 0u, 0u);
        }
    };
    auto stash = [&](int buf) {
#pragma unroll
        for (int i = 0; i < kMfmaSC; ++i) lds[buf * kMfmaStageVecs + i * kMfmaBN + tid] = pre[i];
    };
    // this lane's B operand for codebook slot 4h + j, column tile tn: bvec[j * kMfmaBN + tn * 32]
    const uint4* __restrict__ bbase = lds + (4 * h) * kMfmaBN + wn * 128 + l32;

    // Index words are fetched one stage ahead and BEFORE the B prefetch of the same stage, so that
    // waiting for them never waits for the (younger) B loads: vector memory loads return in order.
    uint32_t next_word[TM];
#pragma unroll
    for (int i = 0; i < TM; ++i) next_word[i] = idx_word(i, 4 * h);
    fetch(0);
    stash(0);
    __syncthreads();

    for (int st = 0; st < stages; ++st) {
        const int buf = st & 1;
        // byte j of w16 = 16 * (index of codebook st*8 + 4h + j) = byte offset into the one-hot table
        uint32_t w16[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) w16[i] = (next_word[i] & 0x0f0f0f0fu) << 4;
        if (st + 1 < stages) {
#pragma unroll
            for (int i = 0; i < TM; ++i) next_word[i] = idx_word(i, (st + 1) * kMfmaSC + 4 * h);
            fetch(st + 1);
        }

        const uint4* __restrict__ bvec = bbase + buf * kMfmaStageVecs;
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            v4i a[TM];
#pragma unroll
            for (int i = 0; i < TM; ++i) {
                const uint32_t off = (w16[i] >> (8 * j)) & 0xffu;
                const uint4 v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(lut) + off);
                a[i] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
            }
            v4i b[4];
#pragma unroll
            for (int tn = 0; tn < 4; ++tn) {
                const uint4 v = bvec[j * kMfmaBN + tn * 32];
                b[tn] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
            }
#pragma unroll
            for (int i = 0; i < TM; ++i)
#pragma unroll
                for (int tn = 0; tn < 4; ++tn)
                    acc[i][tn] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a[i], b[tn], acc[i][tn], 0, 0, 0);
        }

        if (st + 1 < stages) stash(buf ^ 1);
        __syncthreads();
    }
}

// Dequantise (r = s*q, Sec. 3.3), add the bias and store this wave's tiles.
// 32x32 accumulator layout: lane -> column l32, register r -> row 8*(r/4) + 4*h + (r%4).
//   row_base  first row of this wave's row block 0 (row block i starts at row_base + 32*i)
//   col_base  first column of this wave's column tile 0
// The bias values are fetched once, up front, and the stores of a tile that lies wholly inside
// the matrix are issued without any test or wait in between (a wait on the load counter between
// stores would wait for the stores before it as well: they share the counter).  For one (row
// block, register) the TN column tiles are written back to back: TN x 128 contiguous bytes.
// STREAM: Y is far larger than the caches (hundreds of megabytes): non-temporal stores keep it from
// displacing the activations and indices the next launches read (config 5: the encoder of the next
// step runs 4 % faster; the lookup itself is unchanged).
template <int TM, bool BIAS, bool STREAM, int TN = 4>
__device__ __forceinline__ void mfma_store_tile_impl(const v16i (&acc)[TM][TN], float s,
                                                     const float* __restrict__ bias, int M, int64_t N,
                                                     int64_t row_base, int col_base,
                                                     float* __restrict__ Y, int64_t ldy) {
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    float bv[TN];
#pragma unroll
    for (int tn = 0; tn < TN; ++tn) bv[tn] = 0.f;
    if (BIAS) {
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) {
            const int col = col_base + tn * 32 + l32;
            bv[tn] = col < M ? bias[col] : 0.f;
        }
        // have the values here, once, instead of a wait in front of every store
#pragma unroll
        for (int tn = 0; tn < TN; ++tn) asm volatile("" : "+v"(bv[tn]));
    }
    // wave-uniform: whole tile inside the matrix, and byte offsets within it fit 32 bits
    const bool interior = row_base + TM * 32 <= N && col_base + 32 * TN <= M && ldy < (1 << 22);
    if (interior) {
        // uniform base + 32-bit lane offset; rows advance the uniform part
        char* __restrict__ base = reinterpret_cast<char*>(Y + row_base * ldy + col_base);
        const uint32_t voff = (uint32_t)(4 * h * (int)ldy + l32) * 4u;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                char* __restrict__ rowp = base + (int64_t)(i * 32 + 8 * (r >> 2) + (r & 3)) * ldy * 4;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn) {
                    const float a = (float)acc[i][tn][r];
                    const float y = BIAS ? __fmaf_rn(a, s, bv[tn]) : __fmul_rn(a, s);
                    if constexpr (STREAM)
                        __builtin_nontemporal_store(y, reinterpret_cast<float*>(rowp + voff + tn * 128));
                    else
                        *reinterpret_cast<float*>(rowp + voff + tn * 128) = y;
                }
            }
        }
    } else {
        float* __restrict__ p = Y + (row_base + 4 * h) * ldy + col_base + l32;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
#pragma unroll
            for (int r = 0; r < 16; ++r) {
                const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
                if (row_base + 4 * h + rr < N) {
                    float* __restrict__ q = p + (int64_t)rr * ldy;
#pragma unroll
                    for (int tn = 0; tn < TN; ++tn) {
                        if (col_base + tn * 32 + l32 < M) {
                            const float a = (float)acc[i][tn][r];
                            q[tn * 32] = BIAS ? __fmaf_rn(a, s, bv[tn]) : __fmul_rn(a, s);
                        }
                    }
                }
            }
        }
    }
}

// The same tile added into an int32 image of Y (row stride ldy elements) with integer atomics:
// the partial sums of workgroups that share an output tile but split the codebooks.  Integer
// addition is associative, so the result does not depend on the order of arrival.
template <int TM, int TN = 4>
__device__ __forceinline__ void mfma_atomic_add_tile(const v16i (&acc)[TM][TN], int M, int64_t N,
                                                     int64_t row_base, int col_base, int32_t* __restrict__ Yi,
                                                     int64_t ldy) {
    const int lane = threadIdx.x & 63;
    const int l32 = lane & 31, h = lane >> 5;
    int32_t* __restrict__ p = Yi + (row_base + 4 * h) * ldy + col_base + l32;
#pragma unroll
    for (int i = 0; i < TM; ++i) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            const int rr = i * 32 + 8 * (r >> 2) + (r & 3);
            if (row_base + 4 * h + rr < N) {
                int32_t* __restrict__ q = p + (int64_t)rr * ldy;
#pragma unroll
                for (int tn = 0; tn < TN; ++tn)
                    if (col_base + tn * 32 + l32 < M) atomicAdd(q + tn * 32, acc[i][tn][r]);
            }
        }
    }
}

template <int TM, bool STREAM = false, int TN = 4>
__device__ __forceinline__ void mfma_store_tile(const v16i (&acc)[TM][TN], float s,
                                                const float* __restrict__ bias, int M, int64_t N,
                                                int64_t row_base, int col_base, float* __restrict__ Y,
                                                int64_t ldy) {
    if (bias)
        mfma_store_tile_impl<TM, true, STREAM, TN>(acc, s, bias, M, N, row_base, col_base, Y, ldy);
    else
        mfma_store_tile_impl<TM, false, STREAM, TN>(acc, s, bias, M, N, row_base, col_base, Y, ldy);
}

}  // namespace lutnn
