// Encode + table read in ONE launch for small problems (arXiv 2302.03213, Eq. 2 and Eq. 4; the
// fused operator of Fig. 5).
//
// A launch costs ~4.5 us of device time on this chip whatever it does, and a layer at the batch
// sizes of on-device inference (the paper's setting: one image, one sentence) does about a
// microsecond of work in each of its two steps - so for these shapes the second launch IS the
// cost.  Here a workgroup owns R rows and up to 1024 output columns: it first encodes its rows
// against all C codebooks (one thread per (row, codebook), the direct-form search of the encoder),
// leaves the C index bytes of each row in LDS, and after one barrier its wavefronts gather and add
// the selected table rows straight from L2 exactly as the stand-alone gather kernel does (a lane
// owns four columns, sixteen loads in flight, codebook order).  Workgroups that share rows but
// not columns repeat the encoding - cheap while rows x codebooks is small, which is the
// condition under which this kernel is chosen.
//
// Results are bit-identical to lutnn_encode followed by the gather variant of lutnn_lookup: the
// same two device functions run.  The hash encoder (Sec. 2, "Hashing for acceleration") can stand
// in for step 1: the kernels are compiled around the encoder as a type.
#include <algorithm>
#include <type_traits>

#include "encode_tile.h"
#include "gather_row.h"
#include "lutnn_kernels.h"

namespace lutnn {
namespace {

constexpr int kSmallThreads = 256;
constexpr int kSmallWaves = 4;
constexpr int kChunkCols = 256;  // columns a wavefront covers: 64 lanes x 4

// Step 1 of the operator for ONE sub-vector, as a value the kernels below are compiled around:
// the arg-min of Eq. 2 ...
template <int V, int K_T>
struct DistanceSearch {
    static constexpr int kK = K_T;  // table rows per codebook when known at compile time, else 0
    const float* __restrict__ P;    // [C][K][V]
    int K;
    __device__ __forceinline__ int operator()(const float (&x)[V], int c) const {
        const int k = K_T ? K_T : K;
        return nearest_centroid<V, K_T>(x, P + (size_t)c * k * V, k);
    }
};

// ... or the walk down the codebook's threshold tree (Sec. 2, "Hashing for acceleration"; heap
// order, right when the value is greater, a split index outside [0, V) clamped - the same walk as
// the stand-alone hash encoder).  With four levels the fifteen nodes are loaded up front and the
// walk runs on registers: a chain of four dependent trips to L2 would cost as much as the launch
// this kernel saves.
template <int V, int L_T>
struct TreeWalk {
    static constexpr int kK = L_T ? (1 << L_T) : 0;
    const int32_t* __restrict__ split_dim;  // [C][2^levels - 1]
    const float* __restrict__ threshold;    // [C][2^levels - 1]
    int levels;
    // x[min(max(d, 0), V - 1)] by a chain of selects over constant positions: the sub-vector stays
    // in registers (written as a loop, the chain is compiled to an indexed load from a copy of the
    // sub-vector in scratch memory)
    template <int I = 1>
    __device__ __forceinline__ static float pick(const float (&x)[V], int d, float below) {
        if constexpr (I < V)
            return pick<I + 1>(x, d, d >= I ? x[I] : below);
        else
            return below;
    }
    __device__ __forceinline__ static float pick(const float (&x)[V], int d) { return pick<1>(x, d, x[0]); }
    __device__ __forceinline__ int operator()(const float (&x)[V], int c) const {
        if constexpr (L_T != 0) {
            constexpr int NODES = (1 << L_T) - 1;
            const int32_t* __restrict__ dp = split_dim + (size_t)c * NODES;
            const float* __restrict__ tp = threshold + (size_t)c * NODES;
            int d[NODES];
            float t[NODES];
#pragma unroll
            for (int i = 0; i < NODES; ++i) {
                d[i] = dp[i];
                t[i] = tp[i];
            }
            int path = 0;  // the node reached at level l is 2^l - 1 + path
#pragma unroll
            for (int l = 0; l < L_T; ++l) {
                const int first = (1 << l) - 1;
                int dd = d[first];
                float tt = t[first];
#pragma unroll
                for (int q = 1; q < (1 << l); ++q) {
                    const bool here = path == q;
                    dd = here ? d[first + q] : dd;
                    tt = here ? t[first + q] : tt;
                }
                path = 2 * path + (pick(x, dd) > tt ? 1 : 0);
            }
            return path;
        } else {
            const int nodes = (1 << levels) - 1;
            const int32_t* __restrict__ dp = split_dim + (size_t)c * nodes;
            const float* __restrict__ tp = threshold + (size_t)c * nodes;
            int node = 0;
            for (int l = 0; l < levels; ++l) node = 2 * node + 1 + (pick(x, dp[node]) > tp[node] ? 1 : 0);
            return node - nodes;
        }
    }
};

// Step 1 for `rows` rows x C codebooks by the whole workgroup, indices to LDS (sidx[r * Cpad + c]):
// a thread per (row, codebook) runs the encoder's sequential search; neighbouring threads take
// neighbouring codebooks.  (One thread per (row, codebook, centroid) with the arg-min found between
// lanes by DPP exchanges reads the centroids as contiguous memory instead of 64 * V bytes per
// thread, but spends ten times the instructions on addresses and exchanges per distance: measured
// 1.4x slower on BERT's shapes.)
template <int V, typename ENC>
__device__ __forceinline__ void encode_rows_to_lds(const float* __restrict__ X, int64_t ldx, int rows,
                                                   const ENC& enc, int C, uint8_t* __restrict__ sidx,
                                                   int Cpad, int nthreads) {
    for (int pair = threadIdx.x; pair < rows * C; pair += nthreads) {
        const int r = pair / C, c = pair - r * C;
        const float* __restrict__ xp = X + (int64_t)r * ldx + (int64_t)c * V;
        float x[V];
#pragma unroll
        for (int v = 0; v < V; ++v) x[v] = xp[v];
        sidx[r * Cpad + c] = (uint8_t)enc(x, c);
    }
}

//   R                rows per workgroup
//   col_groups       workgroups per row group; each takes chunks_per_group runs of 256 columns
//   lpr              lanes per row when M < 256 (M / 4), else 64
//   Cpad             C rounded up to 4: byte stride of a row's indices in LDS
template <int V, typename ENC, typename TT>
__global__ __launch_bounds__(kSmallThreads) void linear_small_kernel(
    const float* __restrict__ X, int64_t ldx, const ENC enc, const TT* __restrict__ T,
    const float* __restrict__ scale, const float* __restrict__ bias, int C, int K_rt, int M, int64_t N,
    float* __restrict__ Y, int64_t ldy, int R, int col_groups, int chunks_per_group, int lpr, int Cpad) {
    extern __shared__ uint32_t sidx_words[];
    uint8_t* __restrict__ sidx = reinterpret_cast<uint8_t*>(sidx_words);  // [R][Cpad]
    const int K = ENC::kK ? ENC::kK : K_rt;
    const int64_t r0 = (int64_t)(blockIdx.x / col_groups) * R;
    const int cg = (int)(blockIdx.x % col_groups);
    const int rows_here = (int)min((int64_t)R, N - r0);

    encode_rows_to_lds<V>(X + r0 * ldx, ldx, rows_here, enc, C, sidx, Cpad, kSmallThreads);
    __syncthreads();

    // ---- Eq. 4
    const int lane = threadIdx.x & 63;
    const int w = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    if (lpr >= 64) {
        const int chunk0 = cg * chunks_per_group;
        const int chunks_here = min(chunks_per_group, (M + kChunkCols - 1) / kChunkCols - chunk0);
        for (int item = w; item < rows_here * chunks_here; item += kSmallWaves) {
            const int r = item / chunks_here;
            const int m = (chunk0 + item - r * chunks_here) * kChunkCols + lane * 4;
            if (m < M)  // M % 4 == 0: a lane's four columns are all inside or all outside
                gather_row<TT, true, true>(T, scale, bias, C, K, M, sidx + r * Cpad, m, Y + (r0 + r) * ldy);
        }
    } else {
        const int rows_per_wave = 64 / lpr;
        const int sub = lane / lpr;
        for (int first = w * rows_per_wave; first < rows_here; first += kSmallWaves * rows_per_wave) {
            const int r = first + sub;
            if (sub < rows_per_wave && r < rows_here)
                gather_row<TT, true, false>(T, scale, bias, C, K, M, sidx + r * Cpad, (lane - sub * lpr) * 4,
                                            Y + (r0 + r) * ldy);
        }
    }
}

// The same for a handful of rows on a layer with many codebooks: one workgroup per (row, 256
// columns), its SPLIT wavefronts first encode the row between them (each workgroup of the row
// repeats that), then share out the codebooks of the table read as the split gather kernel does.
template <int V, typename ENC, typename TT, int SPLIT>
__global__ __launch_bounds__(64 * SPLIT) void linear_split_kernel(
    const float* __restrict__ X, int64_t ldx, const ENC enc, const TT* __restrict__ T,
    const float* __restrict__ scale, const float* __restrict__ bias, int C, int K_rt, int M,
    float* __restrict__ Y, int64_t ldy, int col_chunks, int per_wave) {
    extern __shared__ uint32_t sidx_words[];
    uint8_t* __restrict__ sidx = reinterpret_cast<uint8_t*>(sidx_words);  // [C], padded to 4
    const int K = ENC::kK ? ENC::kK : K_rt;
    const int64_t row = blockIdx.x / col_chunks;  // < N by construction of the grid
    encode_rows_to_lds<V>(X + row * ldx, ldx, 1, enc, C, sidx, 0, 64 * SPLIT);
    __syncthreads();
    const int m = (int)(blockIdx.x % col_chunks) * kChunkCols + (threadIdx.x & 63) * 4;
    gather_row_split<TT, true, SPLIT>(T, scale, bias, C, K, M, sidx, m, Y + row * ldy, per_wave);
}

// Few (row, 256 columns) pairs and enough codebooks to share out: the split form.
constexpr int64_t kSplitMaxItems = 2049;
constexpr int kSplitMinCodebooks = 64;
inline bool split_form(int C, int M, int64_t N) {
    return M >= kChunkCols && C >= kSplitMinCodebooks && N * ((M + kChunkCols - 1) / kChunkCols) < kSplitMaxItems;
}

struct SmallPlan {
    int R, col_groups, chunks_per_group, lpr, Cpad;
    int64_t blocks;
    size_t shmem;
};

SmallPlan make_plan(int C, int M, int64_t N) {
    SmallPlan p;
    p.Cpad = (C + 3) & ~3;
    if (M >= kChunkCols) {
        const int chunks = (M + kChunkCols - 1) / kChunkCols;
        p.lpr = 64;
        p.chunks_per_group = std::min(chunks, kSmallWaves);
        p.col_groups = (chunks + p.chunks_per_group - 1) / p.chunks_per_group;
        // at least one (row, 256 columns) item per wavefront
        p.R = p.chunks_per_group >= 4 ? 1 : p.chunks_per_group >= 2 ? 2 : 4;
    } else {
        p.lpr = M / 4;
        p.chunks_per_group = 1;
        p.col_groups = 1;
        p.R = kSmallWaves * (64 / p.lpr);
    }
    p.blocks = ((N + p.R - 1) / p.R) * p.col_groups;
    p.shmem = (size_t)p.R * p.Cpad;
    return p;
}

// One launch with the encoder `enc` in front of the table read.
template <int V, typename ENC, typename TT>
hipError_t launch_enc(const ENC& enc, const TT* T, const float* scale, const float* bias, int C, int K, int M,
                      const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
    if (split_form(C, M, N)) {
        const int col_chunks = (M + kChunkCols - 1) / kChunkCols;
        const dim3 grid((unsigned)(N * col_chunks));
        const size_t shmem = (size_t)((C + 3) & ~3);
        if (C >= 256) {  // sixteen codebooks or more per wavefront: one full batch of loads each
            constexpr int SPLIT = 16;
            hipLaunchKernelGGL((linear_split_kernel<V, ENC, TT, SPLIT>), grid, dim3(64 * SPLIT), shmem, s, X, ldx,
                               enc, T, scale, bias, C, K, M, Y, ldy, col_chunks, ((C + SPLIT - 1) / SPLIT + 3) & ~3);
        } else {
            constexpr int SPLIT = 4;
            hipLaunchKernelGGL((linear_split_kernel<V, ENC, TT, SPLIT>), grid, dim3(64 * SPLIT), shmem, s, X, ldx,
                               enc, T, scale, bias, C, K, M, Y, ldy, col_chunks, ((C + SPLIT - 1) / SPLIT + 3) & ~3);
        }
        return hipGetLastError();
    }
    const SmallPlan p = make_plan(C, M, N);
    if (p.blocks > 0x7fffffffLL) return hipErrorInvalidValue;
    hipLaunchKernelGGL((linear_small_kernel<V, ENC, TT>), dim3((unsigned)p.blocks), dim3(kSmallThreads), p.shmem, s,
                       X, ldx, enc, T, scale, bias, C, K, M, N, Y, ldy, p.R, p.col_groups, p.chunks_per_group,
                       p.lpr, p.Cpad);
    return hipGetLastError();
}

// Calls f with the sub-vector length as a compile-time constant.
template <typename F>
hipError_t with_subvector_length(int V, F&& f) {
    switch (V) {
        case 1: return f(std::integral_constant<int, 1>{});
        case 2: return f(std::integral_constant<int, 2>{});
        case 3: return f(std::integral_constant<int, 3>{});
        case 4: return f(std::integral_constant<int, 4>{});
        case 8: return f(std::integral_constant<int, 8>{});
        case 9: return f(std::integral_constant<int, 9>{});
        case 16: return f(std::integral_constant<int, 16>{});
        case 32: return f(std::integral_constant<int, 32>{});
        default: return hipErrorInvalidValue;
    }
}

template <typename TT>
hipError_t launch_t(const float* P, const TT* T, const float* scale, const float* bias, int C, int K, int V,
                    int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
    return with_subvector_length(V, [&](auto v) {
        constexpr int VV = decltype(v)::value;
        if (K == 16)
            return launch_enc<VV>(DistanceSearch<VV, 16>{P, K}, T, scale, bias, C, K, M, X, N, ldx, Y, ldy, s);
        if (K == 8)
            return launch_enc<VV>(DistanceSearch<VV, 8>{P, K}, T, scale, bias, C, K, M, X, N, ldx, Y, ldy, s);
        return launch_enc<VV>(DistanceSearch<VV, 0>{P, K}, T, scale, bias, C, K, M, X, N, ldx, Y, ldy, s);
    });
}

template <typename TT>
hipError_t launch_tree_t(const int32_t* split_dim, const float* threshold, int levels, const TT* T,
                         const float* scale, const float* bias, int C, int V, int M, const float* X, int64_t N,
                         int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
    const int K = 1 << levels;
    return with_subvector_length(V, [&](auto v) {
        constexpr int VV = decltype(v)::value;
        if (levels == 4)
            return launch_enc<VV>(TreeWalk<VV, 4>{split_dim, threshold, levels}, T, scale, bias, C, K, M, X, N,
                                  ldx, Y, ldy, s);
        return launch_enc<VV>(TreeWalk<VV, 0>{split_dim, threshold, levels}, T, scale, bias, C, K, M, X, N, ldx,
                              Y, ldy, s);
    });
}

}  // namespace

// Shapes the kernel can run: fp32 or INT8 table in its plain layout, whole groups of four columns,
// table aligned for a four-column load, a sub-vector length with an unrolled search.
bool linear_small_supported(const void* T, int table_kind, int C, int K, int V, int M) {
    if (!T || (table_kind != 0 && table_kind != 1)) return false;
    if (!(V == 1 || V == 2 || V == 3 || V == 4 || V == 8 || V == 9 || V == 16 || V == 32)) return false;
    if (M % 4 != 0 || K > 256) return false;
    if (M < kChunkCols && 64 % (M / 4) != 0) return false;  // rows narrower than a wavefront must tile it
    if (make_plan(C, M, 1).shmem > 32 * 1024 || C > 32768) return false;  // index bytes must fit LDS
    const uintptr_t align = table_kind == 0 ? 15 : 3;
    return (reinterpret_cast<uintptr_t>(T) & align) == 0;
}

// ... and the shapes on which it beats encode + lookup.  Only where the lookup would be the gather
// anyway (`gather_wins`: the library's own pricing of the gather against the matrix cores), and
// where the encoding that every workgroup repeats stays cheap: a workgroup reads all C*K*V
// centroid values (each thread its own 64*V bytes), which costs more than the launch it saves from
// about 128 KiB on (sweeps over V = 2, 4, 16, C = 64 ... 2048, M = 256 ... 4096, 1 ... 64 rows: the
// one-launch form wins up to C*V of 2048-3072 and loses beyond), and all workgroups together should
// read less than 32 MiB of them; the rows form also wants a short chain of codebooks per row.
bool linear_small_preferred(const void* T, int table_kind, int C, int K, int V, int M, int64_t N,
                            bool gather_wins) {
    if (!gather_wins || !linear_small_supported(T, table_kind, C, K, V, M)) return false;
    if ((int64_t)C * V > 3072) return false;
    const double centroid_bytes = (double)C * K * V * 4;
    if (split_form(C, M, N))
        return (double)N * ((M + kChunkCols - 1) / kChunkCols) * centroid_bytes < 33554432.0;
    const SmallPlan p = make_plan(C, M, N);
    return C <= 128 && (double)N * C * p.col_groups <= 32768.0;
}

hipError_t launch_linear_small_f32(const float* P, const float* T, const float* bias, int C, int K, int V,
                                   int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                                   hipStream_t s) {
    return launch_t<float>(P, T, nullptr, bias, C, K, V, M, X, N, ldx, Y, ldy, s);
}

hipError_t launch_linear_small_i8(const float* P, const int8_t* T, const float* scale, const float* bias, int C,
                                  int K, int V, int M, const float* X, int64_t N, int64_t ldx, float* Y,
                                  int64_t ldy, hipStream_t s) {
    return launch_t<int8_t>(P, T, scale, bias, C, K, V, M, X, N, ldx, Y, ldy, s);
}

// The same kernels with the hash encoder in front (K = 2^levels table rows per codebook).
hipError_t launch_linear_small_tree_f32(const int32_t* split_dim, const float* threshold, int levels,
                                        const float* T, const float* bias, int C, int V, int M, const float* X,
                                        int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s) {
    return launch_tree_t<float>(split_dim, threshold, levels, T, nullptr, bias, C, V, M, X, N, ldx, Y, ldy, s);
}

hipError_t launch_linear_small_tree_i8(const int32_t* split_dim, const float* threshold, int levels,
                                       const int8_t* T, const float* scale, const float* bias, int C, int V,
                                       int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                                       hipStream_t s) {
    return launch_tree_t<int8_t>(split_dim, threshold, levels, T, scale, bias, C, V, M, X, N, ldx, Y, ldy, s);
}

}  // namespace lutnn
