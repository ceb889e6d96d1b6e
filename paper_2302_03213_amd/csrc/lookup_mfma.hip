// Table read and accumulation (arXiv 2302.03213, Eq. 4) as a dense INT8 MFMA contraction, gfx950:
// stand-alone kernels reading the index matrix idx[N][C] from global memory.
//
// Eq. 4 writes the lookup as  g^c(a^c) . h^c(b^c)  with g a one-hot vector of length K: stacked
// over the codebooks this is  OneHot[N x C*K] x T[C*K x M].  With K <= 16 the one-hot slice of one
// (row, codebook) is 16 bytes - exactly one lane's A operand of v_mfma_i32_32x32x32_i8.  The A
// operand is therefore never read from memory: a lane turns one index byte into its 16 operand
// bytes with one read of a 256-byte one-hot table in LDS.  The B operand is the table in the
// packed layout [codebook][m][16 k], staged through LDS without transposition.  Accumulation is
// exact int32; the epilogue dequantises with the layer scale (Sec. 3.3) and adds the bias.
// 15 of every 16 multiplies are by zero; that is the price of running the gather on the matrix
// cores.
//
// Main kernel (needs C % 32 == 0 and a 16-byte aligned idx).  Workgroup = 4 wavefronts (2 x 2),
// one per SIMD, output tile 256 x 256; each wave owns 128 x 128 = 4 x 4 MFMA tiles, i.e. 256
// accumulator registers per lane.  With a single wave per SIMD nothing else hides latency, so the
// codebook loop is software pipelined by hand:
//   - The codebooks are walked in super-stages of 32, each split into 4 stages of 8 codebooks
//     (4 MFMA steps of 2 codebooks).  Stage s' of super-stage u holds codebooks
//     32u + 16h + 4s' + j for lane half h (lanes 0-31 / 32-63) and step j, so the 16 index bytes
//     a lane needs for a whole super-stage are contiguous: one 16-byte load per row block.
//   - Table slabs (32 KiB per stage) and index bytes go global -> LDS directly
//     (global_load_lds_dwordx4), never through registers, into a ring of 4 stage buffers and 2
//     index buffers.  They are issued from inline assembly three stages ahead and waited for with
//     an explicit s_waitcnt vmcnt(N) that leaves the youngest stage in flight; the compiler sees
//     no vector memory loads in the loop and so inserts no waits of its own (left to it, the wait
//     at the loop back-edge becomes vmcnt(0) and drains the prefetch queue every trip).
//   - Stage s+1 is complete in LDS while stage s is computed, so the operands of its first MFMA
//     step are read before the barrier that ends stage s; inside a stage the LDS reads of step
//     j+1 go into a second set of operand registers, spread one per two MFMAs of step j.  The four
//     waves run in lockstep, so bursts of LDS reads or of loads would fill the queues, stall the
//     in-order wave, and let the MFMA pipe, which only ever has one instruction in flight, run
//     dry.
//   - One barrier per stage; it waits for LDS traffic and for the loads of the stage after next.
//
// Fallback kernel (any C, any idx alignment): the simpler two-waves-per-SIMD tile loop of
// mfma_tile.h, 128 x 256 workgroup tile.
#include <type_traits>

#include "lutnn_kernels.h"
#include "mfma_tile.h"

namespace lutnn {
namespace {

static_assert(kMfmaBN == kPackedColPad, "packed column padding must match the column tile");

// ------------------------------------------------------------------------------- main kernel
constexpr int TM = 4;                       // 32-row MFMA blocks per wave
constexpr int BM = 2 * TM * 32;             // rows per workgroup (256)
constexpr int NBUF = 4;                     // LDS ring depth, stages
constexpr int SC = kMfmaSC;                 // codebooks per stage
constexpr int KSTEPS = SC / 2;              // MFMA steps per stage (2 codebooks each)
constexpr int STAGE_VECS = kMfmaStageVecs;  // uint4 per stage buffer
constexpr int SUPER = 4;                    // stages per super-stage (32 codebooks)
static_assert(KSTEPS == 4 && SC == 8 && TM == 4 && NBUF == SUPER, "the schedule below assumes these");

__global__ __launch_bounds__(kMfmaThreads, 1) void lookup_mfma_i8_pipelined_kernel(
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int M, int Mp, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int row_tiles, int64_t tiles) {
    __shared__ uint4 ring[NBUF * STAGE_VECS];  // 4 x 32 KiB table slabs
    __shared__ uint4 ibuf[2][2][TM][64];       // [super-stage parity][wave row][row block][lane]
    __shared__ uint4 lut[kOnehotLutVecs];

    const int64_t t = xcd_tile(tiles);
    if (t < 0) return;
    const int n0 = (int)(t / row_tiles) * kMfmaBN;
    const int64_t m0 = (t % row_tiles) * BM;

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
    const int wm = w >> 1, wn = w & 1;
    const int l32 = lane & 31, h = lane >> 5;
    const int64_t row_base = m0 + wm * (TM * 32);

    init_onehot_lut(lut);

    const int supers = C / (SC * SUPER);  // C % 32 == 0
    const int stages = supers * SUPER;

    // ---- load issue.  Table: this wave copies columns [64w, 64w+64) of each of the 8 codebook
    // slots of a stage; slot g of stage s = 4u + s' is codebook 32u + 16(g>>2) + 4s' + (g&3).
    const uint4* __restrict__ tsrc = packed + n0 + 64 * w;  // wave-uniform
    const uint32_t lane16 = lane * 16;
    const uint32_t ring0 = lds_offset(ring) + 64 * w * 16;
    auto load_b = [&](int s, int g) {
        const int c = 32 * (s >> 2) + 16 * (g >> 2) + 4 * (s & 3) + (g & 3);
        dma16(ring0 + ((s & 3) * STAGE_VECS + g * kMfmaBN) * 16, tsrc + (size_t)c * Mp, lane16);
    };
    // Indices: the two waves of a wave row share one copy; wave column wn fetches row blocks 2wn
    // and 2wn+1.  Rows >= N re-read row N-1 (their results are never stored).
    const uint8_t* __restrict__ isrc = idx + m0 * C;  // wave-uniform
    uint32_t ioff[2];
#pragma unroll
    for (int q = 0; q < 2; ++q) {
        int64_t row = wm * (TM * 32) + (2 * wn + q) * 32 + l32;
        if (m0 + row >= N) row = N - 1 - m0;
        ioff[q] = (uint32_t)(row * C + 16 * h);
    }
    const uint32_t ibuf0 = lds_offset(ibuf);
    auto load_idx = [&](int u, int q) {
        dma16(ibuf0 + ((((u & 1) * 2 + wm) * TM + 2 * wn + q) * 64) * 16, isrc + 32 * u, ioff[q]);
    };

    v16i acc[TM][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // operand registers, double buffered over MFMA steps.  Read r < 4 is B tile r, else A block
    // r-4: the first MFMAs of a step need all four B tiles but only A block 0, so this order gives
    // every operand at least four MFMA groups between its read and its first use.
    v4i a[2][TM], b[2][4];
    const uint4* __restrict__ bbase = ring + (4 * h) * kMfmaBN + wn * 128 + l32;
    // w16 = byte offsets into the one-hot table for the 4 steps of one stage
    auto load_operand = [&](int set, int sbuf, int j, const uint32_t (&w16)[TM], int r) {
        uint4 v;
        if (r >= 4) {
            const uint32_t off = (w16[r - 4] >> (8 * j)) & 0xffu;
            v = *reinterpret_cast<const uint4*>(reinterpret_cast<const char*>(lut) + off);
            a[set][r - 4] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
        } else {
            v = bbase[sbuf * STAGE_VECS + j * kMfmaBN + r * 32];
            b[set][r] = v4i{(int)v.x, (int)v.y, (int)v.z, (int)v.w};
        }
    };
    // index words of a super-stage: wq[i][s'] = one-hot table offsets of row block i, stage s'
    auto read_idx = [&](int u, uint32_t (&wq)[TM][SUPER]) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const uint4 v = ibuf[u & 1][wm][i][lane];
            wq[i][0] = (v.x & 0x0f0f0f0fu) << 4;  // byte j = 16 * index = offset of the table entry
            wq[i][1] = (v.y & 0x0f0f0f0fu) << 4;
            wq[i][2] = (v.z & 0x0f0f0f0fu) << 4;
            wq[i][3] = (v.w & 0x0f0f0f0fu) << 4;
        }
    };

    // ---- prologue: stages 0..2 and the indices of super-stage 0
    load_idx(0, 0);
    load_idx(0, 1);
#pragma unroll
    for (int s = 0; s < 3; ++s)
#pragma unroll
        for (int g = 0; g < SC; ++g) load_b(s, g);
    wait_loads<0>();
    __syncthreads();
    uint32_t wcur[TM][SUPER], wnext[TM][SUPER];
    read_idx(0, wcur);
    {
        uint32_t w0[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) w0[i] = wcur[i][0];
#pragma unroll
        for (int r = 0; r < 8; ++r) load_operand(0, 0, 0, w0, r);
    }

    // One stage s = 4u + SP.  FULL = the ring is in steady state: stage s+3 and super-stage u+1
    // exist for every stage of this super-stage, so nothing in the body is conditional.
    auto run_stage = [&](int u, auto sp_c, auto full) {
        constexpr int SP = decltype(sp_c)::value;
        constexpr bool FULL = decltype(full)::value;
        const int s = SUPER * u + SP;
        const bool do_fetch = FULL || s + 3 < stages;
        const bool do_idx = SP == 0 && (FULL || u + 1 < supers);
        uint32_t wst[TM], wnx[TM];
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            wst[i] = wcur[i][SP];
            wnx[i] = wcur[i][(SP + 1) % SUPER];  // unused when SP is the last stage
        }
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) {
            // in the last stage of a super-stage, pick up the next super-stage's index words
            // (published two barriers ago); past the last super-stage this reads unused data
            if (SP == SUPER - 1 && j == 0) read_idx(u + 1, wnext);
            // 8 groups of two MFMAs; behind each group one LDS read for the next step (in the last
            // step: two, in the first four groups, for the first step of the next stage - they
            // must have returned when the barrier waits for the LDS counter), and at most one
            // load: the texture path serves the four lockstep waves one instruction at a time.
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 2 * g; q < 2 * g + 2; ++q)
                    acc[q >> 2][q & 3] = __builtin_amdgcn_mfma_i32_32x32x32_i8(
                        a[j & 1][q >> 2], b[j & 1][q & 3], acc[q >> 2][q & 3], 0, 0, 0);
                if (j + 1 < KSTEPS) {
                    load_operand((j + 1) & 1, SP, j + 1, wst, g);
                } else if (g < 4) {
                    if (SP + 1 < SUPER) {
                        load_operand(0, SP + 1, 0, wnx, 2 * g);
                        load_operand(0, SP + 1, 0, wnx, 2 * g + 1);
                    } else {
                        uint32_t w0[TM];
#pragma unroll
                        for (int i = 0; i < TM; ++i) w0[i] = wnext[i][0];
                        load_operand(0, 0, 0, w0, 2 * g);
                        load_operand(0, 0, 0, w0, 2 * g + 1);
                    }
                }
                if (do_fetch && (g == 1 || g == 5)) load_b(s + 3, 2 * j + (g == 5));
                if (do_idx && g == 3 && j < 2) load_idx(u + 1, j);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // Before the barrier everything issued before this stage must have landed: stage s+2 is
        // read from the end of stage s+1 on.  This stage's own loads (8, or 10 with the indices)
        // stay in flight.
        if (FULL) {
            if (SP == 0)
                wait_loads<10>();
            else
                wait_loads<8>();
        } else {
            wait_loads<0>();
        }
        __syncthreads();
    };
    auto rotate_idx = [&]() {
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int q = 0; q < SUPER; ++q) wcur[i][q] = wnext[i][q];
    };
    using SP0 = std::integral_constant<int, 0>;
    using SP1 = std::integral_constant<int, 1>;
    using SP2 = std::integral_constant<int, 2>;
    using SP3 = std::integral_constant<int, 3>;

    int u = 0;
    for (; u + 1 < supers; ++u) {
        run_stage(u, SP0{}, std::true_type{});
        run_stage(u, SP1{}, std::true_type{});
        run_stage(u, SP2{}, std::true_type{});
        run_stage(u, SP3{}, std::true_type{});
        rotate_idx();
    }
    run_stage(u, SP0{}, std::false_type{});
    run_stage(u, SP1{}, std::false_type{});
    run_stage(u, SP2{}, std::false_type{});
    run_stage(u, SP3{}, std::false_type{});

    mfma_store_tile<TM>(acc, *scale, bias, M, N, row_base, n0 + wn * 128, Y, ldy);
}

// ----------------------------------------------------------------------------- fallback kernel
constexpr int BM_GENERIC = 128;

__global__ __launch_bounds__(kMfmaThreads, 2) void lookup_mfma_i8_generic_kernel(
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int M, int Mp, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int row_tiles, int64_t tiles) {
    __shared__ uint4 lds[2 * kMfmaStageVecs];
    __shared__ uint4 lut[kOnehotLutVecs];

    const int64_t t = xcd_tile(tiles);
    if (t < 0) return;
    const int n0 = (int)(t / row_tiles) * kMfmaBN;
    const int64_t m0 = (t % row_tiles) * BM_GENERIC;
    const int l32 = threadIdx.x & 31;
    const int64_t row_base = m0 + (threadIdx.x >> 7) * 64;

    init_onehot_lut(lut);  // the barrier inside mfma_lookup_tile's prologue orders it before use
    const uint8_t* irow[2];
#pragma unroll
    for (int i = 0; i < 2; ++i) {
        int64_t row = row_base + i * 32 + l32;
        row = row < N ? row : N - 1;  // never stored
        irow[i] = idx + row * C;
    }
    auto idx_word = [&](int i, int cbase) -> uint32_t {
        uint32_t word = 0;
        for (int b = 0; b < 4; ++b)
            if (cbase + b < C) word |= (uint32_t)irow[i][cbase + b] << (8 * b);
        return word;
    };
    v16i acc[2][4];
    mfma_lookup_tile<2>(packed, C, Mp, n0, lds, lut, idx_word, acc);
    mfma_store_tile<2>(acc, *scale, bias, M, N, row_base, n0 + ((threadIdx.x >> 6) & 1) * 128, Y, ldy);
}

}  // namespace

hipError_t launch_lookup_mfma_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                 int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                 hipStream_t s) {
    if (K > 16) return hipErrorInvalidValue;  // one 16-wide k block per codebook
    const int Mp = (int)packed_cols(M);
    const int64_t col_tiles = Mp / kMfmaBN;
    const bool dw = (C % 32 == 0) && ((reinterpret_cast<uintptr_t>(idx) & 15) == 0);
    const int bm = dw ? BM : BM_GENERIC;
    const int64_t row_tiles = (N + bm - 1) / bm;
    const int64_t tiles = row_tiles * col_tiles;
    const int64_t blocks = (tiles + 7) / 8 * 8;
    if (blocks > 0x7fffffffLL || row_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    if (dw)
        hipLaunchKernelGGL(lookup_mfma_i8_pipelined_kernel, dim3((unsigned)blocks), dim3(kMfmaThreads), 0,
                           s, reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y,
                           ldy, (int)row_tiles, tiles);
    else
        hipLaunchKernelGGL(lookup_mfma_i8_generic_kernel, dim3((unsigned)blocks), dim3(kMfmaThreads), 0, s,
                           reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y, ldy,
                           (int)row_tiles, tiles);
    return hipGetLastError();
}

}  // namespace lutnn
