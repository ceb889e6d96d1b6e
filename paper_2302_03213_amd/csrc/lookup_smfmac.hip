// Table read and accumulation (arXiv 2302.03213, Eq. 4) on the structured-sparse matrix cores of
// gfx950 (v_smfmac_i32_32x32x64_i8).
//
// Eq. 4 is OneHot[N x C*16] x T[C*16 x M].  A one-hot slice of 16 has one non-zero in four groups
// of four, so it trivially meets the 2:4 structured-sparsity format of the SMFMAC instructions:
// per group of 4 consecutive k the A operand stores 2 values plus a 2-bit position for each.  The
// instruction covers k = 64 (four codebooks) in the 32 cycles a dense 32x32x32 MFMA needs for two
// codebooks, so the contraction runs at twice the dense rate with the result unchanged (exact
// int32).  Measured operand layout (lane = 32h + l):
//   A values, lane (row l, half h): stored bytes 0-7  -> k block h     (k = 16h + ...),
//                                   stored bytes 8-15 -> k block 2 + h (k = 32 + 16h + ...);
//                                   stored bytes 2g, 2g+1 belong to group g of the block;
//   A positions: bits [2t+1:2t] of the index register = position (0-3) of stored byte t;
//   B, lane (column l, half h): bytes 0-15 -> k block 2h, bytes 16-31 -> k block 2h + 1;
//   D: as for the dense 32x32 MFMA.
// A lane's operand for one codebook with index p is therefore: stored byte 2(p>>2) = 1 (a 64-bit
// 1 << 16(p>>2)), position field of that byte = p&3, everything else 0.  The values are built in
// registers with one 64-bit shift per codebook; the position words of a whole super-stage are
// looked up (1 KiB table in LDS, indexed by a pair of index bytes) when its index bytes are picked
// up, off the critical path.
//
// Kernel shape.  Workgroup = 4 wavefronts stacked over rows, one per SIMD, output tile 512 rows x
// 128 columns (each wave 128 x 128, 256 accumulator registers): with the matrix pipe twice as
// fast, halving the table bytes per MFMA matters more than re-reading the indices (32 column
// blocks instead of 16).  Codebooks are walked in super-stages of 32 = 2 stages of 16 = 4 steps of
// 4 codebooks; step j of stage s' of super-stage u uses codebooks 32u + 16h + 8s' + 2j + {0,1} for
// lane half h, so a lane's 16 index bytes per super-stage are contiguous.  Table slabs (32 KiB
// per stage) and index bytes go global -> LDS directly (global_load_lds_dwordx4 from inline
// assembly, explicit vmcnt waits) three stages ahead through a ring of four stage buffers; the
// operands of the next step are read from LDS between the MFMAs of the current one.  See
// lookup_mfma.hip for the reasoning behind each of these choices; this kernel has the same
// structure with a different tile and operand format.
//
// Tiles are streamed: when a whole number of 4-stage ring turns fits (C % 64 == 0) the launch has
// one workgroup per compute unit and each workgroup walks several output tiles as ONE continuous
// stage stream - the last three stages of a tile already fetch the first three stages of the next
// one, so there is no pipeline fill per tile, and the stores of a finished tile drain while the
// next tile computes (with one wave per SIMD and all workgroups in step, a separate store phase
// per tile would leave the matrix pipes idle about a sixth of the time).
//
// Needs C % 32 == 0 and a 16-byte aligned idx.
#include <type_traits>

#include "lutnn_kernels.h"
#include "mfma_tile.h"

namespace lutnn {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int TM = 4;                 // 32-row blocks per wave
constexpr int WAVE_ROWS = TM * 32;    // 128
constexpr int BM = 4 * WAVE_ROWS;     // rows per workgroup (512)
constexpr int BN = 128;               // columns per workgroup
constexpr int NBUF = 4;               // LDS ring depth, stages
constexpr int SC = 16;                // codebooks per stage
constexpr int KSTEPS = 4;             // MFMA steps per stage, 4 codebooks each
constexpr int STAGE_VECS = SC * BN;   // uint4 per stage buffer (32 KiB)
constexpr int B_LOADS = 8;            // table loads per wave per stage
constexpr int I_LOADS = TM;           // index loads per wave per super-stage
constexpr int kComputeUnits = 256;    // MI355X: 8 XCDs x 32 CUs

__global__ __launch_bounds__(kMfmaThreads, 1) void lookup_smfmac_i8_kernel(
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int M, int Mp, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int row_tiles, int64_t tiles) {
    __shared__ uint4 ring[NBUF * STAGE_VECS];  // 4 x 32 KiB table slabs
    __shared__ uint4 ibuf[4][TM][64];          // [wave][row block][lane]: one super-stage of indices
    __shared__ uint32_t plut[256];             // position words by byte pair, see IdxWords

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
    const int l32 = lane & 31, h = lane >> 5;

    // XCD-aware tile schedule: consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2).  XCD x owns the contiguous tile range [x*per_xcd, (x+1)*per_xcd), tiles are
    // ordered column-block major, and the workgroups of the XCD take its tiles round robin, so at
    // any time they walk the same slab of the table.
    const int64_t per_xcd = (tiles + 7) / 8;
    const int wg_per_xcd = gridDim.x >> 3;
    const int64_t xcd_end = min(((int64_t)(blockIdx.x & 7) + 1) * per_xcd, tiles);
    int64_t t = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= xcd_end) return;

    // Per-tile addressing.  Indices of super-stage u: lane (row l32 of block i, half h) gets bytes
    // [32u + 16h, +16); rows >= N re-read row N-1 (their results are never stored).
    struct Tile {
        int n0;
        int64_t m0;
        const uint4* tsrc;    // packed + n0 (wave-uniform)
        const uint8_t* isrc;  // idx + m0 * C (wave-uniform)
        uint32_t ioff[TM];    // per-lane byte offset of the lane's index bytes from isrc
    };
    auto setup_tile = [&](int64_t tt, Tile& T) {
        T.n0 = (int)(tt / row_tiles) * BN;
        T.m0 = (tt % row_tiles) * BM;
        T.tsrc = packed + T.n0;
        T.isrc = idx + T.m0 * C;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int64_t row = w * WAVE_ROWS + i * 32 + l32;
            if (T.m0 + row >= N) row = N - 1 - T.m0;
            T.ioff[i] = (uint32_t)(row * C + 16 * h);
        }
    };
    Tile cur, nxt;
    setup_tile(t, cur);
    bool has_next = t + wg_per_xcd < xcd_end;
    setup_tile(has_next ? t + wg_per_xcd : t, nxt);

    const int supers = C / 32;  // C % 32 == 0
    const int stages = 2 * supers;

    {  // position table: entry p0 | p1 << 4
        const uint32_t p0 = tid & 15, p1 = tid >> 4;
        plut[tid] = ((p0 & 3) << (4 * (p0 >> 2))) | ((p1 & 3) << (16 + 4 * (p1 >> 2)));
    }

    // ---- load issue.  Slot g of stage s = 2u + s' holds codebook 32u + 16(g>>3) + 8s' + (g&7).
    // Wave w copies slots 4w .. 4w+3, both 64-column halves: load q -> slot 4w + (q>>1), half q&1.
    // Stage / super-stage numbers past the end of the tile address the next tile of the stream.
    const uint32_t lane16 = lane * 16;
    const uint32_t ring0 = lds_offset(ring);
    auto load_b = [&](int s, int q) {
        const bool in_cur = s < stages;
        const uint4* src = in_cur ? cur.tsrc : nxt.tsrc;
        if (!in_cur) s -= stages;
        const int g = 4 * w + (q >> 1);
        const int c = 32 * (s >> 1) + 16 * (g >> 3) + 8 * (s & 1) + (g & 7);
        dma16(ring0 + ((s & 3) * STAGE_VECS + g * BN + 64 * (q & 1)) * 16,
              src + (size_t)c * Mp + 64 * (q & 1), lane16);
    };
    const uint32_t ibuf0 = lds_offset(ibuf) + w * TM * 64 * 16;
    auto load_idx = [&](int u, int i) {
        const bool in_cur = u < supers;
        dma16(ibuf0 + i * 64 * 16, (in_cur ? cur.isrc : nxt.isrc) + 32 * (in_cur ? u : u - supers),
              in_cur ? cur.ioff[i] : nxt.ioff[i]);
    };

    v16i acc[TM][4];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Operand registers, double buffered over MFMA steps.  B: 8 LDS reads per step, read r is
    // half (r&1) of column tile r>>1.  A: built from the index words, no memory access.
    typedef unsigned long long u64;
    typedef u64 u64x2 __attribute__((ext_vector_type(2)));
    u64x2 a[2][TM];
    v8i b[2][4];
    auto load_b_operand = [&](int set, int sbuf, int j, int r) {
        const int tn = r >> 1, half = r & 1;
        const uint4 v = ring[sbuf * STAGE_VECS + (8 * half + 2 * j + h) * BN + tn * 32 + l32];
        b[set][tn][4 * half + 0] = (int)v.x;
        b[set][tn][4 * half + 1] = (int)v.y;
        b[set][tn][4 * half + 2] = (int)v.z;
        b[set][tn][4 * half + 3] = (int)v.w;
    };
    // Index words of one super-stage, per row block i:
    //   raw[i][d]  the 16 index bytes as loaded
    //   pos[i][t]  position word of step t (0..7 over the two stages): codebook 2t in the low
    //              half, codebook 2t+1 in the high half, each (p & 3) << 4(p >> 2).  Looked up in
    //              a 256-entry table indexed by the byte pair p0 | p1 << 4.
    struct IdxWords {
        uint32_t raw[TM][4];
        uint32_t pos[TM][8];
    };
    auto make_a_operand = [&](int set, int sp, int j, const IdxWords& wq, int i) {
        // values: stored byte 2(p>>2) = 1, i.e. the 64-bit value 1 << 16(p>>2)
        const uint32_t word = wq.raw[i][2 * sp + (j >> 1)];
        const uint32_t s0 = ((word >> (16 * (j & 1))) << 2) & 0x30u;
        const uint32_t s1 = ((word >> (16 * (j & 1) + 8)) << 2) & 0x30u;
        a[set][i][0] = (u64)1 << s0;
        a[set][i][1] = (u64)1 << s1;
    };
    auto read_idx = [&](IdxWords& wq) {
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            const uint4 v = ibuf[w][i][lane];
            const uint32_t raw[4] = {v.x, v.y, v.z, v.w};
#pragma unroll
            for (int d = 0; d < 4; ++d) {
                wq.raw[i][d] = raw[d];
                const uint32_t pair = (raw[d] | (raw[d] >> 4)) << 2;  // bytes 0, 2: (p0 | p1<<4) * 4
                wq.pos[i][2 * d + 0] = *reinterpret_cast<const uint32_t*>(
                    reinterpret_cast<const char*>(plut) + (pair & 0x3fcu));
                wq.pos[i][2 * d + 1] = *reinterpret_cast<const uint32_t*>(
                    reinterpret_cast<const char*>(plut) + ((pair >> 16) & 0x3fcu));
            }
        }
    };

    // ---- prologue: stages 0..2, the indices of super-stage 0 (into registers) and 1 (in flight)
#pragma unroll
    for (int i = 0; i < TM; ++i) load_idx(0, i);
#pragma unroll
    for (int s = 0; s < 3; ++s)
        if (s < stages)
#pragma unroll
            for (int q = 0; q < B_LOADS; ++q) load_b(s, q);
    wait_loads<0>();
    __syncthreads();
    IdxWords wcur, wnext;
    read_idx(wcur);
    __syncthreads();  // every lane has its words before the buffer is refilled
    if (supers > 1 || has_next) {
#pragma unroll
        for (int i = 0; i < TM; ++i) load_idx(1, i);
    }
#pragma unroll
    for (int r = 0; r < 8; ++r) load_b_operand(0, 0, 0, r);
#pragma unroll
    for (int i = 0; i < TM; ++i) make_a_operand(0, 0, 0, wcur, i);

    // One stage s.  SB = s % 4 (ring buffer), SP = s % 2 (stage within the super-stage).
    // FULL = steady state: stage s+3 exists, and in the second stage of a super-stage the
    // super-stage after next exists, so nothing in the body is conditional.
    auto run_stage = [&](int s, auto sb_c, auto full) {
        constexpr int SB = decltype(sb_c)::value;
        constexpr int SP = SB & 1;
        constexpr bool FULL = decltype(full)::value;
        const int u = s >> 1;
        const bool do_fetch = FULL || s + 3 < stages;
        const bool do_idx = SP == 1 && (FULL || u + 2 < supers);
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) {
            // second stage of a super-stage: pick up the next super-stage's index words (their
            // loads were issued a super-stage ago and awaited at the end of the previous stage;
            // past the last super-stage this reads stale, unused data)
            if (SP == 1 && j == 2) read_idx(wnext);
            // 8 groups of two MFMAs; behind each group one LDS read of a B operand for the next
            // step (after the last step: the first step of the next stage, in the first four
            // groups so that the reads have returned when the barrier waits for the LDS counter),
            // half an A operand, and at most one load.
            const int tstep = 4 * SP + j;  // step within the super-stage
#pragma unroll
            for (int g = 0; g < 8; ++g) {
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int q = 2 * g; q < 2 * g + 2; ++q) {
                    // column-tile major: the B tiles are read in this order a step earlier, so
                    // the tile read last is also used last
                    const int i = q & 3, tn = q >> 2;
                    const u64x2 av = a[j & 1][i];
                    const v4i a4 = {(int)(uint32_t)av[0], (int)(uint32_t)(av[0] >> 32),
                                    (int)(uint32_t)av[1], (int)(uint32_t)(av[1] >> 32)};
                    acc[i][tn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(
                        a4, b[j & 1][tn], acc[i][tn], (int)wcur.pos[i][tstep], 0, 0);
                }
                if (j + 1 < KSTEPS) {
                    load_b_operand((j + 1) & 1, SB, j + 1, g);
                    if (g & 1) make_a_operand((j + 1) & 1, SP, j + 1, wcur, g >> 1);
                } else {
                    if (g < 4) {
                        load_b_operand(0, (SB + 1) % NBUF, 0, 2 * g);
                        load_b_operand(0, (SB + 1) % NBUF, 0, 2 * g + 1);
                    }
                    if (g & 1) {
                        if (SP == 0)
                            make_a_operand(0, 1, 0, wcur, g >> 1);
                        else
                            make_a_operand(0, 0, 0, wnext, g >> 1);
                    }
                }
                if (do_fetch && (g == 1 || g == 5)) load_b(s + 3, 2 * j + (g == 5));
                // the index buffer is free once read_idx above has returned (step 2); refill it in
                // step 3 with the super-stage after next
                if (do_idx && j == 3 && g < I_LOADS && g != 1) load_idx(u + 2, g);
                if (do_idx && j == 3 && g == 6) load_idx(u + 2, 1);
            }
        }
        __builtin_amdgcn_sched_barrier(0);
        // Before the barrier everything issued before this stage must have landed (stage s+2 is
        // read from the end of stage s+1 on); this stage's own loads stay in flight.
        if (FULL) {
            if (SP == 1)
                wait_loads<B_LOADS + I_LOADS>();
            else
                wait_loads<B_LOADS>();
        } else {
            wait_loads<0>();
        }
        __syncthreads();
        if (SP == 1) wcur = wnext;
    };
    using B0 = std::integral_constant<int, 0>;
    using B1 = std::integral_constant<int, 1>;
    using B2 = std::integral_constant<int, 2>;
    using B3 = std::integral_constant<int, 3>;

    // The stage stream.  A group of four stages runs unconditionally (FULL) while its last stage
    // still has stage s+3 and super-stage u+2 ahead of it - in this tile, or in the next one when
    // the workgroup streams on (only launched when stages % 4 == 0 and supers >= 2, so that the
    // ring phase and the index look-ahead carry over).
    const float sc = *scale;
    for (;;) {
        int s = 0;
        for (; s < stages && (has_next || (s + 6 < stages && (s + 3) / 2 + 2 < supers)); s += 4) {
            run_stage(s + 0, B0{}, std::true_type{});
            run_stage(s + 1, B1{}, std::true_type{});
            run_stage(s + 2, B2{}, std::true_type{});
            run_stage(s + 3, B3{}, std::true_type{});
        }
        for (; s < stages; s += 4) {
            run_stage(s + 0, B0{}, std::false_type{});
            run_stage(s + 1, B1{}, std::false_type{});  // stages come in pairs
            if (s + 2 < stages) {
                run_stage(s + 2, B2{}, std::false_type{});
                run_stage(s + 3, B3{}, std::false_type{});
            }
        }
        mfma_store_tile<TM>(acc, sc, bias, M, N, cur.m0 + w * WAVE_ROWS, cur.n0, Y, ldy);
        if (!has_next) break;
        // next tile: its first stages and index words are already in LDS / registers
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        t += wg_per_xcd;
        cur = nxt;
        has_next = t + wg_per_xcd < xcd_end;
        if (has_next) setup_tile(t + wg_per_xcd, nxt);
    }
}

}  // namespace

bool smfmac_supported(int C, int K, const uint8_t* idx) {
    return K <= 16 && C % 32 == 0 && (reinterpret_cast<uintptr_t>(idx) & 15) == 0;
}

hipError_t launch_lookup_smfmac_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                   int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                   hipStream_t s) {
    if (!smfmac_supported(C, K, idx)) return hipErrorInvalidValue;
    const int Mp = (int)packed_cols(M);
    const int64_t col_tiles = (M + BN - 1) / BN;  // the packed table is padded to 256 columns
    const int64_t row_tiles = (N + BM - 1) / BM;
    const int64_t tiles = row_tiles * col_tiles;
    int64_t blocks = (tiles + 7) / 8 * 8;
    if (blocks > 0x7fffffffLL || row_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    // Stream several tiles per workgroup when the ring phase carries over from tile to tile:
    // one workgroup per compute unit (the kernel's LDS footprint allows only one anyway).
    if (C % 64 == 0 && blocks > kComputeUnits) blocks = kComputeUnits;
    hipLaunchKernelGGL(lookup_smfmac_i8_kernel, dim3((unsigned)blocks), dim3(kMfmaThreads), 0, s,
                       reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y, ldy,
                       (int)row_tiles, tiles);
    return hipGetLastError();
}

}  // namespace lutnn
