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
// registers with one 64-bit shift per codebook; the position words are looked up in a 1 KiB table
// in LDS indexed by a pair of index bytes.
//
// Kernel shape.  Workgroup = 4 wavefronts stacked over rows, one per SIMD, output tile 512 rows x
// 128 columns (each wave 128 x 128, 256 accumulator registers): with the matrix pipe twice as
// fast, halving the table bytes per MFMA matters more than re-reading the indices (32 column
// blocks instead of 16).  Codebooks are walked in super-stages of 32 = 2 stages of 16 = 4 steps of
// 4 codebooks; step j of stage s' of super-stage u uses codebooks 32u + 16h + 8s' + 2j + {0,1} for
// lane half h, so a lane's 16 index bytes per super-stage are contiguous.  Table slabs (32 KiB
// per stage) and index bytes go global -> LDS directly (global_load_lds_dwordx4 from inline
// assembly, explicit vmcnt waits) three stages ahead through a ring of four stage buffers.
//
// Instruction schedule.  A wave issues in order, and the next SMFMAC cannot issue before the
// previous one has left the pipe (32 cycles, about 8 issue slots).  Whatever sits between two
// SMFMACs beyond ~6 instructions therefore delays the matrix pipe, and whatever is NOT placed
// between two SMFMACs wastes slots that were free.  So the stage body is written as 64 slots of
// "one SMFMAC + its share of the housekeeping", pinned with scheduling barriers, and every piece
// of housekeeping is cut into units of at most ~5 instructions with a fixed slot:
//   even slots          one LDS read of a B operand for the next step
//   slots 2, 10         one table load (DMA) for stage s+3; slot 12 advances the load pointer
//   slots 1, 5, 9, 13   half of the work on one 4-byte index word (position-word look-ups, the
//                       shift word the A values are built from) - 32 such halves per super-stage,
//                       done in the order their results are needed
//   slots 3, 7, 11, 15  the two A values of one row block for the next step
//   stage 1 of a super-stage, step 0: the four 16-byte LDS reads of the next super-stage's
//                       index bytes; step 3: the loads (DMA) of the super-stage after that
//
// Tiles are streamed: when a whole number of 4-stage ring turns fits (C % 64 == 0) the launch has
// one workgroup per compute unit and each workgroup walks several output tiles as ONE continuous
// stage stream - the last three stages of a tile already fetch the first three stages of the next
// one, so there is no pipeline fill per tile.
//
// Needs C % 32 == 0 and a 16-byte aligned idx.
#include <algorithm>
#include <cstdlib>
#include <type_traits>

#include "lutnn_kernels.h"
#include "mfma_tile.h"

namespace lutnn {
namespace {

typedef int v8i __attribute__((ext_vector_type(8)));

constexpr int NBUF = 4;               // LDS ring depth, stages
constexpr int SC = 16;                // codebooks per stage
constexpr int KSTEPS = 4;             // MFMA steps per stage, 4 codebooks each

// 64 lanes x 16 bytes global -> LDS at (lds_base + LDS_IMM) + 16 * lane; see dma16().  GOFF: a constant
// added to every lane's global address through the instruction's offset field, which the hardware
// adds to the LDS address as well: M0 is set lower by as much.
template <int LDS_IMM, int GOFF = 0>
__device__ __forceinline__ void dma16_at(uint32_t lds_base, const void* sbase, uint32_t voff) {
    asm volatile(
        "s_add_u32 m0, %0, %3\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %1, %2 offset:%4"
        :
        : "s"(lds_base), "v"(voff), "s"(sbase), "n"(LDS_IMM - GOFF), "n"(GOFF)
        : "memory", "m0", "scc");
}

// TM = 32-row blocks per wavefront, TN = 32-column tiles per wavefront (4, or 3): the workgroup tile
// is 128*TM rows x 32*TN columns.  (4, 4) is the efficient shape; TM = 3, 2 and 1 exist so that
// problems with few rows still spread over the chip, and TN = 3 (96 columns) for widths where it
// yields a whole number of rounds of tiles and 128 columns do not (M = 3072 at 4096 rows: 256 tiles
// of 512 x 96 against 192 of 512 x 128 on 256 compute units).
// SPLITS > 1 (run-time `splits`, template flag SPLIT): `splits` workgroups share an output tile, each
// contracts C / splits consecutive codebooks and adds its int32 partial sums into Y with atomics; Y
// then holds integers (zeroed beforehand, turned into the final floats by a separate pass).  For
// problems with fewer tiles than compute units: more workgroups stream the table in parallel.
template <int TM, int TN, bool SPLIT = false, bool STREAM = false>
__global__ __launch_bounds__(kMfmaThreads, 1) void lookup_smfmac_i8_kernel(
    const uint4* __restrict__ packed, const float* __restrict__ scale, const float* __restrict__ bias,
    int C, int M, int Mp, const uint8_t* __restrict__ idx, int64_t N, float* __restrict__ Y,
    int64_t ldy, int row_tiles, int64_t tiles, int splits, int row_group) {
    constexpr int WAVE_ROWS = TM * 32;
    constexpr int BM = 4 * WAVE_ROWS;  // rows per workgroup
    static_assert(TN == 4 || (TN == 3 && TM == 4), "column tiles per wavefront");
    constexpr int BN = 32 * TN;          // columns per workgroup
    constexpr int STAGE_VECS = SC * BN;  // uint4 per stage buffer (32 KiB at TN = 4)
    constexpr int B_LOADS = 2 * TN;      // table loads per wave per stage (1 KiB each)
    constexpr int I_LOADS = TM;          // index loads per wave per super-stage
    constexpr int S = TN * TM;           // SMFMAC slots per step
    // index-word half-operations: 8*TM per super-stage, TM per step; the sequence of a super-stage
    // starts at this position of the one before it (after its index bytes were read from LDS in
    // step 0 of the second stage, early enough that the words of d = 0 are finished two steps later)
    constexpr int HSEQ = 8 * TM;
    constexpr int HSTART = TM == 1 ? 5 : 4 * TM + TM / 2;
    __shared__ uint4 ring[NBUF * STAGE_VECS];  // 4 x 32 KiB table slabs
    __shared__ uint4 ibuf[4][TM][64];          // [wave][row block][lane]: one super-stage of indices
    __shared__ uint32_t plut[256];             // position words by byte pair, see IdxWords

    const int tid = threadIdx.x;
    const int lane = tid & 63;
    const int w = __builtin_amdgcn_readfirstlane(tid >> 6);  // wave-uniform
    const int l32 = lane & 31, h = lane >> 5;

    // XCD-aware tile schedule: consecutive workgroup ids land on different XCDs (8 of them, each
    // with its own L2).  XCD x owns the contiguous tile range [x*per_xcd, (x+1)*per_xcd) of the tile
    // order (column-block major, or grouped by row tiles: see aim_loads_at), and the workgroups of
    // the XCD take its tiles round robin, so at any time they share table slabs and index rows.
    const int64_t per_xcd = (tiles + 7) / 8;
    const int wg_per_xcd = gridDim.x >> 3;
    const int64_t xcd_end = min(((int64_t)(blockIdx.x & 7) + 1) * per_xcd, tiles);
    int64_t t = (int64_t)(blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (t >= xcd_end) return;
    bool has_next = t + wg_per_xcd < xcd_end;

    // codebooks of this workgroup: all C, or share `t % splits` of them (C / splits % 32 == 0)
    const int c_count = SPLIT ? C / splits : C;
    const int c_begin = SPLIT ? (int)(t % splits) * c_count : 0;
    const int supers = c_count / 32;  // C % 32 == 0
    const int stages = 2 * supers;

    // ---- the two streams.  Compute works on tile (ct_n0, ct_m0); the loads run three stages
    // ahead and move on to the next tile of this workgroup while the current one is still being
    // computed.  Load state: bp = address of the next table row this wave loads (rows of 128
    // columns x 16 B at packed + n0, one per codebook; the wave owns rows 16(w>>1) + 4(w&1) + 0..3
    // of each stage), ip = index bytes of the next super-stage to load (row 0 of the tile), fioff
    // = per-lane byte offset of the lane's index bytes: lane (row l32 of block i, half h) gets
    // bytes [32u + 16h, +16) of its row; rows >= N re-read row N-1 (never stored).
    int ct_n0, ft_n0;
    int64_t ct_m0, ft_m0;
    const char* bp;
    const uint8_t* ip;
    uint32_t fioff[TM];
    const uint32_t rs1 = (uint32_t)Mp * 16u;  // bytes from one codebook's row to the next
    const int row0 = 16 * (w >> 1) + 4 * (w & 1);
    auto aim_loads_at = [&](int64_t tt) {
        const int64_t tile = SPLIT ? tt / splits : tt;
        if (row_group > 0) {
            // Row tiles in groups of `row_group`, column-block major within a group: the workgroups
            // of an XCD that run at the same time then share `row_group` row tiles' index bytes AND
            // a few column blocks' table slabs, instead of one slab and every row tile's indices.
            const int64_t col_tiles = (SPLIT ? tiles / splits : tiles) / row_tiles;
            const int64_t per_group = (int64_t)row_group * col_tiles;
            const int64_t g = tile / per_group, rem = tile - g * per_group;
            const int64_t rows_here = min((int64_t)row_group, (int64_t)row_tiles - g * row_group);
            ft_n0 = (int)(rem / rows_here) * BN;
            ft_m0 = (g * row_group + rem % rows_here) * BM;
        } else {
            ft_n0 = (int)(tile / row_tiles) * BN;
            ft_m0 = (tile % row_tiles) * BM;
        }
        bp = reinterpret_cast<const char*>(packed + ft_n0) + (size_t)(row0 + c_begin) * rs1;
        ip = idx + ft_m0 * C + c_begin;
#pragma unroll
        for (int i = 0; i < TM; ++i) {
            int64_t row = w * WAVE_ROWS + i * 32 + l32;
            if (ft_m0 + row >= N) row = N - 1 - ft_m0;
            fioff[i] = (uint32_t)(row * C + 16 * h);
        }
    };
    aim_loads_at(t);
    ct_n0 = ft_n0;
    ct_m0 = ft_m0;

    {  // position table: entry p0 | p1 << 4
        const uint32_t p0 = tid & 15, p1 = tid >> 4;
        plut[tid] = ((p0 & 3) << (4 * (p0 >> 2))) | ((p1 & 3) << (16 + 4 * (p1 >> 2)));
    }

    // ---- load issue.  Slot g of stage s = 2u + s' holds codebook 32u + 16(g>>3) + 8s' + (g&7).
    // Wave w copies slots 4w .. 4w+3, both 64-column halves: load q -> slot 4w + (q>>1), half q&1.
    const uint32_t lane16 = lane * 16;
    const uint32_t lane16_hi = lane * 16 + 1024;  // second 64-column half of a row
    const uint32_t ring_w = lds_offset(ring) + 4 * w * BN * 16;
    const uint32_t ibuf_w = lds_offset(ibuf) + w * TM * 64 * 16;
    // TN = 3: a row of 96 columns is 1.5 loads.  The wave's four rows of a stage are 6 KiB = six
    // loads, contiguous in LDS; load q covers rows 2(q/3) and 2(q/3)+1: the first KiB of the first
    // row, then its last half KiB together with the first half KiB of the second (lanes 32-63), then
    // the second row's last KiB.  bp stays at the wave's first row for the whole stage.
    const uint32_t lane16_mid = lane < 32 ? 1024u + lane * 16u : rs1 + (lane - 32) * 16u;
    auto load_b = [&](auto fb_c, auto q_c) {  // load q of the stage that goes to ring buffer FB
        constexpr int FB = decltype(fb_c)::value, Q = decltype(q_c)::value;
        if constexpr (TN == 4) {
            dma16_at<(FB * STAGE_VECS + (Q >> 1) * BN + 64 * (Q & 1)) * 16>(ring_w, bp, (Q & 1) ? lane16_hi : lane16);
        } else {
            constexpr int LDS = FB * STAGE_VECS * 16 + Q * 1024;
            const char* rows = bp + (size_t)(2 * (Q / 3)) * rs1;
            if constexpr (Q % 3 == 0)
                dma16_at<LDS>(ring_w, rows, lane16);
            else if constexpr (Q % 3 == 1)
                dma16_at<LDS>(ring_w, rows, lane16_mid);
            else
                dma16_at<LDS, 512>(ring_w, rows + rs1, lane16);
        }
    };
    auto load_idx = [&](auto i_c) {
        constexpr int I = decltype(i_c)::value;
        dma16_at<I * 64 * 16>(ibuf_w, ip, fioff[I]);
    };
    // after the four rows of a stage: on to the rows of the next stage (+8 codebooks within a
    // super-stage, +24 to the next super-stage)
    auto next_stage_rows = [&](int sp_of_loaded_stage) {
        if constexpr (TN == 4)  // bp has moved on by three rows while the stage was loaded
            bp += (sp_of_loaded_stage == 0) ? 5 * (size_t)rs1 : 21 * (size_t)rs1;
        else
            bp += (sp_of_loaded_stage == 0) ? 8 * (size_t)rs1 : 24 * (size_t)rs1;
    };

    v16i acc[TM][TN];
#pragma unroll
    for (int i = 0; i < TM; ++i)
#pragma unroll
        for (int j = 0; j < TN; ++j)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;

    // Operand registers, double buffered over MFMA steps.  B: 8 LDS reads per step, read r is
    // half (r&1) of column tile r>>1.  A: built from the index words, no memory access.
    typedef unsigned long long u64;
    typedef u64 u64x2 __attribute__((ext_vector_type(2)));
    u64x2 a[2][TM];
    v8i b[2][TN];
    auto load_b_operand = [&](int set, int sbuf, int j, int r) {
        const int tn = r >> 1, half = r & 1;
        const uint4 v = ring[sbuf * STAGE_VECS + (8 * half + 2 * j + h) * BN + tn * 32 + l32];
        b[set][tn][4 * half + 0] = (int)v.x;
        b[set][tn][4 * half + 1] = (int)v.y;
        b[set][tn][4 * half + 2] = (int)v.z;
        b[set][tn][4 * half + 3] = (int)v.w;
    };
    // Index words of one super-stage, per row block i and 4-byte word d (codebooks 4d .. 4d+3 of
    // the lane's 16):
    //   sh[i][d]   first the index bytes as loaded; after the word's second half-operation, byte
    //              b = 16 (p >> 2) of codebook 4d + b: the shift that builds its A values
    //   pos[i][t]  position word of step t (0..7 over the two stages): codebook 2t in the low
    //              half, codebook 2t+1 in the high half, each (p & 3) << 4(p >> 2).  Looked up in
    //              a 256-entry table indexed by the byte pair p0 | p1 << 4.
    struct IdxWords {
        uint32_t sh[TM][4];
        uint32_t pos[TM][8];
    };
    auto read_ibuf = [&](IdxWords& wq, int i) {
        // 384-row tiles: the address is formed here, from the lane's byte offset, every time.  Held
        // in a register of its own across the stage loop it is one live value too many for that
        // instance, and the allocator's way out was a reload from scratch memory inside the loop,
        // whose wait (the vector-memory counter at zero) also waits for every table load in flight.
        // (The other instances keep the plain form: their loops come out shorter with it.)
        uint4 v;
        if constexpr (TM == 3) {
            uint32_t lane_bytes = lane16;
            asm volatile("" : "+v"(lane_bytes));
            typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
            const u32x4 t = *reinterpret_cast<const __attribute__((address_space(3))) u32x4*>(ibuf_w + i * 1024 + lane_bytes);
            v = uint4{t[0], t[1], t[2], t[3]};
        } else {
            v = ibuf[w][i][lane];
        }
        wq.sh[i][0] = v.x;
        wq.sh[i][1] = v.y;
        wq.sh[i][2] = v.z;
        wq.sh[i][3] = v.w;
    };
    // Half-operation k = 0..8*TM-1 of a super-stage's index words: word (i, d) = ((k>>1) % TM, (k>>1) / TM),
    // first half = position word of codebooks 4d, 4d+1; second half = that of 4d+2, 4d+3, and the
    // shift word.  Words are finished in the order d = 0, 1, 2, 3, the order the steps use them.
    uint32_t pair = 0;  // carried from the first half of a word to the second
    // LDS address of the table in a vector register (kept opaque): (x & mask) | base is then one
    // v_and_or_b32 instead of an AND and an OR with a constant that is no inline constant
    uint32_t plut_base = lds_offset(plut);
    asm volatile("" : "+v"(plut_base));
    auto plut_at_addr = [&](uint32_t lds_addr) {
        return *reinterpret_cast<const __attribute__((address_space(3))) uint32_t*>(lds_addr);
    };
    auto idx_halfop = [&](IdxWords& wq, int k) {
        const int d = (k >> 1) / TM, i = (k >> 1) % TM;
        if ((k & 1) == 0) {
            const uint32_t raw = wq.sh[i][d];
            // bits 2-9 = 4 (p0 | p1 << 4), bits 18-25 = 4 (p2 | p3 << 4): byte offsets into plut
            pair = (raw << 2) | (raw >> 2);
            wq.pos[i][2 * d + 0] = plut_at_addr((pair & 0x3fcu) | plut_base);
        } else {
            wq.pos[i][2 * d + 1] = plut_at_addr(((pair >> 16) & 0x3fcu) | plut_base);
            wq.sh[i][d] = (wq.sh[i][d] << 2) & 0x30303030u;
        }
    };
    // A values of row block i for step j of stage sp: stored byte 2(p>>2) = 1, i.e. the 64-bit
    // value 1 << 16(p>>2).  The shift instruction itself takes its amount modulo 64, so the bytes
    // above the one that holds the amount need no masking - which C cannot express (a shift by 64
    // or more is undefined there), hence the instruction is written out: one AND less per value.
    auto one_shl = [](uint32_t amount) {
        u64 r;
        asm("v_lshlrev_b64 %0, %1, 1" : "=v"(r) : "v"(amount));
        return r;
    };
    auto make_a_operand = [&](int set, int sp, int j, const IdxWords& wq, int i) {
        const uint32_t word = wq.sh[i][2 * sp + (j >> 1)];
        a[set][i][0] = one_shl(word >> (16 * (j & 1)));
        a[set][i][1] = one_shl(word >> (16 * (j & 1) + 8));
    };

    using I0 = std::integral_constant<int, 0>;
    using I1 = std::integral_constant<int, 1>;
    using I2 = std::integral_constant<int, 2>;
    using I3 = std::integral_constant<int, 3>;

    // ---- prologue: stages 0..2 and the indices of super-stage 0 (into registers) and 1 (in
    // flight); afterwards the load state points at stage 3 / super-stage 2.
    auto load_idx_all = [&]() {
        load_idx(I0{});
        if constexpr (TM > 1) load_idx(I1{});
        if constexpr (TM > 2) load_idx(I2{});
        if constexpr (TM > 3) load_idx(I3{});
        ip += 32;
    };
    load_idx_all();
    auto load_stage = [&](auto fb_c) {
        load_b(fb_c, I0{});
        load_b(fb_c, I1{});
        if constexpr (TN == 4) bp += rs1;
        load_b(fb_c, std::integral_constant<int, 2>{});
        load_b(fb_c, std::integral_constant<int, 3>{});
        if constexpr (TN == 4) bp += rs1;
        load_b(fb_c, std::integral_constant<int, 4>{});
        load_b(fb_c, std::integral_constant<int, 5>{});
        if constexpr (TN == 4) {
            bp += rs1;
            load_b(fb_c, std::integral_constant<int, 6>{});
            load_b(fb_c, std::integral_constant<int, 7>{});
        }
    };
    load_stage(I0{});
    next_stage_rows(0);
    load_stage(I1{});
    next_stage_rows(1);
    if (stages > 2) {
        load_stage(I2{});
        next_stage_rows(0);
    }
    wait_loads<0>();
    __syncthreads();
    // Index words ping-pong between wq[0] (even super-stages) and wq[1] (odd ones); four stages
    // are two super-stages, so the ring phase SB of a stage also fixes which of the two it uses.
    IdxWords wq[2];
#pragma unroll
    for (int i = 0; i < TM; ++i) read_ibuf(wq[0], i);
#pragma unroll
    for (int k = 0; k < HSEQ - HSTART; ++k) idx_halfop(wq[0], k);  // the stage loop continues from here
    __syncthreads();  // every lane has its words before the buffer is refilled
    if (supers > 1) load_idx_all();
#pragma unroll
    for (int r = 0; r < 2 * TN; ++r) load_b_operand(0, 0, 0, r);
#pragma unroll
    for (int i = 0; i < TM; ++i) make_a_operand(0, 0, 0, wq[0], i);

    // One stage s.  SB = s % 4 (ring buffer), SP = s % 2 (stage within the super-stage).
    // FULL = steady state: stage s+3 exists, and in the second stage of a super-stage the
    // super-stage after next exists, so nothing in the body is conditional.
    auto run_stage = [&](int s, auto sb_c, auto full) {
        constexpr int SB = decltype(sb_c)::value;
        constexpr int SP = SB & 1;
        constexpr int FB = (SB + 3) % NBUF;  // ring buffer of stage s + 3
        constexpr bool FULL = decltype(full)::value;
        IdxWords& wcur = wq[SB >> 1];
        IdxWords& wnext = wq[(SB >> 1) ^ 1];
        const bool do_fetch = FULL || s + 3 < stages;
        const bool do_idx = SP == 1 && (FULL || (s >> 1) + 2 < supers);
        // stage s + 3 is the first stage of the next tile: the loads move on
        if (FULL && SB == 1 && s + 3 == stages) aim_loads_at(t + wg_per_xcd);
#pragma unroll
        for (int j = 0; j < KSTEPS; ++j) {
            const int tstep = 4 * SP + j;  // step within the super-stage
#pragma unroll
            for (int q = 0; q < S; ++q) {
                __builtin_amdgcn_sched_barrier(0);
                {
                    // column-tile major: the B tiles are read in this order a step earlier, so
                    // the tile read last is also used last
                    const int i = q % TM, tn = q / TM;
                    const u64x2 av = a[j & 1][i];
                    const v4i a4 = {(int)(uint32_t)av[0], (int)(uint32_t)(av[0] >> 32),
                                    (int)(uint32_t)av[1], (int)(uint32_t)(av[1] >> 32)};
                    acc[i][tn] = __builtin_amdgcn_smfmac_i32_32x32x64_i8(
                        a4, b[j & 1][tn], acc[i][tn], (int)wcur.pos[i][tstep], 0, 0);
                }
                // B operands of the next step, eight LDS reads spread over the slots; after the
                // last step: the first step of the next stage, in the first slots so that the
                // reads have returned when the barrier waits for the LDS counter
                if (j + 1 < KSTEPS) {
                    if constexpr (S == 16 || TN == 3) {
                        if ((q & 1) == 0) load_b_operand((j + 1) & 1, SB, j + 1, q >> 1);
                    } else if constexpr (S == 12) {
                        if (q % 3 != 2) load_b_operand((j + 1) & 1, SB, j + 1, q - q / 3);
                    } else if constexpr (S == 8) {
                        load_b_operand((j + 1) & 1, SB, j + 1, q);
                    } else {
                        load_b_operand((j + 1) & 1, SB, j + 1, 2 * q);
                        load_b_operand((j + 1) & 1, SB, j + 1, 2 * q + 1);
                    }
                } else {
                    if constexpr (S >= 8) {
                        if (q < 2 * TN) load_b_operand(0, (SB + 1) % NBUF, 0, q);
                    } else {
                        load_b_operand(0, (SB + 1) % NBUF, 0, 2 * q);
                        load_b_operand(0, (SB + 1) % NBUF, 0, 2 * q + 1);
                    }
                }
                // second stage of a super-stage: pick up the next super-stage's index bytes
                // (their loads were issued a super-stage ago and awaited at the end of the
                // previous stage; past the last super-stage this reads stale, unused data)
                if (SP == 1 && j == 0 && (q & 1) == 0 && q / 2 < TM) read_ibuf(wnext, q / 2);
                // index-word half-operations, one every TN-th slot
                if (q % TN == 1) {
                    const int n = (4 * SP + j) * TM + q / TN;
                    idx_halfop(n >= HSTART ? wnext : wcur, (n - HSTART + HSEQ) % HSEQ);
                }
                // A values of the next step, one row block at a time
                if (q % TN == TN - 1) {
                    const int i = q / TN;
                    if (j + 1 < KSTEPS)
                        make_a_operand((j + 1) & 1, SP, j + 1, wcur, i);
                    else if (SP == 0)
                        make_a_operand(0, 1, 0, wcur, i);
                    else
                        make_a_operand(0, 0, 0, wnext, i);
                }
                // table loads of stage s + 3: rows one per step, two halves (TN = 3: six loads,
                // two in steps 0 and 2, one in steps 1 and 3)
                if (do_fetch && TN == 3) {
                    if (q == 2) {
                        if (j == 0) load_b(std::integral_constant<int, FB>{}, I0{});
                        if (j == 1) load_b(std::integral_constant<int, FB>{}, I2{});
                        if (j == 2) load_b(std::integral_constant<int, FB>{}, I3{});
                        if (j == 3) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 5>{});
                    }
                    if (q == 8) {
                        if (j == 0) load_b(std::integral_constant<int, FB>{}, I1{});
                        if (j == 2) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 4>{});
                    }
                    if (q == S - 1 && j + 1 == KSTEPS) next_stage_rows(SP ^ 1);
                }
                if (do_fetch && TN == 4) {
                    if (q == (S >= 8 ? 2 : 0)) {
                        if (j == 0) load_b(std::integral_constant<int, FB>{}, I0{});
                        if (j == 1) load_b(std::integral_constant<int, FB>{}, I2{});
                        if (j == 2) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 4>{});
                        if (j == 3) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 6>{});
                    }
                    if (q == (S >= 8 ? 2 + S / 2 : 2)) {
                        if (j == 0) load_b(std::integral_constant<int, FB>{}, I1{});
                        if (j == 1) load_b(std::integral_constant<int, FB>{}, I3{});
                        if (j == 2) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 5>{});
                        if (j == 3) load_b(std::integral_constant<int, FB>{}, std::integral_constant<int, 7>{});
                    }
                    if (q == S - 1) {
                        if (j + 1 < KSTEPS)
                            bp += rs1;
                        else
                            next_stage_rows(SP ^ 1);  // stage s + 3 has the other parity
                    }
                }
                // the index buffer is free once its reads (step 0) have returned; refill it in
                // step 3 with the super-stage after next
                if (do_idx && j == 3) {
                    if constexpr (TM == 1) {
                        if (q == 3) load_idx(I0{});
                    } else {
                        if (q == 4) load_idx(I0{});
                        if (q == 6) load_idx(I1{});
                    }
                    if constexpr (TM == 3) {
                        if (q == 8) load_idx(I2{});
                    }
                    if constexpr (TM == 4) {
                        if (q == (TN == 4 ? 12 : 8)) load_idx(I2{});
                        if (q == (TN == 4 ? 14 : 10)) load_idx(I3{});
                    }
                    if (q == S - 1) ip += 32;
                }
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
        if constexpr (SPLIT)
            mfma_atomic_add_tile<TM, TN>(acc, M, N, ct_m0 + w * WAVE_ROWS, ct_n0, reinterpret_cast<int32_t*>(Y), ldy);
        else
            mfma_store_tile<TM, STREAM, TN>(acc, sc, bias, M, N, ct_m0 + w * WAVE_ROWS, ct_n0, Y, ldy);
        if (!has_next) break;
        // next tile: its first stages and index words are already in LDS / registers
#pragma unroll
        for (int i = 0; i < TM; ++i)
#pragma unroll
            for (int j = 0; j < TN; ++j)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[i][j][r] = 0;
        t += wg_per_xcd;
        ct_n0 = ft_n0;
        ct_m0 = ft_m0;
        has_next = t + wg_per_xcd < xcd_end;
    }
}

// Y[n][m] = 0 as int32 / Y[n][m] = fma((float)int32, s, bias[m]) in place, over the N x M region of a
// matrix with row stride ldy: the two passes around a codebook-split contraction.
// grid: (blocks of 256 columns, rows).
__global__ __launch_bounds__(256) void zero_rows_kernel(float* __restrict__ Y, int M, int64_t ldy) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m < M) Y[(int64_t)blockIdx.y * ldy + m] = 0.f;
}
__global__ __launch_bounds__(256) void dequant_rows_kernel(float* __restrict__ Y, int M, int64_t ldy,
                                                           const float* __restrict__ scale,
                                                           const float* __restrict__ bias) {
    const int m = blockIdx.x * 256 + threadIdx.x;
    if (m >= M) return;
    float* y = Y + (int64_t)blockIdx.y * ldy + m;
    const float a = (float)__float_as_int(*y);
    *y = bias ? __fmaf_rn(a, *scale, bias[m]) : __fmul_rn(a, *scale);
}

template <int TM, int TN = 4>
hipError_t launch_tm(const int8_t* packed, const float* scale, const float* bias, int C, int M,
                     const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s) {
    constexpr int BM = 128 * TM, BN = 32 * TN;
    const int Mp = (int)packed_cols(M);
    const int64_t col_tiles = (M + BN - 1) / BN;  // the packed table is padded to 256 columns
    if (col_tiles * BN > Mp) return hipErrorInvalidValue;  // 96-column tiles past the padding
    const int64_t row_tiles = (N + BM - 1) / BM;
    const int64_t tiles = row_tiles * col_tiles;
    int64_t blocks = (tiles + 7) / 8 * 8;
    if (blocks > 0x7fffffffLL || row_tiles > 0x7fffffffLL) return hipErrorInvalidValue;
    if ((int64_t)Mp * 16 * 21 > 0xffffffffLL) return hipErrorInvalidValue;  // row strides are 32-bit
    // Few tiles and many codebooks (a small batch on a wide layer): every workgroup would stream
    // 2 KiB x C of table alone while most of the chip idles.  Split the codebooks over `splits`
    // workgroups per tile instead; their int32 partial sums meet in Y through atomics, between a
    // pass that zeroes Y and one that dequantises it.  What it saves is the serial walk over the
    // codebooks, ~24 ns per codebook and workgroup, times (1 - 1/splits); what it costs is two more
    // launches (~6 us) and the atomics and passes over Y, ~14 us per million outputs (fitted to
    // sweeps over 129-4096 rows at (C, M) = (1536, 768), (1024, 4096), (512, 1024): e.g. 0.022
    // against 0.042 ms at 512 rows of the first, break-even at 2048 rows; break-even at 256 rows of
    // the second).  Each share keeps at least 64 codebooks.  LUTNN_SMFMAC_SPLIT = 0 | 1 pins the
    // decision (sweeps, and tests that must reach both paths).
    const int kComputeUnits = compute_units();
    if (TN == 4 && tiles <= kComputeUnits / 2 && C >= 512) {
        const int supers = C / 32;
        int splits = 1;
        for (int cand = (int)std::min<int64_t>(16, kComputeUnits / tiles); cand > 1; --cand)
            if (supers % cand == 0 && supers / cand >= 2) {
                splits = cand;
                break;
            }
        const double saved_us = 0.024 * C * (1.0 - 1.0 / splits);
        const double cost_us = 6.0 + 14e-6 * (double)N * M;
        bool split = saved_us > cost_us;
        if (const int pinned = tunable(kTuneSmfmacSplit); pinned >= 0) split = pinned == 1;
        if (!split) splits = 1;
        if (splits > 1) {
            const dim3 cells((unsigned)((M + 255) / 256), (unsigned)N);
            hipLaunchKernelGGL(zero_rows_kernel, cells, dim3(256), 0, s, Y, M, ldy);
            const int64_t units = tiles * splits;
            hipLaunchKernelGGL((lookup_smfmac_i8_kernel<TM, 4, true>), dim3((unsigned)((units + 7) / 8 * 8)),
                               dim3(kMfmaThreads), 0, s, reinterpret_cast<const uint4*>(packed), scale, bias, C, M,
                               Mp, idx, N, Y, ldy, (int)row_tiles, units, splits, 0);
            hipLaunchKernelGGL(dequant_rows_kernel, cells, dim3(256), 0, s, Y, M, ldy, scale, bias);
            return hipGetLastError();
        }
    }
    // Tile order.  The 32 workgroups of an XCD that run at the same time read R row tiles' index
    // bytes (128*TM*C each) and Q column blocks' table slabs (2048*C each), R*Q = 32: plain
    // column-block-major order is R = 32, Q = 1 (config 5: 18 MiB per round and XCD, the whole index
    // matrix once per column block); groups of 16 row tiles give R = 16, Q = 2 (12 MiB).  Measured on
    // config 5 (rocprofv3 FETCH_SIZE): 605 -> 404 MB fetched per launch, time unchanged (the re-reads
    // come from the Infinity Cache either way).  Only worth it when a launch has several rounds of
    // tiles; LUTNN_SMFMAC_ROW_GROUP pins the group size (0 = plain).
    int row_group = tiles >= 4 * (int64_t)kComputeUnits && row_tiles >= 16 ? 16 : 0;
    if (const int pinned = tunable(kTuneSmfmacRowGroup); pinned >= 0) row_group = pinned;
    // Stream several tiles per workgroup when the ring phase carries over from tile to tile:
    // one workgroup per compute unit (the kernel's LDS footprint allows only one anyway).
    if (C % 64 == 0 && blocks > kComputeUnits) blocks = kComputeUnits;
    // an output of 128 MiB or more cannot stay in any cache: stream it (512-row tiles only, the
    // height such problems take)
    if (TM == 4 && TN == 4 && (double)N * M * 4 >= 134217728.0)
        hipLaunchKernelGGL((lookup_smfmac_i8_kernel<TM, 4, false, TM == 4>), dim3((unsigned)blocks),
                           dim3(kMfmaThreads), 0, s, reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp,
                           idx, N, Y, ldy, (int)row_tiles, tiles, 1, row_group);
    else
        hipLaunchKernelGGL((lookup_smfmac_i8_kernel<TM, TN, false>), dim3((unsigned)blocks), dim3(kMfmaThreads), 0, s,
                           reinterpret_cast<const uint4*>(packed), scale, bias, C, M, Mp, idx, N, Y, ldy,
                           (int)row_tiles, tiles, 1, row_group);
    return hipGetLastError();
}

}  // namespace

bool smfmac_supported(int C, int K, const uint8_t* idx) {
    return K <= 16 && C % 32 == 0 && (reinterpret_cast<uintptr_t>(idx) & 15) == 0;
}

hipError_t launch_lookup_smfmac_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                   int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                   hipStream_t s) {
    if (!smfmac_supported(C, K, idx)) return hipErrorInvalidValue;
    // Tile height.  512 rows amortise the table slab best, but the tiles have to cover the chip:
    // price each height as (rounds of 256 workgroups) x (measured time of one tile relative to
    // the 512-row tile: 0.8 for 384 rows, 0.56 for 256, 0.42 for 128 - the slab traffic does not
    // shrink).
    const int kComputeUnits = compute_units();
    auto cost = [&](int64_t bm, double rel, int bn = 128) {
        const int64_t tiles = ((N + bm - 1) / bm) * ((M + bn - 1) / bn);
        return (double)((tiles + kComputeUnits - 1) / kComputeUnits) * rel;
    };
    // 512 x 96 tiles where the padded table covers them.  Same outputs and matrix instructions as
    // a 384 x 128 tile, but a quarter less of the table to copy and to read per stage: priced 0.75
    // (measured at 4096 rows, 384 codebooks: M = 2304 0.0342 ms against 0.0378 with 384-row and 0.0384
    // with 512 x 128 tiles; M = 3072 0.0405 against 0.0423; at 8192 and 12288 rows of M = 3072 3-10 %
    // ahead; at 16384 rows, where it needs a fourth round, 4 % behind - which the price reproduces).
    // LUTNN_SMFMAC_TILE_COLS = 96 | 128 pins the width of 512-row tiles.
    constexpr double kNarrowRel = 0.75;
    const bool narrow_fits = (int64_t)(M + 95) / 96 * 96 <= (int64_t)packed_cols(M);
    const int pinned_cols = tunable(kTuneSmfmacTileCols);
    // LUTNN_SMFMAC_TILE_ROWS = 128 | 256 | 384 | 512 pins the height (tuning sweeps, and tests that
    // must reach every instance whatever the prices below say); anything else is ignored.
    switch (tunable(kTuneSmfmacTileRows)) {
        case 512:
            if (pinned_cols == 96 && narrow_fits) return launch_tm<4, 3>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
            return launch_tm<4>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
        case 384: return launch_tm<3>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
        case 256: return launch_tm<2>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
        case 128: return launch_tm<1>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
        default: break;
    }
    const double c4 = cost(512, 1.0), c3 = cost(384, 0.8), c2 = cost(256, 0.56), c1 = cost(128, 0.42);
    const double best = std::min(std::min(c4, c3), std::min(c2, c1));
    if (narrow_fits && pinned_cols != 128 && (cost(512, kNarrowRel, 96) < best || (pinned_cols == 96 && c4 == best)))
        return launch_tm<4, 3>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
    if (c4 == best) return launch_tm<4>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
    if (c3 == best) return launch_tm<3>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
    if (c2 == best) return launch_tm<2>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
    return launch_tm<1>(packed, scale, bias, C, M, idx, N, Y, ldy, s);
}

}  // namespace lutnn
