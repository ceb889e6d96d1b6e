// Internal launcher declarations shared by the host dispatch (api.hip) and the kernel files.
// Every launcher assumes its arguments were validated by the caller in api.hip and returns the
// hipError_t of the launch.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace lutnn {

// Column padding of the MFMA operand copy of an INT8 table: [C*Kb][Mp][16], Mp = roundup(M, this).
constexpr int kPackedColPad = 256;

inline int64_t packed_cols(int64_t M) { return (M + kPackedColPad - 1) / kPackedColPad * kPackedColPad; }
inline int kblocks(int K) { return (K + 15) / 16; }

// Tuning switches that pin a launcher's choice (sweeps, and tests that must reach every kernel
// instance).  Each starts from the environment variable of the same name, read once when the first
// switch is asked for, and can be changed through lutnn_set_tunable; -1 = not pinned.  Atomic.
enum Tunable {
    kTuneFusedKernel = 0,   // LUTNN_FUSED_KERNEL: 0 = "tile", 1 = "small"
    kTuneSmfmacSplit,       // LUTNN_SMFMAC_SPLIT: 0 | 1
    kTuneSmfmacTileRows,    // LUTNN_SMFMAC_TILE_ROWS: 128 | 256 | 384 | 512
    kTuneSmfmacRowGroup,    // LUTNN_SMFMAC_ROW_GROUP: row tiles per group of the tile order, 0..64 (0 = plain)
    kTuneSmfmacTileCols,    // LUTNN_SMFMAC_TILE_COLS: 96 | 128, width of the 512-row tiles
    kTuneCount
};
int tunable(int which);

// Compute units of the current device (queried once per device; 256 on an MI355X).
int compute_units();

// A convolution seen as a matrix product (Sec. 4): row n = (image b, output pixel ho, wo),
// column j = (input channel ci, filter row r, filter column s) with ci slowest, element
// input[b][ci][ho*sh + r - ph][wo*sw + s - pw] or 0 outside the image.
struct ConvGeom {
    int Cin, H, W, kh, kw, sh, sw, ph, pw, Ho, Wo;
};

// Eq. 2 on the rows of that matrix, read from the NCHW input without materialising it.
bool encode_conv_supported(int V);
hipError_t launch_encode_conv(const float* P, int C, int K, int V, const float* input, int64_t B,
                              const ConvGeom& g, uint8_t* idx, hipStream_t s);

// Eq. 2.
hipError_t launch_encode(const float* P, int C, int K, int V, const float* X, int64_t N, int64_t ldx,
                         uint8_t* idx, hipStream_t s);

// Hash encoding (Sec. 2, Sec. 7): per codebook a heap-ordered threshold tree with `levels` levels.
hipError_t launch_encode_tree(const int32_t* split_dim, const float* threshold, int C, int levels,
                              int V, const float* X, int64_t N, int64_t ldx, uint8_t* idx,
                              hipStream_t s);

// The same with 16-bit leaves, for trees of up to 12 levels (Sec. 7), and Eq. 4 on 16-bit indices
// (K up to 4096 table rows per codebook, read straight from global memory).
hipError_t launch_encode_tree16(const int32_t* split_dim, const float* threshold, int C, int levels,
                                int V, const float* X, int64_t N, int64_t ldx, uint16_t* idx,
                                hipStream_t s);
hipError_t launch_lookup_wide_i8(const int8_t* T, const float* scale, const float* bias, int C, int K, int M,
                                 const uint16_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s);
hipError_t launch_lookup_wide_f32(const float* T, const float* bias, int C, int K, int M, const uint16_t* idx,
                                  int64_t N, float* Y, int64_t ldy, hipStream_t s);

// Soft-PQ backward (Sec. 3.1-3.2, Eq. 5-6): gradients with respect to the centroids, the layer
// input and the temperature, from Z = dL/dY . W^T.  workspace: softpq_workspace_bytes() bytes.
bool softpq_supported(int K, int V);
size_t softpq_workspace_bytes(int C, int K, int V, int64_t N);
hipError_t launch_softpq_backward(const float* P, int C, int K, int V, float t, const float* X, int64_t N,
                                  int64_t ldx, const float* Z, int64_t ldz, float* dP, float* dX,
                                  int64_t lddx, float* dt, float* workspace, hipStream_t s);

hipError_t launch_encode_tree_conv(const int32_t* split_dim, const float* threshold, int C, int levels,
                                   int V, const float* input, int64_t B, const ConvGeom& g, uint8_t* idx,
                                   hipStream_t s);

// Eq. 3 + Sec. 3.3.
hipError_t launch_build_table_f32(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                  int M, float* T, hipStream_t s);
// bits = 8: T is [C][K][M] int8; bits = 4: T is [C][K][ceil(M/2)] bytes of two nibbles.  The packed
// MFMA operand copy holds one int8 per entry in both cases.
hipError_t launch_build_table_i8(const float* P, const float* W, int64_t ldw, int C, int K, int V,
                                 int M, int8_t* T, int8_t* packed, float* scale, int bits,
                                 hipStream_t s);

// Eq. 4, gather variant.
hipError_t launch_lookup_lds_i8(const int8_t* T, const float* scale, const float* bias, int C, int K,
                                int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                hipStream_t s);
hipError_t launch_lookup_lds_f32(const float* T, const float* bias, int C, int K, int M,
                                 const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s);

hipError_t launch_lookup_lds_i4(const uint8_t* T, const float* scale, const float* bias, int C, int K,
                                int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                hipStream_t s);
// Eq. 4, gather variant with lane = row (256 rows per workgroup share the staged slabs): the shape
// for many rows.  bits = 8: T is [C][K][M] int8; bits = 4: [C][K][ceil(M/2)] nibble pairs.
bool rows_kernel_preferred(int64_t N, int M, int K, bool f32);
hipError_t launch_lookup_rows_i8(const void* T, int bits, const float* scale, const float* bias, int C,
                                 int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                 hipStream_t s);
hipError_t launch_lookup_rows_f32(const float* T, const float* bias, int C, int K, int M,
                                  const uint8_t* idx, int64_t N, float* Y, int64_t ldy, hipStream_t s);

// table_kind: 0 fp32, 1 int8, 2 int4 (nibble pairs)
bool gather_preferred(const void* T, int table_kind, int C, int M, int64_t N, bool sparse_ok);

// Eq. 4, one-hot MFMA variant (INT8).
hipError_t launch_lookup_mfma_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                 int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                 hipStream_t s);

// Eq. 4, one-hot contraction on the 2:4 structured-sparse matrix instructions (INT8).
bool smfmac_supported(int C, int K, const uint8_t* idx);
hipError_t launch_lookup_smfmac_i8(const int8_t* packed, const float* scale, const float* bias, int C,
                                   int K, int M, const uint8_t* idx, int64_t N, float* Y, int64_t ldy,
                                   hipStream_t s);

// Eq. 2 + Eq. 4 in one kernel.
bool fused_supported(int C, int K, int V, int M, int dtype);
hipError_t launch_linear_fused_i8(const float* P, const int8_t* packed, const float* scale,
                                  const float* bias, int C, int K, int V, int M, const float* X,
                                  int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s);
hipError_t launch_linear_fused_f32(const float* P, const float* T, const float* bias, int C, int K,
                                   int V, int M, const float* X, int64_t N, int64_t ldx, float* Y,
                                   int64_t ldy, hipStream_t s);

// Eq. 2 + Eq. 4 in one launch for small problems, reading the plain table (table_kind 0 fp32, 1 int8).
bool linear_small_supported(const void* T, int table_kind, int C, int K, int V, int M);
bool linear_small_preferred(const void* T, int table_kind, int C, int K, int V, int M, int64_t N,
                            bool gather_wins);
hipError_t launch_linear_small_f32(const float* P, const float* T, const float* bias, int C, int K, int V,
                                   int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                                   hipStream_t s);
hipError_t launch_linear_small_i8(const float* P, const int8_t* T, const float* scale, const float* bias, int C,
                                  int K, int V, int M, const float* X, int64_t N, int64_t ldx, float* Y,
                                  int64_t ldy, hipStream_t s);
// ... and with the hash encoder (Sec. 2) as step 1: the trees' K = 2^levels.
hipError_t launch_linear_small_tree_f32(const int32_t* split_dim, const float* threshold, int levels,
                                        const float* T, const float* bias, int C, int V, int M, const float* X,
                                        int64_t N, int64_t ldx, float* Y, int64_t ldy, hipStream_t s);
hipError_t launch_linear_small_tree_i8(const int32_t* split_dim, const float* threshold, int levels,
                                       const int8_t* T, const float* scale, const float* bias, int C, int V,
                                       int M, const float* X, int64_t N, int64_t ldx, float* Y, int64_t ldy,
                                       hipStream_t s);

// probe_smfmac.hip: sink holds 256 * compute_units() ints
hipError_t launch_probe_smfmac_stream(int operands, int iterations, int32_t* sink, hipStream_t s);

}  // namespace lutnn
