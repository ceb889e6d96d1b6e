/*
 * liblutnn — LUT-NN table-lookup linear operator for AMD MI355X (gfx950).
 *
 * C ABI of the inference hot path of LUT-NN (arXiv 2302.03213): a linear operator
 * Y = A x B (an FC layer or an im2col'd convolution, Sec. 4) evaluated by
 *   1. encoding: every row of A is split into C sub-vectors of length V (Sec. 2.1) and
 *      each sub-vector is replaced by the index of its nearest of K centroids (Eq. 2);
 *   2. lookup + aggregation: Y[n][m] = sum_c T[c][idx[n][c]][m] (Eq. 4), where the table
 *      T[c][k][m] = P[c][k] . B[cV:(c+1)V][m] is precomputed (Eq. 3) and optionally
 *      quantised to INT8 or INT4 with one symmetric scale (Sec. 3.3).
 * Around it: the same two steps for a convolution read from its NCHW batch (lutnn_conv2d), the
 * hash (threshold tree) encoder the paper discusses as the alternative to step 1 (lutnn_encode_tree,
 * Sec. 2 and Sec. 7), and the backward pass of soft-PQ training (lutnn_softpq_backward, Sec. 3).
 *
 * Conventions common to every call
 *   - Pointers are DEVICE pointers unless a parameter is marked "host".  The caller owns
 *     every buffer; the library allocates nothing and keeps no reference after the
 *     call returns.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work on that stream; they never synchronise.
 *   - Matrices are row-major with a row stride in ELEMENTS (ldx, ldy, ldw).
 *   - Every call validates its arguments on the host before launching anything and
 *     returns a lutnn_status; on failure nothing has been enqueued and
 *     lutnn_last_error() describes the reason.  No exception crosses this boundary.
 *   - N == 0 is valid: once the layer descriptor has been validated the call returns LUTNN_OK
 *     without looking at the data pointers (an empty batch may have none) or enqueuing anything
 *     (lutnn_softpq_backward still writes its zero sums).
 *   - Inputs are assumed finite.  Non-finite activations never cause an out-of-range
 *     index or an out-of-bounds access; the index chosen for them is unspecified.
 *   - Outputs must not alias inputs.  Some lookups use Y itself as integer scratch before the final
 *     values are written, so Y must not be read by anyone else while a call on it is in flight.
 *   - The library keeps no state between calls (the last-error text is per host thread): calls from
 *     several host threads and on several streams may run concurrently.  The one exception is
 *     lutnn_softpq_backward_static, whose calls share a static scratch array per GPU.
 */
#ifndef LUTNN_H
#define LUTNN_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define LUTNN_API __attribute__((visibility("default")))

typedef enum {
    LUTNN_OK = 0,
    LUTNN_E_NULL = 1,        /* a required pointer is NULL                                   */
    LUTNN_E_SHAPE = 2,       /* a dimension is non-positive, K > 256, or a stride is too small */
    LUTNN_E_UNSUPPORTED = 3, /* no kernel for this (dtype, variant, K) combination           */
    LUTNN_E_ALIGN = 4,       /* a pointer is not aligned as documented                       */
    LUTNN_E_HIP = 5          /* the HIP runtime reported an error on launch                  */
} lutnn_status;

typedef enum {
    LUTNN_TABLE_F32 = 0, /* T[C][K][M] fp32                                   */
    LUTNN_TABLE_I8 = 1,  /* T[C][K][M] int8 + one fp32 scale (Sec. 3.3, n = 8) */
    LUTNN_TABLE_I4 = 2   /* T[C][K][ceil(M/2)] bytes, two 4-bit two's-complement entries per
                            byte, even column in the low nibble, + one fp32 scale (Sec. 3.3 with
                            n = 4: the INT4 table of Sec. 6.4)                        */
} lutnn_table_dtype;

typedef enum {
    LUTNN_VARIANT_AUTO = 0,  /* the library picks                                                  */
    LUTNN_VARIANT_LDS = 1,   /* table tiles staged in LDS, gathered by index, register accumulate   */
    LUTNN_VARIANT_MFMA = 2,  /* Eq. 4 as a dense onehot[N x CK] x T[CK x M] int8 MFMA contraction   */
    LUTNN_VARIANT_FUSED = 3, /* lutnn_linear only: one kernel, indices never leave the chip          */
    LUTNN_VARIANT_SMFMAC = 4 /* as MFMA, on the 2:4 structured-sparse matrix instructions: a one-hot
                                slice is 2:4 sparse by construction, so the result is identical at
                                twice the matrix rate.  Needs C % 32 == 0, 16-byte aligned idx.
                                The rows per workgroup tile and whether a tile's codebooks are
                                shared out over several workgroups are priced by the library;
                                lutnn_set_tunable pins either (results are the same)                */
} lutnn_variant;

/*
 * One LUT layer.  Plain data filled by the caller (host struct holding device pointers);
 * the library only reads it during the call.
 */
typedef struct {
    int32_t C;               /* number of codebooks (sub-vectors per row), D = C * V           */
    int32_t K;               /* centroids per codebook, 1..256 (..4096 for the 16-bit index calls) */
    int32_t V;               /* sub-vector length                                              */
    int32_t M;               /* output width                                                   */
    int32_t table_dtype;     /* lutnn_table_dtype                                              */
    int32_t reserved;        /* must be 0                                                      */
    const float* centroids;  /* P[C][K][V] fp32 (needed by encode / linear)                    */
    const void* table;       /* T[C][K][M], m fastest, in the layout of table_dtype (needed by the
                                LDS variant)                                                   */
    const void* table_packed;/* INT8 / INT4: MFMA operand layout (one int8 per entry for both)
                                written by lutnn_build_table, lutnn_packed_bytes() bytes,
                                16-byte aligned; NULL if absent                                */
    const float* scale;      /* INT8 / INT4: device pointer to the layer's single fp32 scale    */
    const float* bias;       /* [M] fp32 or NULL                                               */
} lutnn_layer;

/* Size in bytes of T[C][K][M] for `dtype`.  Host; returns 0 on invalid arguments. */
LUTNN_API size_t lutnn_table_bytes(int32_t C, int32_t K, int32_t M, int32_t dtype);

/*
 * Size in bytes of the MFMA operand copy of an INT8 or INT4 table (padded; see
 * lutnn_build_table).  Host; returns 0 for fp32 tables or invalid arguments.
 */
LUTNN_API size_t lutnn_packed_bytes(int32_t C, int32_t K, int32_t M, int32_t dtype);

/*
 * Offline table construction (Eq. 3) and, for INT8, symmetric scalar quantisation
 * (Sec. 3.3).  Not part of the timed path.
 *
 *   centroids  P[C][K][V] fp32
 *   W          B[D][M] fp32 row-major (Table 1), row stride ldw >= M, D = C*V
 *   table_out  T[C][K][M]: fp32 entries  T = sum_v P[c][k][v] * W[cV+v][m]  (fp32, v
 *              ascending, fused multiply-add), or for INT8
 *              q = clamp(round_half_even(T / s), -127, 127) with
 *              s = max|T| / 127 over the whole layer (s = 1 when the table is all zero);
 *              for INT4 the same with 7 in place of 127, two entries per byte
 *   packed_out INT8 / INT4, nullable: the same q re-laid out for the MFMA variants, one int8 per
 *              entry for both dtypes:
 *              [C * ceil(K/16)][Mp][16] int8 with Mp = M rounded up to 256, k fastest,
 *              zero padded.  Must be 16-byte aligned.  K <= 256 only.
 *   scale_out  INT8 / INT4: receives s (one fp32).  Also used as scratch during the call.
 * K up to 4096 (the tables behind lutnn_lookup16) with packed_out = NULL.
 *
 * Errors: E_NULL, E_SHAPE, E_UNSUPPORTED (unknown dtype; packed_out with K > 256), E_ALIGN, E_HIP.
 */
LUTNN_API lutnn_status lutnn_build_table(const float* centroids, const float* W, int64_t ldw,
                                         int32_t C, int32_t K, int32_t V, int32_t M,
                                         int32_t dtype, void* table_out, void* packed_out,
                                         float* scale_out, void* stream);

/*
 * Encoding (Eq. 2; "closest centroid search", Sec. 5.1):
 *   idx[n][c] = argmin_k sum_v (X[n][cV+v] - P[c][k][v])^2
 * evaluated in fp32 in exactly this form (v ascending, one fused multiply-add per term);
 * the lowest k wins ties.
 *
 *   X    [N][D] fp32, row stride ldx >= D = C*V
 *   idx  [N][C] uint8, dense
 * Uses layer->centroids, C, K, V.  Errors: E_NULL, E_SHAPE, E_HIP.
 */
LUTNN_API lutnn_status lutnn_encode(const lutnn_layer* layer, const float* X, int64_t N,
                                    int64_t ldx, uint8_t* idx, void* stream);

/*
 * Lookup + aggregation (Eq. 4; "table read and accumulation", Sec. 5.2):
 *   INT8 / INT4: acc = sum_c (int32) q[c][idx[n][c]][m]  (exact),
 *                Y[n][m] = fma((float)acc, s, bias[m])   (or (float)acc * s without bias)
 *   fp32 table:  Y[n][m] = sum_c T[c][idx[n][c]][m] (+ bias[m]), fp32 accumulation
 *
 *   idx  [N][C] uint8, dense; every value must be < K (larger values never cause an
 *        out-of-bounds access but give an unspecified result)
 *   Y    [N][M] fp32, row stride ldy >= M
 *   variant  AUTO, LDS (needs layer->table), MFMA or SMFMAC (INT8 only, K <= 16, need
 *            layer->table_packed; SMFMAC also needs C % 32 == 0 and idx 16-byte aligned).
 * Errors: E_NULL, E_SHAPE, E_UNSUPPORTED, E_ALIGN, E_HIP.
 */
LUTNN_API lutnn_status lutnn_lookup(const lutnn_layer* layer, const uint8_t* idx, int64_t N,
                                    float* Y, int64_t ldy, int32_t variant, void* stream);

/*
 * The whole operator: encode then lookup, Y ~= X . B (+ bias).
 *
 *   variant FUSED  one kernel; the indices stay in LDS.  `idx_workspace` is ignored.  Two forms.
 *                  The one-launch kernel for small problems (fp32 / INT8 table in its plain layout,
 *                  M % 4 == 0) is the form that pays: at on-device batch sizes it beats the two
 *                  launches, and AUTO takes it there.  The tile kernel on the matrix cores (INT8:
 *                  needs table_packed) is strictly the fallback for callers that have no index
 *                  workspace on shapes the one-launch kernel does not take: it re-encodes a row
 *                  block per column split and re-streams the table per row block, and is several
 *                  times slower than encode + lookup on every shape measured - give a workspace
 *                  whenever you can.  lutnn_set_tunable("LUTNN_FUSED_KERNEL", ...) pins the form.
 *   variant LDS / MFMA / SMFMAC  lutnn_encode into idx_workspace, then lutnn_lookup with that
 *                  variant.
 *   variant AUTO   the one-launch kernel where the problem is so small that a second launch would
 *                  be most of the time; else, with a workspace: lutnn_encode, then lutnn_lookup
 *                  with AUTO (the fastest lookup for the shape); without one: FUSED, if a fused
 *                  kernel exists.  lutnn_linear_auto_variant reports the choice.
 *   idx_workspace  [N][C] uint8 device scratch (contents unspecified afterwards); may be NULL
 *                  only for FUSED / AUTO.
 * Errors: as lutnn_encode and lutnn_lookup.
 */
LUTNN_API lutnn_status lutnn_linear(const lutnn_layer* layer, const float* X, int64_t N,
                                    int64_t ldx, float* Y, int64_t ldy, int32_t variant,
                                    uint8_t* idx_workspace, void* stream);

/*
 * Hash encoding (Sec. 2, "Hashing for acceleration"; the alternative to Eq. 2 evaluated in Sec. 7):
 * each codebook owns a balanced binary tree with `levels` levels whose K = 2^levels leaves are the
 * buckets.  A sub-vector starts at the root and at every node compares one of its V values, the
 * node's split index, with the node's threshold:
 *   node <- 2*node + 1 + (x[split_dim[c][node]] > threshold[c][node])   (root 0; a value equal to
 *                                                   the threshold, and a NaN, go to the left child)
 *   idx[n][c] = node - (2^levels - 1) after `levels` steps: the leaf reached, counted from the left.
 * The descriptor lives in host memory, the arrays it points to in device memory, owned by the
 * caller.  The trees come from training, like the centroids; the library does not learn them.
 */
typedef struct {
    int32_t C;       /* codebooks                                                             */
    int32_t V;       /* sub-vector length; D = C*V                                            */
    int32_t levels;  /* 1..8 (..12 for the 16-bit index calls); K = 2^levels buckets           */
    int32_t reserved; /* must be 0                                                            */
    const int32_t* split_dim; /* device, [C][2^levels - 1] heap order; values outside [0, V)
                                 are clamped into it                                          */
    const float* threshold;   /* device, [C][2^levels - 1] fp32                               */
} lutnn_tree;

/*
 *   X    [N][D] fp32, row stride ldx >= D = C*V
 *   idx  [N][C] uint8, dense; usable by lutnn_lookup with a table of K = 2^levels rows
 * Errors: E_NULL, E_SHAPE (C, V < 1, levels outside 1..8, reserved != 0, ldx < D), E_HIP.
 */
LUTNN_API lutnn_status lutnn_encode_tree(const lutnn_tree* tree, const float* X, int64_t N,
                                         int64_t ldx, uint8_t* idx, void* stream);

/*
 * The whole operator with the hash encoder in front: lutnn_encode_tree into idx_workspace, then
 * lutnn_lookup(layer, idx_workspace, ..., variant).  layer->C and V must equal the tree's and
 * layer->K must be 2^levels; layer->centroids is not used (the table rows are the buckets'
 * prototypes times the weights, built by lutnn_build_table from whatever prototypes training
 * assigned to the buckets).
 *   idx_workspace  [N][C] uint8 device scratch; required unless the one-launch kernel runs
 *   variant        AUTO, LDS, MFMA, SMFMAC, or FUSED = the one-launch kernel of lutnn_linear with the
 *                  tree walk as its first step (fp32 or INT8 table in the plain layout, M % 4 == 0,
 *                  V in {1,2,3,4,8,9,16,32}; E_UNSUPPORTED otherwise).  AUTO takes that kernel on
 *                  the shapes where lutnn_linear's AUTO does (lutnn_linear_auto_variant), else
 *                  the two launches; the indices, and with an INT8 table the outputs, are the
 *                  same either way.
 * Errors: as lutnn_encode_tree and lutnn_lookup; E_SHAPE when tree and layer disagree.
 */
LUTNN_API lutnn_status lutnn_linear_tree(const lutnn_layer* layer, const lutnn_tree* tree,
                                         const float* X, int64_t N, int64_t ldx, float* Y,
                                         int64_t ldy, int32_t variant, uint8_t* idx_workspace,
                                         void* stream);

/*
 * The hash encoder with deep trees (Sec. 7 evaluates a 12-level tree: 4096 buckets per codebook)
 * and the lookup behind it, with 16-bit indices.  Same definitions as lutnn_encode_tree,
 * lutnn_lookup and lutnn_linear_tree; what changes is the index width and the limits:
 *   tree->levels  1 .. 12                      layer->K  up to 4096 (= 2^levels for lutnn_linear_tree16)
 *   idx / idx_workspace  [N][C] uint16, dense, 2-byte aligned; values >= K are treated as K - 1
 *   tables        LUTNN_TABLE_I8 or LUTNN_TABLE_F32, layout [C][K][M] as always (INT4: E_UNSUPPORTED);
 *                 lutnn_build_table builds them for K up to 4096 when packed_out is NULL
 * The lookup reads the selected table rows straight from global memory (nothing of a table with
 * thousands of rows per codebook can be staged), codebooks in ascending order: bit-exact int32 sums
 * for INT8, a fixed fp32 summation order for fp32 tables.  There is no variant argument.
 * Up to 8 levels the 8-bit entry points are the faster ones.
 * Errors: as their 8-bit counterparts.
 */
LUTNN_API lutnn_status lutnn_encode_tree16(const lutnn_tree* tree, const float* X, int64_t N,
                                           int64_t ldx, uint16_t* idx, void* stream);
LUTNN_API lutnn_status lutnn_lookup16(const lutnn_layer* layer, const uint16_t* idx, int64_t N,
                                      float* Y, int64_t ldy, void* stream);
LUTNN_API lutnn_status lutnn_linear_tree16(const lutnn_layer* layer, const lutnn_tree* tree,
                                           const float* X, int64_t N, int64_t ldx, float* Y,
                                           int64_t ldy, uint16_t* idx_workspace, void* stream);

/*
 * Soft-PQ backward pass (Sec. 3.1 "Backpropagation through soft-PQ", Eq. 5-6; Sec. 3.2 "Learned
 * temperature").  In training the layer's VALUE is the hard output that lutnn_linear computes, and
 * its GRADIENT is that of the soft output
 *   Ysoft[n][m] = sum_c sum_k s[n][c][k] * T[c][k][m],   s[n][c][:] = softmax_k(-||x_n^c - P^c_k||^2 / t),
 * with the real-valued table T = P . W of Eq. 3 (Sec. 3.3: the backward pass does not quantise).
 * The weights W stay fixed (the tables are rebuilt from the updated centroids), so everything
 * follows from  Z = dL/dY . W^T, the input gradient of the ordinary linear layer with the same
 * weights, which the caller computes with any GEMM:
 *   dP[c][k][v] = dL/dP       gradient for the centroids
 *   dX[n][cV+v] = dL/dX       gradient for the layer input (earlier layers need it)
 *   dt          = dL/dt       gradient for the layer's temperature
 * All arithmetic is fp32; sums over rows are taken in a fixed order (reproducible run to run).
 *
 *   temperature  t > 0
 *   X   [N][D] fp32, row stride ldx >= D = C*V            (the forward pass's input)
 *   Z   [N][D] fp32, row stride ldz >= D
 *   dP  [C][K][V] fp32, overwritten
 *   dX  [N][D] fp32, row stride lddx >= D, overwritten; NULL to skip it
 *   dt  one fp32, overwritten; NULL to skip it
 *   workspace  device scratch of at least lutnn_softpq_workspace_bytes(C, K, V, N) bytes, 4-byte
 *              aligned; contents unspecified afterwards
 * Uses layer->centroids, C, K, V.  Supported: K = 8 or 16 with V in {1,2,3,4,8,9,16,32} (the
 * paper's settings); anything else is E_UNSUPPORTED.
 * Errors: E_NULL, E_SHAPE (also t <= 0, workspace too small), E_UNSUPPORTED, E_ALIGN, E_HIP.
 */
LUTNN_API lutnn_status lutnn_softpq_backward(const lutnn_layer* layer, float temperature,
                                             const float* X, int64_t N, int64_t ldx, const float* Z,
                                             int64_t ldz, float* dP, float* dX, int64_t lddx,
                                             float* dt, void* workspace, size_t workspace_bytes,
                                             void* stream);

/* Host: bytes of workspace lutnn_softpq_backward needs; 0 for unsupported (K, V) or empty shapes. */
LUTNN_API size_t lutnn_softpq_workspace_bytes(int32_t C, int32_t K, int32_t V, int64_t N);

/*
 * lutnn_softpq_backward for callers that cannot allocate device memory and have no workspace to
 * pass: code under HIP graph capture, tight serving or training loops, harnesses that forbid
 * hipMalloc.  Same arguments without the workspace, same kernels, same results bit for bit; the
 * scratch is a static device array of LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES inside the library (one copy
 * on every GPU that loads the library, held until the process ends).  The call allocates nothing
 * and frees nothing.
 *   - A shape whose lutnn_softpq_workspace_bytes(C, K, V, N) exceeds the array is refused with
 *     E_SHAPE before anything is enqueued.  The need grows with N up to a bound that the paper's
 *     settings keep under 17 MB (N = 16384, C = 1024, K = 16, V = 4: 8.4 MB; K = 16, V = 32 with 128
 *     or more codebooks: 16.8 MB); only layers of several million centroid values exceed 32 MiB.
 *   - The device the stream belongs to must be the current device (E_HIP otherwise).  The first
 *     call on a device looks the array's address up once (hipGetSymbolAddress); make that call
 *     outside stream capture.
 *   - All calls on one GPU share the one array: two calls whose kernels may overlap on that GPU
 *     (different streams, or several host threads on different streams) race on it.  Calls on one
 *     stream are ordered and safe.  Contents are unspecified between calls.
 * Errors: as lutnn_softpq_backward.
 */
#define LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES (32u << 20)
LUTNN_API lutnn_status lutnn_softpq_backward_static(const lutnn_layer* layer, float temperature,
                                                    const float* X, int64_t N, int64_t ldx,
                                                    const float* Z, int64_t ldz, float* dP, float* dX,
                                                    int64_t lddx, float* dt, void* stream);

/*
 * A 2-D convolution as the operator above (Sec. 4: a convolution becomes a matrix product by
 * im2col, with M = output channels, D = input channels x filter size and N = output pixels).
 * Row n = (image b, output pixel ho, wo), b slowest; column j = (input channel ci, filter row r,
 * filter column s), ci slowest, holding input[b][ci][ho*stride_h + r - pad_h][wo*stride_w + s - pad_w]
 * or 0 outside the image.  Sub-vector c of a row is columns [c*V, (c+1)*V): with V = kh*kw it is
 * one channel's patch, the paper's (K, V) = (16, 9) for 3x3 filters; with a 1x1 filter and V = 4
 * it is four consecutive channels of one pixel, the paper's (16, 4).
 */
typedef struct {
    int32_t Cin, H, W;          /* input channels, height, width                      */
    int32_t kh, kw;             /* filter height, width                               */
    int32_t stride_h, stride_w; /* >= 1                                               */
    int32_t pad_h, pad_w;       /* zero padding on each side, >= 0                    */
    int32_t reserved;           /* must be 0                                          */
} lutnn_conv2d_geom;

/*
 * Host: rows of the im2col matrix, N = B * Ho * Wo with Ho = (H + 2*pad_h - kh) / stride_h + 1
 * (Wo likewise).  Returns -1 for an invalid geometry or B < 0.
 */
LUTNN_API int64_t lutnn_conv2d_rows(const lutnn_conv2d_geom* geom, int64_t B);

/*
 * lutnn_encode on the rows of the im2col matrix, read straight from the image batch: the matrix
 * (kh*kw times the input) is never written.
 *
 *   input  [B][Cin][H][W] fp32, dense (NCHW)
 *   idx    [N][C] uint8, dense, N = lutnn_conv2d_rows(geom, B)
 * Needs Cin*kh*kw == C*V and V in {1, 2, 3, 4, 8, 9, 16}.
 * Errors: E_NULL, E_SHAPE, E_UNSUPPORTED (V), E_ALIGN, E_HIP.
 */
LUTNN_API lutnn_status lutnn_encode_conv2d(const lutnn_layer* layer, const float* input, int64_t B,
                                           const lutnn_conv2d_geom* geom, uint8_t* idx,
                                           void* stream);

/*
 * The convolution: lutnn_encode_conv2d into idx_workspace, then lutnn_lookup.
 *
 *   Y              [N][M] fp32, row stride ldy >= M: output pixels by output channels (NHWC)
 *   variant        AUTO, LDS, MFMA or SMFMAC (as lutnn_lookup); FUSED is not available
 *   idx_workspace  [N][C] uint8 device scratch, required
 * Errors: as lutnn_encode_conv2d and lutnn_lookup.
 */
LUTNN_API lutnn_status lutnn_conv2d(const lutnn_layer* layer, const float* input, int64_t B,
                                    const lutnn_conv2d_geom* geom, float* Y, int64_t ldy,
                                    int32_t variant, uint8_t* idx_workspace, void* stream);

/*
 * The hash encoder on a convolution's rows (lutnn_encode_tree on the im2col matrix of `input`,
 * which is never written; row and column order as for lutnn_encode_conv2d), and the whole
 * convolution with it: lutnn_encode_tree_conv2d into idx_workspace, then lutnn_lookup.
 *   tree   C * V must equal Cin*kh*kw; V in {1,2,3,4,8,9,16} (E_UNSUPPORTED otherwise)
 *   idx / idx_workspace  [B*Ho*Wo][C] uint8
 * Errors: as lutnn_encode_tree, lutnn_encode_conv2d and lutnn_lookup; E_SHAPE when tree and layer
 * disagree.
 */
LUTNN_API lutnn_status lutnn_encode_tree_conv2d(const lutnn_tree* tree, const float* input, int64_t B,
                                                const lutnn_conv2d_geom* geom, uint8_t* idx, void* stream);
LUTNN_API lutnn_status lutnn_conv2d_tree(const lutnn_layer* layer, const lutnn_tree* tree,
                                         const float* input, int64_t B, const lutnn_conv2d_geom* geom,
                                         float* Y, int64_t ldy, int32_t variant, uint8_t* idx_workspace,
                                         void* stream);

/*
 * Host: the variant that LUTNN_VARIANT_AUTO stands for in lutnn_lookup(layer, idx, N, ...) - and in
 * lutnn_linear when `idx` is its workspace - so that callers (and benchmarks) can report which
 * kernel ran.  Pure function of the descriptor, N and the address of idx; nothing is launched
 * and nothing dereferenced.  Returns LUTNN_VARIANT_LDS, _MFMA or _SMFMAC; for lutnn_linear with a
 * NULL workspace AUTO means LUTNN_VARIANT_FUSED instead.  Returns -1 for a NULL layer.
 */
LUTNN_API int32_t lutnn_auto_variant(const lutnn_layer* layer, const uint8_t* idx, int64_t N);

/*
 * Host: the same for lutnn_linear(layer, X, N, ..., LUTNN_VARIANT_AUTO, idx_workspace, ...):
 * LUTNN_VARIANT_FUSED where one launch does both steps, else what lutnn_auto_variant returns for
 * the lookup that follows the encoding.  Returns -1 for a NULL layer.
 */
LUTNN_API int32_t lutnn_linear_auto_variant(const lutnn_layer* layer, const uint8_t* idx_workspace,
                                            int64_t N);

/* Host: static name of a status code. */
LUTNN_API const char* lutnn_status_string(int32_t status);

/* Host: description of the calling thread's most recent failure ("" if none). */
LUTNN_API const char* lutnn_last_error(void);

/*
 * Host: pins a launcher's choice among its kernel instances, for tuning sweeps and for tests that
 * must reach every instance; not needed in normal use.  Switches (each starts from the environment
 * variable of the same name, which is read once, when the first call needs it):
 *   "LUTNN_FUSED_KERNEL"      "small" | "tile"          which form LUTNN_VARIANT_FUSED runs
 *   "LUTNN_SMFMAC_SPLIT"      "0" | "1"                 codebooks of a tile shared out over workgroups
 *   "LUTNN_SMFMAC_TILE_ROWS"  "128" | "256" | "384" | "512"   tile height of the sparse matrix-core lookup
 *   "LUTNN_SMFMAC_ROW_GROUP"  "0" .. "64"               row tiles per group of its tile order (0 = plain)
 *   "LUTNN_SMFMAC_TILE_COLS"  "96" | "128"              width of its 512-row tiles
 * value NULL or "" returns the switch to "not pinned".  A pinned choice the shape cannot take is
 * ignored.  Process-wide and atomic: safe to call while other threads launch, which then see
 * either the old or the new value.
 * Errors: E_NULL (name), E_UNSUPPORTED (unknown name), E_SHAPE (value not understood).
 */
LUTNN_API lutnn_status lutnn_set_tunable(const char* name, const char* value);

/*
 * Measurement aid, not part of the operator: enqueues a stream of nothing but the 2:4-sparse INT8
 * matrix instruction that the one-hot form of Eq. 4 runs on - one workgroup of four waves per compute
 * unit, 16 * iterations instructions per wave - so that a caller timing it with events learns how fast
 * the matrix pipes go on a kind of operand data (the clock the chip holds depends on it): the floor of
 * the lookup on such data, quoted by the benchmark beside the nominal peak.
 *   operands   0 = the same constants in every instruction; 1 = full-range random INT8 table
 *              values and random one-hot slices, as the lookup feeds them; 2 = as 1, 3-bit values
 *   sink       device, at least 256 ints per compute unit (1 KiB each); written once, content
 *              meaningless (it keeps the instructions alive)
 * Errors: E_NULL, E_SHAPE (operands, iterations outside 0 .. 2^24, sink too small), E_ALIGN, E_HIP.
 */
LUTNN_API lutnn_status lutnn_probe_smfmac_stream(int32_t operands, int32_t iterations, int32_t* sink,
                                                 size_t sink_bytes, void* stream);

/*
 * Host: library version, "major.minor.patch+<source hash>": the hash (12 hex digits) identifies the
 * sources the library was compiled from, so that a loader can tell a stale binary.
 */
LUTNN_API const char* lutnn_version(void);

#ifdef __cplusplus
}
#endif
#endif /* LUTNN_H */
