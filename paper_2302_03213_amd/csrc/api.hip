// Host side of liblutnn: argument validation and dispatch for the C ABI declared in
// include/lutnn.h.  Nothing here allocates device memory or synchronises.
#include <hip/hip_runtime.h>

#include <atomic>
#include <cmath>
#include <cstdarg>
#include <cstdio>
#include <cstdlib>
#include <cstring>
#include <mutex>

#include "lutnn.h"
#include "lutnn_kernels.h"

namespace {

thread_local char g_err[512] = "";

lutnn_status fail(lutnn_status st, const char* fmt, ...) {
    va_list ap;
    va_start(ap, fmt);
    vsnprintf(g_err, sizeof(g_err), fmt, ap);
    va_end(ap);
    return st;
}

lutnn_status hip_result(hipError_t e, const char* what) {
    if (e == hipSuccess) return LUTNN_OK;
    return fail(LUTNN_E_HIP, "%s: %s", what, hipGetErrorString(e));
}

// ---- tuning switches (lutnn_kernels.h)
const char* const kTunableNames[lutnn::kTuneCount] = {"LUTNN_FUSED_KERNEL", "LUTNN_SMFMAC_SPLIT",
                                                      "LUTNN_SMFMAC_TILE_ROWS", "LUTNN_SMFMAC_ROW_GROUP",
                                                      "LUTNN_SMFMAC_TILE_COLS"};
std::atomic<int> g_tunable[lutnn::kTuneCount];
std::once_flag g_tunable_once;

// Text of a switch -> its value; -1 for NULL, empty or anything not understood.
int parse_tunable(int which, const char* text) {
    if (!text || !*text) return -1;
    if (which == lutnn::kTuneFusedKernel) {
        if (std::strcmp(text, "small") == 0) return 1;
        if (std::strcmp(text, "tile") == 0) return 0;
        return -1;
    }
    char* end = nullptr;
    const long v = std::strtol(text, &end, 10);
    if (*end != 0) return -1;
    if (which == lutnn::kTuneSmfmacSplit) return (v == 0 || v == 1) ? (int)v : -1;
    if (which == lutnn::kTuneSmfmacRowGroup) return (v >= 0 && v <= 64) ? (int)v : -1;
    if (which == lutnn::kTuneSmfmacTileCols) return (v == 96 || v == 128) ? (int)v : -1;
    return (v == 128 || v == 256 || v == 384 || v == 512) ? (int)v : -1;
}

void tunables_from_environment() {
    for (int i = 0; i < lutnn::kTuneCount; ++i)
        g_tunable[i].store(parse_tunable(i, std::getenv(kTunableNames[i])), std::memory_order_relaxed);
}

bool aligned(const void* p, uintptr_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) == 0; }

// Dimensions shared by every entry point.  CK*M and N*C style products are formed in int64 by the
// kernels; the individual dimensions must fit comfortably in int32.
constexpr int kMaxK8 = 256;    // uint8 indices
constexpr int kMaxK16 = 4096;  // uint16 indices: the 12-level trees of Sec. 7

lutnn_status check_dims(int32_t C, int32_t K, int32_t V, int32_t M, int32_t kmax = kMaxK8) {
    if (C <= 0 || K <= 0 || V <= 0 || M <= 0)
        return fail(LUTNN_E_SHAPE, "C, K, V, M must be positive (got C=%d K=%d V=%d M=%d)", C, K, V, M);
    if (K > kmax)
        return fail(LUTNN_E_SHAPE, "K=%d exceeds %d (%s)", K, kmax,
                    kmax == kMaxK8 ? "indices are uint8; the ...16 entry points take up to 4096" : "indices are uint16");
    // M: a grid dimension of the table kernels counts blocks of 256 padded columns and stops at 65535
    if ((int64_t)C * V > (1 << 24) || M > (1 << 24) - 512 || C > (1 << 22))
        return fail(LUTNN_E_SHAPE, "dimension too large (C=%d V=%d M=%d)", C, V, M);
    return LUTNN_OK;
}

inline bool is_int_table(int dtype) { return dtype == LUTNN_TABLE_I8 || dtype == LUTNN_TABLE_I4; }

lutnn_status check_layer(const lutnn_layer* L, int32_t kmax = kMaxK8) {
    if (!L) return fail(LUTNN_E_NULL, "layer is NULL");
    if (L->reserved != 0) return fail(LUTNN_E_SHAPE, "layer->reserved must be 0");
    if (L->table_dtype != LUTNN_TABLE_F32 && !is_int_table(L->table_dtype))
        return fail(LUTNN_E_UNSUPPORTED, "unknown table dtype %d", L->table_dtype);
    return check_dims(L->C, L->K, L->V, L->M, kmax);
}

constexpr int64_t kMaxRows = (int64_t)1 << 31;

// Which lookup kernel AUTO resolves to.
int resolve_lookup_variant(const lutnn_layer* L, int variant, const uint8_t* idx, int64_t N) {
    if (variant != LUTNN_VARIANT_AUTO) return variant;
    if (is_int_table(L->table_dtype) && L->table_packed && L->K <= 16) {
        // small problems with few codebooks: rows gathered straight from L2 beat a matrix-core launch
        const bool sparse_ok = lutnn::smfmac_supported(L->C, L->K, idx);
        if (lutnn::gather_preferred(L->table, L->table_dtype == LUTNN_TABLE_I4 ? 2 : 1, L->C, L->M, N, sparse_ok))
            return LUTNN_VARIANT_LDS;
        // the sparse kernel at any N (its 128-row tiles spread even a single row's columns over the
        // chip and stream the table in parallel); the dense one where the sparse one cannot run
        if (sparse_ok) return LUTNN_VARIANT_SMFMAC;
        return LUTNN_VARIANT_MFMA;
    }
    return LUTNN_VARIANT_LDS;
}

lutnn_status check_lookup(const lutnn_layer* L, int variant, const uint8_t* idx, const float* Y,
                          int64_t N, int64_t ldy) {
    if (!Y) return fail(LUTNN_E_NULL, "Y is NULL");
    if (N < 0 || N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=%lld out of range", (long long)N);
    if (ldy < L->M) return fail(LUTNN_E_SHAPE, "ldy=%lld is smaller than M=%d", (long long)ldy, L->M);
    if (!aligned(Y, 4)) return fail(LUTNN_E_ALIGN, "Y must be 4-byte aligned");
    if (L->bias && !aligned(L->bias, 4)) return fail(LUTNN_E_ALIGN, "bias must be 4-byte aligned");
    if (is_int_table(L->table_dtype) && !L->scale)
        return fail(LUTNN_E_NULL, "an integer table needs layer->scale");
    switch (variant) {
        case LUTNN_VARIANT_LDS:
            if (!L->table) return fail(LUTNN_E_NULL, "the LDS variant needs layer->table");
            if (L->table_dtype == LUTNN_TABLE_F32 && !aligned(L->table, 4))
                return fail(LUTNN_E_ALIGN, "fp32 table must be 4-byte aligned");
            break;
        case LUTNN_VARIANT_MFMA:
        case LUTNN_VARIANT_SMFMAC:
            if (!is_int_table(L->table_dtype))
                return fail(LUTNN_E_UNSUPPORTED, "the MFMA variants need an INT8 or INT4 table");
            if (L->K > 16)
                return fail(LUTNN_E_UNSUPPORTED, "the MFMA variants support K <= 16 (got %d)", L->K);
            if (!L->table_packed) return fail(LUTNN_E_NULL, "the MFMA variants need layer->table_packed");
            if (!aligned(L->table_packed, 16))
                return fail(LUTNN_E_ALIGN, "table_packed must be 16-byte aligned");
            if (variant == LUTNN_VARIANT_SMFMAC) {
                if (L->C % 32 != 0)
                    return fail(LUTNN_E_UNSUPPORTED, "the SMFMAC variant needs C %% 32 == 0 (got %d)", L->C);
                if (!aligned(idx, 16)) return fail(LUTNN_E_ALIGN, "the SMFMAC variant needs idx 16-byte aligned");
            }
            break;
        default:
            return fail(LUTNN_E_UNSUPPORTED, "variant %d is not a lookup variant", variant);
    }
    return LUTNN_OK;
}

lutnn_status do_lookup(const lutnn_layer* L, int variant, const uint8_t* idx, int64_t N, float* Y,
                       int64_t ldy, hipStream_t s) {
    hipError_t e;
    if (variant == LUTNN_VARIANT_SMFMAC) {
        e = lutnn::launch_lookup_smfmac_i8(static_cast<const int8_t*>(L->table_packed), L->scale, L->bias,
                                           L->C, L->K, L->M, idx, N, Y, ldy, s);
    } else if (variant == LUTNN_VARIANT_MFMA) {
        e = lutnn::launch_lookup_mfma_i8(static_cast<const int8_t*>(L->table_packed), L->scale, L->bias,
                                         L->C, L->K, L->M, idx, N, Y, ldy, s);
    } else if (L->table_dtype == LUTNN_TABLE_I8) {
        e = lutnn::launch_lookup_lds_i8(static_cast<const int8_t*>(L->table), L->scale, L->bias, L->C,
                                        L->K, L->M, idx, N, Y, ldy, s);
    } else if (L->table_dtype == LUTNN_TABLE_I4) {
        e = lutnn::launch_lookup_lds_i4(static_cast<const uint8_t*>(L->table), L->scale, L->bias, L->C,
                                        L->K, L->M, idx, N, Y, ldy, s);
    } else {
        e = lutnn::launch_lookup_lds_f32(static_cast<const float*>(L->table), L->bias, L->C, L->K, L->M,
                                         idx, N, Y, ldy, s);
    }
    return hip_result(e, "lookup launch");
}

lutnn_status check_encode(const lutnn_layer* L, const float* X, int64_t N, int64_t ldx) {
    if (!L->centroids) return fail(LUTNN_E_NULL, "layer->centroids is NULL");
    if (!X) return fail(LUTNN_E_NULL, "X is NULL");
    if (N < 0 || N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=%lld out of range", (long long)N);
    if (ldx < (int64_t)L->C * L->V)
        return fail(LUTNN_E_SHAPE, "ldx=%lld is smaller than D=C*V=%lld", (long long)ldx,
                    (long long)L->C * L->V);
    if (!aligned(X, 4) || !aligned(L->centroids, 4))
        return fail(LUTNN_E_ALIGN, "X and centroids must be 4-byte aligned");
    return LUTNN_OK;
}

lutnn_status check_tree(const lutnn_tree* T, const float* X, int64_t N, int64_t ldx, int max_levels = 8) {
    if (!T) return fail(LUTNN_E_NULL, "tree is NULL");
    if (T->reserved != 0) return fail(LUTNN_E_SHAPE, "tree->reserved must be 0");
    if (T->levels < 1 || T->levels > max_levels)
        return fail(LUTNN_E_SHAPE, "tree->levels=%d outside 1..%d (%s)", T->levels, max_levels,
                    max_levels == 8 ? "indices are uint8; the ...16 entry points take up to 12 levels"
                                    : "indices are uint16");
    if (lutnn_status st = check_dims(T->C, 1 << T->levels, T->V, 1, kMaxK16)) return st;
    if (N == 0) return LUTNN_OK;
    if (!T->split_dim || !T->threshold) return fail(LUTNN_E_NULL, "tree->split_dim or tree->threshold is NULL");
    if (!X) return fail(LUTNN_E_NULL, "X is NULL");
    if (N < 0 || N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=%lld out of range", (long long)N);
    if (ldx < (int64_t)T->C * T->V)
        return fail(LUTNN_E_SHAPE, "ldx=%lld is smaller than D=C*V=%lld", (long long)ldx,
                    (long long)T->C * T->V);
    if (!aligned(X, 4) || !aligned(T->split_dim, 4) || !aligned(T->threshold, 4))
        return fail(LUTNN_E_ALIGN, "X, split_dim and threshold must be 4-byte aligned");
    return LUTNN_OK;
}

// Validates a convolution geometry against the layer and derives the output size.
lutnn_status check_conv(const lutnn_layer* L, const lutnn_conv2d_geom* g, int64_t B, lutnn::ConvGeom* out,
                        int64_t* rows) {
    if (!g) return fail(LUTNN_E_NULL, "geom is NULL");
    if (g->reserved != 0) return fail(LUTNN_E_SHAPE, "geom->reserved must be 0");
    if (B < 0 || B >= kMaxRows) return fail(LUTNN_E_SHAPE, "B=%lld out of range", (long long)B);
    if (g->Cin <= 0 || g->H <= 0 || g->W <= 0 || g->kh <= 0 || g->kw <= 0 || g->stride_h <= 0 ||
        g->stride_w <= 0 || g->pad_h < 0 || g->pad_w < 0)
        return fail(LUTNN_E_SHAPE, "invalid convolution geometry");
    if (g->kh > 64 || g->kw > 64 || g->pad_h > 64 || g->pad_w > 64)
        return fail(LUTNN_E_SHAPE, "filter size and padding are limited to 64");
    const int64_t eh = (int64_t)g->H + 2 * g->pad_h - g->kh, ew = (int64_t)g->W + 2 * g->pad_w - g->kw;
    if (eh < 0 || ew < 0) return fail(LUTNN_E_SHAPE, "the filter is larger than the padded image");
    const int64_t Ho = eh / g->stride_h + 1, Wo = ew / g->stride_w + 1;
    if (Ho * Wo >= (int64_t)1 << 30 || (int64_t)g->Cin * g->H * g->W >= (int64_t)1 << 31)
        return fail(LUTNN_E_SHAPE, "image too large");
    const int64_t N = B * Ho * Wo;
    if (N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=B*Ho*Wo=%lld out of range", (long long)N);
    if (L) {
        if ((int64_t)g->Cin * g->kh * g->kw != (int64_t)L->C * L->V)
            return fail(LUTNN_E_SHAPE, "Cin*kh*kw=%lld differs from C*V=%lld",
                        (long long)g->Cin * g->kh * g->kw, (long long)L->C * L->V);
        if (!lutnn::encode_conv_supported(L->V))
            return fail(LUTNN_E_UNSUPPORTED, "no convolution encoder for V=%d", L->V);
    }
    if (out)
        *out = lutnn::ConvGeom{g->Cin, g->H,     g->W,     g->kh,   g->kw, g->stride_h,
                               g->stride_w, g->pad_h, g->pad_w, (int)Ho, (int)Wo};
    *rows = N;
    return LUTNN_OK;
}

lutnn_status check_conv_input(const lutnn_layer* L, const float* input) {
    if (!L->centroids) return fail(LUTNN_E_NULL, "layer->centroids is NULL");
    if (!input) return fail(LUTNN_E_NULL, "input is NULL");
    if (!aligned(input, 4) || !aligned(L->centroids, 4))
        return fail(LUTNN_E_ALIGN, "input and centroids must be 4-byte aligned");
    return LUTNN_OK;
}

}  // namespace

namespace lutnn {

int tunable(int which) {
    std::call_once(g_tunable_once, tunables_from_environment);
    return g_tunable[which].load(std::memory_order_relaxed);
}

int compute_units() {
    constexpr int kDevices = 64;
    static std::atomic<int> cached[kDevices];
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kDevices) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

}  // namespace lutnn

extern "C" {

lutnn_status lutnn_set_tunable(const char* name, const char* value) {
    if (!name) return fail(LUTNN_E_NULL, "name is NULL");
    std::call_once(g_tunable_once, tunables_from_environment);
    for (int i = 0; i < lutnn::kTuneCount; ++i)
        if (std::strcmp(name, kTunableNames[i]) == 0) {
            const int v = parse_tunable(i, value);
            if (value && *value && v < 0) return fail(LUTNN_E_SHAPE, "%s does not take the value '%s'", name, value);
            g_tunable[i].store(v, std::memory_order_relaxed);
            return LUTNN_OK;
        }
    return fail(LUTNN_E_UNSUPPORTED, "no tuning switch named '%s'", name);
}

lutnn_status lutnn_probe_smfmac_stream(int32_t operands, int32_t iterations, int32_t* sink, size_t sink_bytes,
                                       void* stream) {
    if (!sink) return fail(LUTNN_E_NULL, "sink is NULL");
    if (operands < 0 || operands > 2) return fail(LUTNN_E_SHAPE, "operands must be 0, 1 or 2 (got %d)", operands);
    if (iterations < 0 || iterations > (1 << 24))
        return fail(LUTNN_E_SHAPE, "iterations must be 0 .. 2^24 (got %d)", iterations);
    if (sink_bytes < (size_t)lutnn::compute_units() * 256 * sizeof(int32_t))
        return fail(LUTNN_E_SHAPE, "sink holds %zu bytes, the probe writes %zu", sink_bytes,
                    (size_t)lutnn::compute_units() * 256 * sizeof(int32_t));
    if (!aligned(sink, 4)) return fail(LUTNN_E_ALIGN, "sink must be 4-byte aligned");
    return hip_result(lutnn::launch_probe_smfmac_stream(operands, iterations, sink, static_cast<hipStream_t>(stream)),
                      "lutnn_probe_smfmac_stream");
}

size_t lutnn_table_bytes(int32_t C, int32_t K, int32_t M, int32_t dtype) {
    if (C <= 0 || K <= 0 || M <= 0) return 0;
    const size_t n = (size_t)C * (size_t)K * (size_t)M;
    if (dtype == LUTNN_TABLE_I8) return n;
    if (dtype == LUTNN_TABLE_I4) return (size_t)C * (size_t)K * (((size_t)M + 1) / 2);
    if (dtype == LUTNN_TABLE_F32) return n * 4;
    return 0;
}

size_t lutnn_packed_bytes(int32_t C, int32_t K, int32_t M, int32_t dtype) {
    if (C <= 0 || K <= 0 || K > 256 || M <= 0 || !is_int_table(dtype)) return 0;
    return (size_t)C * (size_t)lutnn::kblocks(K) * (size_t)lutnn::packed_cols(M) * 16;
}

lutnn_status lutnn_build_table(const float* centroids, const float* W, int64_t ldw, int32_t C,
                               int32_t K, int32_t V, int32_t M, int32_t dtype, void* table_out,
                               void* packed_out, float* scale_out, void* stream) {
    if (!centroids || !W || !table_out) return fail(LUTNN_E_NULL, "centroids, W or table_out is NULL");
    if (lutnn_status st = check_dims(C, K, V, M, kMaxK16)) return st;
    if (K > kMaxK8 && packed_out)
        return fail(LUTNN_E_UNSUPPORTED, "no packed copy for K=%d > 256 (pass packed_out = NULL)", K);
    if (ldw < M) return fail(LUTNN_E_SHAPE, "ldw=%lld is smaller than M=%d", (long long)ldw, M);
    if (!aligned(centroids, 4) || !aligned(W, 4))
        return fail(LUTNN_E_ALIGN, "centroids and W must be 4-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (dtype == LUTNN_TABLE_F32) {
        if (!aligned(table_out, 4)) return fail(LUTNN_E_ALIGN, "table_out must be 4-byte aligned");
        return hip_result(lutnn::launch_build_table_f32(centroids, W, ldw, C, K, V, M,
                                                        static_cast<float*>(table_out), s),
                          "build_table launch");
    }
    if (is_int_table(dtype)) {
        if (!scale_out) return fail(LUTNN_E_NULL, "an integer table needs scale_out");
        if (!aligned(scale_out, 4)) return fail(LUTNN_E_ALIGN, "scale_out must be 4-byte aligned");
        if (packed_out && !aligned(packed_out, 16))
            return fail(LUTNN_E_ALIGN, "packed_out must be 16-byte aligned");
        return hip_result(lutnn::launch_build_table_i8(centroids, W, ldw, C, K, V, M,
                                                       static_cast<int8_t*>(table_out),
                                                       static_cast<int8_t*>(packed_out), scale_out,
                                                       dtype == LUTNN_TABLE_I4 ? 4 : 8, s),
                          "build_table launch");
    }
    return fail(LUTNN_E_UNSUPPORTED, "unknown table dtype %d", dtype);
}

lutnn_status lutnn_encode(const lutnn_layer* layer, const float* X, int64_t N, int64_t ldx,
                          uint8_t* idx, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (N == 0) return LUTNN_OK;  // an empty batch may come with NULL data pointers
    if (lutnn_status st = check_encode(layer, X, N, ldx)) return st;
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    return hip_result(lutnn::launch_encode(layer->centroids, layer->C, layer->K, layer->V, X, N, ldx, idx,
                                           static_cast<hipStream_t>(stream)),
                      "encode launch");
}

lutnn_status lutnn_encode_tree(const lutnn_tree* tree, const float* X, int64_t N, int64_t ldx,
                               uint8_t* idx, void* stream) {
    if (lutnn_status st = check_tree(tree, X, N, ldx)) return st;
    if (N == 0) return LUTNN_OK;
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    return hip_result(lutnn::launch_encode_tree(tree->split_dim, tree->threshold, tree->C, tree->levels,
                                                tree->V, X, N, ldx, idx, static_cast<hipStream_t>(stream)),
                      "tree encode launch");
}

size_t lutnn_softpq_workspace_bytes(int32_t C, int32_t K, int32_t V, int64_t N) {
    if (C <= 0 || K <= 0 || V <= 0 || N <= 0) return 0;
    return lutnn::softpq_workspace_bytes(C, K, V, N);
}

}  // extern "C"

namespace {

// Validation shared by the two forms of the soft-PQ backward entry point; everything but the
// scratch buffer, whose size in bytes the caller of this function has already established.
lutnn_status softpq_backward_checked(const lutnn_layer* layer, float temperature, const float* X, int64_t N,
                                     int64_t ldx, const float* Z, int64_t ldz, float* dP, float* dX,
                                     int64_t lddx, float* dt, void* workspace, size_t workspace_bytes,
                                     const char* what_scratch, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (!(temperature > 0.0f) || !std::isfinite(temperature))
        return fail(LUTNN_E_SHAPE, "temperature must be positive and finite (got %g)", (double)temperature);
    if (!lutnn::softpq_supported(layer->K, layer->V))
        return fail(LUTNN_E_UNSUPPORTED, "soft-PQ backward supports K in {8,16} and V in {1,2,3,4,8,9,16,32} "
                    "(got K=%d V=%d)", layer->K, layer->V);
    if (!dP) return fail(LUTNN_E_NULL, "dP is NULL");
    if (N < 0 || N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=%lld out of range", (long long)N);
    const int64_t D = (int64_t)layer->C * layer->V;
    if (N > 0) {  // an empty batch may come with NULL data pointers
        if (lutnn_status st = check_encode(layer, X, N, ldx)) return st;
        if (!Z) return fail(LUTNN_E_NULL, "Z is NULL");
        if (ldz < D) return fail(LUTNN_E_SHAPE, "ldz=%lld is smaller than D=%lld", (long long)ldz, (long long)D);
        if (dX && lddx < D)
            return fail(LUTNN_E_SHAPE, "lddx=%lld is smaller than D=%lld", (long long)lddx, (long long)D);
        if (!workspace) return fail(LUTNN_E_NULL, "workspace is NULL");
        const size_t need = lutnn::softpq_workspace_bytes(layer->C, layer->K, layer->V, N);
        if (workspace_bytes < need)
            return fail(LUTNN_E_SHAPE, "%s of %zu bytes is smaller than the %zu this shape needs (C=%d K=%d V=%d N=%lld)",
                        what_scratch, workspace_bytes, need, layer->C, layer->K, layer->V, (long long)N);
    }
    if (!aligned(Z, 4) || !aligned(dP, 4) || !aligned(dX, 4) || !aligned(dt, 4) || !aligned(workspace, 4))
        return fail(LUTNN_E_ALIGN, "Z, dP, dX, dt and workspace must be 4-byte aligned");
    hipStream_t s = static_cast<hipStream_t>(stream);
    // N == 0: the launcher only writes the zeros of the empty sums
    return hip_result(lutnn::launch_softpq_backward(layer->centroids, layer->C, layer->K, layer->V, temperature,
                                                    X, N, ldx, Z, ldz, dP, dX, lddx, dt,
                                                    static_cast<float*>(workspace), s),
                      "soft-PQ backward launch");
}

}  // namespace

// Scratch of lutnn_softpq_backward_static: one copy per GPU that loads this library, held until the
// process ends.  In host code this name is only a handle for hipGetSymbolAddress; the address a
// kernel may use is the one that call returns, on the device it was made for.
static __device__ __align__(256) unsigned char scratch[LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES];

namespace {

constexpr int kMaxDevices = 64;
std::mutex g_scratch_mutex;
std::atomic<void*> g_scratch_ptr[kMaxDevices];

// Device address of `scratch` on the current device, looked up once per device.
lutnn_status scratch_of_current_device(void* stream, void** out) {
    int dev = -1;
    if (hipError_t e = hipGetDevice(&dev)) return hip_result(e, "hipGetDevice");
    if (dev < 0 || dev >= kMaxDevices) return fail(LUTNN_E_HIP, "device ordinal %d outside 0..%d", dev, kMaxDevices - 1);
    if (stream) {  // the array is per device: the stream's kernels must run where the address is valid
        hipDevice_t sdev = -1;
        if (hipError_t e = hipStreamGetDevice(static_cast<hipStream_t>(stream), &sdev))
            return hip_result(e, "hipStreamGetDevice");
        if ((int)sdev != dev)
            return fail(LUTNN_E_HIP, "stream belongs to device %d but device %d is current", (int)sdev, dev);
    }
    void* p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!p) {
        std::lock_guard<std::mutex> lock(g_scratch_mutex);
        p = g_scratch_ptr[dev].load(std::memory_order_relaxed);
        if (!p) {
            if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch))) return hip_result(e, "hipGetSymbolAddress");
            if (!p) return fail(LUTNN_E_HIP, "hipGetSymbolAddress returned no address");
            g_scratch_ptr[dev].store(p, std::memory_order_release);
        }
    }
    *out = p;
    return LUTNN_OK;
}

}  // namespace

extern "C" {

lutnn_status lutnn_softpq_backward(const lutnn_layer* layer, float temperature, const float* X, int64_t N,
                                   int64_t ldx, const float* Z, int64_t ldz, float* dP, float* dX,
                                   int64_t lddx, float* dt, void* workspace, size_t workspace_bytes,
                                   void* stream) {
    return softpq_backward_checked(layer, temperature, X, N, ldx, Z, ldz, dP, dX, lddx, dt, workspace,
                                   workspace_bytes, "workspace", stream);
}

lutnn_status lutnn_softpq_backward_static(const lutnn_layer* layer, float temperature, const float* X,
                                          int64_t N, int64_t ldx, const float* Z, int64_t ldz, float* dP,
                                          float* dX, int64_t lddx, float* dt, void* stream) {
    // size first, on the host alone: a shape beyond the static array is refused before anything
    // touches the device
    if (lutnn_status st = check_layer(layer)) return st;
    if (N > 0 && lutnn::softpq_supported(layer->K, layer->V) && N < kMaxRows) {
        const size_t need = lutnn::softpq_workspace_bytes(layer->C, layer->K, layer->V, N);
        if (need > (size_t)LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES)
            return fail(LUTNN_E_SHAPE, "this shape needs %zu bytes of scratch, the static buffer holds %zu "
                        "(C=%d K=%d V=%d N=%lld): use lutnn_softpq_backward with a workspace",
                        need, (size_t)LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES, layer->C, layer->K, layer->V, (long long)N);
    }
    void* ptr = nullptr;
    if (lutnn_status st = scratch_of_current_device(stream, &ptr)) return st;
    // every partial sum the second kernel reads is written by the first in the same call, so
    // nothing of the previous call's contents has to be cleared
    return softpq_backward_checked(layer, temperature, X, N, ldx, Z, ldz, dP, dX, lddx, dt, ptr,
                                   (size_t)LUTNN_SOFTPQ_STATIC_SCRATCH_BYTES, "the static scratch buffer", stream);
}

lutnn_status lutnn_lookup(const lutnn_layer* layer, const uint8_t* idx, int64_t N, float* Y,
                          int64_t ldy, int32_t variant, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (N == 0) return LUTNN_OK;  // an empty batch may come with NULL data pointers
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    if (variant == LUTNN_VARIANT_FUSED)
        return fail(LUTNN_E_UNSUPPORTED, "FUSED is a lutnn_linear variant, not a lookup variant");
    const int v = resolve_lookup_variant(layer, variant, idx, N);
    if (lutnn_status st = check_lookup(layer, v, idx, Y, N, ldy)) return st;
    return do_lookup(layer, v, idx, N, Y, ldy, static_cast<hipStream_t>(stream));
}

namespace {

inline int small_table_kind(const lutnn_layer* L) {
    return L->table_dtype == LUTNN_TABLE_F32 ? 0 : L->table_dtype == LUTNN_TABLE_I8 ? 1 : 2;
}

// The one-launch kernel is worth it where the lookup it replaces would be the gather anyway (the
// indices it would see are 16-byte aligned in LDS, so the sparse kernel counts as available when
// the shape allows it).
bool small_preferred(const lutnn_layer* L, int64_t N) {
    const int kind = small_table_kind(L);
    if (kind == 2) return false;
    const bool sparse_ok = is_int_table(L->table_dtype) && L->table_packed && L->K <= 16 && L->C % 32 == 0;
    const bool matrix_ok = is_int_table(L->table_dtype) && L->table_packed && L->K <= 16;
    const bool gather_wins = !matrix_ok || lutnn::gather_preferred(L->table, kind, L->C, L->M, N, sparse_ok);
    return lutnn::linear_small_preferred(L->table, kind, L->C, L->K, L->V, L->M, N, gather_wins);
}

// Which of the two one-kernel forms FUSED runs: the one-launch kernel for small problems where it
// is the faster one, or where the tile kernel cannot run at all; the switch LUTNN_FUSED_KERNEL =
// small | tile pins the choice (tests that must reach both).
bool fused_takes_small_kernel(const lutnn_layer* L, int64_t N) {
    const int kind = small_table_kind(L);
    const bool can_small = lutnn::linear_small_supported(L->table, kind, L->C, L->K, L->V, L->M);
    const bool can_tile = lutnn::fused_supported(L->C, L->K, L->V, L->M, L->table_dtype) &&
                          (L->table_dtype == LUTNN_TABLE_F32 ? L->table != nullptr : L->table_packed != nullptr);
    const int pinned = lutnn::tunable(lutnn::kTuneFusedKernel);
    if (pinned == 1 && can_small) return true;
    if (pinned == 0 && can_tile) return false;
    if (!can_small) return false;
    return !can_tile || small_preferred(L, N);
}

// What lutnn_linear runs for `variant`.  AUTO: one launch where the problem is small enough that
// the second launch would be the larger part of the time; else encode once, then the fastest
// lookup - over conv-like, BERT-like and FC shapes the two launches are never slower than the tile
// form of the fused kernel (its 64-row workgroups encode all C codebooks serially and re-stream the
// table per row block).  Without a workspace for the indices a fused kernel is the only choice.
int resolve_linear_variant(const lutnn_layer* L, int variant, const uint8_t* idx_workspace, int64_t N) {
    if (variant != LUTNN_VARIANT_AUTO) return variant;
    if (small_preferred(L, N)) return LUTNN_VARIANT_FUSED;
    const bool tile_ok = lutnn::fused_supported(L->C, L->K, L->V, L->M, L->table_dtype) &&
                         (L->table_dtype == LUTNN_TABLE_F32 ? L->table != nullptr : L->table_packed != nullptr);
    const bool small_ok = lutnn::linear_small_supported(L->table, small_table_kind(L), L->C, L->K, L->V, L->M);
    if ((tile_ok || small_ok) && !idx_workspace) return LUTNN_VARIANT_FUSED;
    return resolve_lookup_variant(L, LUTNN_VARIANT_AUTO, idx_workspace, N);
}

}  // namespace

lutnn_status lutnn_linear(const lutnn_layer* layer, const float* X, int64_t N, int64_t ldx, float* Y,
                          int64_t ldy, int32_t variant, uint8_t* idx_workspace, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (N == 0) return LUTNN_OK;  // an empty batch may come with NULL data pointers
    if (lutnn_status st = check_encode(layer, X, N, ldx)) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    const lutnn_layer* L = layer;

    const int v = resolve_linear_variant(L, variant, idx_workspace, N);

    if (v == LUTNN_VARIANT_FUSED) {
        if (!Y) return fail(LUTNN_E_NULL, "Y is NULL");
        if (ldy < L->M) return fail(LUTNN_E_SHAPE, "ldy=%lld is smaller than M=%d", (long long)ldy, L->M);
        if (!aligned(Y, 4)) return fail(LUTNN_E_ALIGN, "Y must be 4-byte aligned");
        if (L->bias && !aligned(L->bias, 4)) return fail(LUTNN_E_ALIGN, "bias must be 4-byte aligned");
        if (is_int_table(L->table_dtype) && !L->scale)
            return fail(LUTNN_E_NULL, "an integer table needs layer->scale");
        if (fused_takes_small_kernel(L, N)) {
            if (L->table_dtype == LUTNN_TABLE_I8)
                return hip_result(lutnn::launch_linear_small_i8(L->centroids, static_cast<const int8_t*>(L->table),
                                                                L->scale, L->bias, L->C, L->K, L->V, L->M, X, N,
                                                                ldx, Y, ldy, s),
                                  "one-launch linear");
            return hip_result(lutnn::launch_linear_small_f32(L->centroids, static_cast<const float*>(L->table),
                                                             L->bias, L->C, L->K, L->V, L->M, X, N, ldx, Y, ldy,
                                                             s),
                              "one-launch linear");
        }
        if (!lutnn::fused_supported(L->C, L->K, L->V, L->M, L->table_dtype))
            return fail(LUTNN_E_UNSUPPORTED, "no fused kernel for C=%d K=%d V=%d M=%d dtype=%d", L->C, L->K,
                        L->V, L->M, L->table_dtype);
        if (is_int_table(L->table_dtype)) {
            if (!L->table_packed) return fail(LUTNN_E_NULL, "the fused INT8 kernel needs layer->table_packed");
            if (!aligned(L->table_packed, 16))
                return fail(LUTNN_E_ALIGN, "table_packed must be 16-byte aligned");
            return hip_result(lutnn::launch_linear_fused_i8(
                                  L->centroids, static_cast<const int8_t*>(L->table_packed), L->scale,
                                  L->bias, L->C, L->K, L->V, L->M, X, N, ldx, Y, ldy, s),
                              "fused linear launch");
        }
        if (!L->table) return fail(LUTNN_E_NULL, "the fused fp32 kernel needs layer->table");
        return hip_result(lutnn::launch_linear_fused_f32(L->centroids, static_cast<const float*>(L->table),
                                                         L->bias, L->C, L->K, L->V, L->M, X, N, ldx, Y,
                                                         ldy, s),
                          "fused linear launch");
    }

    if (!idx_workspace) return fail(LUTNN_E_NULL, "this variant needs idx_workspace");
    if (lutnn_status st = check_lookup(L, v, idx_workspace, Y, N, ldy)) return st;
    if (lutnn_status st = hip_result(
            lutnn::launch_encode(L->centroids, L->C, L->K, L->V, X, N, ldx, idx_workspace, s),
            "encode launch"))
        return st;
    return do_lookup(L, v, idx_workspace, N, Y, ldy, s);
}

lutnn_status lutnn_linear_tree(const lutnn_layer* layer, const lutnn_tree* tree, const float* X,
                               int64_t N, int64_t ldx, float* Y, int64_t ldy, int32_t variant,
                               uint8_t* idx_workspace, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (lutnn_status st = check_tree(tree, X, N, ldx)) return st;
    if (tree->C != layer->C || tree->V != layer->V || (1 << tree->levels) != layer->K)
        return fail(LUTNN_E_SHAPE, "tree (C=%d V=%d levels=%d) does not match layer (C=%d V=%d K=%d)", tree->C,
                    tree->V, tree->levels, layer->C, layer->V, layer->K);
    if (N == 0) return LUTNN_OK;
    hipStream_t s = static_cast<hipStream_t>(stream);
    // One launch (the tree walk, then the gather, in one kernel) where FUSED asks for it or where
    // AUTO would take it with the distance encoder: the rule prices launches and table reads, and
    // a walk costs less than the search it replaces.
    const bool can_small =
        lutnn::linear_small_supported(layer->table, small_table_kind(layer), layer->C, layer->K, layer->V, layer->M);
    if (variant == LUTNN_VARIANT_FUSED && !can_small)
        return fail(LUTNN_E_UNSUPPORTED, "no one-launch kernel with the hash encoder for C=%d K=%d V=%d M=%d dtype=%d",
                    layer->C, layer->K, layer->V, layer->M, layer->table_dtype);
    if (variant == LUTNN_VARIANT_FUSED || (variant == LUTNN_VARIANT_AUTO && small_preferred(layer, N))) {
        if (!Y) return fail(LUTNN_E_NULL, "Y is NULL");
        if (ldy < layer->M) return fail(LUTNN_E_SHAPE, "ldy=%lld is smaller than M=%d", (long long)ldy, layer->M);
        if (!aligned(Y, 4)) return fail(LUTNN_E_ALIGN, "Y must be 4-byte aligned");
        if (layer->bias && !aligned(layer->bias, 4)) return fail(LUTNN_E_ALIGN, "bias must be 4-byte aligned");
        if (layer->table_dtype == LUTNN_TABLE_I8) {
            if (!layer->scale) return fail(LUTNN_E_NULL, "an integer table needs layer->scale");
            return hip_result(lutnn::launch_linear_small_tree_i8(
                                  tree->split_dim, tree->threshold, tree->levels,
                                  static_cast<const int8_t*>(layer->table), layer->scale, layer->bias, layer->C,
                                  layer->V, layer->M, X, N, ldx, Y, ldy, s),
                              "one-launch linear (hash encoder)");
        }
        return hip_result(lutnn::launch_linear_small_tree_f32(
                              tree->split_dim, tree->threshold, tree->levels,
                              static_cast<const float*>(layer->table), layer->bias, layer->C, layer->V, layer->M, X,
                              N, ldx, Y, ldy, s),
                          "one-launch linear (hash encoder)");
    }
    if (!idx_workspace) return fail(LUTNN_E_NULL, "idx_workspace is NULL");
    const int v = resolve_lookup_variant(layer, variant, idx_workspace, N);
    if (lutnn_status st = check_lookup(layer, v, idx_workspace, Y, N, ldy)) return st;
    if (lutnn_status st = hip_result(lutnn::launch_encode_tree(tree->split_dim, tree->threshold, tree->C,
                                                               tree->levels, tree->V, X, N, ldx,
                                                               idx_workspace, s),
                                     "tree encode launch"))
        return st;
    return do_lookup(layer, v, idx_workspace, N, Y, ldy, s);
}

lutnn_status lutnn_encode_tree16(const lutnn_tree* tree, const float* X, int64_t N, int64_t ldx,
                                 uint16_t* idx, void* stream) {
    if (lutnn_status st = check_tree(tree, X, N, ldx, 12)) return st;
    if (N == 0) return LUTNN_OK;
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    if (!aligned(idx, 2)) return fail(LUTNN_E_ALIGN, "idx must be 2-byte aligned");
    return hip_result(lutnn::launch_encode_tree16(tree->split_dim, tree->threshold, tree->C, tree->levels,
                                                  tree->V, X, N, ldx, idx, static_cast<hipStream_t>(stream)),
                      "tree encode launch (16-bit leaves)");
}

namespace {
lutnn_status lookup16_checked(const lutnn_layer* L, const uint16_t* idx, int64_t N, float* Y, int64_t ldy,
                              hipStream_t s) {
    if (L->table_dtype == LUTNN_TABLE_I4)
        return fail(LUTNN_E_UNSUPPORTED, "the 16-bit index lookup reads INT8 and fp32 tables");
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    if (!Y) return fail(LUTNN_E_NULL, "Y is NULL");
    if (!L->table) return fail(LUTNN_E_NULL, "layer->table is NULL");
    if (N < 0 || N >= kMaxRows) return fail(LUTNN_E_SHAPE, "N=%lld out of range", (long long)N);
    if (ldy < L->M) return fail(LUTNN_E_SHAPE, "ldy=%lld is smaller than M=%d", (long long)ldy, L->M);
    if (!aligned(idx, 2) || !aligned(Y, 4) || (L->bias && !aligned(L->bias, 4)))
        return fail(LUTNN_E_ALIGN, "idx must be 2-byte, Y and bias 4-byte aligned");
    if (L->table_dtype == LUTNN_TABLE_I8) {
        if (!L->scale) return fail(LUTNN_E_NULL, "an integer table needs layer->scale");
        return hip_result(lutnn::launch_lookup_wide_i8(static_cast<const int8_t*>(L->table), L->scale, L->bias,
                                                       L->C, L->K, L->M, idx, N, Y, ldy, s),
                          "lookup launch (16-bit indices)");
    }
    if (!aligned(L->table, 4)) return fail(LUTNN_E_ALIGN, "fp32 table must be 4-byte aligned");
    return hip_result(lutnn::launch_lookup_wide_f32(static_cast<const float*>(L->table), L->bias, L->C, L->K,
                                                    L->M, idx, N, Y, ldy, s),
                      "lookup launch (16-bit indices)");
}
}  // namespace

lutnn_status lutnn_lookup16(const lutnn_layer* layer, const uint16_t* idx, int64_t N, float* Y, int64_t ldy,
                            void* stream) {
    if (lutnn_status st = check_layer(layer, kMaxK16)) return st;
    if (N == 0) return LUTNN_OK;
    return lookup16_checked(layer, idx, N, Y, ldy, static_cast<hipStream_t>(stream));
}

lutnn_status lutnn_linear_tree16(const lutnn_layer* layer, const lutnn_tree* tree, const float* X, int64_t N,
                                 int64_t ldx, float* Y, int64_t ldy, uint16_t* idx_workspace, void* stream) {
    if (lutnn_status st = check_layer(layer, kMaxK16)) return st;
    if (lutnn_status st = check_tree(tree, X, N, ldx, 12)) return st;
    if (tree->C != layer->C || tree->V != layer->V || (1 << tree->levels) != layer->K)
        return fail(LUTNN_E_SHAPE, "tree (C=%d V=%d levels=%d) does not match layer (C=%d V=%d K=%d)", tree->C,
                    tree->V, tree->levels, layer->C, layer->V, layer->K);
    if (N == 0) return LUTNN_OK;
    if (!idx_workspace) return fail(LUTNN_E_NULL, "idx_workspace is NULL");
    hipStream_t s = static_cast<hipStream_t>(stream);
    // validate the lookup before anything is enqueued
    if (layer->table_dtype == LUTNN_TABLE_I4)
        return fail(LUTNN_E_UNSUPPORTED, "the 16-bit index lookup reads INT8 and fp32 tables");
    if (!Y || !layer->table) return fail(LUTNN_E_NULL, "Y or layer->table is NULL");
    if (ldy < layer->M) return fail(LUTNN_E_SHAPE, "ldy=%lld is smaller than M=%d", (long long)ldy, layer->M);
    if (layer->table_dtype == LUTNN_TABLE_I8 && !layer->scale)
        return fail(LUTNN_E_NULL, "an integer table needs layer->scale");
    if (!aligned(idx_workspace, 2) || !aligned(Y, 4) || (layer->bias && !aligned(layer->bias, 4)) ||
        !aligned(layer->table, layer->table_dtype == LUTNN_TABLE_F32 ? 4 : 1))
        return fail(LUTNN_E_ALIGN, "idx_workspace must be 2-byte, Y, bias and an fp32 table 4-byte aligned");
    if (lutnn_status st = hip_result(lutnn::launch_encode_tree16(tree->split_dim, tree->threshold, tree->C,
                                                                 tree->levels, tree->V, X, N, ldx,
                                                                 idx_workspace, s),
                                     "tree encode launch (16-bit leaves)"))
        return st;
    return lookup16_checked(layer, idx_workspace, N, Y, ldy, s);
}

const char* lutnn_status_string(int32_t status) {
    switch (status) {
        case LUTNN_OK: return "LUTNN_OK";
        case LUTNN_E_NULL: return "LUTNN_E_NULL";
        case LUTNN_E_SHAPE: return "LUTNN_E_SHAPE";
        case LUTNN_E_UNSUPPORTED: return "LUTNN_E_UNSUPPORTED";
        case LUTNN_E_ALIGN: return "LUTNN_E_ALIGN";
        case LUTNN_E_HIP: return "LUTNN_E_HIP";
        default: return "LUTNN_E_UNKNOWN";
    }
}

int64_t lutnn_conv2d_rows(const lutnn_conv2d_geom* geom, int64_t B) {
    int64_t rows = -1;
    return check_conv(nullptr, geom, B, nullptr, &rows) == LUTNN_OK ? rows : -1;
}

lutnn_status lutnn_encode_conv2d(const lutnn_layer* layer, const float* input, int64_t B,
                                 const lutnn_conv2d_geom* geom, uint8_t* idx, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    lutnn::ConvGeom g;
    int64_t N = 0;
    if (lutnn_status st = check_conv(layer, geom, B, &g, &N)) return st;
    if (N == 0) return LUTNN_OK;
    if (lutnn_status st = check_conv_input(layer, input)) return st;
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    return hip_result(lutnn::launch_encode_conv(layer->centroids, layer->C, layer->K, layer->V, input, B,
                                                g, idx, static_cast<hipStream_t>(stream)),
                      "convolution encode launch");
}

namespace {
// The shape part of a tree, as the layer view check_conv wants (it reads C and V only).
lutnn_layer shape_of(const lutnn_tree* T) {
    lutnn_layer l{};
    l.C = T->C;
    l.V = T->V;
    l.K = 1 << T->levels;
    l.M = 1;
    return l;
}
lutnn_status check_tree_shape(const lutnn_tree* T) {
    if (!T) return fail(LUTNN_E_NULL, "tree is NULL");
    if (T->reserved != 0) return fail(LUTNN_E_SHAPE, "tree->reserved must be 0");
    if (T->levels < 1 || T->levels > 8)
        return fail(LUTNN_E_SHAPE, "tree->levels=%d outside 1..8 (indices are uint8)", T->levels);
    return check_dims(T->C, 1 << T->levels, T->V, 1);
}
}  // namespace

lutnn_status lutnn_encode_tree_conv2d(const lutnn_tree* tree, const float* input, int64_t B,
                                      const lutnn_conv2d_geom* geom, uint8_t* idx, void* stream) {
    if (lutnn_status st = check_tree_shape(tree)) return st;
    const lutnn_layer shape = shape_of(tree);
    lutnn::ConvGeom g;
    int64_t N = 0;
    if (lutnn_status st = check_conv(&shape, geom, B, &g, &N)) return st;
    if (N == 0) return LUTNN_OK;
    if (!tree->split_dim || !tree->threshold) return fail(LUTNN_E_NULL, "tree->split_dim or tree->threshold is NULL");
    if (!input) return fail(LUTNN_E_NULL, "input is NULL");
    if (!idx) return fail(LUTNN_E_NULL, "idx is NULL");
    if (!aligned(input, 4) || !aligned(tree->split_dim, 4) || !aligned(tree->threshold, 4))
        return fail(LUTNN_E_ALIGN, "input, split_dim and threshold must be 4-byte aligned");
    return hip_result(lutnn::launch_encode_tree_conv(tree->split_dim, tree->threshold, tree->C, tree->levels,
                                                     tree->V, input, B, g, idx, static_cast<hipStream_t>(stream)),
                      "convolution tree encode launch");
}

lutnn_status lutnn_conv2d_tree(const lutnn_layer* layer, const lutnn_tree* tree, const float* input, int64_t B,
                               const lutnn_conv2d_geom* geom, float* Y, int64_t ldy, int32_t variant,
                               uint8_t* idx_workspace, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    if (lutnn_status st = check_tree_shape(tree)) return st;
    if (tree->C != layer->C || tree->V != layer->V || (1 << tree->levels) != layer->K)
        return fail(LUTNN_E_SHAPE, "tree (C=%d V=%d levels=%d) does not match layer (C=%d V=%d K=%d)", tree->C,
                    tree->V, tree->levels, layer->C, layer->V, layer->K);
    lutnn::ConvGeom g;
    int64_t N = 0;
    if (lutnn_status st = check_conv(layer, geom, B, &g, &N)) return st;
    if (N == 0) return LUTNN_OK;
    if (variant == LUTNN_VARIANT_FUSED)
        return fail(LUTNN_E_UNSUPPORTED, "there is no fused kernel for the hash encoder on a convolution");
    if (!idx_workspace) return fail(LUTNN_E_NULL, "idx_workspace is NULL");
    const int v = resolve_lookup_variant(layer, variant, idx_workspace, N);
    if (lutnn_status st = check_lookup(layer, v, idx_workspace, Y, N, ldy)) return st;
    if (lutnn_status st = lutnn_encode_tree_conv2d(tree, input, B, geom, idx_workspace, stream)) return st;
    return do_lookup(layer, v, idx_workspace, N, Y, ldy, static_cast<hipStream_t>(stream));
}

lutnn_status lutnn_conv2d(const lutnn_layer* layer, const float* input, int64_t B,
                          const lutnn_conv2d_geom* geom, float* Y, int64_t ldy, int32_t variant,
                          uint8_t* idx_workspace, void* stream) {
    if (lutnn_status st = check_layer(layer)) return st;
    lutnn::ConvGeom g;
    int64_t N = 0;
    if (lutnn_status st = check_conv(layer, geom, B, &g, &N)) return st;
    if (N == 0) return LUTNN_OK;
    if (lutnn_status st = check_conv_input(layer, input)) return st;
    if (variant == LUTNN_VARIANT_FUSED)
        return fail(LUTNN_E_UNSUPPORTED, "there is no fused convolution kernel");
    if (!idx_workspace) return fail(LUTNN_E_NULL, "lutnn_conv2d needs idx_workspace");
    const int v = resolve_lookup_variant(layer, variant, idx_workspace, N);
    if (lutnn_status st = check_lookup(layer, v, idx_workspace, Y, N, ldy)) return st;
    hipStream_t s = static_cast<hipStream_t>(stream);
    if (lutnn_status st = hip_result(lutnn::launch_encode_conv(layer->centroids, layer->C, layer->K,
                                                               layer->V, input, B, g, idx_workspace, s),
                                     "convolution encode launch"))
        return st;
    return do_lookup(layer, v, idx_workspace, N, Y, ldy, s);
}

int32_t lutnn_auto_variant(const lutnn_layer* layer, const uint8_t* idx, int64_t N) {
    if (!layer) return -1;
    return resolve_lookup_variant(layer, LUTNN_VARIANT_AUTO, idx, N);
}

int32_t lutnn_linear_auto_variant(const lutnn_layer* layer, const uint8_t* idx_workspace, int64_t N) {
    if (!layer) return -1;
    return resolve_linear_variant(layer, LUTNN_VARIANT_AUTO, idx_workspace, N);
}

const char* lutnn_last_error(void) { return g_err; }

#ifndef LUTNN_SOURCE_HASH
#define LUTNN_SOURCE_HASH "unknown"
#endif
const char* lutnn_version(void) { return "0.2.0+" LUTNN_SOURCE_HASH; }

}  // extern "C"
