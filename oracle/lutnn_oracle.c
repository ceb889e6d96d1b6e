/*
 * LUT-NN table-lookup linear operator: plain CPU oracle.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, obviously-correct
 * definition that the GPU library is checked against.  Nothing in the product
 * path may call it, and it shares no code, header, table or constant with the
 * HIP implementation.  All pointers are host pointers.
 *
 * What it computes follows the LUT-NN paper (arXiv 2302.03213):
 *   - sub-vector split  D = C*V                      (Sec. 2.1)
 *   - encoding  g^c(a^c) = argmin_k ||a^c - P^c_k||^2 (Eq. 2)
 *   - table construction h^c(b^c)[k] = P^c_k . b^c    (Eq. 3)
 *   - symmetric scalar quantisation of the table      (Sec. 3.3)
 *   - lookup + aggregation  a.b ~= sum_c T[c][g^c][m] (Eq. 4)
 *   - hash (threshold tree) encoding as the alternative g^c (Sec. 2, Sec. 7)
 *
 * Readings taken where the paper is silent (each is listed in the design
 * document of this repository):
 *   - distances use the direct form of Eq. 2, evaluated in fp32 with one fused
 *     multiply-add per element, v ascending; the arg-min keeps the lowest k on
 *     ties (strict "<" while k ascends);
 *   - weights are B[D][M] row-major as in Table 1, with row stride ldw;
 *   - one scale per layer: s = max|T| / 127 (n = 8), s = 1 for an all-zero
 *     table; q = round-half-even(T / s) clamped to [-127, 127];
 *   - INT8 output  Y = fma((float)acc_int32, s, bias)  (bias optional:
 *     Y = (float)acc * s); fp32-table output is the double-precision sum
 *     rounded once to fp32.
 *
 * Every function here is pinned by tests/test_oracle_*.py against something
 * other than itself (fp64 brute force, library GEMM / cdist, closed forms,
 * the reconstruction identity Y == Xhat . W).  No function is "parity
 * unpinned".
 *
 * Build: gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC (see oracle/build.py).
 * -ffp-contract=off matters: the only fused operations are the explicit fmaf().
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define ORACLE_API __attribute__((visibility("default")))

/* Number of threads the row-parallel loops will use (reported by the bench). */
ORACLE_API int lutnn_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

ORACLE_API void lutnn_oracle_set_threads(int n) {
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
#else
    (void)n;
#endif
}

/*
 * Eq. 3: Tf[c][k][m] = sum_v P[c][k][v] * W[c*V+v][m].
 * P is [C][K][V], W is [D][M] with row stride ldw (elements), Tf is [C][K][M].
 * fp32, v ascending, one fmaf per term.
 */
ORACLE_API void lutnn_oracle_build_table_f32(const float* P, const float* W, int64_t ldw,
                                             int C, int K, int V, int M, float* Tf) {
    for (int c = 0; c < C; ++c)
        for (int k = 0; k < K; ++k)
            for (int m = 0; m < M; ++m) {
                float acc = 0.0f;
                for (int v = 0; v < V; ++v) {
                    float p = P[((size_t)c * K + k) * V + v];
                    float w = W[(size_t)(c * V + v) * (size_t)ldw + m];
                    acc = fmaf(p, w, acc);
                }
                Tf[((size_t)c * K + k) * M + m] = acc;
            }
}

/*
 * Sec. 3.3: r = s*(q - z) with z = 0 and n bits: s = max|value| / (2^(n-1) - 1),
 * q = round(value / s) in [-(2^(n-1) - 1), 2^(n-1) - 1].  One scale for the whole layer table of
 * `count` entries; q is returned one entry per int8 whatever n is (2 <= n <= 8).
 */
ORACLE_API void lutnn_oracle_quantize(const float* Tf, int64_t count, int bits, int8_t* q,
                                      float* scale_out) {
    const float qmax = (float)((1 << (bits - 1)) - 1);
    float amax = 0.0f;
    for (int64_t i = 0; i < count; ++i) {
        float a = fabsf(Tf[i]);
        if (a > amax) amax = a;
    }
    float s = (amax == 0.0f) ? 1.0f : amax / qmax;
    for (int64_t i = 0; i < count; ++i) {
        float r = nearbyintf(Tf[i] / s); /* default rounding mode: half to even */
        if (r > qmax) r = qmax;
        if (r < -qmax) r = -qmax;
        q[i] = (int8_t)r;
    }
    *scale_out = s;
}

/* n = 8, the paper's deployed setting. */
ORACLE_API void lutnn_oracle_quantize_i8(const float* Tf, int64_t count, int8_t* q,
                                         float* scale_out) {
    lutnn_oracle_quantize(Tf, count, 8, q, scale_out);
}

/*
 * Eq. 2: idx[n][c] = argmin_k sum_v (X[n][c*V+v] - P[c][k][v])^2, lowest k on ties.
 * X is [N][D] with row stride ldx, idx is [N][C] uint8 (K <= 256).
 */
ORACLE_API void lutnn_oracle_encode(const float* P, int C, int K, int V, const float* X,
                                    int64_t N, int64_t ldx, uint8_t* idx) {
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float* x = X + (size_t)n * (size_t)ldx;
        for (int c = 0; c < C; ++c) {
            int best = 0;
            float best_d = INFINITY;
            for (int k = 0; k < K; ++k) {
                const float* p = P + ((size_t)c * K + k) * V;
                float d = 0.0f;
                for (int v = 0; v < V; ++v) {
                    float t = x[c * V + v] - p[v];
                    d = fmaf(t, t, d);
                }
                if (d < best_d || k == 0) {
                    best_d = d;
                    best = k;
                }
            }
            idx[(size_t)n * C + c] = (uint8_t)best;
        }
    }
}

/*
 * Hash encoding (Sec. 2, "Hashing for acceleration"; evaluated in Sec. 7): in place of the
 * arg-min of Eq. 2 every codebook owns a balanced binary tree with `levels` levels whose
 * 2^levels leaves are the buckets.  A sub-vector starts at the root; at each node it looks at ONE
 * of its V values (the node's split index) and moves to the right child when that value lies above
 * the node's threshold, to the left child otherwise.  The leaf it reaches, counted from the left,
 * is idx[n][c].
 *
 * Readings: nodes are stored in heap order (node i has children 2i+1 and 2i+2, root 0), so a
 * codebook has 2^levels - 1 (split index, threshold) pairs; "above" is the strict x > t, so a
 * value equal to the threshold, and a NaN, go left.
 *   split_dim  [C][2^levels - 1] int32, every value in [0, V)
 *   threshold  [C][2^levels - 1] fp32
 *   idx        [N][C] uint16: Sec. 7 evaluates trees of up to 12 levels, i.e. 4096 buckets (levels <= 16)
 */
ORACLE_API void lutnn_oracle_encode_tree(const int32_t* split_dim, const float* threshold, int C,
                                         int levels, int V, const float* X, int64_t N,
                                         int64_t ldx, uint16_t* idx) {
    const int nodes = (1 << levels) - 1;
#pragma omp parallel for schedule(static)
    for (int64_t n = 0; n < N; ++n) {
        const float* x = X + (size_t)n * (size_t)ldx;
        for (int c = 0; c < C; ++c) {
            const int32_t* dim = split_dim + (size_t)c * nodes;
            const float* thr = threshold + (size_t)c * nodes;
            int node = 0;
            for (int l = 0; l < levels; ++l) {
                const int right = x[c * V + dim[node]] > thr[node];
                node = 2 * node + 1 + right;
            }
            idx[(size_t)n * C + c] = (uint16_t)(node - nodes);
        }
    }
}

/*
 * Diagnostic: the K squared distances of sub-vector (n, c) in double precision,
 * used by the tests to decide whether an index disagreement is a near-tie.
 */
ORACLE_API void lutnn_oracle_distances_f64(const float* P, int C, int K, int V,
                                           const float* X, int64_t ldx, int64_t n, int c,
                                           double* d_out) {
    (void)C;
    const float* x = X + (size_t)n * (size_t)ldx;
    for (int k = 0; k < K; ++k) {
        const float* p = P + ((size_t)c * K + k) * V;
        double d = 0.0;
        for (int v = 0; v < V; ++v) {
            double t = (double)x[c * V + v] - (double)p[v];
            d += t * t;
        }
        d_out[k] = d;
    }
}

/*
 * Eq. 4 with an INT8 table: acc[n][m] = sum_c q[c][idx[n][c]][m] (exact int32);
 * Y[n][m] = fma((float)acc, s, bias[m]), or (float)acc * s when bias is NULL.
 * q is [C][K][M], Y is [N][M] with row stride ldy; idx is [N][C] uint16 (K up to 65536: the hash
 * encoder's 12-level trees have 4096 buckets, Sec. 7; Eq. 2's indices are widened by the caller).
 * acc_out (nullable) receives the raw int32 sums, [N][M] dense.
 */
ORACLE_API void lutnn_oracle_lookup_i8(const int8_t* q, float scale, const float* bias, int C,
                                       int K, int M, const uint16_t* idx, int64_t N, float* Y,
                                       int64_t ldy, int32_t* acc_out) {
#pragma omp parallel
    {
        int32_t* acc = (int32_t*)malloc((size_t)M * sizeof(int32_t));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            memset(acc, 0, (size_t)M * sizeof(int32_t));
            for (int c = 0; c < C; ++c) {
                const int8_t* row = q + ((size_t)c * K + idx[(size_t)n * C + c]) * M;
                for (int m = 0; m < M; ++m) acc[m] += (int32_t)row[m];
            }
            for (int m = 0; m < M; ++m) {
                float a = (float)acc[m];
                Y[(size_t)n * (size_t)ldy + m] = bias ? fmaf(a, scale, bias[m]) : a * scale;
                if (acc_out) acc_out[(size_t)n * M + m] = acc[m];
            }
        }
        free(acc);
    }
}

/*
 * Eq. 4 with an fp32 table: Y[n][m] = (float)( sum_c (double)Tf[c][idx[n][c]][m] + bias[m] ).
 */
ORACLE_API void lutnn_oracle_lookup_f32(const float* Tf, const float* bias, int C, int K, int M,
                                        const uint16_t* idx, int64_t N, float* Y, int64_t ldy) {
#pragma omp parallel
    {
        double* acc = (double*)malloc((size_t)M * sizeof(double));
#pragma omp for schedule(static)
        for (int64_t n = 0; n < N; ++n) {
            for (int m = 0; m < M; ++m) acc[m] = 0.0;
            for (int c = 0; c < C; ++c) {
                const float* row = Tf + ((size_t)c * K + idx[(size_t)n * C + c]) * M;
                for (int m = 0; m < M; ++m) acc[m] += (double)row[m];
            }
            for (int m = 0; m < M; ++m) {
                double y = bias ? acc[m] + (double)bias[m] : acc[m];
                Y[(size_t)n * (size_t)ldy + m] = (float)y;
            }
        }
        free(acc);
    }
}
