"""Pins for the oracle's table construction (Eq. 3), quantisation (Sec. 3.3), lookup (Eq. 4) and
the end-to-end operator of arXiv 2302.03213, each against something other than the oracle."""
import numpy as np
import pytest

import lutnn_workloads as wl
import oracle


# ---------------------------------------------------------------- Eq. 3: table construction
@pytest.mark.parametrize("C,K,V,M", [(3, 16, 9, 5), (4, 7, 2, 11), (2, 16, 4, 33), (1, 1, 1, 1)])
def test_build_table_matches_batched_gemm(C, K, V, M):
    w = wl.make_layer("t", 1, C, K, V, M, "f32", seed=21)
    Tf = oracle.build_table_f32(w.P, w.W)
    assert Tf.shape == (C, K, M) and Tf.dtype == np.float32
    ref = np.einsum("ckv,cvm->ckm", w.P.astype(np.float64),
                    w.W.reshape(C, V, M).astype(np.float64))
    np.testing.assert_allclose(Tf, ref, rtol=1e-5, atol=1e-6)


def test_build_table_entry_is_a_dot_product():
    w = wl.make_layer("t", 1, 3, 16, 9, 5, "f32", seed=22)
    Tf = oracle.build_table_f32(w.P, w.W)
    for c, k, m in [(0, 0, 0), (1, 7, 3), (2, 15, 4)]:
        ref = np.dot(w.P[c, k].astype(np.float64), w.W[c * 9:(c + 1) * 9, m].astype(np.float64))
        assert abs(Tf[c, k, m] - ref) <= 1e-6 * max(1.0, abs(ref))


def test_build_table_exact_on_dyadic_inputs():
    rng = np.random.default_rng(23)
    C, K, V, M = 3, 5, 4, 6
    P = (rng.integers(-8, 9, (C, K, V)) / 4.0).astype(np.float32)
    W = (rng.integers(-8, 9, (C * V, M)) / 4.0).astype(np.float32)
    ref = np.einsum("ckv,cvm->ckm", P.astype(np.float64), W.reshape(C, V, M).astype(np.float64))
    np.testing.assert_array_equal(oracle.build_table_f32(P, W).astype(np.float64), ref)


# ---------------------------------------------------------------- Sec. 3.3: quantisation
def test_quantize_closed_forms():
    w = wl.make_layer("t", 1, 5, 16, 4, 37, "i8", seed=31)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize_i8(Tf)
    amax = np.abs(Tf).max()
    assert q.dtype == np.int8 and q.shape == Tf.shape
    assert s == np.float32(amax) / np.float32(127.0)  # s = max|value| / (2^(n-1) - 1), n = 8
    where = np.unravel_index(np.abs(Tf).argmax(), Tf.shape)
    assert abs(int(q[where])) == 127  # the extreme entry lands on the end of the range
    assert np.sign(q[where]) == np.sign(Tf[where])
    assert q.min() >= -127 and q.max() <= 127
    # r = s*q reconstructs every entry to within half a step (plus fp32 slack)
    err = np.abs(q.astype(np.float64) * float(s) - Tf.astype(np.float64))
    assert err.max() <= float(s) * 0.5 * (1 + 1e-5)


def test_quantize_rounds_half_to_even_and_handles_zero_table():
    # s = 127/127 = 1 -> q = rint(T): halves go to the even neighbour.
    Tf = np.array([127.0, 0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.49, -126.5], dtype=np.float32)
    q, s = oracle.quantize_i8(Tf)
    assert s == np.float32(1.0)
    np.testing.assert_array_equal(q, [127, 0, 2, 2, 0, -2, -2, 3, -126])
    q, s = oracle.quantize_i8(np.zeros((2, 3, 4), np.float32))
    assert s == np.float32(1.0) and not q.any()


@pytest.mark.parametrize("bits", [4, 8, 6])
def test_quantize_n_bits_closed_forms(bits):
    """Sec. 3.3 with n bits: s = max|value| / (2^(n-1) - 1); checked for n = 4 (the INT4 table of
    Sec. 6.4) against the same closed forms as n = 8."""
    qmax = 2 ** (bits - 1) - 1
    w = wl.make_layer("t", 1, 5, 16, 4, 37, "i8", seed=34)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize(Tf, bits)
    assert s == np.float32(np.abs(Tf).max()) / np.float32(qmax)
    where = np.unravel_index(np.abs(Tf).argmax(), Tf.shape)
    assert int(q[where]) == qmax * int(np.sign(Tf[where]))
    assert q.min() >= -qmax and q.max() <= qmax
    err = np.abs(q.astype(np.float64) * float(s) - Tf.astype(np.float64))
    assert err.max() <= float(s) * 0.5 * (1 + 1e-5)
    # independent formula, evaluated in double where the fp32 quotient is far from a half
    ratio = Tf.astype(np.float64) / float(s)
    safe = np.abs(ratio - np.floor(ratio) - 0.5) > 1e-3
    np.testing.assert_array_equal(q[safe], np.rint(ratio[safe]).astype(np.int8))
    if bits == 8:
        q8, s8 = oracle.quantize_i8(Tf)
        assert s8 == s
        np.testing.assert_array_equal(q8, q)


def test_quantize_4_bits_half_to_even_and_nibble_packing():
    Tf = np.array([[7.0, 0.5, 1.5, 2.5, -0.5], [-1.5, -2.5, 3.49, -6.5, -7.0]], dtype=np.float32)
    q, s = oracle.quantize(Tf, 4)
    assert s == np.float32(1.0)
    np.testing.assert_array_equal(q, [[7, 0, 2, 2, 0], [-2, -2, 3, -6, -7]])
    packed = oracle.pack_nibbles(q)  # even column in the low nibble, two's complement, zero padded
    assert packed.dtype == np.uint8 and packed.shape == (2, 3)
    np.testing.assert_array_equal(packed, [[0x07, 0x22, 0x00], [0xEE, 0xA3, 0x09]])
    q0, s0 = oracle.quantize(np.zeros((3, 4), np.float32), 4)
    assert s0 == np.float32(1.0) and not q0.any()


def test_quantize_is_symmetric():
    w = wl.make_layer("t", 1, 3, 16, 2, 9, "i8", seed=33)
    Tf = oracle.build_table_f32(w.P, w.W)
    q1, s1 = oracle.quantize_i8(Tf)
    q2, s2 = oracle.quantize_i8(-Tf)
    assert s1 == s2
    np.testing.assert_array_equal(q1.astype(np.int32), -q2.astype(np.int32))


# ---------------------------------------------------------------- Eq. 4: lookup + aggregation
def onehot(idx, K):
    N, C = idx.shape
    G = np.zeros((N, C * K), dtype=np.int64)
    G[np.arange(N)[:, None], np.arange(C)[None] * K + idx] = 1
    return G


@pytest.mark.parametrize("N,C,K,M", [(9, 5, 16, 7), (4, 3, 4, 130), (1, 1, 1, 1), (33, 17, 16, 3)])
def test_lookup_i8_is_onehot_times_table(N, C, K, M):
    # Eq. 4 literally: onehot(g) [N x CK] @ T [CK x M] with an exact int64 library GEMM.
    q = wl.random_table_i8(C, K, M, seed=41)
    idx = wl.random_indices(N, C, K, seed=42)
    rng = np.random.default_rng(43)
    bias = rng.standard_normal(M).astype(np.float32)
    s = np.float32(0.0123)
    ref_acc = onehot(idx, K) @ q.reshape(C * K, M).astype(np.int64)
    Y, acc = oracle.lookup_i8(q, s, idx, bias, return_acc=True)
    np.testing.assert_array_equal(acc.astype(np.int64), ref_acc)
    ref_y = ref_acc.astype(np.float64) * float(s) + bias.astype(np.float64)
    np.testing.assert_allclose(Y, ref_y, rtol=1e-6, atol=1e-6)
    Y0 = oracle.lookup_i8(q, s, idx, None)
    np.testing.assert_array_equal(Y0, (ref_acc.astype(np.float32) * s).astype(np.float32))


def test_lookup_i8_naive_triple_loop():
    C, K, M, N = 4, 5, 6, 3
    q = wl.random_table_i8(C, K, M, seed=44)
    idx = wl.random_indices(N, C, K, seed=45)
    _, acc = oracle.lookup_i8(q, 1.0, idx, None, return_acc=True)
    for n in range(N):
        for m in range(M):
            tot = 0
            for c in range(C):
                tot += int(q[c, idx[n, c], m])
            assert acc[n, m] == tot


def test_lookup_i8_extreme_sum_is_exact():
    # Every entry +127 (or -127) over C = 1536 codebooks: |acc| = 195072, no 16-bit wrap.
    C, K, M = 1536, 2, 3
    q = np.full((C, K, M), 127, np.int8)
    q[:, 1] = -127
    idx = np.zeros((2, C), np.uint8)
    idx[1] = 1
    _, acc = oracle.lookup_i8(q, 1.0, idx, None, return_acc=True)
    np.testing.assert_array_equal(acc[0], 127 * C)
    np.testing.assert_array_equal(acc[1], -127 * C)


@pytest.mark.parametrize("N,C,K,M", [(9, 5, 16, 7), (4, 3, 4, 130)])
def test_lookup_f32_is_onehot_times_table(N, C, K, M):
    rng = np.random.default_rng(46)
    Tf = rng.standard_normal((C, K, M)).astype(np.float32)
    bias = rng.standard_normal(M).astype(np.float32)
    idx = wl.random_indices(N, C, K, seed=47)
    ref = onehot(idx, K).astype(np.float64) @ Tf.reshape(C * K, M).astype(np.float64)
    np.testing.assert_allclose(oracle.lookup_f32(Tf, idx, None), ref, rtol=1e-6, atol=1e-7)
    np.testing.assert_allclose(oracle.lookup_f32(Tf, idx, bias), ref + bias, rtol=1e-6, atol=1e-7)


def test_lookup_single_centroid_sums_the_table():
    rng = np.random.default_rng(48)
    Tf = rng.standard_normal((6, 1, 10)).astype(np.float32)
    idx = np.zeros((4, 6), np.uint8)
    Y = oracle.lookup_f32(Tf, idx, None)
    np.testing.assert_allclose(Y, np.broadcast_to(Tf.astype(np.float64).sum(0)[0], (4, 10)),
                               rtol=1e-6)


def test_lookup_is_linear_in_the_table():
    C, K, M, N = 5, 16, 12, 20
    qa = (wl.random_table_i8(C, K, M, seed=49) // 2).astype(np.int8)
    qb = (wl.random_table_i8(C, K, M, seed=50) // 2).astype(np.int8)
    idx = wl.random_indices(N, C, K, seed=51)
    _, a = oracle.lookup_i8(qa, 1.0, idx, None, return_acc=True)
    _, b = oracle.lookup_i8(qb, 1.0, idx, None, return_acc=True)
    _, ab = oracle.lookup_i8((qa + qb).astype(np.int8), 1.0, idx, None, return_acc=True)
    np.testing.assert_array_equal(ab, a + b)


# ---------------------------------------------------------------- end to end
@pytest.mark.parametrize("C,K,V,M", [(6, 16, 4, 10), (3, 16, 9, 7), (8, 5, 2, 17)])
def test_reconstruction_identity(C, K, V, M):
    # Exact algebra behind Eq. 3 + Eq. 4: the fp32-table output equals Xhat . W (+ bias), where
    # Xhat replaces every sub-vector by its chosen centroid.
    w = wl.make_layer("t", 40, C, K, V, M, "f32", seed=61)
    Tf = oracle.build_table_f32(w.P, w.W)
    idx = oracle.encode(w.P, w.X)
    Xhat = w.P[np.arange(C)[None], idx].reshape(w.N, C * V).astype(np.float64)
    ref = Xhat @ w.W.astype(np.float64) + w.bias.astype(np.float64)
    np.testing.assert_allclose(oracle.linear_f32(w.P, Tf, w.X, w.bias), ref, rtol=1e-5, atol=1e-5)


def test_centroid_inputs_reproduce_the_exact_matmul():
    # If every sub-vector IS a centroid, the approximation of Eq. 4 is exact: Y == X . W + bias.
    w = wl.make_layer("t", 1, 12, 16, 4, 20, "f32", seed=62)
    X, _ = wl.rows_from_centroids(w.P, 64, seed=63)
    Tf = oracle.build_table_f32(w.P, w.W)
    ref = X.astype(np.float64) @ w.W.astype(np.float64) + w.bias.astype(np.float64)
    np.testing.assert_allclose(oracle.linear_f32(w.P, Tf, X, w.bias), ref, rtol=1e-5, atol=1e-5)


def test_int8_output_within_quantisation_bound_of_fp32_output():
    w = wl.make_layer("t", 50, 16, 16, 4, 24, "i8", seed=64)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize_i8(Tf)
    y8 = oracle.linear_i8(w.P, q, s, w.X, w.bias).astype(np.float64)
    yf = oracle.linear_f32(w.P, Tf, w.X, w.bias).astype(np.float64)
    assert np.abs(y8 - yf).max() <= w.C * float(s) / 2 * (1 + 1e-4) + 1e-5


def test_approximation_improves_with_kmeans_like_centroids():
    # Sanity of the whole method (Sec. 2.2): with centroids drawn from the data the LUT output is
    # closer to X.W than with unrelated centroids, and exact for the rows the centroids came from.
    w = wl.make_layer("t", 300, 8, 16, 2, 16, "f32", seed=65)
    exact = w.X.astype(np.float64) @ w.W.astype(np.float64)
    P_data = wl.centroids_from_rows(w.X, w.C, w.K, w.V, seed=66)
    far = (w.P + 50.0).astype(np.float32)
    e_data = np.abs(oracle.linear_f32(P_data, oracle.build_table_f32(P_data, w.W), w.X) - exact)
    e_far = np.abs(oracle.linear_f32(far, oracle.build_table_f32(far, w.W), w.X) - exact)
    assert e_data.mean() < 0.2 * e_far.mean()
