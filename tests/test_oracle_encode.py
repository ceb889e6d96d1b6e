"""Pins for the oracle's encoder (arXiv 2302.03213, Eq. 2) against things other than itself."""
import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle


def brute_force_f64(P, X):
    """argmin_k ||x - p_k||^2 in double, first minimum, written straight from Eq. 2."""
    C, K, V = P.shape
    N = X.shape[0]
    Xs = X.reshape(N, C, V).astype(np.float64)
    d = ((Xs[:, :, None, :] - P[None].astype(np.float64)) ** 2).sum(-1)  # [N, C, K]
    return d.argmin(-1).astype(np.uint8), d


def dyadic(rng, shape, lo=-16, hi=16, den=8.0):
    """Small dyadic rationals: every fp32 sub / fma on them is exact, so fp32 == fp64."""
    return (rng.integers(lo, hi + 1, size=shape) / den).astype(np.float32)


@pytest.mark.parametrize("N,C,K,V", [(8, 3, 16, 9), (5, 2, 7, 4), (7, 4, 16, 2), (3, 1, 5, 1),
                                     (6, 2, 256, 3)])
def test_exact_arithmetic_matches_brute_force(N, C, K, V):
    # Dyadic inputs: no rounding anywhere, so the fp32 oracle must equal the fp64 brute force
    # bit for bit, exact ties included (many occur on this coarse grid -> lowest index).
    rng = np.random.default_rng(100 + N + K)
    P = dyadic(rng, (C, K, V))
    X = dyadic(rng, (N, C * V))
    ref, d = brute_force_f64(P, X)
    got = oracle.encode(P, X)
    assert got.dtype == np.uint8 and got.shape == (N, C)
    np.testing.assert_array_equal(got, ref)


def test_exact_ties_take_lowest_index():
    # V = 1, centroids +1 and -1 (in both orders), x = 0: equidistant -> index 0.
    P = np.array([[[1.0], [-1.0]], [[-1.0], [1.0]]], dtype=np.float32)  # C=2, K=2, V=1
    X = np.zeros((3, 2), dtype=np.float32)
    np.testing.assert_array_equal(oracle.encode(P, X), np.zeros((3, 2), np.uint8))
    # Duplicated centroid: the lower of the two equal indices wins.
    rng = np.random.default_rng(1)
    P = rng.standard_normal((2, 6, 4)).astype(np.float32)
    P[:, 4] = P[:, 1]
    X = np.concatenate([P[0, 1], P[1, 4]])[None].astype(np.float32)
    np.testing.assert_array_equal(oracle.encode(P, X), [[1, 1]])


def test_random_inputs_match_cdist_up_to_near_ties():
    # Library routine: torch.cdist in fp64, squared, argmin.  Any disagreement must be a near-tie
    # (relative gap of the two fp64 distances below 1e-6).
    w = wl.make_layer("t", 257, 5, 16, 9, 8, "f32", seed=3)
    got = oracle.encode(w.P, w.X)
    Xs = torch.from_numpy(w.X.reshape(w.N, w.C, w.V)).double().permute(1, 0, 2)  # [C, N, V]
    d = torch.cdist(Xs, torch.from_numpy(w.P).double()) ** 2  # [C, N, K]
    ref = d.argmin(-1).t().numpy()
    bad = np.argwhere(got != ref)
    for n, c in bad:
        dd = oracle.distances_f64(w.P, w.X, n, c)
        a, b = dd[got[n, c]], dd[ref[n, c]]
        assert abs(a - b) <= 1e-6 * max(a, b)
    assert len(bad) <= 2


def test_distances_f64_matches_numpy():
    w = wl.make_layer("t", 4, 3, 16, 9, 8, "f32", seed=5)
    _, d = brute_force_f64(w.P, w.X)
    for n in range(w.N):
        for c in range(w.C):
            np.testing.assert_allclose(oracle.distances_f64(w.P, w.X, n, c), d[n, c], rtol=1e-13)


def test_inputs_that_are_centroids_encode_to_themselves():
    w = wl.make_layer("t", 1, 7, 16, 4, 8, "f32", seed=7)
    X, choice = wl.rows_from_centroids(w.P, 64, seed=8)
    np.testing.assert_array_equal(oracle.encode(w.P, X), choice)


def test_single_centroid_gives_zero():
    w = wl.make_layer("t", 9, 3, 1, 4, 8, "f32", seed=9)
    np.testing.assert_array_equal(oracle.encode(w.P, w.X), np.zeros((9, 3), np.uint8))


def test_scalar_subvectors_reduce_to_searchsorted():
    # V = 1: the nearest of K sorted scalars is found by bisecting on the midpoints.
    rng = np.random.default_rng(11)
    C, K, N = 4, 16, 200
    P = np.sort(rng.standard_normal((C, K)).astype(np.float32), axis=1)[..., None]
    X = (rng.standard_normal((N, C)) * 1.5).astype(np.float32)
    got = oracle.encode(P, X)
    for c in range(C):
        cent = P[c, :, 0].astype(np.float64)
        mid = (cent[1:] + cent[:-1]) / 2
        ref = np.searchsorted(mid, X[:, c].astype(np.float64), side="left")
        safe = np.min(np.abs(X[:, c, None].astype(np.float64) - mid[None]), axis=1) > 1e-6
        np.testing.assert_array_equal(got[safe, c], ref[safe])
        assert safe.sum() > N * 0.9


def test_permuting_centroids_permutes_indices():
    w = wl.make_layer("t", 50, 6, 16, 2, 8, "f32", seed=13)
    rng = np.random.default_rng(14)
    base = oracle.encode(w.P, w.X)
    P2 = np.empty_like(w.P)
    perms = []
    for c in range(w.C):
        perm = rng.permutation(w.K)  # new position j holds old centroid perm[j]
        P2[c] = w.P[c, perm]
        perms.append(np.argsort(perm))  # old index -> new index
    got = oracle.encode(P2, w.X)
    for c in range(w.C):
        np.testing.assert_array_equal(got[:, c], perms[c][base[:, c]])


def test_subvector_split_uses_contiguous_columns():
    # Sec. 2.1: sub-vector c is columns [cV, (c+1)V).  Make only one codebook's columns matter.
    C, K, V = 3, 4, 2
    P = np.zeros((C, K, V), dtype=np.float32)
    P[1] = [[0, 0], [10, 0], [0, 10], [10, 10]]
    X = np.zeros((4, C * V), dtype=np.float32)
    X[:, 2:4] = [[1, 1], [9, 1], [1, 9], [9, 9]]
    got = oracle.encode(P, X)
    np.testing.assert_array_equal(got[:, 1], [0, 1, 2, 3])
    np.testing.assert_array_equal(got[:, [0, 2]], 0)


def test_row_stride_and_empty():
    w = wl.make_layer("t", 0, 3, 16, 4, 8, "f32", seed=1)
    assert oracle.encode(w.P, w.X).shape == (0, 3)
