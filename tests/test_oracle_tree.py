"""Pins for the oracle's hash (threshold tree) encoder, Sec. 2 "Hashing for acceleration" and Sec. 7
of arXiv 2302.03213.  None of them walks a tree the way the oracle does: they use sorted-threshold
bucketing (numpy.searchsorted), sign bits, the region each leaf owns, and the balance of a tree
built from medians."""
import numpy as np
import pytest

import lutnn_workloads as wl
import oracle


def _inorder(levels):
    """Heap indices of a complete tree with `levels` levels, listed left to right."""
    out = []

    def visit(i, depth):
        if depth == levels:
            return
        visit(2 * i + 1, depth + 1)
        out.append(i)
        visit(2 * i + 2, depth + 1)

    visit(0, 0)
    return out


@pytest.mark.parametrize("levels", [1, 2, 4, 6, 8, 9, 12])
def test_one_split_index_is_sorted_threshold_bucketing(levels):
    # Every node tests the same value; thresholds sorted along the in-order walk make the tree a
    # binary search, so the bucket is the number of thresholds strictly below the value.
    C, V, N = 5, 4, 700
    rng = np.random.default_rng(levels)
    nodes = (1 << levels) - 1
    X = rng.standard_normal((N, C * V)).astype(np.float32)
    dims = np.empty((C, nodes), np.int32)
    thr = np.empty((C, nodes), np.float32)
    sorted_thr = np.sort(rng.standard_normal((C, nodes)).astype(np.float32), axis=1)
    order = _inorder(levels)
    for c in range(C):
        dims[c, :] = c % V
        thr[c, order] = sorted_thr[c]
    # plant exact ties: a value equal to a threshold stays left of it
    X[:50, 0] = sorted_thr[0, rng.integers(0, nodes, 50)]
    got = oracle.encode_tree(dims, thr, X, V)
    assert got.dtype == (np.uint8 if levels <= 8 else np.uint16)
    for c in range(C):
        want = np.searchsorted(sorted_thr[c], X[:, c * V + c % V], side="left")
        np.testing.assert_array_equal(got[:, c], want)
    if levels > 8:  # 700 points over 512 or 4096 buckets: indices beyond one byte do occur
        assert got.max() > 255


def test_level_l_splits_on_value_l_at_zero_gives_the_sign_bits():
    # Level l looks at value l with threshold 0: the bucket's bits, first level most significant,
    # are the signs of the first `levels` values.
    C, V, levels, N = 3, 4, 4, 500
    rng = np.random.default_rng(7)
    X = rng.standard_normal((N, C * V)).astype(np.float32)
    X[:20] = 0.0  # zero is not above zero: all-left, bucket 0
    nodes = (1 << levels) - 1
    level_of = np.floor(np.log2(np.arange(nodes) + 1)).astype(np.int32)
    dims = np.tile(level_of, (C, 1)).astype(np.int32)
    thr = np.zeros((C, nodes), np.float32)
    got = oracle.encode_tree(dims, thr, X, V)
    Xs = X.reshape(N, C, V)
    want = np.zeros((N, C), np.int64)
    for l in range(levels):
        want |= (Xs[:, :, l] > 0).astype(np.int64) << (levels - 1 - l)
    np.testing.assert_array_equal(got, want)
    assert (got[:20] == 0).all()


def test_twelve_levels_give_the_sign_bits_of_twelve_values():
    # The paper's deepest setting (Sec. 7: 12 levels): level l looks at value l with threshold 0, so
    # the 12-bit bucket is the sign pattern of the sub-vector's first twelve values.
    C, V, levels, N = 2, 16, 12, 3000
    rng = np.random.default_rng(12)
    X = rng.standard_normal((N, C * V)).astype(np.float32)
    nodes = (1 << levels) - 1
    level_of = np.floor(np.log2(np.arange(nodes) + 1)).astype(np.int32)
    dims = np.tile(level_of, (C, 1)).astype(np.int32)
    got = oracle.encode_tree(dims, np.zeros((C, nodes), np.float32), X, V)
    Xs = X.reshape(N, C, V)
    want = np.zeros((N, C), np.int64)
    for l in range(levels):
        want |= (Xs[:, :, l] > 0).astype(np.int64) << (levels - 1 - l)
    assert got.dtype == np.uint16
    np.testing.assert_array_equal(got, want)
    assert len(np.unique(got)) > 1500  # the buckets beyond 255 are really in use


@pytest.mark.parametrize("levels,V", [(3, 4), (4, 9), (5, 2), (9, 3), (12, 32)])
def test_each_point_lies_in_the_region_of_exactly_the_leaf_reported(levels, V):
    # Set definition instead of a walk: leaf b owns the points that satisfy every inequality on the
    # path from the root to b.  The regions partition the space, and the oracle's answer must be
    # the one region containing the point.
    C, N = (4, 300) if levels <= 8 else (2, 120)
    dims, thr = wl.random_tree(C, V, levels, seed=11)
    rng = np.random.default_rng(3)
    X = rng.standard_normal((N, C * V)).astype(np.float32)
    got = oracle.encode_tree(dims, thr, X, V)
    nodes = (1 << levels) - 1
    Xs = X.reshape(N, C, V)
    for c in range(C):
        member = np.zeros((N, 1 << levels), bool)
        for b in range(1 << levels):
            inside = np.ones(N, bool)
            child = b + nodes  # heap index of the leaf
            while child > 0:
                parent = (child - 1) // 2
                above = Xs[:, c, dims[c, parent]] > thr[c, parent]
                inside &= above if child == 2 * parent + 2 else ~above
                child = parent
            member[:, b] = inside
        assert (member.sum(axis=1) == 1).all()
        np.testing.assert_array_equal(got[:, c], member.argmax(axis=1))


def test_tree_of_medians_fills_its_buckets_evenly():
    # A tree whose every node splits its own points at their median (the balanced tree of the cited
    # hashing work) must put N / 2^levels points in every bucket when N is a multiple of it and the
    # values are distinct.  Built here by recursion over point sets; a heap-order or child-order
    # slip in the oracle sends points through the wrong thresholds and unbalances the buckets.
    C, V, levels = 3, 4, 4
    N = 64 << levels
    rng = np.random.default_rng(5)
    X = rng.standard_normal((N, C * V)).astype(np.float32)
    nodes = (1 << levels) - 1
    dims = np.zeros((C, nodes), np.int32)
    thr = np.zeros((C, nodes), np.float32)
    Xs = X.reshape(N, C, V)
    for c in range(C):
        def build(node, rows, depth):
            if depth == levels:
                return
            d = int(rng.integers(0, V))
            vals = np.sort(Xs[rows, c, d])
            half = len(rows) // 2
            t = vals[half - 1]  # the lower half is "not above t"
            assert vals[half] > t
            dims[c, node], thr[c, node] = d, t
            above = Xs[rows, c, d] > t
            build(2 * node + 1, rows[~above], depth + 1)
            build(2 * node + 2, rows[above], depth + 1)

        build(0, np.arange(N), 0)
    got = oracle.encode_tree(dims, thr, X, V)
    for c in range(C):
        np.testing.assert_array_equal(np.bincount(got[:, c], minlength=1 << levels),
                                      np.full(1 << levels, N >> levels))


def test_nan_goes_left_and_infinity_goes_right():
    C, V, levels = 2, 4, 4
    dims, thr = wl.random_tree(C, V, levels, seed=2)
    X = np.full((3, C * V), np.nan, np.float32)
    assert (oracle.encode_tree(dims, thr, X, V) == 0).all()
    X = np.full((3, C * V), np.inf, np.float32)
    assert (oracle.encode_tree(dims, thr, X, V) == (1 << levels) - 1).all()
