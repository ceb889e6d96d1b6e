"""GPU parity of the hash (threshold tree) encoder, Sec. 2 and Sec. 7 of arXiv 2302.03213, against
the CPU oracle through the C ABI.  The walk is comparisons only, so the bar is bit-exact indices;
with an INT8 table the outputs of lutnn_linear_tree are bit-exact too."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle
from gpu_util import OracleLayer, dev, host

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return lut_mod


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield


def device_tree(lut, dims, thr, V):
    return lut.LutTree(dev(dims), dev(thr), V)


TREE_SHAPES = [
    # N, C, V, levels
    (1, 1, 4, 4), (63, 5, 4, 4), (64, 32, 4, 4), (65, 33, 4, 4), (200, 128, 4, 4), (2100, 70, 4, 4),
    (130, 64, 9, 4), (77, 17, 9, 4), (300, 384, 2, 4), (129, 70, 2, 3), (100, 9, 1, 4),
    (100, 35, 3, 2), (100, 20, 8, 4), (50, 3, 16, 4), (40, 2, 32, 4), (300, 24, 32, 5),
    (200, 48, 16, 6), (150, 12, 4, 1), (150, 40, 4, 6), (70, 33, 4, 7), (90, 70, 4, 8),
    (130, 9, 9, 8), (60, 66, 1, 8), (90, 130, 2, 8), (64, 5, 32, 8),
    # sub-vector lengths without a tiled kernel
    (90, 7, 5, 4), (33, 4, 7, 8), (41, 3, 12, 3),
    # grids of 1024 workgroups and more take the full tile width
    (4160, 600, 4, 4), (4100, 512, 4, 8), (2100, 320, 9, 4),
    # thousands of tiles: ragged rows and codebooks, byte-wise index stores, deep trees on narrow
    # tiles, V = 9
    (8250, 1030, 4, 4), (8250, 1030, 4, 8), (16500, 300, 9, 4), (5000, 2048, 2, 5),
]


@pytest.mark.parametrize("N,C,V,levels", TREE_SHAPES)
def test_encode_tree_matches_oracle(lut, N, C, V, levels):
    seed = N * 31 + C * 7 + V + levels
    dims, thr = wl.random_tree(C, V, levels, seed=seed, level_dims=bool(seed & 1))
    X = wl.make_layer("t", N, C, 1 << levels, V, 1, "i8", seed=seed).X
    ref = oracle.encode_tree(dims, thr, X, V)
    got = host(lut.encode_tree(device_tree(lut, dims, thr, V), dev(X)))
    np.testing.assert_array_equal(got, ref)
    assert len(np.unique(ref)) > 1 or N * C < 4  # the trees do spread the rows over buckets


def test_encode_tree_values_on_thresholds_nan_and_infinities(lut):
    N, C, V, levels = 300, 20, 4, 4
    dims, thr = wl.random_tree(C, V, levels, seed=9)
    X = wl.make_layer("t", N, C, 16, V, 1, "i8", seed=9).X.copy()
    rng = np.random.default_rng(1)
    # a third of the values sit exactly on a threshold of their own codebook
    Xs = X.reshape(N, C, V)
    for c in range(C):
        pick = rng.random((N, V)) < 0.33
        Xs[:, c, :][pick] = thr[c, rng.integers(0, thr.shape[1], pick.sum())]
    X[5] = np.nan
    X[6] = np.inf
    X[7] = -np.inf
    X[8, ::3] = np.nan
    ref = oracle.encode_tree(dims, thr, X, V)
    got = host(lut.encode_tree(device_tree(lut, dims, thr, V), dev(X)))
    np.testing.assert_array_equal(got, ref)
    assert (got[5] == 0).all() and (got[6] == 15).all() and (got[7] == 0).all()


def test_encode_tree_row_stride_misaligned_rows_and_odd_index_address(lut):
    N, C, V, levels = 130, 33, 4, 4
    dims, thr = wl.random_tree(C, V, levels, seed=3)
    X = wl.make_layer("t", N, C, 16, V, 1, "i8", seed=3).X
    ref = oracle.encode_tree(dims, thr, X, V)
    tree = device_tree(lut, dims, thr, V)
    big = torch.zeros((N, C * V + 7), dtype=torch.float32, device="cuda")
    big[:, 3:3 + C * V] = dev(X)
    np.testing.assert_array_equal(host(lut.encode_tree(tree, big[:, 3:3 + C * V])), ref)
    # index matrix at an odd byte address: the byte-wise store path
    raw = torch.zeros(N * C + 1, dtype=torch.uint8, device="cuda")
    out = raw[1:].view(N, C)
    lut.encode_tree(tree, dev(X), out=out)
    np.testing.assert_array_equal(host(out), ref)
    assert int(raw[0]) == 0


def test_encode_tree_clamps_split_indices_outside_the_subvector(lut):
    N, C, V, levels = 100, 6, 4, 4
    dims, thr = wl.random_tree(C, V, levels, seed=4)
    bad = dims.copy()
    bad[dims == 0] = -5
    bad[dims == V - 1] = V + 100
    X = wl.make_layer("t", N, C, 16, V, 1, "i8", seed=4).X
    ref = oracle.encode_tree(dims, thr, X, V)  # the clamped tree
    got = host(lut.encode_tree(device_tree(lut, bad, thr, V), dev(X)))
    np.testing.assert_array_equal(got, ref)
    # and on the kernel without tiles
    V2 = 5
    dims2, thr2 = wl.random_tree(C, V2, levels, seed=5)
    bad2 = dims2.copy()
    bad2[dims2 == 0] = -1
    bad2[dims2 == V2 - 1] = 1 << 20
    X2 = wl.make_layer("t", N, C, 16, V2, 1, "i8", seed=5).X
    got2 = host(lut.encode_tree(device_tree(lut, bad2, thr2, V2), dev(X2)))
    np.testing.assert_array_equal(got2, oracle.encode_tree(dims2, thr2, X2, V2))


LINEAR_TREE_SHAPES = [
    # N, C, V, levels, M, dtype
    (130, 32, 4, 4, 96, "i8"), (600, 64, 4, 4, 320, "i8"), (77, 17, 9, 4, 64, "i8"),
    (100, 24, 32, 4, 50, "i8"), (90, 12, 4, 3, 40, "i8"), (64, 8, 4, 6, 33, "i8"),
    (130, 32, 4, 4, 96, "f32"), (50, 6, 2, 8, 20, "f32"),
    # shapes of the one-launch kernel: one row of a BERT layer (codebooks shared out over sixteen
    # and over four wavefronts), rows narrower than a wavefront, whole rows per wavefront, trees
    # walked from memory (levels != 4), every sub-vector length it unrolls
    (1, 384, 2, 4, 768, "i8"), (3, 384, 2, 4, 2304, "i8"), (5, 128, 4, 4, 512, "f32"),
    (200, 32, 4, 4, 64, "i8"), (7, 70, 4, 3, 260, "i8"), (9, 16, 32, 5, 256, "f32"),
    (4, 24, 16, 8, 128, "i8"), (33, 20, 8, 4, 1024, "i8"), (70, 10, 1, 4, 32, "f32"),
    (6, 12, 3, 2, 16, "i8"), (130, 64, 9, 4, 128, "i8"), (2, 530, 2, 4, 300, "f32"),
]


def one_launch_supported(V, M):
    return V in (1, 2, 3, 4, 8, 9, 16, 32) and M % 4 == 0 and (M >= 256 or 64 % (M // 4) == 0)


@pytest.mark.parametrize("N,C,V,levels,M,dtype", LINEAR_TREE_SHAPES)
def test_linear_tree_matches_oracle(lut, N, C, V, levels, M, dtype):
    K = 1 << levels
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=N + C + M)
    dims, thr = wl.random_tree(C, V, levels, seed=N + C)
    ol = OracleLayer(w)  # table rows = bucket prototypes (w.P) times the weights
    idx_ref = oracle.encode_tree(dims, thr, w.X, V)
    ref = ol.lookup(idx_ref)
    tree = device_tree(lut, dims, thr, V)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8 if dtype == "i8" else lut.TABLE_F32,
                            bias=dev(w.bias))
    variants = ["auto", "lds", "mfma"] if dtype == "i8" and K <= 16 else ["auto", "lds"]
    if dtype == "i8" and K <= 16 and C % 32 == 0:
        variants.append("smfmac")
    if one_launch_supported(V, M):
        variants.append("fused")
    for v in variants:
        got = host(lut.linear_tree(layer, tree, dev(w.X), v))
        if dtype == "i8":
            np.testing.assert_array_equal(got, ref, err_msg=v)
        else:
            np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-4, err_msg=v)


def test_fc_large_with_the_hash_encoder_sampled_rows(lut):
    # the benchmark workload with 4-level trees in front of the same INT8 table, in the launch
    # configuration bench.py --tree times; the oracle's lookup runs on a sample of rows
    w = wl.fc_large(0)
    dims, thr = wl.random_tree(w.C, w.V, 4, seed=0)
    ol = OracleLayer(w)
    idx_ref = oracle.encode_tree(dims, thr, w.X, w.V)
    tree = device_tree(lut, dims, thr, w.V)
    Xd = dev(w.X)
    np.testing.assert_array_equal(host(lut.encode_tree(tree, Xd)), idx_ref)
    rng = np.random.default_rng(0)
    rows = np.sort(rng.choice(w.N, size=256, replace=False))
    rows[-1] = w.N - 1
    ref = ol.lookup(idx_ref[rows])
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    got = host(lut.linear_tree(layer, tree, Xd, "auto"))[rows]
    np.testing.assert_array_equal(got, ref)


def test_tree_error_statuses_and_empty_batch(lut):
    C, V, levels = 4, 4, 4
    dims, thr = wl.random_tree(C, V, levels, seed=1)
    tree = device_tree(lut, dims, thr, V)
    X = dev(np.zeros((8, C * V), np.float32))
    assert lut.encode_tree(tree, X[:0]).shape == (0, C)
    w = wl.make_layer("t", 8, C, 8, V, 16, "i8", seed=1)  # K = 8 != 2^4
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear_tree(layer, tree, X)
    assert e.value.status == 2
    w16 = wl.make_layer("t", 8, C, 16, V, 18, "i8", seed=1)  # M % 4 != 0: no one-launch kernel
    layer16 = lut.build_table(dev(w16.P), dev(w16.W), lut.TABLE_I8)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear_tree(layer16, tree, X, "fused")
    assert e.value.status == 3
    w4 = wl.make_layer("t", 8, C, 16, V, 16, "i4", seed=1)  # nor for INT4 storage
    layer4 = lut.build_table(dev(w4.P), dev(w4.W), lut.TABLE_I4)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear_tree(layer4, tree, X, "fused")
    assert e.value.status == 3


def test_linear_tree_one_launch_strides_no_bias_and_no_workspace(lut):
    # row strides on X and Y, a layer without bias; the one-launch kernel takes no index workspace
    # (the binding passes NULL for "fused")
    N, C, V, levels, M = 6, 96, 4, 4, 512
    w = wl.make_layer("t", N, C, 16, V, M, "i8", seed=77)
    dims, thr = wl.random_tree(C, V, levels, seed=77)
    ref = OracleLayer(w).lookup(oracle.encode_tree(dims, thr, w.X, V), bias=None)
    tree = device_tree(lut, dims, thr, V)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8)
    Xbig = torch.zeros((N, C * V + 12), dtype=torch.float32, device="cuda")
    Xbig[:, 4:4 + C * V] = dev(w.X)
    Ybig = torch.full((N, M + 8), -7.0, dtype=torch.float32, device="cuda")
    lut.linear_tree(layer, tree, Xbig[:, 4:4 + C * V], "fused", out=Ybig[:, :M])
    np.testing.assert_array_equal(host(Ybig[:, :M]), ref)
    assert (host(Ybig[:, M:]) == -7.0).all()
    # AUTO takes the same kernel on this shape, and equals the two launches
    assert lut.linear_auto_variant(layer, N) == "fused"
    np.testing.assert_array_equal(host(lut.linear_tree(layer, tree, dev(w.X), "auto")), ref)
    np.testing.assert_array_equal(host(lut.linear_tree(layer, tree, dev(w.X), "lds")), ref)


@pytest.mark.parametrize("levels", [4, 3])
def test_linear_tree_one_launch_clamps_split_indices_and_walks_non_finite_values(lut, levels):
    # the walk inside the one-launch kernel (from registers for four levels, from memory otherwise)
    # treats split indices outside [0, V), NaN and the infinities as the stand-alone encoder does
    N, C, V, M = 40, 24, 4, 256
    K = 1 << levels
    w = wl.make_layer("t", N, C, K, V, M, "i8", seed=5 + levels)
    dims, thr = wl.random_tree(C, V, levels, seed=6 + levels)
    bad = dims.copy()
    bad[dims == 0] = -3
    bad[dims == V - 1] = V + 50
    X = w.X.copy()
    X[3] = np.nan
    X[4] = np.inf
    X[5] = -np.inf
    X[6, ::3] = np.nan
    Xs = X.reshape(N, C, V)
    Xs[10:20, :, 1] = thr[:, 0][None, :]  # values exactly on the root's threshold go left
    idx_ref = oracle.encode_tree(dims, thr, X, V)
    ref = OracleLayer(w).lookup(idx_ref)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    got = host(lut.linear_tree(layer, device_tree(lut, bad, thr, V), dev(X), "fused"))
    np.testing.assert_array_equal(got, ref)
    assert (idx_ref[3] == 0).all() and (idx_ref[4] == K - 1).all() and (idx_ref[5] == 0).all()


def _unfold_rows(inp, kernel, stride, pad):
    cols = torch.nn.functional.unfold(torch.from_numpy(inp), kernel, padding=pad, stride=stride)
    return cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous().numpy()


TREE_CONV_SHAPES = [
    # B, Cin, H, W, kernel, stride, pad, V, levels
    (1, 16, 13, 17, (3, 3), (1, 1), (1, 1), 9, 4), (2, 8, 20, 20, (3, 3), (2, 2), (1, 1), 9, 3),
    (3, 16, 9, 11, (1, 1), (1, 1), (0, 0), 4, 4), (2, 4, 15, 9, (3, 5), (2, 1), (1, 2), 2, 6),
    (1, 64, 56, 56, (3, 3), (1, 1), (1, 1), 9, 4), (4, 32, 30, 30, (3, 3), (1, 1), (1, 1), 16, 8),
]


@pytest.mark.parametrize("B,Cin,H,W,kernel,stride,pad,V,levels", TREE_CONV_SHAPES)
def test_encode_tree_conv2d_matches_oracle_on_unfolded_rows(lut, B, Cin, H, W, kernel, stride, pad, V, levels):
    rng = np.random.default_rng(B + Cin + H)
    inp = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    X = _unfold_rows(inp, kernel, stride, pad)
    C = X.shape[1] // V
    assert C * V == X.shape[1]
    dims, thr = wl.random_tree(C, V, levels, seed=H + W)
    ref = oracle.encode_tree(dims, thr, X, V)
    tree = device_tree(lut, dims, thr, V)
    np.testing.assert_array_equal(host(lut.encode_tree_conv2d(tree, dev(inp), kernel, stride, pad)), ref)
    # the same indices as the matrix form of the encoder on the unfolded rows
    np.testing.assert_array_equal(host(lut.encode_tree(tree, dev(X))), ref)


def test_conv2d_tree_matches_oracle(lut):
    B, Cin, H, W, M, levels = 2, 16, 14, 12, 40, 4
    rng = np.random.default_rng(3)
    inp = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    X = _unfold_rows(inp, (3, 3), (1, 1), (1, 1))
    w = wl.make_layer("t", 1, Cin, 16, 9, M, "i8", seed=9)
    dims, thr = wl.random_tree(Cin, 9, levels, seed=9)
    ol = OracleLayer(w)
    ref = ol.lookup(oracle.encode_tree(dims, thr, X, 9))
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    tree = device_tree(lut, dims, thr, 9)
    for v in ("auto", "lds", "mfma"):
        np.testing.assert_array_equal(host(lut.conv2d_tree(layer, tree, dev(inp), 3, 1, 1, v)), ref, err_msg=v)
    with pytest.raises(lut.LutnnError) as e:  # V = 32 has no convolution form
        lut.encode_tree_conv2d(device_tree(lut, *wl.random_tree(1, 32, 4, seed=1), 32),
                               dev(rng.standard_normal((1, 32, 8, 8)).astype(np.float32)), 1, 1, 0)
    assert e.value.status == 3
