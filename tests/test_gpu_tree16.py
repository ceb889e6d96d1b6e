"""GPU parity of the 16-bit index forms - the hash encoder with trees of up to 12 levels (Sec. 7 of
arXiv 2302.03213 evaluates 12: 4096 buckets per codebook) and the lookup of Eq. 4 behind it -
against the CPU oracle through the C ABI.  Comparisons and integer sums only: indices and INT8
outputs are bit-exact; fp32-table outputs within the fp32 bar of the 8-bit lookups."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle
from gpu_util import dev, host

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


def u16(t):
    """A torch int16 tensor carries the library's uint16 bits."""
    return host(t).view(np.uint16)


def dev16(a):
    return torch.from_numpy(np.ascontiguousarray(a, dtype=np.uint16).view(np.int16)).cuda()


TREE16_SHAPES = [
    # N, C, V, levels
    (1, 1, 4, 12), (63, 5, 4, 9), (130, 33, 4, 12), (300, 70, 2, 10), (100, 9, 1, 11), (100, 35, 3, 9),
    (200, 20, 8, 12), (77, 17, 9, 12), (150, 6, 16, 12), (4100, 24, 32, 12), (90, 7, 5, 12), (33, 4, 7, 9),
    # the depths the 8-bit form also takes give the same leaves
    (150, 12, 4, 1), (200, 40, 4, 4), (129, 19, 9, 8),
    # many tiles, ragged rows and codebooks
    (8250, 130, 4, 12), (5000, 96, 32, 12),
]


@pytest.mark.parametrize("N,C,V,levels", TREE16_SHAPES)
def test_encode_tree16_matches_oracle(lut, N, C, V, levels):
    seed = N * 31 + C * 7 + V + levels
    dims, thr = wl.random_tree(C, V, levels, seed=seed, level_dims=bool(seed & 1))
    X = wl.make_layer("t", N, C, 2, V, 1, "i8", seed=seed).X
    ref = oracle.encode_tree(dims, thr, X, V).astype(np.uint16)
    tree = lut.LutTree(dev(dims), dev(thr), V)
    got = u16(lut.encode_tree16(tree, dev(X)))
    np.testing.assert_array_equal(got, ref)
    if levels <= 8:
        np.testing.assert_array_equal(host(lut.encode_tree(tree, dev(X))), ref.astype(np.uint8))
    elif N * C >= 4000:
        assert ref.max() > 255  # the buckets beyond one byte are in use


def test_encode_tree16_ties_nan_infinities_strides_and_clamped_split_indices(lut):
    N, C, V, levels = 300, 10, 4, 12
    dims, thr = wl.random_tree(C, V, levels, seed=9)
    X = wl.make_layer("t", N, C, 2, V, 1, "i8", seed=9).X.copy()
    rng = np.random.default_rng(1)
    Xs = X.reshape(N, C, V)
    for c in range(C):  # a third of the values sit exactly on a threshold of their own codebook
        pick = rng.random((N, V)) < 0.33
        Xs[:, c, :][pick] = thr[c, rng.integers(0, thr.shape[1], pick.sum())]
    X[5] = np.nan
    X[6] = np.inf
    X[7] = -np.inf
    ref = oracle.encode_tree(dims, thr, X, V)
    bad = dims.copy()  # split indices outside [0, V) are clamped into it
    bad[dims == 0] = -3
    bad[dims == V - 1] = V + 50
    tree = lut.LutTree(dev(bad), dev(thr), V)
    big = torch.zeros((N, C * V + 7), dtype=torch.float32, device="cuda")
    big[:, 3:3 + C * V] = dev(X)  # row stride 47 floats, rows 4-byte aligned only
    got = u16(lut.encode_tree16(tree, big[:, 3:3 + C * V]))
    np.testing.assert_array_equal(got, ref)
    assert (got[5] == 0).all() and (got[6] == 4095).all() and (got[7] == 0).all()
    assert lut.encode_tree16(tree, dev(X)[:0]).shape == (0, C)


LOOKUP16_SHAPES = [
    # N, C, K, M, dtype
    (70, 5, 300, 37, "i8"), (129, 9, 512, 64, "i8"), (33, 3, 4096, 520, "i8"), (300, 24, 4096, 256, "i8"),
    (1, 1, 1, 1, "i8"), (50, 7, 1000, 130, "f32"), (65, 4, 4096, 96, "f32"), (40, 6, 16, 33, "f32"),
]


@pytest.mark.parametrize("N,C,K,M,dtype", LOOKUP16_SHAPES)
def test_lookup16_matches_oracle(lut, N, C, K, M, dtype):
    rng = np.random.default_rng(N + C + K + M)
    idx = rng.integers(0, K, (N, C)).astype(np.uint16)
    bias = rng.standard_normal(M).astype(np.float32)
    P = dev(np.zeros((C, K, 1), np.float32))
    for b in (bias, None):
        if dtype == "i8":
            q = rng.integers(-127, 128, (C, K, M)).astype(np.int8)
            s = np.float32(0.0173)
            layer = lut.LutLayer(P, dev(q), lut.TABLE_I8, M, scale=dev(np.array([s], np.float32)), bias=dev(b))
            ref = oracle.lookup_i8(q, s, idx, b)
        else:
            Tf = rng.standard_normal((C, K, M)).astype(np.float32)
            layer = lut.LutLayer(P, dev(Tf), lut.TABLE_F32, M, bias=dev(b))
            ref = oracle.lookup_f32(Tf, idx, b)
        buf = torch.full((N + 2, M + 5), -7.0, dtype=torch.float32, device="cuda")
        lut.lookup16(layer, dev16(idx), out=buf[1:N + 1, 2:M + 2])
        got = host(buf)
        if dtype == "i8":
            np.testing.assert_array_equal(got[1:N + 1, 2:M + 2], ref)
        else:
            np.testing.assert_allclose(got[1:N + 1, 2:M + 2], ref, rtol=1e-5, atol=1e-4)
        guard = np.ones_like(got, bool)
        guard[1:N + 1, 2:M + 2] = False
        assert (got[guard] == -7.0).all(), "wrote outside its output"
    # indices past K are the caller's bug: treated as K - 1, nothing read out of bounds
    if K > 1 and dtype == "i8":
        bad = idx.copy()
        bad[0, 0] = 65535
        clamped = idx.copy()
        clamped[0, 0] = K - 1
        np.testing.assert_array_equal(host(lut.lookup16(layer, dev16(bad))), oracle.lookup_i8(q, s, clamped, None))


def test_build_table_beyond_256_rows_per_codebook(lut):
    # tables for the 16-bit lookup come from the same Eq. 3 / Sec. 3.3 kernels, without the packed copy
    C, K, V, M = 3, 700, 4, 50
    w = wl.make_layer("t", 1, C, K, V, M, "i8", seed=77)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize_i8(Tf)
    l8 = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8)
    assert l8.packed is None and host(l8.scale)[0] == s
    np.testing.assert_array_equal(host(l8.table), q)
    np.testing.assert_array_equal(host(lut.build_table(dev(w.P), dev(w.W), lut.TABLE_F32).table), Tf)


@pytest.mark.parametrize("dtype", ["i8", "f32"])
def test_linear_tree16_twelve_levels_on_a_bert_shape(lut, dtype):
    """The paper's hashing experiment (Sec. 7): 12-level trees.  BERT-base FFN-up rows (D = 768) at
    V = 32: 24 codebooks of 4096 buckets each; the table is built from seeded bucket prototypes."""
    N, C, V, levels, M = 4096, 24, 32, 12, 256
    K = 1 << levels
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=5)
    dims, thr = wl.random_tree(C, V, levels, seed=6)
    Tf = oracle.build_table_f32(w.P, w.W)
    idx_ref = oracle.encode_tree(dims, thr, w.X, V)
    assert idx_ref.dtype == np.uint16 and idx_ref.max() > 255
    tree = lut.LutTree(dev(dims), dev(thr), V)
    if dtype == "i8":
        q, s = oracle.quantize_i8(Tf)
        ref = oracle.lookup_i8(q, s, idx_ref, w.bias)
        layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
        np.testing.assert_array_equal(host(layer.table), q)
    else:
        ref = oracle.lookup_f32(Tf, idx_ref, w.bias)
        layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_F32, bias=dev(w.bias))
    ws = torch.zeros((N, C), dtype=torch.int16, device="cuda")
    got = host(lut.linear_tree16(layer, tree, dev(w.X), idx_workspace=ws))
    np.testing.assert_array_equal(u16(ws), idx_ref)
    if dtype == "i8":
        assert np.array_equal(got, ref), "%d elements differ" % (got != ref).sum()
    else:
        np.testing.assert_allclose(got, ref, rtol=1e-5, atol=1e-4)
    # the 8-bit entry points refuse what only the 16-bit ones take
    with pytest.raises(lut.LutnnError) as e:
        lut.encode_tree(tree, dev(w.X))
    assert e.value.name == "LUTNN_E_SHAPE"
    shallow = lut.LutTree(dev(dims[:, :15]), dev(thr[:, :15]), V)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear_tree16(layer, shallow, dev(w.X))
    assert e.value.name == "LUTNN_E_SHAPE"  # 4 levels against K = 4096
