"""GPU parity on seeded random shapes: the whole operator (arXiv 2302.03213 Eq. 2 + Eq. 4) through
every lookup variant the shape admits, the hash encoder of Sec. 2 / Sec. 7 in front of it, and the
convolution form of Sec. 4, against the CPU oracle.  The hand-picked shapes of the other
files aim at known tile edges; these draws are there for the combinations nobody thought of (a
launcher's price list picking an unusual tile for a ragged shape, a fallback taken for an odd
alignment).  Same bars as everywhere: indices bit-exact except counted near-ties, INT8-table outputs
bit-exact, fp32-table outputs within 1e-5 relative / 1e-4 absolute."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
from gpu_util import OracleLayer, dev, host, near_tie_report

pytestmark = pytest.mark.gpu

F32_RTOL, F32_ATOL = 1e-5, 1e-4


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return lut_mod


def draw_shape(seed):
    """One shape per seed, sized so that the oracle needs at most a few seconds."""
    rng = np.random.default_rng(1000 + seed)
    dtype = rng.choice(["i8", "i8", "i8", "f32"])
    K = int(rng.choice([16, 16, 16, 8, int(rng.integers(1, 16)), int(rng.integers(17, 65)), 256]))
    V = int(rng.choice([1, 2, 3, 4, 4, 5, 8, 9, 9, 16, 32]))
    if rng.random() < 0.5:
        C = 32 * int(rng.integers(1, 13))          # the sparse matrix-core lookup needs C % 32 == 0
    else:
        C = int(rng.integers(1, 200))
    # a third of the draws small in either direction, the rest large enough for several tiles
    N = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(9000.0))))
    M = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(4300.0))))
    # bound the oracle's work: encode N*C*K*V, lookup N*C*M
    while N * C * K * V > 1.5e9 or N * C * M > 2.5e9:
        N = max(1, N // 2)
    return N, C, K, V, M, str(dtype)


@pytest.mark.parametrize("seed", range(48))
def test_linear_on_a_random_shape(lut, seed):
    N, C, K, V, M, dtype = draw_shape(seed)
    print("\n[case] seed %d: N=%d C=%d K=%d V=%d M=%d %s" % (seed, N, C, K, V, M, dtype),
          file=sys.stderr, flush=True)
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=seed, bias=bool(seed & 1))
    ol = OracleLayer(w)
    idx_ref = ol.encode()
    ref = ol.lookup(idx_ref, bias=w.bias)
    table_dtype = lut.TABLE_I8 if dtype == "i8" else lut.TABLE_F32
    layer = lut.build_table(dev(w.P), dev(w.W), table_dtype, bias=dev(w.bias))
    Xd = dev(w.X)
    idx_gpu = host(lut.encode(layer, Xd))
    flips = near_tie_report(w, idx_gpu, idx_ref)
    assert flips <= max(1, idx_ref.size // 10000), "%d near-ties" % flips
    clean = (idx_gpu == idx_ref).all(axis=1)
    ran = []
    for variant in ("auto", "lds", "mfma", "smfmac", "fused"):
        Ybig = torch.full((N, M + 3), -7.25, dtype=torch.float32, device="cuda")
        try:
            lut.linear(layer, Xd, variant, out=Ybig[:, :M])
        except lut.LutnnError as e:
            assert variant != "auto" and e.name == "LUTNN_E_UNSUPPORTED", (variant, str(e))
            continue
        ran.append(variant)
        got = host(Ybig[:, :M])
        assert (host(Ybig[:, M:]) == -7.25).all(), "variant %s wrote past its rows" % variant
        if dtype == "i8":
            bad = got[clean] != ref[clean]
            assert not bad.any(), "variant %s: %d elements differ" % (variant, bad.sum())
        else:
            np.testing.assert_allclose(got[clean], ref[clean], rtol=F32_RTOL, atol=F32_ATOL,
                                       err_msg="variant %s" % variant)
    assert "auto" in ran and "lds" in ran


def draw_tree_shape(seed):
    rng = np.random.default_rng(5000 + seed)
    levels = int(rng.choice([1, 2, 3, 4, 4, 4, 5, 6, 8, 9, 10, 12]))
    V = int(rng.choice([1, 2, 3, 4, 4, 8, 9, 16, 32]))
    C = 32 * int(rng.integers(1, 9)) if rng.random() < 0.5 else int(rng.integers(1, 150))
    N = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(6000.0))))
    M = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(3000.0))))
    dtype = str(rng.choice(["i8", "i8", "f32"]))
    K = 1 << levels
    while N * C * M > 1.5e9 or C * K * M > 6e7 or N * C * V > 3e7:
        if C * K * M > 6e7 and M > 64:
            M //= 2
        elif C > 8 and C * K * M > 6e7:
            C //= 2
        else:
            N = max(1, N // 2)
    return N, C, V, levels, M, dtype


@pytest.mark.parametrize("seed", range(32))
def test_linear_tree_on_a_random_shape(lut, seed):
    """The hash encoder (Sec. 2 "Hashing for acceleration", Sec. 7) in front of every lookup the shape
    admits: comparisons only, so indices and INT8 outputs are bit-exact; trees of more than eight
    levels take the 16-bit index calls."""
    import oracle
    N, C, V, levels, M, dtype = draw_tree_shape(seed)
    K = 1 << levels
    print("\n[case] seed %d: N=%d C=%d V=%d levels=%d M=%d %s" % (seed, N, C, V, levels, M, dtype),
          file=sys.stderr, flush=True)
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=seed + 77, bias=bool(seed & 1))
    dims, thr = wl.random_tree(C, V, levels, seed=seed)
    ol = OracleLayer(w)
    idx_ref = oracle.encode_tree(dims, thr, w.X, V)
    ref = ol.lookup(idx_ref, bias=w.bias)
    tree = lut.LutTree(dev(dims), dev(thr), V)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8 if dtype == "i8" else lut.TABLE_F32, bias=dev(w.bias))
    Xd = dev(w.X)

    def check(got, what):
        if dtype == "i8":
            bad = got != ref
            assert not bad.any(), "%s: %d elements differ" % (what, bad.sum())
        else:
            np.testing.assert_allclose(got, ref, rtol=F32_RTOL, atol=F32_ATOL, err_msg=what)

    if levels > 8:
        idx = host(lut.encode_tree16(tree, Xd)).view(np.uint16)
        np.testing.assert_array_equal(idx, idx_ref)
        check(host(lut.linear_tree16(layer, tree, Xd)), "linear_tree16")
        return
    np.testing.assert_array_equal(host(lut.encode_tree(tree, Xd)), idx_ref)
    ran = []
    for variant in ("auto", "lds", "mfma", "smfmac", "fused"):
        try:
            got = host(lut.linear_tree(layer, tree, Xd, variant))
        except lut.LutnnError as e:
            assert variant != "auto" and e.name == "LUTNN_E_UNSUPPORTED", (variant, str(e))
            continue
        ran.append(variant)
        check(got, variant)
    assert "auto" in ran and "lds" in ran


@pytest.mark.parametrize("seed", range(24))
def test_conv2d_on_a_random_geometry(lut, seed):
    """Convolutions read from the NCHW batch (Sec. 4): random image sizes, filters, strides and
    paddings; the rows must be those of torch's unfold, encoded and looked up as the oracle does."""
    import oracle
    rng = np.random.default_rng(9000 + seed)
    kh, kw = [(3, 3), (3, 3), (1, 1), (5, 5), (3, 1), (1, 3), (2, 2), (3, 5)][int(rng.integers(0, 8))]
    taps = kh * kw
    V = int(rng.choice([v for v in (1, 2, 3, 4, 8, 9, 16) if (taps % v == 0 or v % taps == 0)]))
    chan_per_sub = max(1, V // taps)                 # a sub-vector spans whole filters' worth of channels
    Cin = chan_per_sub * int(rng.integers(1, 40 // chan_per_sub + 2))
    if (Cin * taps) % V:
        Cin *= V
    B = int(rng.integers(1, 4))
    H, W = int(rng.integers(kh, 40)), int(rng.integers(kw, 40))
    stride = (int(rng.integers(1, 3)), int(rng.integers(1, 3)))
    pad = (int(rng.integers(0, kh)), int(rng.integers(0, kw)))
    K = int(rng.choice([16, 16, 8, 5]))
    M = int(rng.choice([1, 8, 64, 100, 256]))
    print("\n[case] seed %d: B=%d Cin=%d H=%d W=%d filter %dx%d stride %s pad %s V=%d K=%d M=%d"
          % (seed, B, Cin, H, W, kh, kw, stride, pad, V, K, M), file=sys.stderr, flush=True)
    inp = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    cols = torch.nn.functional.unfold(torch.from_numpy(inp), (kh, kw), padding=pad, stride=stride)
    X = cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous().numpy()
    C = X.shape[1] // V
    w = wl.make_layer("t", 1, C, K, V, M, "i8", seed=seed + 5)
    w.X, w.N = X, X.shape[0]
    ol = OracleLayer(w)
    idx_ref = ol.encode(X)
    ref = ol.lookup(idx_ref, bias=w.bias)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    idx = host(lut.encode_conv2d(layer, dev(inp), (kh, kw), stride, pad))
    assert idx.shape == idx_ref.shape
    flips = near_tie_report(w, idx, idx_ref, X)
    assert flips <= max(1, idx_ref.size // 10000)
    clean = (idx == idx_ref).all(axis=1)
    got = host(lut.conv2d(layer, dev(inp), (kh, kw), stride, pad))
    bad = got[clean] != ref[clean]
    assert not bad.any(), "%d elements differ" % bad.sum()
