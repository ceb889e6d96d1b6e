"""GPU parity: the HIP library (through its C ABI) against the CPU oracle, element by element, on
identical seeded inputs.  Bars (arXiv 2302.03213 leaves precision open; these are this project's):
indices bit-exact except counted near-ties (fp64 distance gap < 1e-6 relative); INT8-table
outputs bit-exact; fp32-table outputs within 1e-5 relative / 1e-4 absolute."""
import os
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle
from gpu_util import (OracleLayer, dev, device_layer_from_oracle, host, near_tie_report,
                      packed_from_q)

pytestmark = pytest.mark.gpu

F32_RTOL, F32_ATOL = 1e-5, 1e-4


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return lut_mod


@pytest.fixture(autouse=True)
def announce(request):
    print("\n[case] %s" % request.node.nodeid, file=sys.stderr, flush=True)
    yield


@pytest.fixture
def pin(lut):
    """pin(NAME, value): sets one of the library's tuning switches for the rest of the test."""
    names = []

    def set_one(name, value):
        lut.set_tunable(name, value)
        names.append(name)
    yield set_one
    for name in names:
        lut.set_tunable(name, None)


def assert_f32_close(got, ref):
    np.testing.assert_allclose(got, ref, rtol=F32_RTOL, atol=F32_ATOL)


# ------------------------------------------------------------------ lutnn_build_table (Eq. 3, Sec. 3.3)
@pytest.mark.parametrize("C,K,V,M", [(5, 16, 4, 37), (3, 16, 9, 64), (8, 7, 2, 300), (2, 33, 3, 5),
                                     (64, 16, 9, 64), (1, 1, 1, 1)])
def test_build_table_matches_oracle(lut, C, K, V, M):
    w = wl.make_layer("t", 1, C, K, V, M, "i8", seed=C * 1000 + M)
    ol = OracleLayer(w)
    P, W = dev(w.P), dev(w.W)
    lf = lut.build_table(P, W, lut.TABLE_F32)
    np.testing.assert_array_equal(host(lf.table), ol.Tf)  # same fma chain -> bit-exact
    l8 = lut.build_table(P, W, lut.TABLE_I8)
    assert host(l8.scale)[0] == ol.s
    np.testing.assert_array_equal(host(l8.table), ol.q)
    Kb, Mp = (K + 15) // 16, (M + 255) // 256 * 256
    assert l8.packed.numel() == C * Kb * Mp * 16 == lut.packed_bytes(C, K, M, lut.TABLE_I8)
    np.testing.assert_array_equal(host(l8.packed).reshape(C * Kb, Mp, 16), packed_from_q(ol.q))


def test_build_table_strided_weights_and_zero_table(lut):
    w = wl.make_layer("t", 1, 4, 16, 4, 20, "i8", seed=5)
    Wbig = np.zeros((16, 31), np.float32)
    Wbig[:, :20] = w.W
    layer = lut.build_table(dev(w.P), dev(Wbig)[:, :20], lut.TABLE_I8)
    ol = OracleLayer(w)
    np.testing.assert_array_equal(host(layer.table), ol.q)
    zero = lut.build_table(dev(w.P), dev(np.zeros_like(w.W)), lut.TABLE_I8)
    assert host(zero.scale)[0] == np.float32(1.0) and not host(zero.table).any()


# ------------------------------------------------------------------ lutnn_encode (Eq. 2)
ENC_SHAPES = [
    # N, C, K, V
    (1, 1, 16, 4), (63, 5, 16, 4), (64, 32, 16, 4), (65, 33, 16, 4), (200, 128, 16, 4),
    (130, 64, 16, 9), (77, 17, 16, 9), (300, 384, 16, 2), (129, 70, 16, 2), (100, 9, 16, 1),
    (100, 35, 16, 3), (100, 20, 16, 8), (90, 7, 16, 5), (50, 3, 16, 16), (40, 2, 16, 32),
    (150, 12, 8, 4), (150, 12, 5, 9), (60, 6, 1, 4), (60, 6, 256, 2), (33, 4, 100, 7),
    # the paper's own settings: (K, V) = (16, 32), (16, 16), (8, 9)
    (300, 24, 16, 32), (130, 7, 16, 32), (200, 48, 16, 16), (67, 9, 16, 16), (130, 12, 8, 16),
    (130, 64, 8, 9), (90, 5, 5, 32),
]


@pytest.mark.parametrize("N,C,K,V", ENC_SHAPES)
def test_encode_matches_oracle(lut, N, C, K, V):
    w = wl.make_layer("t", N, C, K, V, 8, "f32", seed=N + 7 * C + K + V)
    ref = oracle.encode(w.P, w.X)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, w.M)
    got = host(lut.encode(layer, dev(w.X)))
    assert got.max() < K
    ties = near_tie_report(w, got, ref)
    assert ties <= max(1, N * C // 10000), "%d near-ties" % ties


def test_encode_ties_and_centroid_inputs(lut):
    # exact ties (duplicated centroids, equidistant grid points) must resolve to the lowest index
    rng = np.random.default_rng(3)
    C, K, V, N = 6, 16, 4, 500
    P = (rng.integers(-4, 5, (C, K, V)) / 2.0).astype(np.float32)
    P[:, 9] = P[:, 2]
    X = (rng.integers(-8, 9, (N, C * V)) / 4.0).astype(np.float32)
    layer = lut.LutLayer(dev(P), None, lut.TABLE_F32, 8)
    np.testing.assert_array_equal(host(lut.encode(layer, dev(X))), oracle.encode(P, X))
    w = wl.make_layer("t", 1, 40, 16, 9, 8, "f32", seed=4)
    Xc, choice = wl.rows_from_centroids(w.P, 333, seed=5)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    np.testing.assert_array_equal(host(lut.encode(layer, dev(Xc))), choice)


def test_encode_row_stride_and_misaligned_rows(lut):
    w = wl.make_layer("t", 150, 32, 16, 4, 8, "f32", seed=6)
    ref = oracle.encode(w.P, w.X)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    big = torch.zeros((150, 128 + 13), dtype=torch.float32, device="cuda")
    big[:, 1:129] = dev(w.X)  # row stride 141 floats, first element 4-byte aligned only
    got = host(lut.encode(layer, big[:, 1:129]))
    np.testing.assert_array_equal(got, ref)


def test_encode_nonfinite_inputs_stay_in_range(lut):
    w = wl.make_layer("t", 64, 8, 16, 4, 8, "f32", seed=7)
    X = w.X.copy()
    X[3, 5] = np.nan
    X[10, 0] = np.inf
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    got = host(lut.encode(layer, dev(X)))
    assert got.max() < 16
    ref = oracle.encode(w.P, w.X)
    clean = np.ones(64, bool)
    clean[[3, 10]] = False
    np.testing.assert_array_equal(got[clean], ref[clean])


# ------------------------------------------------------------------ lutnn_lookup (Eq. 4)
LOOKUP_SHAPES = [
    # N, C, K, M
    (1, 1, 16, 1), (130, 8, 16, 64), (257, 37, 16, 250), (64, 5, 16, 300), (200, 64, 16, 64),
    (129, 384, 16, 513), (70, 300, 16, 100), (90, 12, 7, 40), (50, 9, 1, 33), (128, 128, 16, 512),
    # large enough grids for the LDS-staged kernels (few-row problems take the direct gather)
    (2048, 8, 16, 4096), (1030, 6, 16, 2048),
]


@pytest.mark.parametrize("variant", ["lds", "mfma"])
@pytest.mark.parametrize("N,C,K,M", LOOKUP_SHAPES)
def test_lookup_i8_bit_exact(lut, variant, N, C, K, M):
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=11 + N + C + M)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=12 + C)  # full-range table, arbitrary scale
    ol.s = np.float32(0.0371)
    idx = wl.random_indices(N, C, K, seed=13 + N)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        got = host(lut.lookup(layer, dev(idx), variant))
        ref = oracle.lookup_i8(ol.q, ol.s, idx, w.bias if with_bias else None)
        np.testing.assert_array_equal(got, ref)


SMFMAC_SHAPES = [
    # N, C, K, M   (C % 32 == 0)
    (1, 32, 16, 1), (130, 64, 16, 64), (513, 96, 16, 250), (1025, 384, 16, 513), (700, 32, 7, 100),
    (512, 160, 16, 128), (300, 128, 1, 40), (2000, 224, 16, 130),
    # larger grids, where the launcher prices taller tiles (every height is also pinned below)
    (2100, 64, 16, 3968), (4700, 64, 16, 4096), (2100, 64, 16, 6400), (1000, 64, 16, 8192),
]


@pytest.mark.parametrize("rows", [128, 256, 384, 512])
@pytest.mark.parametrize("N,C,K,M", [(1500, 96, 16, 300), (2100, 64, 16, 3968), (4700, 64, 16, 4096)])
def test_lookup_smfmac_every_tile_height(lut, pin, rows, N, C, K, M):
    """Each tile height on ragged rows / columns, one tile per workgroup (C % 64 != 0 or few tiles)
    and several (the last shape), pinned through the library's tuning switch."""
    pin("LUTNN_SMFMAC_TILE_ROWS", rows)
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + rows)
    ol = OracleLayer(w)
    idx = wl.random_indices(N, C, K, seed=N + rows)
    layer = device_layer_from_oracle(lut, ol)
    np.testing.assert_array_equal(host(lut.lookup(layer, dev(idx), "smfmac")), ol.lookup(idx))


@pytest.mark.parametrize("group", [0, 1, 3, 8, 64])
@pytest.mark.parametrize("N,C,K,M,rows", [(4700, 64, 16, 4096, 512), (2100, 96, 16, 3968, 128),
                                          (9000, 128, 16, 1100, 256), (1500, 32, 7, 300, 384)])
def test_lookup_smfmac_tile_orders(lut, pin, group, N, C, K, M, rows):
    """The grouped tile order (row tiles in groups, column-block major within a group) against the
    plain one: every tile is visited exactly once whatever the group size, with ragged last groups,
    with tiles streamed through a workgroup (C % 64 == 0 and more tiles than compute units) and
    without."""
    pin("LUTNN_SMFMAC_ROW_GROUP", group)
    pin("LUTNN_SMFMAC_TILE_ROWS", rows)
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + group)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=C + M)
    ol.s = np.float32(0.031)
    idx = wl.random_indices(N, C, K, seed=N + 3)
    layer = device_layer_from_oracle(lut, ol)
    got = host(lut.lookup(layer, dev(idx), "smfmac"))
    ref = ol.lookup(idx)
    assert np.array_equal(got, ref), "%d elements differ" % (got != ref).sum()


@pytest.mark.parametrize("N,C,K,M,group", [(4700, 64, 16, 3072, -1), (2100, 96, 16, 3968, 0),
                                           (9000, 128, 16, 1100, 3), (1500, 32, 7, 300, 0),
                                           (4096, 192, 16, 3072, -1), (600, 32, 16, 4096, 0),
                                           (513, 64, 16, 96, 0), (70, 32, 16, 97, 0)])
def test_lookup_smfmac_tiles_of_96_columns(lut, pin, N, C, K, M, group):
    """512 x 96 tiles (three column tiles per wavefront; table rows of 1.5 KiB copied as one and a
    half loads): bit-exact against the oracle, with and without bias, into a strided Y whose guard
    band must stay untouched - widths that are and are not multiples of 96, tiles streamed through a
    workgroup and not, plain and grouped tile order.  M = 4096 has no room for a 43rd tile in the
    table's padding and takes 128-column tiles whatever the switch says."""
    pin("LUTNN_SMFMAC_TILE_ROWS", 512)
    pin("LUTNN_SMFMAC_TILE_COLS", 96)
    if group >= 0:
        pin("LUTNN_SMFMAC_ROW_GROUP", group)
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + C)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=C + M + 1)
    ol.s = np.float32(0.017)
    idx = wl.random_indices(N, C, K, seed=N + 11)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        Ybig = torch.full((N, M + 8), 3.5, dtype=torch.float32, device="cuda")
        lut.lookup(layer, dev(idx), "smfmac", out=Ybig[:, :M])
        ref = ol.lookup(idx, bias="layer" if with_bias else None)
        got = host(Ybig[:, :M])
        assert np.array_equal(got, ref), "%d elements differ" % (got != ref).sum()
        assert (host(Ybig[:, M:]) == 3.5).all()


@pytest.mark.parametrize("N,C,K,M,rows", [(33, 1024, 16, 4096, 0), (100, 512, 16, 300, 0),
                                          (128, 544, 16, 1000, 0), (64, 576, 7, 130, 0),
                                          (1, 2048, 16, 256, 0), (77, 1536, 16, 768, 0),
                                          (700, 1536, 16, 768, 0), (1029, 512, 16, 260, 0),
                                          (700, 1536, 16, 768, 256), (1029, 1024, 16, 260, 384),
                                          (1300, 1536, 16, 300, 512)])
def test_lookup_smfmac_codebooks_split_over_workgroups(lut, pin, N, C, K, M, rows):
    """Few tiles, many codebooks: several workgroups share an output tile, each with a range of the
    codebooks, and add int32 partial sums into Y (zeroed before, dequantised after).  Bit-exact, with
    and without bias, into a strided Y whose guard band must stay untouched.  (544 codebooks = 17
    groups of 32 cannot be split evenly: that shape takes the unsplit kernel.)  The split is pinned
    through the library's tuning switch so that the test does not depend on its price list; the
    last cases also pin the tile height to reach the taller split instances."""
    pin("LUTNN_SMFMAC_SPLIT", 1)
    if rows:
        pin("LUTNN_SMFMAC_TILE_ROWS", rows)
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + C + M)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=C + M)
    ol.s = np.float32(0.0213)
    idx = wl.random_indices(N, C, K, seed=N + 5)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        Ybig = torch.full((N, M + 8), 3.5, dtype=torch.float32, device="cuda")
        lut.lookup(layer, dev(idx), "smfmac", out=Ybig[:, :M])
        np.testing.assert_array_equal(host(Ybig[:, :M]), ol.lookup(idx, bias="layer" if with_bias else None))
        assert (host(Ybig[:, M:]) == 3.5).all()


@pytest.mark.parametrize("N,C,K,M", SMFMAC_SHAPES)
def test_lookup_smfmac_bit_exact(lut, N, C, K, M):
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=71 + N + C + M)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=72 + C)
    ol.s = np.float32(0.0123)
    idx = wl.random_indices(N, C, K, seed=73 + N)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        got = host(lut.lookup(layer, dev(idx), "smfmac"))
        ref = oracle.lookup_i8(ol.q, ol.s, idx, w.bias if with_bias else None)
        np.testing.assert_array_equal(got, ref)


def test_smfmac_needs_whole_super_stages(lut):
    w = wl.make_layer("t", 1, 40, 16, 2, 64, "i8", seed=74)
    layer = device_layer_from_oracle(lut, OracleLayer(w), True)
    with pytest.raises(lut.LutnnError) as e:
        lut.lookup(layer, dev(wl.random_indices(10, 40, 16)), "smfmac")
    assert e.value.name == "LUTNN_E_UNSUPPORTED"


@pytest.mark.parametrize("variant", ["lds", "mfma", "smfmac"])
def test_lookup_i8_extreme_sums_do_not_wrap(lut, variant):
    # all entries +-127 over C = 1536 codebooks (the deepest layer of the BERT workload):
    # 16-bit partial sums would overflow many times over.
    C, K, M, N = 1536, 16, 96, 70
    q = np.full((C, K, M), 127, np.int8)
    q[:, 1::2] = -127
    w = wl.make_layer("t", 1, C, K, 1, M, "i8", seed=1)
    ol = OracleLayer.__new__(OracleLayer)
    ol.w, ol.q, ol.s, ol.Tf = w, q, np.float32(1.0), None
    idx = np.zeros((N, C), np.uint8)
    idx[1::2] = 1
    idx[2] = wl.random_indices(1, C, K, seed=2)[0]
    layer = device_layer_from_oracle(lut, ol, False)
    got = host(lut.lookup(layer, dev(idx), variant))
    ref = oracle.lookup_i8(q, 1.0, idx, None)
    np.testing.assert_array_equal(got, ref)
    assert got[0, 0] == 127.0 * C and got[1, 0] == -127.0 * C


@pytest.mark.parametrize("N,C,K,M", LOOKUP_SHAPES + [(40, 6, 40, 70)])
def test_lookup_f32_within_tolerance(lut, N, C, K, M):
    w = wl.make_layer("t", 1, C, K, 4, M, "f32", seed=21 + N + C + M)
    ol = OracleLayer(w)
    idx = wl.random_indices(N, C, K, seed=23 + N)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        got = host(lut.lookup(layer, dev(idx), "lds"))
        assert_f32_close(got, oracle.lookup_f32(ol.Tf, idx, w.bias if with_bias else None))


MANY_ROWS_SHAPES = [
    # N, C, K, M: enough rows and tiles for the lane = row gather kernels (256 rows per workgroup)
    (2100, 33, 16, 8200), (4200, 64, 16, 4096), (2100, 12, 40, 8200), (1100, 5, 200, 16400),
    (2500, 7, 1, 8192), (2100, 18, 16, 8195),
]


@pytest.mark.parametrize("N,C,K,M", MANY_ROWS_SHAPES)
def test_lookup_many_rows_gather_i8_i4_f32(lut, N, C, K, M):
    idx = wl.random_indices(N, C, K, seed=N + C)
    # INT8, full-range table, strided output with a guard band
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + M)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=C + K)
    ol.s = np.float32(0.031)
    layer = device_layer_from_oracle(lut, ol)
    ref = ol.lookup(idx)
    Ybig = torch.full((N, M + 4), -7.0, dtype=torch.float32, device="cuda")
    lut.lookup(layer, dev(idx), "lds", out=Ybig[:, :M])
    np.testing.assert_array_equal(host(Ybig[:, :M]), ref)
    assert (host(Ybig[:, M:]) == -7.0).all()
    # index matrix at an odd address
    raw = torch.zeros(N * C + 1, dtype=torch.uint8, device="cuda")
    raw[1:] = dev(idx).flatten()
    np.testing.assert_array_equal(host(lut.lookup(layer, raw[1:].view(N, C), "lds")), ref)
    # INT4 (same codes, clamped to the 4-bit range, nibble storage)
    q4 = np.clip(ol.q, -7, 7).astype(np.int8)
    l4 = lut.LutLayer(dev(w.P), dev(oracle.pack_nibbles(q4)), lut.TABLE_I4, M,
                      scale=dev(np.array([ol.s], np.float32)), bias=dev(w.bias))
    np.testing.assert_array_equal(host(lut.lookup(l4, dev(idx), "lds")),
                                  oracle.lookup_i8(q4, ol.s, idx, w.bias))
    # fp32
    wf = wl.make_layer("t", 1, C, K, 2, M, "f32", seed=N + M + 1)
    olf = OracleLayer(wf)
    lf = device_layer_from_oracle(lut, olf)
    assert_f32_close(host(lut.lookup(lf, dev(idx), "lds")), oracle.lookup_f32(olf.Tf, idx, wf.bias))


@pytest.mark.parametrize("N,C,K,M", [(1, 1024, 16, 4096), (1, 64, 16, 256), (3, 513, 16, 260), (7, 100, 40, 1028),
                                     (2, 2048, 5, 512), (5, 70, 16, 4100), (6, 96, 16, 1032)])
def test_lookup_few_rows_split_gather(lut, N, C, K, M):
    """A handful of rows: the workgroup's wavefronts split the codebooks and meet in LDS (int8 exact,
    fp32 in a fixed order within the usual tolerance); index matrix also at an odd address."""
    idx = wl.random_indices(N, C, K, seed=N + C + M)
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=N + M)
    ol = OracleLayer(w)
    ol.q = wl.random_table_i8(C, K, M, seed=C + K)
    ol.s = np.float32(0.017)
    ref = ol.lookup(idx)
    for with_bias in (True, False):
        layer = device_layer_from_oracle(lut, ol, with_bias)
        np.testing.assert_array_equal(host(lut.lookup(layer, dev(idx), "lds")),
                                      ref if with_bias else ol.lookup(idx, bias=None))
    raw = torch.zeros(N * C + 1, dtype=torch.uint8, device="cuda")
    raw[1:] = dev(idx).flatten()
    np.testing.assert_array_equal(host(lut.lookup(device_layer_from_oracle(lut, ol), raw[1:].view(N, C), "lds")), ref)
    wf = wl.make_layer("t", 1, C, K, 2, M, "f32", seed=N + M + 1)
    olf = OracleLayer(wf)
    got = host(lut.lookup(device_layer_from_oracle(lut, olf), dev(idx), "lds"))
    assert_f32_close(got, oracle.lookup_f32(olf.Tf, idx, wf.bias))
    again = host(lut.lookup(device_layer_from_oracle(lut, olf), dev(idx), "lds"))
    np.testing.assert_array_equal(got, again)  # fixed summation order
    # INT4 storage of the same codes clamped to 4 bits (the split form needs M % 8 == 0, M >= 512)
    q4 = np.clip(ol.q, -7, 7).astype(np.int8)
    l4 = lut.LutLayer(dev(w.P), dev(oracle.pack_nibbles(q4)), lut.TABLE_I4, M,
                      scale=dev(np.array([ol.s], np.float32)), bias=dev(w.bias))
    np.testing.assert_array_equal(host(lut.lookup(l4, dev(idx), "lds")), oracle.lookup_i8(q4, ol.s, idx, w.bias))


def test_lookup_index_matrix_at_odd_address(lut):
    # idx only byte aligned: the dword / 16-byte index fetches must not be used
    w = wl.make_layer("t", 1, 32, 16, 2, 128, "i8", seed=35)
    ol = OracleLayer(w)
    layer = device_layer_from_oracle(lut, ol, True)
    for N in (100, 4100):  # direct gather / LDS-staged for the "lds" variant
        idx = wl.random_indices(N, 32, 16, seed=36 + N)
        raw = torch.zeros(N * 32 + 1, dtype=torch.uint8, device="cuda")
        raw[1:] = dev(idx).reshape(-1)
        view = raw[1:].view(N, 32)
        ref = ol.lookup(idx)
        for variant in ("lds", "mfma"):
            np.testing.assert_array_equal(host(lut.lookup(layer, view, variant)), ref)
        with pytest.raises(lut.LutnnError) as e:
            lut.lookup(layer, view, "smfmac")
        assert e.value.name == "LUTNN_E_ALIGN"


def test_lookup_large_k_uses_global_gather(lut):
    N, C, K, M = 50, 5, 200, 130
    q = wl.random_table_i8(C, K, M, seed=31)
    idx = wl.random_indices(N, C, K, seed=32)
    w = wl.make_layer("t", 1, C, K, 1, M, "i8", seed=33)
    ol = OracleLayer.__new__(OracleLayer)
    ol.w, ol.q, ol.s, ol.Tf = w, q, np.float32(0.5), None
    layer = device_layer_from_oracle(lut, ol, True)
    np.testing.assert_array_equal(host(lut.lookup(layer, dev(idx), "lds")),
                                  oracle.lookup_i8(q, 0.5, idx, w.bias))
    with pytest.raises(lut.LutnnError) as e:
        lut.lookup(layer, dev(idx), "mfma")
    assert e.value.name == "LUTNN_E_UNSUPPORTED"


def test_lookup_output_stride_and_guard_band(lut):
    N, C, K, M = 100, 32, 16, 70
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=41)
    ol = OracleLayer(w)
    idx = wl.random_indices(N, C, K, seed=42)
    layer = device_layer_from_oracle(lut, ol, True)
    ref = ol.lookup(idx)
    for variant in ("lds", "mfma", "smfmac"):
        buf = torch.full((N + 8, M + 9), -777.0, dtype=torch.float32, device="cuda")
        lut.lookup(layer, dev(idx), variant, out=buf[4:4 + N, 3:3 + M])
        got = host(buf)
        np.testing.assert_array_equal(got[4:4 + N, 3:3 + M], ref)
        mask = np.ones_like(got, bool)
        mask[4:4 + N, 3:3 + M] = False
        assert (got[mask] == -777.0).all(), "%s wrote outside its output" % variant


def test_lookup_out_of_range_indices_are_harmless(lut):
    # idx >= K is the caller's bug: result unspecified, but in-bounds rows must be right and
    # nothing may be read or written out of bounds.
    N, C, K, M = 64, 8, 5, 64
    w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=51)
    ol = OracleLayer(w)
    idx = wl.random_indices(N, C, K, seed=52)
    bad = idx.copy()
    bad[7, 3] = 250
    layer = device_layer_from_oracle(lut, ol, True)
    ref = ol.lookup(idx)
    for variant in ("lds", "mfma"):
        got = host(lut.lookup(layer, dev(bad), variant))
        keep = np.arange(N) != 7
        np.testing.assert_array_equal(got[keep], ref[keep])
        assert np.isfinite(got).all()
    # 32 codebooks, K = 16, 16-byte aligned index rows: the shape the sparse matrix-core kernel
    # takes; also enough rows for more than one of its tiles
    for N, C, K, M in ((200, 32, 16, 300), (700, 64, 9, 128)):
        w = wl.make_layer("t", 1, C, K, 2, M, "i8", seed=53 + C)
        ol = OracleLayer(w)
        idx = wl.random_indices(N, C, K, seed=54)
        bad = idx.copy()
        rows = np.array([0, 7, N // 2, N - 1])
        bad[rows, [3, 0, C - 1, 17]] = [250, 16, 255, 128]
        layer = device_layer_from_oracle(lut, ol, True)
        ref = ol.lookup(idx)
        keep = np.ones(N, bool)
        keep[rows] = False
        for variant in ("smfmac", "mfma", "lds", "auto"):
            got = host(lut.lookup(layer, dev(bad), variant))
            np.testing.assert_array_equal(got[keep], ref[keep], err_msg=variant)
            assert np.isfinite(got).all()


# ------------------------------------------------------------------ lutnn_linear (whole operator)
def check_linear(lut, w, variants, X=None):
    ol = OracleLayer(w)
    X = w.X if X is None else X
    idx_ref = ol.encode(X)
    ref = ol.lookup(idx_ref)
    P, W, Xd = dev(w.P), dev(w.W), dev(X)
    dt = lut.TABLE_I8 if w.table_dtype == "i8" else lut.TABLE_F32
    layer = lut.build_table(P, W, dt, bias=dev(w.bias))
    idx_gpu = host(lut.encode(layer, Xd))
    flips = near_tie_report(w, idx_gpu, idx_ref, X)
    clean = (idx_gpu == idx_ref).all(axis=1)
    assert flips <= max(1, idx_ref.size // 10000)
    # "fused" has two forms (a one-launch kernel for small problems, a tile kernel); the library's
    # tuning switch pins each in turn where it can run, so both are compared whatever AUTO prefers
    runs = []
    for v in variants:
        runs += [(v, form) for form in ("tile", "small")] if v == "fused" else [(v, None)]
    for v, form in runs:
        lut.set_tunable("LUTNN_FUSED_KERNEL", form)
        try:
            got = host(lut.linear(layer, Xd, v))
        finally:
            lut.set_tunable("LUTNN_FUSED_KERNEL", None)
        if w.table_dtype == "i8":
            np.testing.assert_array_equal(got[clean], ref[clean], err_msg="variant %s %s" % (v, form))
            # rows holding a flipped near-tie: one table entry swapped per flip
            assert np.abs(got[~clean] - ref[~clean]).max(initial=0.0) <= 2 * 127 * float(ol.s) * 4
        else:
            assert_f32_close(got[clean], ref[clean])
    return flips


LINEAR_SHAPES = [
    # N, C, K, V, M, dtype
    (1, 1, 16, 4, 1, "i8"), (70, 5, 16, 4, 37, "i8"), (129, 33, 16, 9, 64, "i8"),
    (257, 100, 16, 2, 300, "i8"), (100, 20, 7, 3, 40, "i8"), (64, 16, 16, 8, 512, "i8"),
    (70, 5, 16, 4, 37, "f32"), (129, 33, 16, 9, 130, "f32"), (200, 70, 16, 2, 64, "f32"),
    (50, 9, 5, 1, 20, "f32"),
    (130, 24, 16, 32, 96, "i8"), (70, 5, 16, 16, 40, "i8"), (100, 10, 8, 9, 64, "i8"),
    (90, 6, 16, 32, 50, "f32"), (65, 9, 8, 16, 33, "f32"),
]


@pytest.mark.parametrize("N,C,K,V,M,dtype", LINEAR_SHAPES)
def test_linear_small_shapes(lut, N, C, K, V, M, dtype):
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=N + C + M)
    variants = ["auto", "lds", "fused"] + (["mfma"] if dtype == "i8" else [])
    check_linear(lut, w, variants)


def test_linear_generic_subvector_length(lut):
    # V = 5 has no tiled encoder: split path works, fused is refused with a clear status.
    w = wl.make_layer("t", 90, 7, 16, 5, 40, "i8", seed=8)
    check_linear(lut, w, ["auto", "lds", "mfma"])
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear(layer, dev(w.X), "fused")
    assert e.value.name == "LUTNN_E_UNSUPPORTED"


def test_config1_fc_small_fp32(lut):
    flips = check_linear(lut, wl.fc_small(0), ["auto", "lds", "fused"])
    print("config 1 near-ties: %d" % flips)


def test_config2_conv_int8(lut):
    flips = check_linear(lut, wl.conv_resnet18(0), ["auto", "lds", "mfma", "smfmac", "fused"])
    print("config 2 near-ties: %d" % flips)


def test_config3_bert_ffn_up_int8(lut):
    flips = check_linear(lut, wl.bert_ffn_up(0), ["auto", "lds", "mfma", "smfmac", "fused"])
    print("config 3 near-ties: %d" % flips)


def test_paper_kv_space_layers_int8(lut):
    # (K, V) = (16, 32), (16, 16), (8, 9), (16, 4): the settings of the paper's own evaluation
    for w in wl.paper_kv_space(0):
        variants = ["auto", "lds", "mfma", "fused"] + (["smfmac"] if w.C % 32 == 0 else [])
        flips = check_linear(lut, w, variants)
        print("%s near-ties: %d" % (w.name, flips))


def check_every_row(lut, w, variants):
    """Full-size parity: every element of every variant's output against the oracle's (its lookup of
    16,384 x 4,096 outputs takes a second or two on the host cores), in the launch configuration
    bench.py times.  Returns (near-ties, variants the library refused as unsupported)."""
    ol = OracleLayer(w)
    idx_ref = ol.encode()
    ref = ol.lookup(idx_ref)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    np.testing.assert_array_equal(host(layer.table), ol.q)
    Xd = dev(w.X)
    idx_gpu = host(lut.encode(layer, Xd))
    flips = near_tie_report(w, idx_gpu, idx_ref)
    assert flips <= max(1, idx_ref.size // 10000)
    clean = (idx_gpu == idx_ref).all(axis=1)
    refused = []
    for v in variants:
        print("  %s: variant %s, %d rows" % (w.name, v, w.N), file=sys.stderr, flush=True)
        try:
            got = host(lut.linear(layer, Xd, v))
        except lut.LutnnError as e:
            assert e.name == "LUTNN_E_UNSUPPORTED", e
            refused.append(v)
            continue
        assert got.shape == ref.shape
        if clean.all():
            assert np.array_equal(got, ref), "variant %s: %d elements differ" % (v, (got != ref).sum())
        else:
            np.testing.assert_array_equal(got[clean], ref[clean], err_msg="variant %s" % v)
        # the lookup alone, on the oracle's indices: every row comparable whatever the encoder did
        if v != "fused":
            got = host(lut.lookup(layer, dev(idx_ref), v))
            assert np.array_equal(got, ref), "lookup %s: %d elements differ" % (v, (got != ref).sum())
    return flips, refused


def test_config4_bert_layer_linears_int8(lut):
    for w in wl.bert_layer(0):
        flips, refused = check_every_row(lut, w, ["auto", "mfma", "smfmac", "lds", "fused"])
        assert not refused, refused
        print("config 4 %s near-ties: %d refused: %s" % (w.name, flips, refused))


def test_config5_fc_large_int8(lut):
    # the benchmark workload, in the launch configuration bench.py times (variant auto)
    w = wl.fc_large(0)
    flips, refused = check_every_row(lut, w, ["auto", "smfmac", "mfma", "lds", "fused"])
    assert not refused
    print("config 5 near-ties: %d" % flips)


# ------------------------------------------------------------------ INT4 tables (Sec. 3.3, n = 4)
I4_SHAPES = [
    # N, C, K, V, M
    (70, 5, 16, 4, 37), (129, 32, 16, 4, 64), (300, 64, 16, 2, 520), (50, 9, 5, 1, 21),
    (2100, 8, 16, 4, 4096), (600, 96, 16, 4, 264), (40, 6, 40, 2, 70), (33, 4, 100, 2, 30),
]


@pytest.mark.parametrize("N,C,K,V,M", I4_SHAPES)
def test_int4_table_build_and_every_lookup(lut, N, C, K, V, M):
    w = wl.make_layer("t", N, C, K, V, M, "i8", seed=N + C + M + 4)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize(Tf, 4)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I4, bias=dev(w.bias))
    assert host(layer.scale)[0] == s
    np.testing.assert_array_equal(host(layer.table), oracle.pack_nibbles(q))  # storage format
    if K <= 16:
        ref_packed = packed_from_q(q)
        np.testing.assert_array_equal(host(layer.packed).reshape(ref_packed.shape), ref_packed)
    idx_ref = oracle.encode(w.P, w.X)
    ref = oracle.lookup_i8(q, s, idx_ref, w.bias)
    variants = ["auto", "lds"] + (["mfma"] if K <= 16 else []) + \
        (["smfmac"] if K <= 16 and C % 32 == 0 else [])
    for v in variants:
        np.testing.assert_array_equal(host(lut.lookup(layer, dev(idx_ref), v)), ref, err_msg=v)
    idx_gpu = host(lut.encode(layer, dev(w.X)))
    clean = (idx_gpu == idx_ref).all(axis=1)
    assert clean.mean() > 0.99
    for v in ["auto"] + (["fused"] if K <= 16 else []):
        np.testing.assert_array_equal(host(lut.linear(layer, dev(w.X), v))[clean], ref[clean], err_msg=v)
    # the 4-bit table approximates the fp32 one to within half a (coarser) step per codebook
    exact = oracle.lookup_f32(Tf, idx_ref, w.bias)
    assert np.abs(ref - exact).max() <= C * float(s) / 2 * (1 + 1e-4) + 1e-4


# ------------------------------------------------------------------ convolutions (Sec. 4: im2col)
def unfold_rows(inp, kernel, stride, pad):
    """The im2col matrix with torch's own unfold: rows (b, ho, wo), columns (ci, r, s)."""
    cols = torch.nn.functional.unfold(torch.from_numpy(inp), kernel, padding=pad, stride=stride)
    return cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous().numpy()


CONV_SHAPES = [
    # B, Cin, H, W, kernel, stride, pad, V, K
    (1, 16, 13, 17, (3, 3), (1, 1), (1, 1), 9, 16),   # the paper's 3x3 setting, ragged image
    (2, 8, 20, 20, (3, 3), (2, 2), (1, 1), 9, 8),     # stride 2, (K, V) = (8, 9)
    (3, 16, 9, 11, (1, 1), (1, 1), (0, 0), 4, 16),    # 1x1 filter, V = 4 spans four channels
    (1, 12, 10, 10, (3, 3), (1, 1), (0, 0), 3, 16),   # no padding, sub-vector = one filter row
    (2, 4, 15, 9, (3, 5), (2, 1), (1, 2), 2, 16),     # rectangular filter, mixed stride / padding
    (1, 32, 8, 8, (1, 1), (2, 2), (0, 0), 16, 16),    # strided 1x1, V = 16
    (1, 5, 6, 6, (5, 5), (1, 1), (2, 2), 1, 5),       # padding wider than the image border, V = 1
    # nine-tap filters with V = 9: input rows staged once (band kernel)
    (2, 10, 7, 7, (3, 3), (1, 1), (1, 1), 9, 16),     # 49 pixels per image: a tile spans 7+ rows
    (1, 6, 5, 150, (3, 3), (1, 1), (1, 1), 9, 16),    # wide image: tiles inside one row and across two
    (1, 20, 9, 70, (3, 3), (2, 2), (0, 0), 9, 5),     # stride 2, no padding, run-time K, ragged channels
    (1, 8, 12, 40, (1, 9), (1, 1), (0, 4), 9, 16),    # 1 x 9 filter
    (1, 8, 40, 12, (9, 1), (1, 2), (4, 0), 9, 8),     # 9 x 1 filter, mixed strides
    (3, 33, 14, 14, (3, 3), (1, 1), (1, 1), 9, 16),   # batch of 3, 33 channels
]


@pytest.mark.parametrize("B,Cin,H,W,kernel,stride,pad,V,K", CONV_SHAPES)
def test_encode_conv2d_matches_oracle_on_unfolded_rows(lut, B, Cin, H, W, kernel, stride, pad, V, K):
    rng = np.random.default_rng(B + Cin + H + W + V)
    inp = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    X = unfold_rows(inp, kernel, stride, pad)
    C = X.shape[1] // V
    P = rng.standard_normal((C, K, V)).astype(np.float32)
    layer = lut.LutLayer(dev(P), None, lut.TABLE_F32, 8)
    got = host(lut.encode_conv2d(layer, dev(inp), kernel, stride, pad))
    assert got.shape == (X.shape[0], C)
    np.testing.assert_array_equal(got, oracle.encode(P, X))
    # and it is the same encoder as the one for a materialised matrix
    np.testing.assert_array_equal(got, host(lut.encode(layer, dev(X))))


def test_conv2d_config2_from_the_image(lut):
    """Config 2 without the im2col matrix: same indices and outputs as lutnn_linear on it."""
    w = wl.conv_resnet18(0)
    inp = wl.conv_resnet18_input(0)
    np.testing.assert_array_equal(unfold_rows(inp, (3, 3), (1, 1), (1, 1)), w.X)
    ol = OracleLayer(w)
    idx_ref = ol.encode()
    ref = ol.lookup(idx_ref)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    idx = host(lut.encode_conv2d(layer, dev(inp), 3, 1, 1))
    clean = (idx == idx_ref).all(axis=1)
    assert near_tie_report(w, idx, idx_ref) <= 1
    for variant in ("auto", "lds", "mfma", "smfmac"):
        got = host(lut.conv2d(layer, dev(inp), 3, 1, 1, variant))
        np.testing.assert_array_equal(got[clean], ref[clean], err_msg=variant)
    # a batch of images: rows of image b follow those of image b-1
    batch = np.concatenate([inp, inp[:, ::-1].copy()], axis=0)
    got = host(lut.conv2d(layer, dev(batch), 3, 1, 1))
    np.testing.assert_array_equal(got[:w.N][clean], ref[clean])
    Xb = unfold_rows(batch, (3, 3), (1, 1), (1, 1))
    np.testing.assert_array_equal(host(lut.encode_conv2d(layer, dev(batch), 3, 1, 1)),
                                  oracle.encode(w.P, Xb))


def test_identity_on_centroid_inputs(lut):
    # end-to-end property independent of the oracle: rows made of centroids reproduce X @ W + b
    w = wl.make_layer("t", 1, 24, 16, 4, 80, "f32", seed=9)
    X, _ = wl.rows_from_centroids(w.P, 200, seed=10)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_F32, bias=dev(w.bias))
    ref = X.astype(np.float64) @ w.W.astype(np.float64) + w.bias.astype(np.float64)
    for v in ("lds", "fused"):
        np.testing.assert_allclose(host(lut.linear(layer, dev(X), v)), ref, rtol=1e-5, atol=1e-5)


def test_empty_batch_and_determinism(lut):
    w = wl.make_layer("t", 300, 64, 16, 4, 256, "i8", seed=12)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    X = dev(w.X)
    for v in ("lds", "mfma", "smfmac", "fused"):
        assert lut.linear(layer, X[:0], v).shape == (0, 256)
        a = host(lut.linear(layer, X, v))
        b = host(lut.linear(layer, X, v))
        np.testing.assert_array_equal(a, b)
    assert lut.encode(layer, X[:0]).shape == (0, 64)


def test_error_statuses(lut):
    w = wl.make_layer("t", 10, 4, 16, 4, 8, "i8", seed=13)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8)
    X = dev(w.X)
    with pytest.raises(lut.LutnnError) as e:
        lut.lookup(layer, dev(wl.random_indices(10, 4, 16)), "fused")
    assert e.value.name == "LUTNN_E_UNSUPPORTED"
    no_packed = lut.LutLayer(layer.centroids, layer.table, lut.TABLE_I8, 8, None, layer.scale)
    with pytest.raises(lut.LutnnError) as e:
        lut.linear(no_packed, X, "mfma")
    assert e.value.name == "LUTNN_E_NULL"
    np.testing.assert_array_equal(host(lut.linear(no_packed, X, "auto")),
                                  host(lut.linear(layer, X, "lds")))
