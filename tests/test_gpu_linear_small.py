"""GPU parity of the one-launch form of lutnn_linear (encode + table read in one kernel for small
problems; arXiv 2302.03213, Eq. 2 + Eq. 4, Fig. 5) against the CPU oracle.  The form is pinned
through the library's tuning variable so that the cases do not depend on what AUTO prefers.
Bars as everywhere: INT8 tables bit-exact on rows without a near-tie flip, fp32 tables within
1e-5 relative / 1e-4 absolute."""
import numpy as np
import pytest
import torch

import lutnn_workloads as wl
from gpu_util import OracleLayer, dev, host, near_tie_report

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return lut_mod


@pytest.fixture(autouse=True)
def pin_small(lut):
    lut.set_tunable("LUTNN_FUSED_KERNEL", "small")
    yield
    lut.set_tunable("LUTNN_FUSED_KERNEL", None)


def run_case(lut, w, with_bias=True, x_pad=0, y_pad=0):
    ol = OracleLayer(w)
    idx_ref = ol.encode(w.X)
    ref = ol.lookup(idx_ref, bias="layer" if with_bias else None)
    dt = lut.TABLE_I8 if w.table_dtype == "i8" else lut.TABLE_F32
    layer = lut.build_table(dev(w.P), dev(w.W), dt, bias=dev(w.bias) if with_bias else None)
    Xbig = torch.full((w.N, w.D + x_pad), 7.0, dtype=torch.float32, device="cuda")
    Xbig[:, :w.D] = dev(w.X)
    Ybig = torch.full((w.N, w.M + y_pad), -3.5, dtype=torch.float32, device="cuda")
    lut.linear(layer, Xbig[:, :w.D], "fused", out=Ybig[:, :w.M])
    got = host(Ybig[:, :w.M])
    assert (host(Ybig[:, w.M:]) == -3.5).all()  # the guard band of a strided Y stays untouched
    idx_gpu = host(lut.encode(layer, dev(w.X)))
    flips = near_tie_report(w, idx_gpu, idx_ref, w.X)
    assert flips <= max(1, idx_ref.size // 10000)
    clean = (idx_gpu == idx_ref).all(axis=1)
    if w.table_dtype == "i8":
        np.testing.assert_array_equal(got[clean], ref[clean])
    else:
        np.testing.assert_allclose(got[clean], ref[clean], rtol=1e-5, atol=1e-4)
    return layer, got


SHAPES = [
    # N, C, K, V, M, dtype: rows narrower than a wavefront (M = 4 ... 128), exactly one chunk, several
    # chunks with a ragged last one, more than four chunks (several workgroups per row group)
    (1, 1, 16, 4, 4, "i8"), (70, 5, 16, 4, 8, "i8"), (129, 33, 16, 9, 64, "i8"), (300, 64, 16, 9, 64, "i8"),
    (77, 20, 7, 3, 128, "i8"), (64, 16, 16, 8, 256, "i8"), (257, 100, 16, 2, 300, "i8"),
    (33, 128, 16, 4, 512, "f32"), (256, 128, 16, 4, 512, "f32"), (19, 40, 16, 2, 1028, "i8"),
    (5, 384, 16, 2, 2304, "i8"), (1, 384, 16, 2, 3072, "i8"), (3, 512, 16, 2, 768, "i8"),
    (50, 9, 5, 1, 20, "f32"), (90, 6, 16, 32, 52, "f32"), (65, 9, 8, 16, 32, "f32"),
    (130, 24, 16, 32, 96 * 4, "i8"), (40, 7, 33, 4, 260, "i8"), (21, 10, 200, 3, 16, "i8"),
    # the split form: few rows, 64 codebooks or more, 256 columns or more (4 and 16 wavefronts)
    (2, 64, 16, 4, 256, "i8"), (7, 1024, 16, 4, 4096, "i8"), (1, 1536, 16, 2, 768, "i8"),
    (3, 2050, 16, 1, 260, "i8"), (4, 70, 7, 9, 520, "f32"), (2, 530, 33, 2, 300, "f32"),
]


@pytest.mark.parametrize("N,C,K,V,M,dtype", SHAPES)
def test_one_launch_linear_matches_oracle(lut, N, C, K, V, M, dtype):
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=N + C + M)
    run_case(lut, w)


def test_one_launch_linear_strides_and_no_bias(lut):
    w = wl.make_layer("t", 67, 48, 16, 4, 516, "i8", seed=5)
    run_case(lut, w, with_bias=False, x_pad=3, y_pad=8)
    w = wl.make_layer("t", 45, 31, 16, 2, 64, "f32", seed=6)
    run_case(lut, w, with_bias=False, x_pad=1, y_pad=4)


def test_one_launch_equals_encode_then_gather(lut):
    """Same device functions as lutnn_encode + the gather lookup: identical bits for integer tables;
    fp32 sums may be split over wavefronts differently, so those are compared to rounding."""
    for dtype, N, C, M in (("i8", 143, 72, 512), ("i8", 143, 72, 64), ("i8", 9, 600, 1024), ("f32", 143, 72, 512),
                           ("f32", 40, 30, 144)):
        w = wl.make_layer("t", N, C, 16, 4, M, dtype, seed=M + C)
        layer, got = run_case(lut, w)
        two = host(lut.lookup(layer, lut.encode(layer, dev(w.X)), "lds"))
        if dtype == "i8":
            np.testing.assert_array_equal(got, two)
        else:
            np.testing.assert_allclose(got, two, rtol=1e-5, atol=1e-5)


def test_auto_takes_one_launch_for_small_problems(lut):
    lut.set_tunable("LUTNN_FUSED_KERNEL", None)
    w = wl.fc_small(0)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_F32, bias=dev(w.bias))
    ws = torch.empty((w.N, w.C), dtype=torch.uint8, device="cuda")
    assert lut.linear_auto_variant(layer, w.N, ws) == "fused"
    big = wl.make_layer("t", 4, 1024, 16, 4, 4096, "i8", seed=1)
    layer = lut.build_table(dev(big.P), dev(big.W), lut.TABLE_I8)
    ws = torch.empty((4096, big.C), dtype=torch.uint8, device="cuda")
    assert lut.linear_auto_variant(layer, 4096, ws) == "smfmac"
    assert lut.linear_auto_variant(layer, 4096, None) == "fused"  # no workspace: a fused kernel or nothing


def test_unsupported_shapes_fall_back_or_refuse(lut):
    # M % 4 != 0: the one-launch form cannot run; pinned or not, FUSED takes the tile kernel
    w = wl.make_layer("t", 50, 8, 16, 4, 37, "i8", seed=2)
    ol = OracleLayer(w)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    got = host(lut.linear(layer, dev(w.X), "fused"))
    idx = host(lut.encode(layer, dev(w.X)))
    np.testing.assert_array_equal(got, ol.lookup(idx))
