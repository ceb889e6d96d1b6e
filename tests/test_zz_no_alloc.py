"""lutnn_softpq_backward_static: the soft-PQ backward pass (Sec. 3.1-3.2, Eq. 5-6 of arXiv 2302.03213)
for callers that cannot allocate, against lutnn_softpq_backward with a caller workspace.  Both run
the same kernels in the same fixed summation order, so the bar is bit equality; the workspace form
is itself held to the fp64 oracle in test_gpu_softpq.py, and one case here repeats that check."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
from gpu_util import dev, host
from oracle import softpq as osp

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


def both_forms(lut, N, C, K, V, M, t, seed, oracle_too=False):
    w = wl.make_layer("t", N, C, K, V, M, "f32", seed=seed)
    G = np.random.default_rng(seed).standard_normal((N, M))
    Z = (G @ w.W.astype(np.float64).T).astype(np.float32)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, M)
    Xd, Zd = dev(w.X), dev(Z)
    ref = lut.softpq_backward(layer, t, Xd, Zd)
    # outputs allocated by the caller beforehand and poisoned: the call itself allocates nothing
    dP = torch.full((C, K, V), float("nan"), dtype=torch.float32, device="cuda")
    dX = torch.full((N, C * V), float("nan"), dtype=torch.float32, device="cuda")
    dt = torch.full((1,), float("nan"), dtype=torch.float32, device="cuda")
    # torch's count of allocations it has ever made (monotonic: frees by the garbage collector do
    # not touch it) must not move across the call
    before = torch.cuda.memory_stats().get("allocation.all.allocated", 0)
    got = lut.softpq_backward_static(layer, t, Xd, Zd, dP=dP, dX=dX, dt=dt)
    assert torch.cuda.memory_stats().get("allocation.all.allocated", 0) == before
    for a, b, name in zip(got, ref, ("dP", "dX", "dt")):
        np.testing.assert_array_equal(host(a), host(b), err_msg=name)
    if oracle_too:
        dP_ref, dX_ref, dt_ref = osp.backward(w.P, w.W, w.X, t, G)
        for a, r in ((got[0], dP_ref), (got[1], dX_ref)):
            assert np.abs(host(a) - r).max() <= 5e-5 * np.abs(r).max()
    return layer, Xd, Zd


def test_static_scratch_form_equals_workspace_form_on_two_calls_in_a_row(lut):
    # the second call is smaller: it must not see anything the first left in the shared array
    both_forms(lut, 4200, 64, 16, 4, 24, 1.0, seed=5)
    both_forms(lut, 300, 17, 16, 9, 12, 2.0, seed=6, oracle_too=True)
    # ... and a larger one again, other K, without the input gradient
    layer, Xd, Zd = both_forms(lut, 9000, 40, 8, 16, 10, 0.7, seed=7)
    a = lut.softpq_backward_static(layer, 0.7, Xd, Zd, need_dx=False)
    b = lut.softpq_backward(layer, 0.7, Xd, Zd, need_dx=False)
    assert a[1] is None
    np.testing.assert_array_equal(host(a[0]), host(b[0]))
    np.testing.assert_array_equal(host(a[2]), host(b[2]))


def test_static_scratch_form_empty_batch_and_benchmark_size(lut):
    both_forms(lut, 16384, 1024, 16, 4, 8, 1.0, seed=8)  # 8.4 MB of the 32 MiB array
    both_forms(lut, 4200, 128, 16, 32, 8, 4.0, seed=10)  # 16.8 MB: the largest need of the paper's settings
    w = wl.make_layer("t", 4, 8, 16, 4, 8, "f32", seed=9)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    dP, dX, dt = lut.softpq_backward_static(layer, 1.0, dev(w.X)[:0], dev(w.X)[:0])
    assert not host(dP).any() and dX.shape == (0, 32) and host(dt)[0] == 0.0


def test_static_scratch_form_refuses_what_does_not_fit(lut):
    # 2^23 centroid values: 32 MiB of partial sums for the centroid gradient alone
    C, K, V, N = 131072, 16, 4, 8
    assert lut.softpq_workspace_bytes(C, K, V, N) > 32 << 20
    P = torch.zeros((C, K, V), dtype=torch.float32, device="cuda")
    X = torch.zeros((N, C * V), dtype=torch.float32, device="cuda")
    layer = lut.LutLayer(P, None, lut.TABLE_F32, 8)
    with pytest.raises(lut.LutnnError) as e:
        lut.softpq_backward_static(layer, 1.0, X, X)
    assert e.value.name == "LUTNN_E_SHAPE" and "static buffer" in str(e.value)
    # the other errors are those of the workspace form
    small = lut.LutLayer(P[:4], None, lut.TABLE_F32, 8)
    with pytest.raises(lut.LutnnError) as e:
        lut.softpq_backward_static(small, 0.0, X[:8, :16], X[:8, :16])
    assert e.value.name == "LUTNN_E_SHAPE"
