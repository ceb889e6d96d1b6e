"""GPU parity of the soft-PQ backward pass (Sec. 3.1-3.2, Eq. 5-6 of arXiv 2302.03213) against the
fp64 oracle.  The kernel works in fp32 from Z = G . W^T (formed here in fp64 and rounded once); the
oracle applies the chain rule through the table T = P . W without that factoring.

Bar (the paper fixes no precision for training): every gradient within 5e-5 of the largest
magnitude of its tensor.  The softmax weights carry a relative error of about (d/t) * 2^-23 plus the
2 ulp of the hardware exponential, i.e. up to 1e-5 for exponents of a few tens; a sum of N such
terms in fp32 adds at most N * 2^-24 relative to the sum of magnitudes (1e-3 for N = 16384 in the
worst case, ~sqrt(N) * 2^-24 = 8e-6 typically).  Observed: 2e-7 to 8e-7 for dP and dX.

dt (Sec. 3.2, the learned temperature) is one sum over all N * C * K terms dz_k d_k / t^2 with
cancellation, so its error is measured against S = sum |dz_k d_k| / t^2, the magnitude it is summed
from.  A term carries the relative error of its softmax weight (the exponent (d - d_min)/t is known
to about (d/t) * 2^-23, i.e. 1e-6 for exponents of ten, plus 2 ulp of the exponential) and the fp32
summation adds about sqrt(terms) * 2^-24 of S: both near 1e-6 * S.  The bar is 1e-5 * S, ten times
that; wherever the gradient is not itself a cancellation residue (|dt| >= 1e-2 * S) it must also hold
to 1e-3 relative.  |dt| / S is 3e-5 to 0.3 on the cases below (computed with the oracle), so a
kernel returning 0 or the wrong sign misses the bar on every one of them.  Observed error: 1e-10 to
8e-8 of S."""
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


def close(got, ref, frac=5e-5):
    scale = max(np.abs(ref).max(), 1e-30)
    err = np.abs(got - ref).max() / scale
    assert err <= frac, "normalised error %.3e" % err
    return err


def dt_magnitude(w, t, G):
    """S = sum |dz_k d_k| / t^2: the magnitude the temperature gradient is summed from."""
    s, d, _ = osp.soft_encoding(w.P, w.X, t)
    P64, Wc = w.P.astype(np.float64), w.W.astype(np.float64).reshape(w.C, w.V, -1)
    ds = np.einsum("nm,ckm->nck", G, np.einsum("ckv,cvm->ckm", P64, Wc))
    dz = s * (ds - (s * ds).sum(-1, keepdims=True))
    return np.abs(dz * d).sum() / (t * t)


def check_dt(got, ref, S, frac=1e-5):
    """|dt - dt_ref| <= frac * S, and <= 1e-3 * |dt_ref| where dt_ref is not a cancellation residue."""
    err = abs(float(got) - float(ref))
    print("dt %.6e ref %.6e  err/S %.2e  |ref|/S %.2e" % (got, ref, err / max(S, 1e-300),
                                                        abs(ref) / max(S, 1e-300)))
    assert err <= frac * S, "dt %.8e, oracle %.8e, error %.2e of S" % (got, ref, err / S)
    if abs(ref) >= 1e-2 * S:
        assert err <= 1e-3 * abs(ref), "dt %.8e, oracle %.8e" % (got, ref)
    return err / max(S, 1e-300)


def run_case(lut, N, C, K, V, M, t, seed, strided=False):
    w = wl.make_layer("t", N, C, K, V, M, "f32", seed=seed)
    G = np.random.default_rng(seed).standard_normal((N, M))
    Z = (G @ w.W.astype(np.float64).T).astype(np.float32)
    dP_ref, dX_ref, dt_ref = osp.backward(w.P, w.W, w.X, t, G)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, M)
    if strided:
        Xb = torch.zeros((N, C * V + 5), dtype=torch.float32, device="cuda")
        Zb = torch.zeros((N, C * V + 3), dtype=torch.float32, device="cuda")
        Xb[:, 1:1 + C * V] = dev(w.X)
        Zb[:, 3:3 + C * V] = dev(Z)
        Xd, Zd = Xb[:, 1:1 + C * V], Zb[:, 3:3 + C * V]
    else:
        Xd, Zd = dev(w.X), dev(Z)
    dP, dX, dt = lut.softpq_backward(layer, t, Xd, Zd)
    e1 = close(host(dP), dP_ref)
    e2 = close(host(dX), dX_ref)
    check_dt(host(dt)[0], dt_ref, dt_magnitude(w, t, G))
    # without the input gradient the other two are unchanged, bit for bit (fixed summation order)
    dP2, none, dt2 = lut.softpq_backward(layer, t, Xd, Zd, need_dx=False)
    assert none is None
    np.testing.assert_array_equal(host(dP2), host(dP))
    np.testing.assert_array_equal(host(dt2), host(dt))
    return e1, e2


SOFTPQ_SHAPES = [
    # N, C, K, V, M, t
    (1, 1, 16, 4, 3, 1.0), (63, 5, 16, 4, 7, 1.0), (64, 16, 16, 4, 20, 0.5), (200, 33, 16, 4, 16, 2.0),
    (130, 17, 16, 9, 12, 1.0), (130, 8, 8, 9, 12, 3.0), (150, 40, 16, 2, 9, 1.0), (100, 9, 16, 1, 5, 0.3),
    (100, 35, 16, 3, 6, 1.0), (100, 20, 16, 8, 6, 4.0), (70, 6, 16, 16, 8, 8.0), (70, 5, 16, 32, 8, 16.0),
    (90, 12, 8, 4, 10, 1.0), (90, 7, 8, 16, 10, 6.0), (66, 3, 8, 32, 4, 20.0), (120, 70, 8, 2, 5, 1.0),
    # several row tiles per chunk, several chunks, ragged tail
    (4200, 64, 16, 4, 24, 1.0), (9000, 8, 16, 9, 16, 2.0),
]


@pytest.mark.parametrize("N,C,K,V,M,t", SOFTPQ_SHAPES)
def test_softpq_backward_matches_oracle(lut, N, C, K, V, M, t):
    e = run_case(lut, N, C, K, V, M, t, seed=N + C + K + V)
    print("normalised errors dP %.2e dX %.2e" % e)


def test_softpq_backward_strided_and_misaligned_operands(lut):
    run_case(lut, 130, 9, 16, 4, 11, 1.0, seed=3, strided=True)
    run_case(lut, 77, 5, 16, 9, 6, 1.5, seed=4, strided=True)


def test_softpq_backward_small_temperature_is_finite_and_matches(lut):
    # t = 0.05: exponents of several hundred; the max-subtracted softmax must not overflow
    run_case(lut, 128, 8, 16, 4, 8, 0.05, seed=6)


def test_softpq_backward_is_reproducible_and_handles_an_empty_batch(lut):
    w = wl.make_layer("t", 3000, 32, 16, 4, 8, "f32", seed=1)
    Z = dev(np.random.default_rng(1).standard_normal((3000, 128)).astype(np.float32))
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    a = lut.softpq_backward(layer, 1.0, dev(w.X), Z)
    b = lut.softpq_backward(layer, 1.0, dev(w.X), Z)
    for x, y in zip(a, b):
        np.testing.assert_array_equal(host(x), host(y))
    dP, dX, dt = lut.softpq_backward(layer, 1.0, dev(w.X)[:0], Z[:0])
    assert not host(dP).any() and dX.shape == (0, 128) and host(dt)[0] == 0.0


def test_softpq_backward_at_the_benchmark_size(lut):
    """N, C, K, V of the benchmark workload in the launch configuration bench.py times (the kernel
    never sees M, so a narrow output keeps the oracle affordable).  dX is per row: three sampled
    128-row blocks are compared with the oracle.  dP and dt are sums over rows: the full launch must
    equal the sum of launches over a partition of the rows (additivity, which holds at any size), and
    one block of that kind is already pinned to the oracle by the cases above."""
    N, C, K, V, M, t = 16384, 1024, 16, 4, 16, 1.0
    w = wl.make_layer("t", N, C, K, V, M, "f32", seed=21)
    G = np.random.default_rng(21).standard_normal((N, M))
    Z = (G @ w.W.astype(np.float64).T).astype(np.float32)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, M)
    Xd, Zd = dev(w.X), dev(Z)
    dP, dX, dt = lut.softpq_backward(layer, t, Xd, Zd)
    dXh = host(dX)
    for b0 in (0, 7040, N - 128):
        _, dX_ref, _ = osp.backward(w.P, w.W, w.X[b0:b0 + 128], t, G[b0:b0 + 128])
        close(dXh[b0:b0 + 128], dX_ref)
    parts = [lut.softpq_backward(layer, t, Xd[r0:r0 + 2048], Zd[r0:r0 + 2048], need_dx=False)
             for r0 in range(0, N, 2048)]
    dP_sum = sum(host(p[0]).astype(np.float64) for p in parts)
    dt_sum = sum(float(host(p[2])[0]) for p in parts)
    close(host(dP), dP_sum, 1e-5)
    assert abs(float(host(dt)[0]) - dt_sum) <= 1e-4 * max(abs(dt_sum), 1e-6) + 1e-3 * sum(
        abs(float(host(p[2])[0])) for p in parts)


def test_softpq_backward_unsupported_and_bad_arguments(lut):
    w = wl.make_layer("t", 8, 4, 5, 4, 8, "f32", seed=1)  # K = 5
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    Z = dev(np.zeros((8, 16), np.float32))
    with pytest.raises(lut.LutnnError) as e:
        lut.softpq_backward(layer, 1.0, dev(w.X), Z)
    assert e.value.status == 3
    w = wl.make_layer("t", 8, 4, 16, 4, 8, "f32", seed=1)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    for bad_t in (0.0, -1.0, float("nan"), float("inf")):
        with pytest.raises(lut.LutnnError) as e:
            lut.softpq_backward(layer, bad_t, dev(w.X), Z)
        assert e.value.status == 2
    with pytest.raises(lut.LutnnError) as e:
        lut.softpq_backward(layer, 1.0, dev(w.X), Z, workspace=torch.empty(16, dtype=torch.uint8, device="cuda"))
    assert e.value.status == 2


def test_autograd_wrapper_trains_centroids_and_temperature(lut):
    """The module form: hard forward (INT8 table), soft backward.  Gradients match the oracle, and
    a few steps of gradient descent on the centroids lower the soft loss the gradients belong to."""
    from paper_2302_03213_amd.softpq import SoftPQLinear
    N, C, K, V, M, t = 512, 16, 16, 4, 24, 1.0
    w = wl.make_layer("t", N, C, K, V, M, "i8", seed=12)
    target = w.X.astype(np.float64) @ w.W.astype(np.float64) + w.bias
    layer = SoftPQLinear(dev(w.P), dev(w.W), dev(w.bias), temperature=t, table_dtype=lut.TABLE_I8)
    X = dev(w.X).requires_grad_(True)
    Y = layer(X)
    # value of the forward pass = the hard INT8 operator
    ref_layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    np.testing.assert_array_equal(host(Y.detach()), host(lut.linear(ref_layer, dev(w.X))))
    G = (Y.detach().double() - dev(target.astype(np.float32)).double()).float() / N  # dL/dY of 0.5*MSE
    Y.backward(G)
    dP_ref, dX_ref, dt_ref = osp.backward(w.P, w.W, w.X, t, host(G).astype(np.float64))
    close(host(layer.centroids.grad), dP_ref, 5e-4)  # Z comes from torch's fp32 GEMM here
    close(host(X.grad), dX_ref, 5e-4)
    # Z comes from torch's fp32 GEMM here (relative error ~1e-6 per element): the same bar holds
    check_dt(layer.temperature.grad.item(), dt_ref, dt_magnitude(w, t, host(G).astype(np.float64)))
    np.testing.assert_allclose(host(layer.bias.grad), host(G).sum(axis=0), rtol=1e-4, atol=1e-6)

    def soft_loss(P):
        return 0.5 * ((osp.soft_forward(P, w.W, w.X, t, w.bias) - target) ** 2).sum() / N

    before = soft_loss(w.P)
    opt = torch.optim.SGD([layer.centroids], lr=0.5)
    for _ in range(5):
        opt.zero_grad()
        Y = layer(dev(w.X))
        Ysoft = osp.soft_forward(host(layer.centroids.detach()), w.W, w.X, t, w.bias)
        Y.backward(dev(((Ysoft - target) / N).astype(np.float32)))  # gradient of the soft loss
        opt.step()
    after = soft_loss(host(layer.centroids.detach()))
    assert after < before, (before, after)


def test_autograd_conv2d_module_matches_oracle_on_unfolded_rows(lut):
    """SoftPQConv2d: value = the hard convolution read from NCHW; gradients = the oracle's on the
    im2col rows, the input gradient folded back onto the image (fold is unfold's adjoint)."""
    from paper_2302_03213_amd.softpq import SoftPQConv2d
    B, Cin, H, W, M, K, t = 2, 8, 11, 9, 12, 16, 1.3
    kernel, stride, pad = (3, 3), (2, 1), (1, 1)
    rng = np.random.default_rng(31)
    inp = rng.standard_normal((B, Cin, H, W)).astype(np.float32)
    w = wl.make_layer("t", 1, Cin, K, 9, M, "i8", seed=31)  # V = 9: one channel's patch per sub-vector
    cols = torch.nn.functional.unfold(torch.from_numpy(inp), kernel, padding=pad, stride=stride)
    X = cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous().numpy()
    Ho = (H + 2 * pad[0] - kernel[0]) // stride[0] + 1
    Wo = (W + 2 * pad[1] - kernel[1]) // stride[1] + 1
    mod = SoftPQConv2d(dev(w.P), dev(w.W), kernel, stride, pad, bias=dev(w.bias), temperature=t,
                       table_dtype=lut.TABLE_I8)
    x = dev(inp).requires_grad_(True)
    Y = mod(x)
    assert Y.shape == (B, M, Ho, Wo)
    ref_layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    hard = lut.conv2d(ref_layer, dev(inp), kernel, stride, pad).view(B, Ho, Wo, M).permute(0, 3, 1, 2)
    np.testing.assert_array_equal(host(Y.detach()), host(hard))
    G = rng.standard_normal((B, M, Ho, Wo)).astype(np.float32)
    Y.backward(dev(G))
    G2 = np.ascontiguousarray(G.transpose(0, 2, 3, 1).reshape(-1, M)).astype(np.float64)
    dP_ref, dX_ref, dt_ref = osp.backward(w.P, w.W, X, t, G2)
    dcols = torch.from_numpy(dX_ref).view(B, Ho * Wo, -1).permute(0, 2, 1)
    dinp_ref = torch.nn.functional.fold(dcols, (H, W), kernel, padding=pad, stride=stride).numpy()
    close(host(mod.centroids.grad), dP_ref, 5e-4)  # Z comes from torch's fp32 GEMM here
    close(host(x.grad), dinp_ref, 5e-4)
    w.X = X
    check_dt(mod.temperature.grad.item(), dt_ref, dt_magnitude(w, t, G2))
    np.testing.assert_allclose(host(mod.bias.grad), G2.sum(axis=0), rtol=1e-4, atol=1e-5)


def draw_softpq_shape(seed):
    rng = np.random.default_rng(3000 + seed)
    K = int(rng.choice([16, 16, 8]))
    V = int(rng.choice([1, 2, 3, 4, 4, 8, 9, 16, 32]))
    C = int(rng.integers(1, 90))
    N = int(np.exp(rng.uniform(0.0, np.log(5000.0))))
    M = int(rng.integers(1, 40))
    # temperatures from sharp to flat relative to the typical squared distance (about 2 V)
    t = float(np.exp(rng.uniform(np.log(0.15 * V), np.log(8.0 * V))))
    while N * C * K * max(V, M) > 6e7:
        N = max(1, N // 2)
    return N, C, K, V, M, t


@pytest.mark.parametrize("seed", range(20))
def test_softpq_backward_on_a_random_shape(lut, seed):
    N, C, K, V, M, t = draw_softpq_shape(seed)
    print("seed %d: N=%d C=%d K=%d V=%d M=%d t=%.3f" % (seed, N, C, K, V, M, t), file=sys.stderr, flush=True)
    run_case(lut, N, C, K, V, M, t, seed=900 + seed, strided=bool(seed & 1))
