"""Pins for the soft-PQ oracle (oracle/softpq.py), Sec. 3.1-3.2 and Eq. 5-6 of arXiv 2302.03213:
reverse-mode autodiff of a forward written with different primitives, finite differences, a closed
form and the two temperature limits."""
import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle
from oracle import softpq


def _case(N, C, K, V, M, seed):
    w = wl.make_layer("t", N, C, K, V, M, "f32", seed=seed)
    g = np.random.default_rng(seed).standard_normal((N, M))
    return w, g


@pytest.mark.parametrize("N,C,K,V,M,t", [(7, 3, 16, 4, 5, 1.0), (5, 2, 8, 9, 6, 0.5), (9, 4, 5, 2, 3, 3.0),
                                         (4, 2, 16, 32, 4, 20.0)])
def test_backward_equals_autodiff_of_an_independent_forward(N, C, K, V, M, t):
    w, G = _case(N, C, K, V, M, seed=N + C + K)
    P = torch.tensor(w.P, dtype=torch.float64, requires_grad=True)
    X = torch.tensor(w.X, dtype=torch.float64, requires_grad=True)
    tt = torch.tensor(t, dtype=torch.float64, requires_grad=True)
    W = torch.tensor(w.W, dtype=torch.float64)
    # forward from library pieces: cdist for the distances, softmax, one matmul per codebook
    Y = torch.zeros((N, M), dtype=torch.float64)
    for c in range(C):
        dist2 = torch.cdist(X[:, c * V:(c + 1) * V], P[c]) ** 2
        Y = Y + torch.softmax(-dist2 / tt, dim=1) @ (P[c] @ W[c * V:(c + 1) * V])
    np.testing.assert_allclose(Y.detach().numpy(), softpq.soft_forward(w.P, w.W, w.X, t), rtol=1e-9, atol=1e-11)
    (Y * torch.tensor(G)).sum().backward()
    dP, dX, dt = softpq.backward(w.P, w.W, w.X, t, G)
    np.testing.assert_allclose(dP, P.grad.numpy(), rtol=1e-7, atol=1e-10)
    np.testing.assert_allclose(dX, X.grad.numpy(), rtol=1e-7, atol=1e-10)
    np.testing.assert_allclose(dt, tt.grad.item(), rtol=1e-7, atol=1e-10)


def test_backward_equals_central_differences_of_the_soft_forward():
    N, C, K, V, M, t = 6, 3, 16, 4, 5, 0.8
    w, G = _case(N, C, K, V, M, seed=3)
    dP, dX, dt = softpq.backward(w.P, w.W, w.X, t, G)
    P64, X64 = w.P.astype(np.float64), w.X.astype(np.float64)

    def loss(P=P64, X=X64, t=t):
        return (softpq.soft_forward(P, w.W, X, t) * G).sum()

    h = 1e-6
    rng = np.random.default_rng(0)
    for _ in range(12):
        c, k, v = rng.integers(C), rng.integers(K), rng.integers(V)
        e = np.zeros_like(P64)
        e[c, k, v] = h
        np.testing.assert_allclose((loss(P=P64 + e) - loss(P=P64 - e)) / (2 * h), dP[c, k, v], rtol=1e-5, atol=1e-7)
        n, j = rng.integers(N), rng.integers(C * V)
        e = np.zeros_like(X64)
        e[n, j] = h
        np.testing.assert_allclose((loss(X=X64 + e) - loss(X=X64 - e)) / (2 * h), dX[n, j], rtol=1e-5, atol=1e-7)
    np.testing.assert_allclose((loss(t=t + h) - loss(t=t - h)) / (2 * h), dt, rtol=1e-5, atol=1e-7)


def test_single_centroid_closed_form():
    # K = 1: the encoding is the constant 1, so Ysoft = sum_c P[c][0] . W^c does not depend on X or
    # t, and dL/dP[c][0][v] = sum_n (G W^T)[n][cV+v].
    N, C, V, M = 11, 4, 3, 6
    w, G = _case(N, C, 1, V, M, seed=8)
    dP, dX, dt = softpq.backward(w.P, w.W, w.X, 0.7, G)
    np.testing.assert_allclose(dX, 0.0, atol=1e-12)
    assert abs(dt) < 1e-12
    np.testing.assert_allclose(dP[:, 0, :], (G @ w.W.astype(np.float64).T).sum(axis=0).reshape(C, V), rtol=1e-10)


def test_temperature_limits_hard_lookup_and_uniform_average():
    # t -> 0: the softmax becomes the one-hot arg-min and Ysoft the hard output of Eq. 2 + Eq. 4
    # (the C oracle's, through its own code); t -> inf: every centroid weighs 1/K.
    N, C, K, V, M = 40, 6, 16, 4, 9
    w, _ = _case(N, C, K, V, M, seed=5)
    Tf = oracle.build_table_f32(w.P, w.W)
    hard = oracle.lookup_f32(Tf, oracle.encode(w.P, w.X), w.bias)
    np.testing.assert_allclose(softpq.soft_forward(w.P, w.W, w.X, 1e-4, w.bias), hard, rtol=1e-5, atol=1e-5)
    s, d, _ = softpq.soft_encoding(w.P, w.X, 1e-4)
    np.testing.assert_array_equal(s.argmax(axis=-1), oracle.encode(w.P, w.X))
    uniform = Tf.astype(np.float64).mean(axis=1).sum(axis=0) + w.bias
    np.testing.assert_allclose(softpq.soft_forward(w.P, w.W, w.X, 1e12, w.bias),
                               np.broadcast_to(uniform, (N, M)), rtol=1e-6, atol=1e-6)


def test_encoding_is_a_probability_vector_and_orders_like_the_distances():
    w, _ = _case(30, 5, 16, 4, 3, seed=2)
    s, d, _ = softpq.soft_encoding(w.P, w.X, 0.9)
    np.testing.assert_allclose(s.sum(axis=-1), 1.0, rtol=1e-12)
    assert (s > 0).all()
    np.testing.assert_array_equal(np.argsort(-s, axis=-1, kind="stable"), np.argsort(d, axis=-1, kind="stable"))
