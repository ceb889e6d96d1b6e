"""Soft-PQ (arXiv 2302.03213, Sec. 3.1-3.3): the differentiable stand-in for the table lookup
operator that training back-propagates through.  Plain numpy in double precision.

TEST INFRASTRUCTURE ONLY, like the rest of this package: the product never imports it.

Eq. 5 replaces the one-hot arg-min encoding by a softmax over the same K squared distances,
    g~^c(a^c)_k = softmax_k( -||a^c - P^c_k||^2 / t ),
and Eq. 6 writes a layer's output as  soft - sg(soft - hard):  its VALUE is the hard (arg-min)
result, its GRADIENT is that of the soft output
    Ysoft[n][m] = sum_c sum_k g~^c(x_n^c)_k * T[c][k][m] (+ bias[m]),   T = P . W  (Eq. 3, real valued:
    Sec. 3.3 keeps the tables un-quantised in the backward pass).
`backward` is the chain rule through exactly these formulas, for the parameters the paper learns by
back-propagation: the centroids P and the layer's temperature t (Sec. 3.2), plus the gradient with
respect to the layer input that earlier layers need.

Readings: the weights W are the pre-trained model's and stay fixed (the paper rebuilds the tables
from the updated centroids); t itself is the learned parameter (no re-parameterisation is given);
softmax is evaluated with the usual max subtraction.

Pinned in tests/test_oracle_softpq.py by reverse-mode autodiff of an independently written forward
(torch, fp64), central finite differences, the K = 1 closed form and the t -> 0 / t -> inf limits.
"""
import numpy as np


def _split(P, W, X):
    P = np.asarray(P, np.float64)
    W = np.asarray(W, np.float64)
    X = np.asarray(X, np.float64)
    C, K, V = P.shape
    N, D = X.shape
    assert D == C * V and W.shape[0] == D
    return P, W.reshape(C, V, -1), X.reshape(N, C, V)


def soft_encoding(P, X, t):
    """Eq. 5: s[n][c][k] = softmax_k(-||X[n, cV:(c+1)V] - P[c][k]||^2 / t); also returns the distances."""
    P = np.asarray(P, np.float64)
    C, K, V = P.shape
    Xs = np.asarray(X, np.float64).reshape(-1, C, V)
    diff = Xs[:, :, None, :] - P[None, :, :, :]          # [N, C, K, V]
    d = (diff * diff).sum(axis=-1)                       # [N, C, K]
    z = -d / float(t)
    z = z - z.max(axis=-1, keepdims=True)
    e = np.exp(z)
    return e / e.sum(axis=-1, keepdims=True), d, diff


def soft_forward(P, W, X, t, bias=None):
    """The soft output of Eq. 6: Ysoft[n][m] = sum_c s[n][c][:] . T[c][:][m] (+ bias), T = P . W."""
    Pd, Wc, _ = _split(P, W, X)
    s, _, _ = soft_encoding(P, X, t)
    T = np.einsum("ckv,cvm->ckm", Pd, Wc)                # Eq. 3
    Y = np.einsum("nck,ckm->nm", s, T)
    if bias is not None:
        Y = Y + np.asarray(bias, np.float64)[None, :]
    return Y


def backward(P, W, X, t, G):
    """Gradients of a loss L through Ysoft, given G = dL/dY [N][M].
    Returns (dP [C][K][V], dX [N][D], dt scalar)."""
    Pd, Wc, Xs = _split(P, W, X)
    G = np.asarray(G, np.float64)
    t = float(t)
    s, d, diff = soft_encoding(P, X, t)
    T = np.einsum("ckv,cvm->ckm", Pd, Wc)
    ds = np.einsum("nm,ckm->nck", G, T)                  # dL/ds
    dT = np.einsum("nck,nm->ckm", s, G)                  # dL/dT
    # softmax: dL/dz_k = s_k (dL/ds_k - sum_j s_j dL/ds_j),  z = -d / t
    dz = s * (ds - (s * ds).sum(axis=-1, keepdims=True))
    dd = -dz / t                                         # dL/d(distance)
    dt = (dz * d).sum() / (t * t)                        # dz/dt = d / t^2
    # distance: d = sum_v (x_v - p_kv)^2
    dP = np.einsum("ckm,cvm->ckv", dT, Wc) + (dd[..., None] * (-2.0 * diff)).sum(axis=0)
    dX = (dd[..., None] * (2.0 * diff)).sum(axis=2).reshape(Xs.shape[0], -1)
    return dP, dX, dt
