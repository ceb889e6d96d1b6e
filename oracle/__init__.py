"""ctypes front end of the CPU oracle (oracle/lutnn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, __graft_entry__.smoke() and the
cpu_baseline leg of bench.py.  The product package never imports this module and
this module never imports the product package.

All arrays are numpy, host memory.  Shapes follow the paper's notation
(arXiv 2302.03213, Sec. 2.1-2.2, Table 1): N rows, D = C*V inputs, K centroids per
codebook, M outputs; P[C][K][V] codebooks, W[D][M] weights, T[C][K][M] table.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None

_f32p = ctypes.POINTER(ctypes.c_float)
_f64p = ctypes.POINTER(ctypes.c_double)
_u8p = ctypes.POINTER(ctypes.c_uint8)
_u16p = ctypes.POINTER(ctypes.c_uint16)
_i8p = ctypes.POINTER(ctypes.c_int8)
_i32p = ctypes.POINTER(ctypes.c_int32)


def _lib():
    global _LIB
    if _LIB is None:
        sanitize = os.environ.get("LUTNN_ORACLE_SANITIZE") == "1"  # see build.py
        path = _build.LIB_SAN if sanitize else _build.LIB
        if not os.path.exists(path) or os.path.getmtime(path) < os.path.getmtime(_build.SRC):
            _build.build(force=True, sanitize=sanitize)
        lib = ctypes.CDLL(path)
        lib.lutnn_oracle_threads.restype = ctypes.c_int
        lib.lutnn_oracle_set_threads.argtypes = [ctypes.c_int]
        lib.lutnn_oracle_build_table_f32.argtypes = [_f32p, _f32p, ctypes.c_int64, ctypes.c_int,
                                                     ctypes.c_int, ctypes.c_int, ctypes.c_int, _f32p]
        lib.lutnn_oracle_quantize_i8.argtypes = [_f32p, ctypes.c_int64, _i8p, _f32p]
        lib.lutnn_oracle_quantize.argtypes = [_f32p, ctypes.c_int64, ctypes.c_int, _i8p, _f32p]
        lib.lutnn_oracle_encode.argtypes = [_f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, _f32p,
                                            ctypes.c_int64, ctypes.c_int64, _u8p]
        lib.lutnn_oracle_encode_tree.argtypes = [_i32p, _f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                 _f32p, ctypes.c_int64, ctypes.c_int64, _u16p]
        lib.lutnn_oracle_distances_f64.argtypes = [_f32p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
                                                   _f32p, ctypes.c_int64, ctypes.c_int64,
                                                   ctypes.c_int, _f64p]
        lib.lutnn_oracle_lookup_i8.argtypes = [_i8p, ctypes.c_float, _f32p, ctypes.c_int,
                                               ctypes.c_int, ctypes.c_int, _u16p, ctypes.c_int64,
                                               _f32p, ctypes.c_int64, _i32p]
        lib.lutnn_oracle_lookup_f32.argtypes = [_f32p, _f32p, ctypes.c_int, ctypes.c_int,
                                                ctypes.c_int, _u16p, ctypes.c_int64, _f32p,
                                                ctypes.c_int64]
        _LIB = lib
    return _LIB


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


def _ptr(a, t):
    return a.ctypes.data_as(t)


def threads():
    return int(_lib().lutnn_oracle_threads())


def set_threads(n):
    _lib().lutnn_oracle_set_threads(int(n))


def build_table_f32(P, W):
    """Eq. 3: Tf[c,k,m] = P[c,k,:] . W[c*V:(c+1)*V, m]  (fp32)."""
    P = _c(P, np.float32)
    W = _c(W, np.float32)
    C, K, V = P.shape
    D, M = W.shape
    assert D == C * V, "D must equal C*V"
    Tf = np.empty((C, K, M), dtype=np.float32)
    _lib().lutnn_oracle_build_table_f32(_ptr(P, _f32p), _ptr(W, _f32p), M, C, K, V, M,
                                        _ptr(Tf, _f32p))
    return Tf


def quantize_i8(Tf):
    """Sec. 3.3: symmetric INT8, one scale per layer.  Returns (q int8, s float32)."""
    Tf = _c(Tf, np.float32)
    q = np.empty(Tf.shape, dtype=np.int8)
    s = np.zeros(1, dtype=np.float32)
    _lib().lutnn_oracle_quantize_i8(_ptr(Tf, _f32p), Tf.size, _ptr(q, _i8p), _ptr(s, _f32p))
    return q, np.float32(s[0])


def quantize(Tf, bits):
    """Sec. 3.3 with n = bits: symmetric, one scale per layer, |q| <= 2^(bits-1) - 1.  Returns
    (q int8 - one entry per byte also for bits < 8 -, s float32)."""
    assert 2 <= bits <= 8
    Tf = _c(Tf, np.float32)
    q = np.empty(Tf.shape, dtype=np.int8)
    s = np.zeros(1, dtype=np.float32)
    _lib().lutnn_oracle_quantize(_ptr(Tf, _f32p), Tf.size, bits, _ptr(q, _i8p), _ptr(s, _f32p))
    return q, np.float32(s[0])


def pack_nibbles(q):
    """Storage format of a 4-bit table: [..., M] int8 in [-8, 7] -> [..., ceil(M/2)] uint8, even
    column in the low nibble, two's complement.  Layout only, no arithmetic of the method."""
    q = np.asarray(q, dtype=np.int8)
    if q.shape[-1] % 2:
        q = np.concatenate([q, np.zeros(q.shape[:-1] + (1,), np.int8)], axis=-1)
    u = q.astype(np.uint8) & 0xF
    return (u[..., 0::2] | (u[..., 1::2] << 4)).astype(np.uint8)


def encode(P, X):
    """Eq. 2: idx[n,c] = argmin_k ||X[n, cV:(c+1)V] - P[c,k]||^2 (fp32, lowest k on ties)."""
    P = _c(P, np.float32)
    X = _c(X, np.float32)
    C, K, V = P.shape
    N, D = X.shape
    assert D == C * V and K <= 256
    idx = np.empty((N, C), dtype=np.uint8)
    _lib().lutnn_oracle_encode(_ptr(P, _f32p), C, K, V, _ptr(X, _f32p), N, D, _ptr(idx, _u8p))
    return idx


def encode_tree(split_dim, threshold, X, V):
    """Hash encoding (Sec. 2, Sec. 7): walk each codebook's balanced threshold tree (heap order,
    right when x[split] > threshold); idx[n,c] = the leaf reached, counted from the left.  uint8 for
    up to 8 levels, uint16 for the deeper trees of Sec. 7 (12 levels = 4096 buckets)."""
    split_dim = _c(split_dim, np.int32)
    threshold = _c(threshold, np.float32)
    X = _c(X, np.float32)
    C, nodes = split_dim.shape
    levels = (nodes + 1).bit_length() - 1
    assert threshold.shape == (C, nodes) and nodes == (1 << levels) - 1 and 1 <= levels <= 16
    N, D = X.shape
    assert D == C * V
    assert split_dim.min() >= 0 and split_dim.max() < V
    idx = np.empty((N, C), dtype=np.uint16)
    _lib().lutnn_oracle_encode_tree(_ptr(split_dim, _i32p), _ptr(threshold, _f32p), C, levels, V,
                                    _ptr(X, _f32p), N, D, _ptr(idx, _u16p))
    return idx.astype(np.uint8) if levels <= 8 else idx


def distances_f64(P, X, n, c):
    """The K squared distances of sub-vector (n, c), double precision (near-tie diagnosis)."""
    P = _c(P, np.float32)
    X = _c(X, np.float32)
    C, K, V = P.shape
    d = np.empty(K, dtype=np.float64)
    _lib().lutnn_oracle_distances_f64(_ptr(P, _f32p), C, K, V, _ptr(X, _f32p), X.shape[1], int(n),
                                      int(c), _ptr(d, _f64p))
    return d


def lookup_i8(q, scale, idx, bias=None, return_acc=False):
    """Eq. 4 on an INT8 table: exact int32 sum, then Y = fma(acc, s, bias).  idx: uint8 or uint16."""
    q = _c(q, np.int8)
    assert np.asarray(idx).dtype in (np.uint8, np.uint16)
    idx = _c(idx, np.uint16)  # widened, values unchanged
    C, K, M = q.shape
    N = idx.shape[0]
    assert idx.shape[1] == C
    assert idx.size == 0 or int(idx.max()) < K
    Y = np.empty((N, M), dtype=np.float32)
    acc = np.empty((N, M), dtype=np.int32) if return_acc else None
    b = None if bias is None else _c(bias, np.float32)
    _lib().lutnn_oracle_lookup_i8(_ptr(q, _i8p), ctypes.c_float(float(scale)),
                                  None if b is None else _ptr(b, _f32p), C, K, M,
                                  _ptr(idx, _u16p), N, _ptr(Y, _f32p), M,
                                  None if acc is None else _ptr(acc, _i32p))
    return (Y, acc) if return_acc else Y


def lookup_f32(Tf, idx, bias=None):
    """Eq. 4 on an fp32 table: double-precision sum rounded once to fp32.  idx: uint8 or uint16."""
    Tf = _c(Tf, np.float32)
    assert np.asarray(idx).dtype in (np.uint8, np.uint16)
    idx = _c(idx, np.uint16)  # widened, values unchanged
    C, K, M = Tf.shape
    N = idx.shape[0]
    assert idx.shape[1] == C
    assert idx.size == 0 or int(idx.max()) < K
    Y = np.empty((N, M), dtype=np.float32)
    b = None if bias is None else _c(bias, np.float32)
    _lib().lutnn_oracle_lookup_f32(_ptr(Tf, _f32p), None if b is None else _ptr(b, _f32p), C, K, M,
                                   _ptr(idx, _u16p), N, _ptr(Y, _f32p), M)
    return Y


def linear_i8(P, q, scale, X, bias=None):
    """encode (Eq. 2) then INT8 lookup (Eq. 4)."""
    return lookup_i8(q, scale, encode(P, X), bias)


def linear_f32(P, Tf, X, bias=None):
    """encode (Eq. 2) then fp32 lookup (Eq. 4)."""
    return lookup_f32(Tf, encode(P, X), bias)
