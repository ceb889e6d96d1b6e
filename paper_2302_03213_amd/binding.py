"""Thin ctypes binding of liblutnn.so (C ABI in include/lutnn.h).

Argument marshalling only: every step of the operator runs in the HIP kernels.  PyTorch is used
for device memory and streams.  There is no CPU fallback: if the shared library cannot be loaded
the import of this module fails.

Names and notation follow arXiv 2302.03213: N rows, D = C*V inputs, K centroids per codebook,
M outputs; codebooks P[C][K][V], weights W[D][M] (Table 1), table T[C][K][M] (Eq. 3).
"""
import ctypes
import os

import torch

from . import build as _build

TABLE_F32 = 0
TABLE_I8 = 1
TABLE_I4 = 2

VARIANT_AUTO = 0
VARIANT_LDS = 1
VARIANT_MFMA = 2
VARIANT_FUSED = 3
VARIANT_SMFMAC = 4

VARIANTS = {"auto": VARIANT_AUTO, "lds": VARIANT_LDS, "mfma": VARIANT_MFMA, "fused": VARIANT_FUSED,
            "smfmac": VARIANT_SMFMAC}

EXPORTS = ["lutnn_softpq_backward_static", "lutnn_set_tunable", "lutnn_encode_tree16", "lutnn_lookup16",
           "lutnn_linear_tree16", "lutnn_table_bytes", "lutnn_packed_bytes", "lutnn_build_table", "lutnn_encode",
           "lutnn_lookup", "lutnn_linear", "lutnn_encode_tree", "lutnn_linear_tree",
           "lutnn_softpq_backward", "lutnn_softpq_workspace_bytes",
           "lutnn_encode_tree_conv2d", "lutnn_conv2d_tree", "lutnn_conv2d_rows", "lutnn_encode_conv2d", "lutnn_conv2d",
           "lutnn_auto_variant", "lutnn_linear_auto_variant", "lutnn_status_string", "lutnn_last_error", "lutnn_version",
           "lutnn_probe_smfmac_stream"]


class LutnnError(RuntimeError):
    def __init__(self, status, name, detail):
        super().__init__("%s: %s" % (name, detail))
        self.status = status
        self.name = name


class _CLayer(ctypes.Structure):
    _fields_ = [("C", ctypes.c_int32), ("K", ctypes.c_int32), ("V", ctypes.c_int32),
                ("M", ctypes.c_int32), ("table_dtype", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("centroids", ctypes.c_void_p),
                ("table", ctypes.c_void_p), ("table_packed", ctypes.c_void_p),
                ("scale", ctypes.c_void_p), ("bias", ctypes.c_void_p)]


class _CConvGeom(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("Cin", "H", "W", "kh", "kw", "stride_h", "stride_w",
                                              "pad_h", "pad_w", "reserved")]


class _CTree(ctypes.Structure):
    _fields_ = [("C", ctypes.c_int32), ("V", ctypes.c_int32), ("levels", ctypes.c_int32),
                ("reserved", ctypes.c_int32), ("split_dim", ctypes.c_void_p),
                ("threshold", ctypes.c_void_p)]


def _is_current(path):
    """True if the library file was compiled from the sources as they are now: its version string
    (lutnn_version()) ends in their hash.  Read from the file, so a stale library is never mapped."""
    with open(path, "rb") as f:
        return (b"+" + _build.source_hash().encode() + b"\0") in f.read()


def _load():
    path = _build.LIB
    if not os.path.exists(path) or not _is_current(path):
        _build.build()  # raises if hipcc is missing or the compile fails
    lib = ctypes.CDLL(path)
    missing = [name for name in EXPORTS if not hasattr(lib, name)]
    if missing:
        raise ImportError("liblutnn.so lacks %s" % ", ".join(missing))
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.lutnn_table_bytes.restype = ctypes.c_size_t
    lib.lutnn_table_bytes.argtypes = [i32, i32, i32, i32]
    lib.lutnn_packed_bytes.restype = ctypes.c_size_t
    lib.lutnn_packed_bytes.argtypes = [i32, i32, i32, i32]
    lib.lutnn_build_table.restype = i32
    lib.lutnn_build_table.argtypes = [vp, vp, i64, i32, i32, i32, i32, i32, vp, vp, vp, vp]
    lib.lutnn_encode.restype = i32
    lib.lutnn_encode.argtypes = [ctypes.POINTER(_CLayer), vp, i64, i64, vp, vp]
    lib.lutnn_lookup.restype = i32
    lib.lutnn_lookup.argtypes = [ctypes.POINTER(_CLayer), vp, i64, vp, i64, i32, vp]
    lib.lutnn_linear.restype = i32
    lib.lutnn_linear.argtypes = [ctypes.POINTER(_CLayer), vp, i64, i64, vp, i64, i32, vp, vp]
    lib.lutnn_encode_tree.restype = i32
    lib.lutnn_encode_tree.argtypes = [ctypes.POINTER(_CTree), vp, i64, i64, vp, vp]
    lib.lutnn_linear_tree.restype = i32
    lib.lutnn_linear_tree.argtypes = [ctypes.POINTER(_CLayer), ctypes.POINTER(_CTree), vp, i64, i64, vp,
                                      i64, i32, vp, vp]
    lib.lutnn_encode_tree16.restype = i32
    lib.lutnn_encode_tree16.argtypes = [ctypes.POINTER(_CTree), vp, i64, i64, vp, vp]
    lib.lutnn_lookup16.restype = i32
    lib.lutnn_lookup16.argtypes = [ctypes.POINTER(_CLayer), vp, i64, vp, i64, vp]
    lib.lutnn_linear_tree16.restype = i32
    lib.lutnn_linear_tree16.argtypes = [ctypes.POINTER(_CLayer), ctypes.POINTER(_CTree), vp, i64, i64, vp, i64,
                                        vp, vp]
    lib.lutnn_softpq_workspace_bytes.restype = ctypes.c_size_t
    lib.lutnn_softpq_workspace_bytes.argtypes = [i32, i32, i32, i64]
    lib.lutnn_softpq_backward.restype = i32
    lib.lutnn_softpq_backward.argtypes = [ctypes.POINTER(_CLayer), ctypes.c_float, vp, i64, i64, vp, i64, vp,
                                          vp, i64, vp, vp, ctypes.c_size_t, vp]
    lib.lutnn_softpq_backward_static.restype = i32
    lib.lutnn_softpq_backward_static.argtypes = [ctypes.POINTER(_CLayer), ctypes.c_float, vp, i64, i64, vp, i64,
                                                 vp, vp, i64, vp, vp]
    lib.lutnn_encode_tree_conv2d.restype = i32
    lib.lutnn_encode_tree_conv2d.argtypes = [ctypes.POINTER(_CTree), vp, i64, ctypes.POINTER(_CConvGeom), vp, vp]
    lib.lutnn_conv2d_tree.restype = i32
    lib.lutnn_conv2d_tree.argtypes = [ctypes.POINTER(_CLayer), ctypes.POINTER(_CTree), vp, i64,
                                      ctypes.POINTER(_CConvGeom), vp, i64, i32, vp, vp]
    lib.lutnn_conv2d_rows.restype = i64
    lib.lutnn_conv2d_rows.argtypes = [ctypes.POINTER(_CConvGeom), i64]
    lib.lutnn_encode_conv2d.restype = i32
    lib.lutnn_encode_conv2d.argtypes = [ctypes.POINTER(_CLayer), vp, i64, ctypes.POINTER(_CConvGeom), vp, vp]
    lib.lutnn_conv2d.restype = i32
    lib.lutnn_conv2d.argtypes = [ctypes.POINTER(_CLayer), vp, i64, ctypes.POINTER(_CConvGeom), vp, i64,
                                 i32, vp, vp]
    lib.lutnn_auto_variant.restype = i32
    lib.lutnn_auto_variant.argtypes = [ctypes.POINTER(_CLayer), vp, i64]
    lib.lutnn_linear_auto_variant.restype = i32
    lib.lutnn_linear_auto_variant.argtypes = [ctypes.POINTER(_CLayer), vp, i64]
    lib.lutnn_status_string.restype = ctypes.c_char_p
    lib.lutnn_status_string.argtypes = [i32]
    lib.lutnn_last_error.restype = ctypes.c_char_p
    lib.lutnn_version.restype = ctypes.c_char_p
    lib.lutnn_set_tunable.restype = i32
    lib.lutnn_set_tunable.argtypes = [ctypes.c_char_p, ctypes.c_char_p]
    lib.lutnn_probe_smfmac_stream.restype = i32
    lib.lutnn_probe_smfmac_stream.argtypes = [i32, i32, vp, ctypes.c_size_t, vp]
    return lib


LIB = _load()


def _check(status):
    if status != 0:
        raise LutnnError(status, LIB.lutnn_status_string(status).decode(),
                         LIB.lutnn_last_error().decode())


def _stream():
    return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _variant(v):
    return VARIANTS[v] if isinstance(v, str) else int(v)


def set_tunable(name, value=None):
    """lutnn_set_tunable: pin ("small", "1", "256", ...) or release (None) a launcher's choice."""
    _check(LIB.lutnn_set_tunable(name.encode(), None if value is None else str(value).encode()))


def probe_smfmac_stream(operands, iterations, sink):
    """lutnn_probe_smfmac_stream: 16 * iterations matrix instructions per wave on every SIMD; `sink` is an
    int32 device tensor of at least 256 elements per compute unit."""
    assert sink.is_cuda and sink.dtype == torch.int32 and sink.is_contiguous()
    _check(LIB.lutnn_probe_smfmac_stream(operands, iterations, _ptr(sink), sink.numel() * 4, _stream()))


class tunables:
    """Context manager: pins the given switches for the block, releases them afterwards."""

    def __init__(self, **pins):
        self.pins = pins

    def __enter__(self):
        for name, value in self.pins.items():
            set_tunable(name, value)
        return self

    def __exit__(self, *exc):
        for name in self.pins:
            set_tunable(name, None)
        return False


def version():
    return LIB.lutnn_version().decode()


def table_bytes(C, K, M, dtype):
    return int(LIB.lutnn_table_bytes(C, K, M, dtype))


def packed_bytes(C, K, M, dtype):
    return int(LIB.lutnn_packed_bytes(C, K, M, dtype))


class LutLayer:
    """Device buffers of one LUT layer plus the C descriptor that points at them."""

    def __init__(self, centroids, table, table_dtype, M, packed=None, scale=None, bias=None):
        C, K, V = centroids.shape
        self.C, self.K, self.V, self.M = int(C), int(K), int(V), int(M)
        self.table_dtype = int(table_dtype)
        self.centroids, self.table, self.packed, self.scale, self.bias = \
            centroids, table, packed, scale, bias
        self.c = _CLayer(self.C, self.K, self.V, self.M, self.table_dtype, 0, _ptr(centroids),
                         _ptr(table), _ptr(packed), _ptr(scale), _ptr(bias))

    @property
    def D(self):
        return self.C * self.V


def build_table(centroids, W, table_dtype, bias=None, packed=True):
    """lutnn_build_table: Eq. 3 (+ Sec. 3.3 for INT8 / INT4).  centroids [C,K,V], W [D,M] on the GPU."""
    assert centroids.is_cuda and W.is_cuda and centroids.dtype == torch.float32
    assert centroids.is_contiguous() and W.dtype == torch.float32 and W.stride(1) == 1
    C, K, V = centroids.shape
    D, M = W.shape
    if D != C * V:
        raise ValueError("W has %d rows, expected C*V = %d" % (D, C * V))
    dev = centroids.device
    if table_dtype == TABLE_F32:
        table = torch.empty((C, K, M), dtype=torch.float32, device=dev)
        pk, scale = None, None
    else:
        if table_dtype == TABLE_I4:  # two 4-bit entries per byte, even column in the low nibble
            table = torch.empty((C, K, (M + 1) // 2), dtype=torch.uint8, device=dev)
        else:
            table = torch.empty((C, K, M), dtype=torch.int8, device=dev)
        scale = torch.empty(1, dtype=torch.float32, device=dev)
        pk = None
        if packed and K <= 256:  # the matrix-core operand copy exists for 8-bit indices only
            nbytes = packed_bytes(C, K, M, table_dtype)
            pk = torch.empty(nbytes, dtype=torch.int8, device=dev)
    _check(LIB.lutnn_build_table(_ptr(centroids), _ptr(W), W.stride(0), C, K, V, M, table_dtype,
                                 _ptr(table), _ptr(pk), _ptr(scale), _stream()))
    return LutLayer(centroids, table, table_dtype, M, pk, scale, bias)


def encode(layer, X, out=None):
    """lutnn_encode: Eq. 2.  X [N, D] fp32 (row stride free) -> idx [N, C] uint8."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, layer.C), dtype=torch.uint8, device=X.device)
    assert out.is_contiguous() and out.shape == (N, layer.C) and out.dtype == torch.uint8
    _check(LIB.lutnn_encode(ctypes.byref(layer.c), _ptr(X), N, X.stride(0), _ptr(out), _stream()))
    return out


def lookup(layer, idx, variant="auto", out=None):
    """lutnn_lookup: Eq. 4.  idx [N, C] uint8 -> Y [N, M] fp32."""
    assert idx.is_cuda and idx.dtype == torch.uint8 and idx.is_contiguous()
    N = idx.shape[0]
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=idx.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    _check(LIB.lutnn_lookup(ctypes.byref(layer.c), _ptr(idx), N, _ptr(out), out.stride(0),
                            _variant(variant), _stream()))
    return out


class LutTree:
    """Device buffers of the hash encoder's threshold trees (Sec. 2) plus their C descriptor.
    split_dim [C, 2^levels - 1] int32 and threshold (same shape) fp32, heap order."""

    def __init__(self, split_dim, threshold, V):
        assert split_dim.is_cuda and threshold.is_cuda
        assert split_dim.dtype == torch.int32 and threshold.dtype == torch.float32
        assert split_dim.shape == threshold.shape and split_dim.dim() == 2
        C, nodes = split_dim.shape
        levels = (nodes + 1).bit_length() - 1
        assert nodes == (1 << levels) - 1, "a tree has 2^levels - 1 nodes"
        self.C, self.V, self.levels, self.K = int(C), int(V), levels, 1 << levels
        self.split_dim = split_dim.contiguous()
        self.threshold = threshold.contiguous()
        self.c = _CTree(self.C, self.V, levels, 0, self.split_dim.data_ptr(), self.threshold.data_ptr())


def encode_tree(tree, X, out=None):
    """lutnn_encode_tree: hash encoding.  X [N, D] fp32 (row stride free) -> idx [N, C] uint8."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, tree.C), dtype=torch.uint8, device=X.device)
    assert out.is_contiguous() and out.shape == (N, tree.C) and out.dtype == torch.uint8
    _check(LIB.lutnn_encode_tree(ctypes.byref(tree.c), _ptr(X), N, X.stride(0), _ptr(out), _stream()))
    return out


def linear_tree(layer, tree, X, variant="auto", out=None, idx_workspace=None):
    """lutnn_linear_tree: hash encoding, then the table lookup of Eq. 4."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=X.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    v = _variant(variant)
    if idx_workspace is None and v != VARIANT_FUSED:
        idx_workspace = torch.empty((N, layer.C), dtype=torch.uint8, device=X.device)
    _check(LIB.lutnn_linear_tree(ctypes.byref(layer.c), ctypes.byref(tree.c), _ptr(X), N, X.stride(0),
                                 _ptr(out), out.stride(0), v, _ptr(idx_workspace), _stream()))
    return out


def encode_tree16(tree, X, out=None):
    """lutnn_encode_tree16: the hash encoder with 16-bit leaves (trees of up to 12 levels)."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, tree.C), dtype=torch.int16, device=X.device)
    assert out.dtype == torch.int16 and out.is_contiguous() and out.shape == (N, tree.C)
    _check(LIB.lutnn_encode_tree16(ctypes.byref(tree.c), _ptr(X), N, X.stride(0), _ptr(out), _stream()))
    return out


def lookup16(layer, idx, out=None):
    """lutnn_lookup16: Eq. 4 on 16-bit indices (torch has no uint16 arithmetic: an int16 tensor
    carries the bits)."""
    assert idx.is_cuda and idx.dtype == torch.int16 and idx.is_contiguous()
    N = idx.shape[0]
    assert idx.shape == (N, layer.C)
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=idx.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    _check(LIB.lutnn_lookup16(ctypes.byref(layer.c), _ptr(idx), N, _ptr(out), out.stride(0), _stream()))
    return out


def linear_tree16(layer, tree, X, out=None, idx_workspace=None):
    """lutnn_linear_tree16: deep-tree hash encoding, then the 16-bit index lookup."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=X.device)
    if idx_workspace is None:
        idx_workspace = torch.empty((N, layer.C), dtype=torch.int16, device=X.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    _check(LIB.lutnn_linear_tree16(ctypes.byref(layer.c), ctypes.byref(tree.c), _ptr(X), N, X.stride(0),
                                   _ptr(out), out.stride(0), _ptr(idx_workspace), _stream()))
    return out


def softpq_workspace_bytes(C, K, V, N):
    return int(LIB.lutnn_softpq_workspace_bytes(C, K, V, N))


def softpq_backward(layer, temperature, X, Z, need_dx=True, workspace=None):
    """lutnn_softpq_backward: gradients of the soft output (Eq. 5-6) from Z = dL/dY @ W^T.
    Returns (dP [C, K, V], dX [N, D] or None, dt [1])."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    assert Z.is_cuda and Z.dtype == torch.float32 and Z.stride(1) == 1 and Z.shape == X.shape
    N = X.shape[0]
    dP = torch.empty((layer.C, layer.K, layer.V), dtype=torch.float32, device=X.device)
    dX = torch.empty((N, layer.C * layer.V), dtype=torch.float32, device=X.device) if need_dx else None
    dt = torch.empty(1, dtype=torch.float32, device=X.device)
    need = softpq_workspace_bytes(layer.C, layer.K, layer.V, N)
    if workspace is None:
        workspace = torch.empty(max(need, 4), dtype=torch.uint8, device=X.device)
    assert workspace.is_cuda and workspace.is_contiguous()
    _check(LIB.lutnn_softpq_backward(ctypes.byref(layer.c), float(temperature), _ptr(X), N, X.stride(0),
                                     _ptr(Z), Z.stride(0), _ptr(dP), _ptr(dX),
                                     dX.stride(0) if need_dx else 0, _ptr(dt), _ptr(workspace),
                                     workspace.numel() * workspace.element_size(), _stream()))
    return dP, dX, dt


def softpq_backward_static(layer, temperature, X, Z, need_dx=True, dP=None, dX=None, dt=None):
    """lutnn_softpq_backward_static: the same gradients with the library's static scratch array in
    place of a workspace.  Pass dP, dX, dt to have the call itself allocate nothing."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    assert Z.is_cuda and Z.dtype == torch.float32 and Z.stride(1) == 1 and Z.shape == X.shape
    N = X.shape[0]
    if dP is None:
        dP = torch.empty((layer.C, layer.K, layer.V), dtype=torch.float32, device=X.device)
    if dX is None and need_dx:
        dX = torch.empty((N, layer.C * layer.V), dtype=torch.float32, device=X.device)
    if dt is None:
        dt = torch.empty(1, dtype=torch.float32, device=X.device)
    assert dP.is_contiguous() and dP.shape == (layer.C, layer.K, layer.V) and dt.numel() == 1
    assert not need_dx or (dX.stride(1) == 1 and dX.shape == (N, layer.C * layer.V))
    _check(LIB.lutnn_softpq_backward_static(ctypes.byref(layer.c), float(temperature), _ptr(X), N, X.stride(0),
                                            _ptr(Z), Z.stride(0), _ptr(dP), _ptr(dX) if need_dx else None,
                                            dX.stride(0) if need_dx else 0, _ptr(dt), _stream()))
    return dP, (dX if need_dx else None), dt


def _pair(v):
    return (int(v), int(v)) if isinstance(v, int) else (int(v[0]), int(v[1]))


def conv_geom(inp, kernel, stride=1, pad=0):
    """Geometry descriptor for an NCHW batch `inp` and a kh x kw filter."""
    (kh, kw), (sh, sw), (ph, pw) = _pair(kernel), _pair(stride), _pair(pad)
    return _CConvGeom(inp.shape[1], inp.shape[2], inp.shape[3], kh, kw, sh, sw, ph, pw, 0)


def conv2d_rows(geom, B):
    return int(LIB.lutnn_conv2d_rows(ctypes.byref(geom), B))


def encode_conv2d(layer, inp, kernel, stride=1, pad=0, out=None):
    """lutnn_encode_conv2d: Eq. 2 on the rows of the im2col matrix of `inp` [B, Cin, H, W], read
    in place.  Returns idx [B*Ho*Wo, C] uint8."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 4
    geom = conv_geom(inp, kernel, stride, pad)
    N = conv2d_rows(geom, inp.shape[0])
    if N < 0:
        raise ValueError("invalid convolution geometry")
    if out is None:
        out = torch.empty((N, layer.C), dtype=torch.uint8, device=inp.device)
    assert out.is_contiguous() and out.shape == (N, layer.C) and out.dtype == torch.uint8
    _check(LIB.lutnn_encode_conv2d(ctypes.byref(layer.c), _ptr(inp), inp.shape[0], ctypes.byref(geom),
                                   _ptr(out), _stream()))
    return out


def conv2d(layer, inp, kernel, stride=1, pad=0, variant="auto", out=None, idx_workspace=None):
    """lutnn_conv2d: the convolution, Y [B*Ho*Wo, M] (output pixels by output channels)."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 4
    geom = conv_geom(inp, kernel, stride, pad)
    N = conv2d_rows(geom, inp.shape[0])
    if N < 0:
        raise ValueError("invalid convolution geometry")
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=inp.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    if idx_workspace is None:
        idx_workspace = torch.empty((N, layer.C), dtype=torch.uint8, device=inp.device)
    _check(LIB.lutnn_conv2d(ctypes.byref(layer.c), _ptr(inp), inp.shape[0], ctypes.byref(geom), _ptr(out),
                            out.stride(0), _variant(variant), _ptr(idx_workspace), _stream()))
    return out


def encode_tree_conv2d(tree, inp, kernel, stride=1, pad=0, out=None):
    """lutnn_encode_tree_conv2d: hash encoding of the im2col rows of `inp` [B, Cin, H, W], read in place."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 4
    geom = conv_geom(inp, kernel, stride, pad)
    N = conv2d_rows(geom, inp.shape[0])
    if N < 0:
        raise ValueError("invalid convolution geometry")
    if out is None:
        out = torch.empty((N, tree.C), dtype=torch.uint8, device=inp.device)
    assert out.is_contiguous() and out.shape == (N, tree.C) and out.dtype == torch.uint8
    _check(LIB.lutnn_encode_tree_conv2d(ctypes.byref(tree.c), _ptr(inp), inp.shape[0], ctypes.byref(geom),
                                        _ptr(out), _stream()))
    return out


def conv2d_tree(layer, tree, inp, kernel, stride=1, pad=0, variant="auto", out=None, idx_workspace=None):
    """lutnn_conv2d_tree: the convolution with the hash encoder, Y [B*Ho*Wo, M]."""
    assert inp.is_cuda and inp.dtype == torch.float32 and inp.is_contiguous() and inp.dim() == 4
    geom = conv_geom(inp, kernel, stride, pad)
    N = conv2d_rows(geom, inp.shape[0])
    if N < 0:
        raise ValueError("invalid convolution geometry")
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=inp.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    if idx_workspace is None:
        idx_workspace = torch.empty((N, layer.C), dtype=torch.uint8, device=inp.device)
    _check(LIB.lutnn_conv2d_tree(ctypes.byref(layer.c), ctypes.byref(tree.c), _ptr(inp), inp.shape[0],
                                 ctypes.byref(geom), _ptr(out), out.stride(0), _variant(variant),
                                 _ptr(idx_workspace), _stream()))
    return out


def auto_variant(layer, N, idx=None):
    """lutnn_auto_variant: name of the lookup variant that "auto" stands for at this shape."""
    code = LIB.lutnn_auto_variant(ctypes.byref(layer.c), _ptr(idx), N)
    return {v: k for k, v in VARIANTS.items()}[code]


def linear_auto_variant(layer, N, idx_workspace=None):
    """lutnn_linear_auto_variant: name of what lutnn_linear runs for "auto" at this shape ("fused" =
    one launch does both steps)."""
    code = LIB.lutnn_linear_auto_variant(ctypes.byref(layer.c), _ptr(idx_workspace), N)
    return {v: k for k, v in VARIANTS.items()}[code]


def linear(layer, X, variant="auto", out=None, idx_workspace=None):
    """lutnn_linear: the whole operator, Y ~= X @ W (+ bias)."""
    assert X.is_cuda and X.dtype == torch.float32 and X.stride(1) == 1
    N = X.shape[0]
    if out is None:
        out = torch.empty((N, layer.M), dtype=torch.float32, device=X.device)
    assert out.dtype == torch.float32 and out.stride(1) == 1 and out.shape == (N, layer.M)
    v = _variant(variant)
    if idx_workspace is None and v != VARIANT_FUSED:
        idx_workspace = torch.empty((N, layer.C), dtype=torch.uint8, device=X.device)
    _check(LIB.lutnn_linear(ctypes.byref(layer.c), _ptr(X), N, X.stride(0), _ptr(out),
                            out.stride(0), v, _ptr(idx_workspace), _stream()))
    return out
