"""Helpers shared by the GPU parity tests: move seeded inputs to the device, build both sides'
layers, and classify index disagreements as near-ties.  Expected values always come from the
oracle (or numpy on oracle outputs); nothing computed by the HIP path is ever fed to the oracle."""
import numpy as np
import torch

import oracle


def dev(a):
    if a is None:
        return None
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t):
    torch.cuda.synchronize()
    return t.cpu().numpy()


class OracleLayer:
    """Oracle-side tables of a workload."""

    def __init__(self, w):
        self.w = w
        self.Tf = oracle.build_table_f32(w.P, w.W)
        if w.table_dtype == "i8":
            self.q, self.s = oracle.quantize_i8(self.Tf)
        else:
            self.q, self.s = None, None

    def encode(self, X=None):
        return oracle.encode(self.w.P, self.w.X if X is None else X)

    def lookup(self, idx, bias="layer"):
        b = self.w.bias if isinstance(bias, str) else bias
        if self.w.table_dtype == "i8":
            return oracle.lookup_i8(self.q, self.s, idx, b)
        return oracle.lookup_f32(self.Tf, idx, b)


def packed_from_q(q, mp_pad=256):
    """Numpy re-layout of an oracle INT8 table into the documented MFMA operand layout
    [C * ceil(K/16)][Mp][16], k fastest, zero padded (include/lutnn.h, lutnn_build_table)."""
    C, K, M = q.shape
    Kb = (K + 15) // 16
    Mp = (M + mp_pad - 1) // mp_pad * mp_pad
    out = np.zeros((C, Kb, Mp, 16), dtype=np.int8)
    for k in range(K):
        out[:, k // 16, :M, k % 16] = q[:, k, :]
    return out.reshape(C * Kb, Mp, 16)


def device_layer_from_oracle(lut, ol, with_bias=True):
    """A lutnn LutLayer whose tables are the ORACLE's (so a lookup test isolates the lookup)."""
    w = ol.w
    bias = dev(w.bias) if (with_bias and w.bias is not None) else None
    if w.table_dtype == "i8":
        return lut.LutLayer(dev(w.P), dev(ol.q), lut.TABLE_I8, w.M, packed=dev(packed_from_q(ol.q)),
                            scale=dev(np.array([ol.s], np.float32)), bias=bias)
    return lut.LutLayer(dev(w.P), dev(ol.Tf), lut.TABLE_F32, w.M, bias=bias)


def near_tie_report(w, idx_gpu, idx_ref, X=None, rel=1e-6):
    """Every disagreement must be a near-tie: the two candidates' fp64 distances differ by less
    than `rel` relative.  Returns the number of (counted, documented) near-ties."""
    X = w.X if X is None else X
    bad = np.argwhere(idx_gpu != idx_ref)
    for n, c in bad:
        d = oracle.distances_f64(w.P, X, n, c)
        a, b = d[idx_gpu[n, c]], d[idx_ref[n, c]]
        assert abs(a - b) <= rel * max(a, b), \
            "index mismatch at row %d codebook %d is not a near-tie: %r vs %r" % (n, c, a, b)
    return len(bad)
