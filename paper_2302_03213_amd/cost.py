"""Cost model of a LUT-NN linear operator (arXiv 2302.03213, Sec. 4, Table 1) and the work /
traffic figures the benchmark prices against the MI355X rooflines.  Pure host arithmetic."""

# MI355X published peaks used as roofline denominators.
PEAK_HBM_BYTES_PER_S = 8.0e12
PEAK_MFMA_INT8_OPS_PER_S = 5.0e15
PEAK_VALU_F32_LANE_OPS_PER_S = 256 * 64 * 2.4e9  # 256 CUs x 64 lanes x 2.4 GHz, one op per lane-clock
PEAK_LDS_BYTES_PER_S = 256 * 128 * 2.4e9         # 256 CUs x 128 bytes per clock x 2.4 GHz = 78.6 TB/s

# One 32x32 int8 matrix instruction - dense v_mfma_i32_32x32x32_i8 or 2:4-sparse
# v_smfmac_i32_32x32x64_i8 - holds its SIMD's matrix pipe for 32 cycles, the time in which the dense
# form performs 2*32*32*32 = 65,536 ops.  1024 SIMDs x 65,536 / 32 cycles x 2.4 GHz = 5.03e15: the
# published dense peak, so pricing every issued instruction at 65,536 ops against that peak gives the
# share of the pipes' time the kernel's instructions occupy.
MFMA_I8_32X32_OPS_PER_PIPE_SLOT = 2 * 32 * 32 * 32


def lut_flops(N, D, M, K, V):
    """Table 1, "Ours": N*D*K (encoding) + N*M*D/V (lookup + aggregation); a multiply-add counts 1."""
    return N * D * K + N * M * D // V


def mm_flops(N, D, M):
    """Table 1, "MM": N*D*M."""
    return N * D * M


def flops_reduction(M, K, V):
    """Sec. 6.2: M / (K + M/V)."""
    return M / (K + M / V)


def lut_size_bytes(D, M, K, V):
    """Table 1, "Ours": 4*D*K (fp32 codebooks) + D*M*K/V (INT8 table)."""
    return 4 * D * K + D * M * K // V


def mm_size_bytes(D, M):
    """Table 1, "MM": 4*D*M."""
    return 4 * D * M


def equivalent_flops(N, D, M):
    """FLOPs of the dense product the operator replaces, multiply and add counted separately."""
    return 2 * N * D * M


def encode_bytes(N, C, V):
    """Algorithmic HBM bytes of the encoder: read X once (4*D per row), write idx (C per row)."""
    return N * (4 * C * V + C)


def encode_lane_ops(N, C, K, V):
    """VALU lane-ops of the direct-form distance + arg-min: per (row, codebook, centroid)
    V subtracts + V fused multiply-adds + one compare + one select."""
    return N * C * K * (2 * V + 2)


def softpq_backward_lane_ops(N, C, K, V):
    """VALU lane-ops of the soft-PQ backward formulas (Eq. 5-6) per (row, codebook): per centroid
    3V for the distance and dL/ds (subtract, two fused multiply-adds per element), 4V for the input
    gradient and the centroid contribution (subtract, multiply, add, fused multiply-add), and about 10
    for the softmax and its derivative (min, scale, exponential, sum, normalise, mean, difference,
    product, temperature term, sign/scale).  The sums over rows are not counted."""
    return N * C * K * (7 * V + 10)


def softpq_backward_bytes(N, C, V, with_dx=True):
    """Algorithmic HBM bytes: read X and Z once, write dX once (4 bytes each per element)."""
    return N * C * V * 4 * (3 if with_dx else 2)


def lookup_entries(N, C, M):
    """Table entries read and added by Eq. 4."""
    return N * C * M


def lookup_mfma_ops(N, C, M, kpad=16):
    """Dense INT8 ops of the one-hot contraction: 2 * N * (C*kpad) * M (1/kpad of them useful)."""
    return 2 * N * C * kpad * M


# Measured, not published: a loop of nothing but v_smfmac_i32_32x32x64_i8 (16 independent accumulators,
# one wave per SIMD, every SIMD of the chip busy) on full-range random INT8 B operands and random
# one-hot A operands issues one instruction per SIMD every 19.0 ns (32.8 cycles at the 1.66-1.72 GHz
# the chip holds under that load; 13.8-15 ns on constant operands).  The floor of the one-hot
# contraction on such data, whatever feeds the pipes.
SMFMAC_I8_STREAM_SECONDS_RANDOM_OPERANDS = 19.0e-9
SIMDS = 1024


def lookup_matrix_instructions(N, C, M, sparse, kpad=16):
    """32x32 int8 matrix instructions of the one-hot contraction OneHot[N x C*kpad] x T[C*kpad x M]: a
    dense instruction covers 32 of the contraction's C*kpad positions (two codebooks at kpad = 16), a
    2:4-sparse one 64 (four codebooks).  Unpadded (algorithmic) count; may be fractional."""
    per = 64 if sparse else 32
    return N * M * C * kpad / (32 * 32 * per)


def lookup_lds_floor_s(N, C, M, table_elem_bytes):
    """Time for Eq. 4's N*C*M table entries to cross the LDS once at its peak rate: the floor of a
    gather kernel that reads every entry it adds from LDS."""
    return N * C * M * table_elem_bytes / PEAK_LDS_BYTES_PER_S


def lookup_hbm_bytes(N, C, K, M, table_elem_bytes):
    """Algorithmic HBM bytes of the lookup: idx in, Y out, the table once."""
    return N * C + 4 * N * M + C * K * M * table_elem_bytes
