"""GPU parity on seeded random shapes: the whole operator (arXiv 2302.03213 Eq. 2 + Eq. 4) through
every lookup variant the shape admits, against the CPU oracle.  The hand-picked shapes of the other
files aim at known tile edges; these draws are there for the combinations nobody thought of (a
launcher's price list picking an unusual tile for a ragged shape, a fallback taken for an odd
alignment).  Same bars as everywhere: indices bit-exact except counted near-ties, INT8-table outputs
bit-exact, fp32-table outputs within 1e-5 relative / 1e-4 absolute."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
from gpu_util import OracleLayer, dev, host, near_tie_report

pytestmark = pytest.mark.gpu

F32_RTOL, F32_ATOL = 1e-5, 1e-4


@pytest.fixture(scope="module")
def lut():
    import paper_2302_03213_amd as lut_mod
    assert torch.cuda.is_available(), "GPU tests need a GPU"
    return lut_mod


def draw_shape(seed):
    """One shape per seed, sized so that the oracle needs at most a few seconds."""
    rng = np.random.default_rng(1000 + seed)
    dtype = rng.choice(["i8", "i8", "i8", "f32"])
    K = int(rng.choice([16, 16, 16, 8, int(rng.integers(1, 16)), int(rng.integers(17, 65)), 256]))
    V = int(rng.choice([1, 2, 3, 4, 4, 5, 8, 9, 9, 16, 32]))
    if rng.random() < 0.5:
        C = 32 * int(rng.integers(1, 13))          # the sparse matrix-core lookup needs C % 32 == 0
    else:
        C = int(rng.integers(1, 200))
    # a third of the draws small in either direction, the rest large enough for several tiles
    N = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(9000.0))))
    M = int(np.exp(rng.uniform(0.0, np.log(64.0)) if rng.random() < 0.3 else rng.uniform(np.log(64.0), np.log(4300.0))))
    # bound the oracle's work: encode N*C*K*V, lookup N*C*M
    while N * C * K * V > 1.5e9 or N * C * M > 2.5e9:
        N = max(1, N // 2)
    return N, C, K, V, M, str(dtype)


@pytest.mark.parametrize("seed", range(48))
def test_linear_on_a_random_shape(lut, seed):
    N, C, K, V, M, dtype = draw_shape(seed)
    print("\n[case] seed %d: N=%d C=%d K=%d V=%d M=%d %s" % (seed, N, C, K, V, M, dtype),
          file=sys.stderr, flush=True)
    w = wl.make_layer("t", N, C, K, V, M, dtype, seed=seed, bias=bool(seed & 1))
    ol = OracleLayer(w)
    idx_ref = ol.encode()
    ref = ol.lookup(idx_ref, bias=w.bias)
    table_dtype = lut.TABLE_I8 if dtype == "i8" else lut.TABLE_F32
    layer = lut.build_table(dev(w.P), dev(w.W), table_dtype, bias=dev(w.bias))
    Xd = dev(w.X)
    idx_gpu = host(lut.encode(layer, Xd))
    flips = near_tie_report(w, idx_gpu, idx_ref)
    assert flips <= max(1, idx_ref.size // 10000), "%d near-ties" % flips
    clean = (idx_gpu == idx_ref).all(axis=1)
    ran = []
    for variant in ("auto", "lds", "mfma", "smfmac", "fused"):
        Ybig = torch.full((N, M + 3), -7.25, dtype=torch.float32, device="cuda")
        try:
            lut.linear(layer, Xd, variant, out=Ybig[:, :M])
        except lut.LutnnError as e:
            assert variant != "auto" and e.name == "LUTNN_E_UNSUPPORTED", (variant, str(e))
            continue
        ran.append(variant)
        got = host(Ybig[:, :M])
        assert (host(Ybig[:, M:]) == -7.25).all(), "variant %s wrote past its rows" % variant
        if dtype == "i8":
            bad = got[clean] != ref[clean]
            assert not bad.any(), "variant %s: %d elements differ" % (variant, bad.sum())
        else:
            np.testing.assert_allclose(got[clean], ref[clean], rtol=F32_RTOL, atol=F32_ATOL,
                                       err_msg="variant %s" % variant)
    assert "auto" in ran and "lds" in ran
