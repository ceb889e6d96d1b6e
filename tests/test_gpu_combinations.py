"""GPU parity of combinations of the library's options that the per-feature tests do not pair up
(convolution input with fp32 / INT4 tables, hash encoder with INT4 tables), and of the entry points
under HIP graph capture.  Same bars as tests/test_gpu_parity.py."""
import sys

import numpy as np
import pytest
import torch

import lutnn_workloads as wl
import oracle
from gpu_util import dev, host, near_tie_report

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


def unfold_rows(inp, kernel, stride, pad):
    cols = torch.nn.functional.unfold(torch.from_numpy(inp), kernel, padding=pad, stride=stride)
    return cols.permute(0, 2, 1).reshape(-1, cols.shape[1]).contiguous().numpy()


@pytest.mark.parametrize("dtype", ["f32", "i4"])
def test_conv2d_with_fp32_and_int4_tables(lut, dtype):
    B, Cin, H, W, M = 2, 16, 14, 12, 40
    g = np.random.default_rng(3)
    inp = g.standard_normal((B, Cin, H, W)).astype(np.float32)
    w = wl.make_layer("t", 1, Cin, 16, 9, M, "f32", seed=9)
    X = unfold_rows(inp, (3, 3), (1, 1), (1, 1))
    idx_ref = oracle.encode(w.P, X)
    Tf = oracle.build_table_f32(w.P, w.W)
    if dtype == "f32":
        ref = oracle.lookup_f32(Tf, idx_ref, w.bias)
        layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_F32, bias=dev(w.bias))
    else:
        q, s = oracle.quantize(Tf, 4)
        ref = oracle.lookup_i8(q, s, idx_ref, w.bias)
        layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I4, bias=dev(w.bias))
    idx = host(lut.encode_conv2d(layer, dev(inp), 3, 1, 1))
    w.X = X
    assert near_tie_report(w, idx, idx_ref) <= 1
    clean = (idx == idx_ref).all(axis=1)
    variants = ["auto", "lds"] if dtype == "f32" else ["auto", "lds", "mfma"]
    for v in variants:
        got = host(lut.conv2d(layer, dev(inp), 3, 1, 1, v))
        if dtype == "f32":
            np.testing.assert_allclose(got[clean], ref[clean], rtol=1e-5, atol=1e-4, err_msg=v)
        else:
            np.testing.assert_array_equal(got[clean], ref[clean], err_msg=v)


def test_linear_tree_with_an_int4_table(lut):
    N, C, V, levels, M = 700, 64, 4, 4, 264
    w = wl.make_layer("t", N, C, 16, V, M, "i8", seed=31)
    dims, thr = wl.random_tree(C, V, levels, seed=31)
    q, s = oracle.quantize(oracle.build_table_f32(w.P, w.W), 4)
    ref = oracle.lookup_i8(q, s, oracle.encode_tree(dims, thr, w.X, V), w.bias)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I4, bias=dev(w.bias))
    tree = lut.LutTree(dev(dims), dev(thr), V)
    for v in ("auto", "lds", "mfma", "smfmac"):
        np.testing.assert_array_equal(host(lut.linear_tree(layer, tree, dev(w.X), v)), ref, err_msg=v)


def test_small_batch_paths_replayed_from_a_hip_graph(lut):
    """The small-batch paths under capture: 64 rows on a wide layer (codebooks split over workgroups:
    a zeroing pass, integer atomics into Y, a dequantising pass - every replay must start from
    zero again) and 4 rows (split gather)."""
    C, K, V, M = 1024, 16, 4, 512
    w = wl.make_layer("t", 64, C, K, V, M, "i8", seed=19)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    for N in (64, 4):
        X = dev(w.X[:N]).clone()
        Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
        ws = torch.empty((N, C), dtype=torch.uint8, device="cuda")
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            lut.linear(layer, X, "auto", out=Y, idx_workspace=ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lut.linear(layer, X, "auto", out=Y, idx_workspace=ws)
        rng = np.random.default_rng(N)
        for rep in range(4):
            Xn = rng.standard_normal((N, C * V)).astype(np.float32)
            X.copy_(dev(Xn))
            graph.replay()
            torch.cuda.synchronize()
            got = host(Y)
            idx_ref = oracle.encode(w.P, Xn)
            q, s = oracle.quantize_i8(oracle.build_table_f32(w.P, w.W))
            ref = oracle.lookup_i8(q, s, idx_ref, w.bias)
            clean = (host(ws) == idx_ref).all(axis=1)
            assert clean.mean() > 0.9
            np.testing.assert_array_equal(got[clean], ref[clean], err_msg="N=%d replay %d" % (N, rep))


@pytest.mark.parametrize("variant", ["auto", "smfmac", "mfma", "lds", "fused"])
def test_linear_replayed_from_a_hip_graph(lut, variant):
    """The entry points allocate nothing, clear nothing with memset nodes and never synchronise, so a
    captured lutnn_linear can be replayed; every replay, with fresh inputs written into the captured
    buffers and eager work in between, must equal the eager result."""
    N, C, K, V, M = 700, 64, 16, 4, 320
    w = wl.make_layer("t", N, C, K, V, M, "i8", seed=17)
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    X = dev(w.X).clone()
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    ws = torch.empty((N, C), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up on the capture stream, as torch asks
        lut.linear(layer, X, variant, out=Y, idx_workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lut.linear(layer, X, variant, out=Y, idx_workspace=ws)
    rng = np.random.default_rng(5)
    for rep in range(4):
        Xn = rng.standard_normal((N, C * V)).astype(np.float32)
        X.copy_(dev(Xn))
        Y.fill_(float("nan"))
        graph.replay()
        torch.cuda.synchronize()
        got = host(Y)
        eager = host(lut.linear(layer, dev(Xn), variant))
        np.testing.assert_array_equal(got, eager, err_msg="replay %d" % rep)
        float((dev(Xn) * 2).sum())  # unrelated eager work and a synchronisation between replays


def test_softpq_backward_and_tree_encode_replayed_from_a_hip_graph(lut):
    N, C, K, V = 1500, 32, 16, 4
    w = wl.make_layer("t", N, C, K, V, 8, "f32", seed=23)
    dims, thr = wl.random_tree(C, V, 4, seed=23)
    tree = lut.LutTree(dev(dims), dev(thr), V)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    X = dev(w.X).clone()
    Z = dev(np.random.default_rng(2).standard_normal((N, C * V)).astype(np.float32))
    ws = torch.empty(lut.softpq_workspace_bytes(C, K, V, N), dtype=torch.uint8, device="cuda")
    idx = torch.empty((N, C), dtype=torch.uint8, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lut.softpq_backward(layer, 1.0, X, Z, workspace=ws)
        lut.encode_tree(tree, X, out=idx)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        dP, dX, dt = lut.softpq_backward(layer, 1.0, X, Z, workspace=ws)
        lut.encode_tree(tree, X, out=idx)
    rng = np.random.default_rng(6)
    for rep in range(3):
        Xn = rng.standard_normal((N, C * V)).astype(np.float32)
        X.copy_(dev(Xn))
        graph.replay()
        torch.cuda.synchronize()
        e = lut.softpq_backward(layer, 1.0, dev(Xn), Z)
        for a, b in zip((dP, dX, dt), e):
            np.testing.assert_array_equal(host(a), host(b), err_msg="replay %d" % rep)
        np.testing.assert_array_equal(host(idx), oracle.encode_tree(dims, thr, Xn, V))


def test_static_scratch_backward_and_deep_tree_linear_replayed_from_a_hip_graph(lut):
    """The callers lutnn_softpq_backward_static exists for: captured once (after a first eager call,
    which looks the scratch array's address up), replayed with fresh inputs; and the 16-bit index
    operator (12-level trees) in the same graph."""
    N, C, K, V, M, levels = 1500, 32, 16, 4, 40, 12
    w = wl.make_layer("t", N, C, K, V, 8, "f32", seed=29)
    layer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, 8)
    X = dev(w.X).clone()
    Z = dev(np.random.default_rng(3).standard_normal((N, C * V)).astype(np.float32))
    dP = torch.empty((C, K, V), dtype=torch.float32, device="cuda")
    dX = torch.empty((N, C * V), dtype=torch.float32, device="cuda")
    dt = torch.empty(1, dtype=torch.float32, device="cuda")
    wt = wl.make_layer("t", 1, C, 1 << levels, V, M, "i8", seed=30)
    dims, thr = wl.random_tree(C, V, levels, seed=30)
    tree = lut.LutTree(dev(dims), dev(thr), V)
    deep = lut.build_table(dev(wt.P), dev(wt.W), lut.TABLE_I8, bias=dev(wt.bias))
    Y = torch.empty((N, M), dtype=torch.float32, device="cuda")
    ws16 = torch.empty((N, C), dtype=torch.int16, device="cuda")
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):  # warm-up outside capture
        lut.softpq_backward_static(layer, 1.0, X, Z, dP=dP, dX=dX, dt=dt)
        lut.linear_tree16(deep, tree, X, out=Y, idx_workspace=ws16)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lut.softpq_backward_static(layer, 1.0, X, Z, dP=dP, dX=dX, dt=dt)
        lut.linear_tree16(deep, tree, X, out=Y, idx_workspace=ws16)
    rng = np.random.default_rng(8)
    q, s = oracle.quantize_i8(oracle.build_table_f32(wt.P, wt.W))
    for rep in range(3):
        Xn = rng.standard_normal((N, C * V)).astype(np.float32)
        X.copy_(dev(Xn))
        graph.replay()
        torch.cuda.synchronize()
        e = lut.softpq_backward(layer, 1.0, dev(Xn), Z)
        for a, b in zip((dP, dX, dt), e):
            np.testing.assert_array_equal(host(a), host(b), err_msg="replay %d" % rep)
        idx_ref = oracle.encode_tree(dims, thr, Xn, V)
        np.testing.assert_array_equal(host(ws16).view(np.uint16), idx_ref)
        np.testing.assert_array_equal(host(Y), oracle.lookup_i8(q, s, idx_ref, wt.bias), err_msg="replay %d" % rep)
        float((dev(Xn) * 2).sum())  # unrelated eager work and a synchronisation between replays


def test_four_million_rows_cross_the_32_bit_byte_offsets(lut):
    """N = 2^22 + 77: X, Y and dX are larger than 2 GiB each, so every row offset the kernels form
    must be 64-bit.  The oracle checks the first and the last rows and a sample in between."""
    N, C, K, V, M = (1 << 22) + 77, 32, 16, 4, 128
    w = wl.make_layer("t", 1, C, K, V, M, "i8", seed=41)
    g = torch.Generator(device="cpu")
    g.manual_seed(41)
    X = torch.randn((N, C * V), generator=g, dtype=torch.float32)
    Xd = X.cuda()
    layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
    rows = np.unique(np.concatenate([np.arange(64), np.arange(N - 600, N),
                                     np.random.default_rng(1).integers(0, N, 2000),
                                     np.arange((1 << 21) - 32, (1 << 21) + 32)]))
    Xs = X.numpy()[rows]
    idx_ref = oracle.encode(w.P, Xs)
    Tf = oracle.build_table_f32(w.P, w.W)
    q, s = oracle.quantize_i8(Tf)
    ref = oracle.lookup_i8(q, s, idx_ref, w.bias)
    idx = lut.encode(layer, Xd)
    w.X = Xs
    got_idx = host(idx[torch.from_numpy(rows).cuda()])
    assert near_tie_report(w, got_idx, idx_ref) <= 1
    clean = (got_idx == idx_ref).all(axis=1)
    rows_d = torch.from_numpy(rows).cuda()
    for v in ("smfmac", "mfma", "lds"):
        Y = lut.lookup(layer, idx, v)
        np.testing.assert_array_equal(host(Y[rows_d])[clean], ref[clean], err_msg=v)
        del Y
    dims, thr = wl.random_tree(C, V, 4, seed=41)
    tidx = lut.encode_tree(lut.LutTree(dev(dims), dev(thr), V), Xd)
    np.testing.assert_array_equal(host(tidx[rows_d]), oracle.encode_tree(dims, thr, Xs, V))
    del tidx, idx
    # soft-PQ: dX rows are per-row quantities; compare the sampled ones with the fp64 oracle
    from oracle import softpq as osp
    G = np.random.default_rng(2).standard_normal((len(rows), M))
    Zs = (G @ w.W.astype(np.float64).T).astype(np.float32)
    Zd = torch.zeros((N, C * V), dtype=torch.float32, device="cuda")
    Zd[rows_d] = dev(Zs)
    flayer = lut.LutLayer(dev(w.P), None, lut.TABLE_F32, M)
    dP, dX, dt = lut.softpq_backward(flayer, 1.0, Xd, Zd)
    dP_ref, dX_ref, dt_ref = osp.backward(w.P, w.W, Xs, 1.0, G)  # rows with Z = 0 contribute nothing
    got = host(dX[rows_d])
    assert np.abs(got - dX_ref).max() <= 5e-5 * np.abs(dX_ref).max()
    assert np.abs(host(dP) - dP_ref).max() <= 5e-5 * np.abs(dP_ref).max()


def test_two_host_threads_on_two_streams(lut):
    """No state between calls: two host threads, each on its own stream with its own layer, get the
    results of a serial run (the second uses the small-batch path whose Y doubles as scratch)."""
    import threading
    cases = []
    for seed, (N, C, M) in enumerate([(700, 64, 320), (64, 1024, 512)]):
        w = wl.make_layer("t", N, C, 16, 4, M, "i8", seed=50 + seed)
        layer = lut.build_table(dev(w.P), dev(w.W), lut.TABLE_I8, bias=dev(w.bias))
        X = dev(w.X)
        cases.append((layer, X, host(lut.linear(layer, X))))
    torch.cuda.synchronize()
    results, errors = [None, None], []

    def work(i):
        try:
            layer, X, _ = cases[i]
            stream = torch.cuda.Stream()
            with torch.cuda.stream(stream):
                for _ in range(40):
                    Y = lut.linear(layer, X)
                stream.synchronize()
            results[i] = host(Y)
        except Exception as e:  # surfaced in the main thread below
            errors.append(e)

    threads = [threading.Thread(target=work, args=(i,)) for i in range(2)]
    for t in threads:
        t.start()
    for t in threads:
        t.join()
    assert not errors, errors
    for i in range(2):
        np.testing.assert_array_equal(results[i], cases[i][2])


def test_stream_probe_runs_and_fills_its_sink(lut):
    """lutnn_probe_smfmac_stream is a measurement aid; what can be checked is that it runs to the end
    on every kind of operand and writes the whole sink (constant operands: every matrix instruction adds
    the same products, so the sums it leaves grow with the iteration count)."""
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.full((256 * cus,), -1, dtype=torch.int32, device="cuda")
    sums = []
    for iterations in (1, 3):
        lut.probe_smfmac_stream(0, iterations, sink)
        torch.cuda.synchronize()
        sums.append(sink.to(torch.int64).sum().item())
    assert sums[0] != -256 * cus and sums[1] == 3 * sums[0]
    for operands in (1, 2):
        sink.fill_(-1)
        lut.probe_smfmac_stream(operands, 50, sink)
        torch.cuda.synchronize()
    with pytest.raises(lut.LutnnError):
        lut.probe_smfmac_stream(1, 10, sink[:100])
