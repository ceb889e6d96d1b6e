#!/usr/bin/env python3
"""Benchmark of the LUT-NN linear operator (arXiv 2302.03213, Eq. 2 + Eq. 4) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--variant V]

A step is one pass of the whole hot path - lutnn_linear: encode, then lookup-accumulate - over one
batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line:
throughput in rows/s (value), equivalent TFLOP/s (2*N*D*M/t), the roofline fraction of the
dominant kernel measured with HIP events, and the CPU oracle timed on a bounded row sample.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

# HBM bytes per launch of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE and
# WRITE_SIZE runs, scaled by the same counters on a copy kernel of known size); the summaries
# are under profiles/.  Keyed by (workload, kernel).  None = not measured.
MEASURED_TRAFFIC_BYTES = {
    # profiles/lutnn_linear_fc_large.md: fetch 605,123,584 (295,471 KiB raw x 2.0) + write 268,566,118
    ("fc_large", "lookup_smfmac_i8"): 873689702,
    # dense MFMA variant, measured before the sparse kernel became the default:
    # fetch 403,578,922 (197,084 KiB raw x 2.0) + write 268,435,456
    ("fc_large", "lookup_mfma_i8"): 672014378,
}


def workload_by_name(name):
    import lutnn_workloads as wl
    table = {
        "fc_large": wl.fc_large, "fc_small": wl.fc_small, "conv_resnet18": wl.conv_resnet18,
        "bert_ffn_up": wl.bert_ffn_up, "conv_resnet18_b32": wl.conv_resnet18_batch,
    }
    if name == "bert_layer":
        return wl.bert_layer(0)
    if name == "paper_kv":
        return wl.paper_kv_space(0)
    return [table[name](0)]


def bench_softpq_backward(args, w, lut, cost, np, torch):
    """One step = one lutnn_softpq_backward call (both kernels) on the layer's activations and a
    seeded Z = dL/dY . W^T, everything resident in HBM."""
    assert not w.conv, "softpq_backward is benchmarked on matrix workloads"
    g = torch.Generator(device="cpu")
    g.manual_seed(1)
    layer = lut.LutLayer(torch.from_numpy(w.P).cuda(), None, lut.TABLE_F32, w.M)
    X0 = torch.from_numpy(w.X).cuda()
    Z0 = (torch.randn((w.N, w.D), generator=g, dtype=torch.float32) * 0.1).cuda()
    Xs, Zs = [X0, X0.flip(0).contiguous()], [Z0, Z0.flip(0).contiguous()]
    ws = torch.empty(max(lut.softpq_workspace_bytes(w.C, w.K, w.V, w.N), 4), dtype=torch.uint8, device="cuda")
    temperature = 1.0

    def step(i):
        return lut.softpq_backward(layer, temperature, Xs[i & 1], Zs[i & 1], workspace=ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    sec = (time.perf_counter() - t0) / args.steps
    acc = 0.0
    for i in range(args.steps):
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        ev[0].record()
        out = step(i)
        ev[1].record()
        ev[1].synchronize()
        acc += ev[0].elapsed_time(ev[1])
    k_ms = acc / args.steps
    lane_ops = cost.softpq_backward_lane_ops(w.N, w.C, w.K, w.V)
    byts = cost.softpq_backward_bytes(w.N, w.C, w.V)
    peak = cost.PEAK_VALU_F32_LANE_OPS_PER_S / 1e12
    achieved = lane_ops / (k_ms * 1e-3) / 1e12
    roofline = {"kernel": "softpq_backward (+ reduce)", "bound": "alu", "achieved": round(achieved, 3),
                "peak": round(peak, 2), "unit": "T lane-ops/s", "frac": round(achieved / peak, 4),
                "traffic": None, "kernel_ms": round(k_ms, 4), "ops_per_launch": lane_ops,
                "hbm_GBps": round(byts / (k_ms * 1e-3) / 1e9, 1),
                "hbm_frac": round(byts / (k_ms * 1e-3) / cost.PEAK_HBM_BYTES_PER_S, 4),
                "note": "lane-ops of the backward formulas themselves (sums over rows not counted); peak = "
                        "256 CUs x 64 lanes x 2.4 GHz"}
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        from oracle import softpq as osp
        n = min(w.N, 128)
        G = np.random.default_rng(0).standard_normal((n, w.M))
        c0 = time.perf_counter()
        dP, dX, dt = osp.backward(w.P, w.W, w.X[:n], temperature, G)
        t_cpu = time.perf_counter() - c0
        # cheap sanity link on the same rows (not a parity test): feed the GPU the Z of this G
        Zs_ = torch.from_numpy((G @ w.W.astype(np.float64).T).astype(np.float32)).cuda()
        got = lut.softpq_backward(layer, temperature, X0[:n].contiguous(), Zs_)
        err = np.abs(got[0].cpu().numpy() - dP).max() / max(np.abs(dP).max(), 1e-30)
        assert err < 1e-4, "GPU soft-PQ backward disagrees with the oracle (%.2e)" % err
        cpu = {"value": round(n / t_cpu, 1), "unit": "rows/s", "cores": oracle.threads(), "kind": "oracle",
               "sample": "first %d rows of %s, fp64 chain rule through the full table (numpy); %.2f s wall"
                         % (n, w.name, t_cpu)}
    out = {
        "metric": "softpq_backward_rows_per_s", "value": round(w.N / sec, 1), "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(sec * 1e3, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": "%s N=%d D=%d V=%d C=%d K=%d" % (w.name, w.N, w.D, w.V, w.C, w.K),
                   "step": "lutnn_softpq_backward (dP, dX, dt from X and Z = dL/dY . W^T), inputs resident in "
                           "HBM, two rotating X/Z buffer sets; the GEMM that forms Z is not part of it"},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="fc_large",
                    choices=["fc_large", "fc_small", "conv_resnet18", "bert_ffn_up", "bert_layer",
                             "paper_kv", "conv_resnet18_b32"])
    ap.add_argument("--variant", default="auto", choices=["auto", "lds", "mfma", "smfmac", "fused"])
    ap.add_argument("--int4", action="store_true",
                    help="quantise the INT8 workloads' tables to 4 bits instead (Sec. 3.3 with n = 4)")
    ap.add_argument("--encoder", default="distance", choices=["distance", "tree"],
                    help="tree: the hash encoder of Sec. 2 / Sec. 7 (seeded random threshold trees with "
                         "log2 K levels) in place of the distance search of Eq. 2")
    ap.add_argument("--op", default="linear", choices=["linear", "softpq_backward"],
                    help="softpq_backward: time lutnn_softpq_backward (the training operator of Sec. 3) on "
                         "the workload's first layer instead of the inference step")
    ap.add_argument("--rows", type=int, default=0,
                    help="use only the first ROWS rows of the workload (small-batch latency of the same layer)")
    ap.add_argument("--graph", type=int, default=0, metavar="G",
                    help="launch the timed steps as replays of one HIP graph of G steps (steps is rounded "
                         "down to a multiple of G): device time per call without the host's launch cost, "
                         "for the launch-bound small workloads")
    ap.add_argument("--cpu-sample-rows", type=int, default=16384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device-to-device copy (untimed): the known-size kernel "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the operator shards by rows with no "
              "communication; multi-GPU runs are not part of it). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import lutnn_workloads as wl
    import paper_2302_03213_amd as lut
    from paper_2302_03213_amd import cost

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    layers = workload_by_name(args.workload)
    if args.rows:  # a smaller batch of the same layer(s): per-call latency at N = --rows
        for w in layers:
            assert not w.conv, "--rows applies to matrix workloads"
            w.N = min(w.N, args.rows)
            w.X = np.ascontiguousarray(w.X[:w.N])
    if args.op == "softpq_backward":
        return bench_softpq_backward(args, layers[0], lut, cost, np, torch)

    # ---- device-side set-up (untimed): tables, two rotating activation / output buffer sets
    dev_layers, trees = [], {}
    for w in layers:
        dt = lut.TABLE_I8 if w.table_dtype == "i8" else lut.TABLE_F32
        if args.int4 and dt == lut.TABLE_I8:
            dt = lut.TABLE_I4
        P, W = torch.from_numpy(w.P).cuda(), torch.from_numpy(w.W).cuda()
        bias = torch.from_numpy(w.bias).cuda() if w.bias is not None else None
        layer = lut.build_table(P, W, dt, bias=bias)
        X0 = torch.from_numpy(w.conv["inp"] if w.conv else w.X).cuda()
        Xs = [X0, X0.flip(0).contiguous()]
        Ys = [torch.empty((w.N, w.M), dtype=torch.float32, device="cuda") for _ in range(2)]
        ws = torch.empty((w.N, w.C), dtype=torch.uint8, device="cuda")
        if args.encoder == "tree":
            levels = w.K.bit_length() - 1
            assert not w.conv and w.K == 1 << levels, "--encoder tree needs K = 2^levels and matrix input"
            dims, thr = wl.random_tree(w.C, w.V, levels, seed=0)
            trees[w.name] = (lut.LutTree(torch.from_numpy(dims).cuda(), torch.from_numpy(thr).cuda(), w.V),
                             dims, thr)
        dev_layers.append((w, layer, Xs, Ys, ws))
        del W
    torch.cuda.synchronize()
    if args.copy_calibration:
        src = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    def run_layer(w, layer, X, variant, Y, ws):
        if args.encoder == "tree":
            lut.linear_tree(layer, trees[w.name][0], X, variant, out=Y, idx_workspace=ws)
        elif w.conv:  # the image batch, no im2col matrix
            lut.conv2d(layer, X, w.conv["kernel"], w.conv["stride"], w.conv["pad"], variant, out=Y,
                       idx_workspace=ws)
        else:
            lut.linear(layer, X, variant, out=Y, idx_workspace=ws)

    def run_encode(w, layer, X, ws):
        if args.encoder == "tree":
            lut.encode_tree(trees[w.name][0], X, out=ws)
        elif w.conv:
            lut.encode_conv2d(layer, X, w.conv["kernel"], w.conv["stride"], w.conv["pad"], out=ws)
        else:
            lut.encode(layer, X, out=ws)

    def step(i):
        for (w, layer, Xs, Ys, ws) in dev_layers:
            run_layer(w, layer, Xs[i & 1], args.variant, Ys[i & 1], ws)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    if args.graph > 0:
        # the same steps recorded once (the entry points allocate nothing and never synchronise, so
        # they can be captured) and replayed; G even keeps the two buffer sets alternating
        G = args.graph
        args.steps = max(G, args.steps // G * G)
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            for i in range(G):
                step(i)
        graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps // G):
            graph.replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    else:
        t0 = time.perf_counter()
        for i in range(args.steps):
            step(i)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
    sec_per_step = (t1 - t0) / args.steps

    rows = sum(w.N for (w, *_r) in dev_layers)
    eq_flops = sum(cost.equivalent_flops(w.N, w.D, w.M) for (w, *_r) in dev_layers)

    # ---- per-kernel durations with HIP events on the launch stream (same kernels, same inputs):
    # encode and lookup of the FIRST (for bert_layer: every) layer, split as lutnn_linear splits them
    enc_ms, look_ms, fused_ms = [], [], []
    variant_used, spread = {}, {}
    for (w, layer, Xs, Ys, ws) in dev_layers:
        fused = args.variant == "fused"
        if fused:
            variant_used[w.name] = "fused"
        elif args.variant == "auto":  # what the library's AUTO rule picks at this shape
            variant_used[w.name] = lut.auto_variant(layer, w.N, ws)
            if not w.conv and lut.linear_auto_variant(layer, w.N, ws) == "fused":
                fused = True  # lutnn_linear / lutnn_linear_tree do both steps in one launch here
                variant_used[w.name] = "fused"
        else:
            variant_used[w.name] = args.variant
        e_acc = l_acc = f_acc = 0.0
        e_all, l_all = [], []
        for i in range(args.steps):
            ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
            if fused:
                ev[0].record()
                run_layer(w, layer, Xs[i & 1], "fused", Ys[i & 1], ws)
                ev[1].record()
                ev[1].synchronize()
                f_acc += ev[0].elapsed_time(ev[1])
            else:
                ev[0].record()
                run_encode(w, layer, Xs[i & 1], ws)
                ev[1].record()
                lut.lookup(layer, ws, variant_used[w.name], out=Ys[i & 1])
                ev[2].record()
                ev[2].synchronize()
                e_all.append(ev[0].elapsed_time(ev[1]))
                l_all.append(ev[1].elapsed_time(ev[2]))
                e_acc += e_all[-1]
                l_acc += l_all[-1]
        spread[w.name] = ({"encode_ms_min": round(min(e_all), 4), "encode_ms_median": round(float(np.median(e_all)), 4),
                           "lookup_ms_min": round(min(l_all), 4), "lookup_ms_median": round(float(np.median(l_all)), 4)}
                          if e_all else {})
        enc_ms.append(e_acc / args.steps)
        look_ms.append(l_acc / args.steps)
        fused_ms.append(f_acc / args.steps)

    # ---- roofline of the dominant kernel (of the first layer for multi-layer workloads)
    w0 = dev_layers[0][0]
    v0 = variant_used[w0.name]
    if v0 in ("mfma", "smfmac"):
        ops = cost.lookup_mfma_ops(w0.N, w0.C, w0.M)
        achieved = ops / (look_ms[0] * 1e-3) / 1e12
        kname = "lookup_mfma_i8" if v0 == "mfma" else "lookup_smfmac_i8"
        roofline = {"kernel": kname, "bound": "mfma", "achieved": round(achieved, 2),
                    "peak": cost.PEAK_MFMA_INT8_OPS_PER_S / 1e12, "unit": "TOP/s",
                    "frac": round(achieved * 1e12 / cost.PEAK_MFMA_INT8_OPS_PER_S, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, kname)),
                    "kernel_ms": round(look_ms[0], 4),
                    "ops_per_launch": ops,
                    "note": "dense-equivalent int8 ops of the one-hot contraction 2*N*C*16*M (1/16 of "
                            "them carry a table entry, N*C*M entries per launch), priced against "
                            "the DENSE int8 MFMA peak"}
        if v0 == "smfmac":
            roofline["note"] += ("; the kernel issues v_smfmac_i32_32x32x64_i8 (2:4 structured-sparse "
                                 "A, which a one-hot slice satisfies exactly), i.e. half as many "
                                 "matrix instructions as the dense form")
            roofline["frac_of_sparse_peak"] = round(achieved * 1e12 / (2 * cost.PEAK_MFMA_INT8_OPS_PER_S), 4)
    elif v0 == "lds":
        entries = cost.lookup_entries(w0.N, w0.C, w0.M)
        achieved = entries / (look_ms[0] * 1e-3) / 1e12
        peak = cost.PEAK_VALU_F32_LANE_OPS_PER_S / 1e12
        roofline = {"kernel": "lookup_lds", "bound": "alu", "achieved": round(achieved, 3),
                    "peak": round(peak, 2), "unit": "T entry-adds/s (1 VALU lane-op each)",
                    "frac": round(achieved / peak, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, "lookup_lds")),
                    "kernel_ms": round(look_ms[0], 4)}
    else:
        byts = 4 * w0.N * w0.D + 4 * w0.N * w0.M + w0.C * w0.K * w0.M * (
            1 if w0.table_dtype == "i8" else 4)
        achieved = byts / (fused_ms[0] * 1e-3) / 1e9
        roofline = {"kernel": "linear_fused", "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": cost.PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                    "frac": round(achieved * 1e9 / cost.PEAK_HBM_BYTES_PER_S, 4),
                    "traffic": MEASURED_TRAFFIC_BYTES.get((args.workload, "linear_fused")),
                    "kernel_ms": round(fused_ms[0], 4)}
    # when the encoder of that layer takes longer than its lookup, the encoder is the dominant
    # kernel: VALU-issue bound (Eq. 2 in the direct form is K*(2V+2) lane-operations per sub-vector)
    if args.encoder == "tree" and enc_ms[0] > look_ms[0]:
        byts = cost.encode_bytes(w0.N, w0.C, w0.V)
        achieved = byts / (enc_ms[0] * 1e-3) / 1e9
        roofline = {"kernel": "encode_tree", "bound": "hbm", "achieved": round(achieved, 1),
                    "peak": cost.PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                    "frac": round(achieved * 1e9 / cost.PEAK_HBM_BYTES_PER_S, 4), "traffic": None,
                    "kernel_ms": round(enc_ms[0], 4), "lookup": roofline}
    elif v0 != "fused" and enc_ms[0] > look_ms[0]:
        lane_ops = cost.encode_lane_ops(w0.N, w0.C, w0.K, w0.V)
        achieved = lane_ops / (enc_ms[0] * 1e-3) / 1e12
        peak = cost.PEAK_VALU_F32_LANE_OPS_PER_S / 1e12
        roofline = {"kernel": "encode", "bound": "alu", "achieved": round(achieved, 3),
                    "peak": round(peak, 2), "unit": "T lane-ops/s",
                    "frac": round(achieved / peak, 4), "traffic": None,
                    "kernel_ms": round(enc_ms[0], 4), "ops_per_launch": lane_ops,
                    "note": "arg-min by definition: per sub-vector and centroid V subtract + V fused "
                            "multiply-add + one compare + one select; peak = 256 CUs x 64 lanes x "
                            "2.4 GHz (packed-fp32 instructions are compiled out)",
                    "lookup": roofline}
    kernels = {}
    for (w, *_r), e, l, f in zip(dev_layers, enc_ms, look_ms, fused_ms):
        if variant_used[w.name] == "fused":
            kernels[w.name] = {"fused_ms": round(f, 4)}
        else:
            eb = cost.encode_bytes(w.N, w.C, w.V)
            if w.conv:  # the image is read instead of the kh*kw times larger matrix
                eb = 4 * w.conv["inp"].size + 4 * w.C * w.K * w.V + w.N * w.C
            kernels[w.name] = {"encode_ms": round(e, 4), "lookup_ms": round(l, 4),
                               "encode_hbm_GBps": round(eb / (e * 1e-3) / 1e9, 1),
                               "encode_hbm_frac": round(eb / (e * 1e-3) / cost.PEAK_HBM_BYTES_PER_S, 4)}
            kernels[w.name].update(spread[w.name])

    # ---- CPU baseline: the oracle, as it stands, on a bounded row sample of the same workload
    cpu = None
    if not args.no_cpu_baseline:
        import oracle
        t_cpu, n_cpu = 0.0, 0
        for (w, *_r) in dev_layers:
            n = min(w.N, len(w.X), args.cpu_sample_rows)
            Tf = oracle.build_table_f32(w.P, w.W)  # offline, untimed like on the GPU
            Xs = np.ascontiguousarray(w.X[:n])
            if args.encoder == "tree":
                _t, dims, thr = trees[w.name]
                if w.table_dtype == "i8":
                    q, s = oracle.quantize(Tf, 4 if args.int4 else 8)
                c0 = time.perf_counter()
                idx = oracle.encode_tree(dims, thr, Xs, w.V)
                y = (oracle.lookup_i8(q, s, idx, w.bias) if w.table_dtype == "i8"
                     else oracle.lookup_f32(Tf, idx, w.bias))
            elif w.table_dtype == "i8":
                q, s = oracle.quantize(Tf, 4 if args.int4 else 8)
                c0 = time.perf_counter()
                y = oracle.linear_i8(w.P, q, s, Xs, w.bias)
            else:
                c0 = time.perf_counter()
                y = oracle.linear_f32(w.P, Tf, Xs, w.bias)
            t_cpu += time.perf_counter() - c0
            n_cpu += n
            # cheap sanity link between the two sides on the sampled rows (not a parity test)
            got = dev_layers[[d[0].name for d in dev_layers].index(w.name)][3][0][:64].cpu().numpy()
            exp = y[:64]
            close = np.isclose(got, exp, rtol=1e-5, atol=1e-4).mean()
            assert close > 0.99, "GPU output disagrees with the oracle on %s" % w.name
        cpu = {"value": round(n_cpu / t_cpu, 1), "unit": "rows/s", "cores": oracle.threads(),
               "kind": "oracle",
               "sample": "first %d rows of each layer of %s, encode+lookup, tables prebuilt; "
                         "%.2f s wall" % (n_cpu // len(dev_layers), args.workload, t_cpu)}
        # the same oracle on one core, on a 1024-row slice of the first layer (distance encoder)
        w = dev_layers[0][0]
        if args.encoder == "distance":
            all_threads = oracle.threads()
            oracle.set_threads(1)
            n1 = min(1024, w.N, len(w.X))
            Tf = oracle.build_table_f32(w.P, w.W)
            X1 = np.ascontiguousarray(w.X[:n1])
            if w.table_dtype == "i8":
                q, s = oracle.quantize(Tf, 4 if args.int4 else 8)
                c0 = time.perf_counter()
                oracle.linear_i8(w.P, q, s, X1, w.bias)
            else:
                c0 = time.perf_counter()
                oracle.linear_f32(w.P, Tf, X1, w.bias)
            t1 = time.perf_counter() - c0
            oracle.set_threads(all_threads)
            cpu["single_thread"] = {"value": round(n1 / t1, 1), "unit": "rows/s",
                                    "sample": "first %d rows of %s; %.2f s" % (n1, w.name, t1)}

    w_desc = "; ".join("%s N=%d D=%d M=%d V=%d C=%d K=%d %s table" %
                       (w.name, w.N, w.D, w.M, w.V, w.C, w.K,
                        "i4" if (args.int4 and w.table_dtype == "i8") else w.table_dtype)
                       for (w, *_r) in dev_layers)
    out = {
        "metric": "lut_linear_rows_per_s", "value": round(rows / sec_per_step, 1), "unit": "rows/s",
        "equiv_tflops": round(eq_flops / sec_per_step / 1e12, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(sec_per_step * 1e3, 4), "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "i8" if w0.table_dtype == "i8" else "f32",
        "data": "synthetic",
        "config": {"workload": w_desc, "variant": args.variant, "variant_used": variant_used,
                   "encoder": args.encoder,
                   "step": ("lutnn_linear_tree per layer: hash encode + lookup" if args.encoder == "tree" else
                            "lutnn_linear (lutnn_conv2d for an image batch) per layer: encode fp32 + "
                            "lookup") + ", inputs resident in HBM, two rotating X/Y buffer sets",
                   "launch": ("replays of a HIP graph of %d steps" % args.graph) if args.graph > 0 else
                             "one host call per layer and step"},
        "roofline": roofline, "kernels": kernels, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
