#!/usr/bin/env python3
"""Benchmark of the LUT-NN linear operator (arXiv 2302.03213, Eq. 2 + Eq. 4) on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--variant V]

A step is one pass of the whole hot path - lutnn_linear: encode, then lookup-accumulate - over one
batch of seeded synthetic input that is already resident in HBM.  Prints ONE JSON line:
throughput in rows/s (value), equivalent TFLOP/s (2*N*D*M/t), the roofline fraction of the
dominant kernel measured with HIP events, the CPU oracle timed on a bounded row sample, and (for
the default workload) short runs of the other benchmark configurations and lookup variants.

Order of a measurement: an untimed settle phase (the same steps, so that the clocks the timed
region sees are the ones a long run sees), W untimed warm-up steps, K timed steps between two
synchronisations (value, ms_per_step), then K more steps with an event between every two
(ms_per_step_median / _min) and K more with events between the two kernels of each layer
(kernels, roofline).
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
# are under profiles/.  Keyed by (workload, kernel): (bytes, summary).  Not measured in this run.
MEASURED_TRAFFIC_BYTES = {
    # fetch 403,435,520 (196,990 KiB raw x 2.0) + write 268,687,360 (262,390 KiB raw x 1.0)
    ("fc_large", "lookup_smfmac_i8"): (672020480, "profiles/lutnn_linear_fc_large.md"),
    # dense MFMA variant: fetch 403,578,922 (197,084 KiB raw x 2.0) + write 268,435,456
    ("fc_large", "lookup_mfma_i8"): (672014378, "profiles/lutnn_lookup_variants_fc_large.md"),
}

WORKLOADS = ["fc_large", "fc_small", "conv_resnet18", "bert_ffn_up", "bert_layer", "paper_kv",
             "conv_resnet18_b32", "tree12"]


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
    if name == "tree12":  # runs with --encoder tree: 12-level trees, 16-bit indices
        return [wl.bert_ffn_down_tree12(0)]
    return [table[name](0)]


def kernel_roofline(cost, workload, w, kind, ms):
    """Roofline record of one kernel launch of layer `w` that took `ms`.
    kind: smfmac | mfma | lds | wide | fused | encode | encode_tree."""
    sec = ms * 1e-3
    table_bytes = 1 if w.table_dtype == "i8" else 4
    look_bytes = cost.lookup_hbm_bytes(w.N, w.C, w.K, w.M, table_bytes)
    if kind in ("smfmac", "mfma"):
        kname = "lookup_smfmac_i8" if kind == "smfmac" else "lookup_mfma_i8"
        insts = cost.lookup_matrix_instructions(w.N, w.C, w.M, sparse=(kind == "smfmac"))
        pipe_ops = insts * cost.MFMA_I8_32X32_OPS_PER_PIPE_SLOT
        achieved = pipe_ops / sec / 1e12
        peak = cost.PEAK_MFMA_INT8_OPS_PER_S / 1e12
        traffic, source = MEASURED_TRAFFIC_BYTES.get((workload, kname), (None, None))
        useful = 2 * cost.lookup_entries(w.N, w.C, w.M)
        r = {"kernel": kname, "bound": "mfma", "achieved": round(achieved, 2), "peak": peak, "unit": "TOP/s",
             "frac": round(achieved / peak, 4), "traffic": traffic, "kernel_ms": round(ms, 4),
             "matrix_instructions": insts,
             "useful_frac": round(useful / sec / cost.PEAK_MFMA_INT8_OPS_PER_S, 4),
             "hbm_frac": round(look_bytes / sec / cost.PEAK_HBM_BYTES_PER_S, 4),
             "algorithmic_bytes": look_bytes,
             "traffic_ratio": round(traffic / look_bytes, 2) if traffic else None,
             "traffic_source": (source + " (rocprofv3 --pmc, not this run)") if traffic else None,
             "lds_bound_ratio": round(cost.lookup_lds_floor_s(w.N, w.C, w.M, table_bytes) / sec, 3),
             "note": "frac = share of the matrix pipes' time the issued instructions hold: every 32x32 int8 "
                     "matrix instruction (dense 32x32x32 or 2:4-sparse 32x32x64) occupies its SIMD's pipe for "
                     "32 cycles, the time of 65,536 dense int8 ops; achieved = instructions x 65,536 / kernel "
                     "time against the dense 5.0 POP/s peak (= 1024 SIMDs x 65,536 ops / 32 cycles x 2.4 GHz), "
                     "so frac <= 1 by construction.  useful_frac counts only Eq. 4's own N*C*M multiply-adds "
                     "(the one-hot operand is 15/16 zeros); hbm_frac = idx + Y + table once against 8 TB/s; "
                     "lds_bound_ratio = (N*C*M table bytes through LDS at 78.6 TB/s) / kernel time, above 1 "
                     "because the matrix cores replace the gather"}
        if kind == "smfmac":
            floor = insts / cost.SIMDS * cost.SMFMAC_I8_STREAM_SECONDS_RANDOM_OPERANDS
            r["stream_floor_ms"] = round(floor * 1e3, 4)
            r["frac_of_stream_floor"] = round(floor / sec, 4)
            r["stream_floor_source"] = ("a loop of this matrix instruction alone on random INT8 operands, "
                                        "19.0 ns per instruction and SIMD at the 1.66-1.72 GHz the chip then "
                                        "holds (a microbenchmark of its own, not this run)")
        return r
    if kind == "wide":  # 16-bit indices: every selected table row is read from global memory
        # distinct table rows N*C uniformly drawn (row, codebook) pairs select, in expectation
        distinct = w.C * w.K * (1.0 - (1.0 - 1.0 / w.K) ** w.N)
        byts = distinct * w.M * table_bytes + 2 * w.N * w.C + 4 * w.N * w.M
        gathered = cost.lookup_entries(w.N, w.C, w.M) * table_bytes
        achieved = byts / sec / 1e9
        return {"kernel": "lookup_wide (16-bit indices)", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": cost.PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                "frac": round(achieved * 1e9 / cost.PEAK_HBM_BYTES_PER_S, 4), "traffic": None,
                "kernel_ms": round(ms, 4), "algorithmic_bytes": int(byts),
                "gathered_GBps": round(gathered / sec / 1e9, 1),
                "note": "algorithmic bytes = the distinct table rows the batch selects (expected number under "
                        "uniform indices) once + indices + Y; gathered_GBps counts every one of the N*C row "
                        "reads of M entries, repeats served by the caches"}
    if kind == "lds":
        entries = cost.lookup_entries(w.N, w.C, w.M)
        achieved = entries / sec / 1e12
        peak = cost.PEAK_VALU_F32_LANE_OPS_PER_S / 1e12
        return {"kernel": "lookup_lds (gather)", "bound": "alu", "achieved": round(achieved, 3),
                "peak": round(peak, 2), "unit": "T entry-adds/s (1 VALU lane-op each)",
                "frac": round(achieved / peak, 4), "traffic": None, "kernel_ms": round(ms, 4),
                "lds_frac": round(cost.lookup_lds_floor_s(w.N, w.C, w.M, table_bytes) / sec, 4),
                "hbm_frac": round(look_bytes / sec / cost.PEAK_HBM_BYTES_PER_S, 4)}
    if kind == "fused":
        byts = 4 * w.N * w.D + 4 * w.N * w.M + w.C * w.K * w.M * table_bytes
        achieved = byts / sec / 1e9
        return {"kernel": "linear_fused (one launch)", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": cost.PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                "frac": round(achieved * 1e9 / cost.PEAK_HBM_BYTES_PER_S, 4), "traffic": None,
                "kernel_ms": round(ms, 4)}
    if kind == "encode_tree":
        byts = cost.encode_bytes(w.N, w.C, w.V)
        achieved = byts / sec / 1e9
        return {"kernel": "encode_tree", "bound": "hbm", "achieved": round(achieved, 1),
                "peak": cost.PEAK_HBM_BYTES_PER_S / 1e9, "unit": "GB/s",
                "frac": round(achieved * 1e9 / cost.PEAK_HBM_BYTES_PER_S, 4), "traffic": None,
                "kernel_ms": round(ms, 4)}
    lane_ops = cost.encode_lane_ops(w.N, w.C, w.K, w.V)
    achieved = lane_ops / sec / 1e12
    peak = cost.PEAK_VALU_F32_LANE_OPS_PER_S / 1e12
    return {"kernel": "encode", "bound": "alu", "achieved": round(achieved, 3), "peak": round(peak, 2),
            "unit": "T lane-ops/s", "frac": round(achieved / peak, 4), "traffic": None,
            "kernel_ms": round(ms, 4), "ops_per_launch": lane_ops,
            "hbm_frac": round(cost.encode_bytes(w.N, w.C, w.V) / sec / cost.PEAK_HBM_BYTES_PER_S, 4),
            "note": "arg-min by definition: per sub-vector and centroid V subtract + V fused multiply-add + "
                    "one compare + one select; peak = 256 CUs x 64 lanes x 2.4 GHz (packed-fp32 instructions "
                    "are compiled out)"}


class Bench:
    """Device-side set-up of a workload (untimed) and the measurement passes over it."""

    def __init__(self, name, layers, variant="auto", int4=False, encoder="distance"):
        import numpy as np
        import torch

        import lutnn_workloads as wl
        import paper_2302_03213_amd as lut
        from paper_2302_03213_amd import cost
        self.np, self.torch, self.lut, self.cost = np, torch, lut, cost
        self.name, self.variant, self.int4, self.encoder = name, variant, int4, encoder
        self.layers, self.trees = [], {}
        for w in layers:
            dt = lut.TABLE_I8 if w.table_dtype == "i8" else lut.TABLE_F32
            if int4 and dt == lut.TABLE_I8:
                dt = lut.TABLE_I4
            P, W = torch.from_numpy(w.P).cuda(), torch.from_numpy(w.W).cuda()
            bias = torch.from_numpy(w.bias).cuda() if w.bias is not None else None
            layer = lut.build_table(P, W, dt, bias=bias, packed=w.K <= 256)
            X0 = torch.from_numpy(w.conv["inp"] if w.conv else w.X).cuda()
            Xs = [X0, X0.flip(0).contiguous()]  # two rotating activation / output buffer sets
            Ys = [torch.empty((w.N, w.M), dtype=torch.float32, device="cuda") for _ in range(2)]
            # more than 256 buckets per codebook (trees deeper than 8 levels): the 16-bit index calls
            wide = w.K > 256
            assert not wide or encoder == "tree", "K > 256 comes from the hash encoder: use --encoder tree"
            ws = torch.empty((w.N, w.C), dtype=torch.int16 if wide else torch.uint8, device="cuda")
            if encoder == "tree":
                levels = w.K.bit_length() - 1
                assert not w.conv and w.K == 1 << levels, "--encoder tree needs K = 2^levels and matrix input"
                dims, thr = wl.random_tree(w.C, w.V, levels, seed=0)
                self.trees[w.name] = (lut.LutTree(torch.from_numpy(dims).cuda(), torch.from_numpy(thr).cuda(), w.V),
                                      dims, thr)
            self.layers.append((w, layer, Xs, Ys, ws))
            del W
        torch.cuda.synchronize()

    # ---- the calls
    def run_layer(self, w, layer, X, variant, Y, ws):
        lut = self.lut
        if w.K > 256:
            lut.linear_tree16(layer, self.trees[w.name][0], X, out=Y, idx_workspace=ws)
        elif self.encoder == "tree":
            lut.linear_tree(layer, self.trees[w.name][0], X, variant, out=Y, idx_workspace=ws)
        elif w.conv:  # the image batch, no im2col matrix
            lut.conv2d(layer, X, w.conv["kernel"], w.conv["stride"], w.conv["pad"], variant, out=Y,
                       idx_workspace=ws)
        else:
            lut.linear(layer, X, variant, out=Y, idx_workspace=ws)

    def run_encode(self, w, layer, X, ws):
        lut = self.lut
        if w.K > 256:
            lut.encode_tree16(self.trees[w.name][0], X, out=ws)
        elif self.encoder == "tree":
            lut.encode_tree(self.trees[w.name][0], X, out=ws)
        elif w.conv:
            lut.encode_conv2d(layer, X, w.conv["kernel"], w.conv["stride"], w.conv["pad"], out=ws)
        else:
            lut.encode(layer, X, out=ws)

    def step(self, i):
        for (w, layer, Xs, Ys, ws) in self.layers:
            self.run_layer(w, layer, Xs[i & 1], self.variant, Ys[i & 1], ws)

    # ---- the passes
    def settle(self, seconds):
        """Untimed: the same steps for `seconds` of wall time, so that the timed region starts at the
        clocks a long run holds.  Returns the number of steps taken."""
        torch, n, t0 = self.torch, 0, time.perf_counter()
        while time.perf_counter() - t0 < seconds:
            for _ in range(10):
                self.step(n)
                n += 1
            torch.cuda.synchronize()
        return n

    def timed(self, steps, warmup, graph=0):
        """ms per step over `steps` steps between two synchronisations, after `warmup` untimed ones.
        graph = G > 0: the steps are replays of one HIP graph of G steps."""
        torch = self.torch
        for i in range(warmup):
            self.step(i)
        torch.cuda.synchronize()
        if graph > 0:
            # the entry points allocate nothing and never synchronise, so they can be captured;
            # G even keeps the two buffer sets alternating
            steps = max(graph, steps // graph * graph)
            g = torch.cuda.CUDAGraph()
            with torch.cuda.graph(g):
                for i in range(graph):
                    self.step(i)
            g.replay()
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(steps // graph):
                g.replay()
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        else:
            t0 = time.perf_counter()
            for i in range(steps):
                self.step(i)
            torch.cuda.synchronize()
            t1 = time.perf_counter()
        return (t1 - t0) / steps * 1e3, steps

    def per_step_events(self, steps):
        """The same steps with a HIP event between every two (no synchronisation in between):
        per-step durations on the launch stream."""
        torch = self.torch
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(steps + 1)]
        ev[0].record()
        for i in range(steps):
            self.step(i)
            ev[i + 1].record()
        ev[-1].synchronize()
        return [ev[i].elapsed_time(ev[i + 1]) for i in range(steps)]

    def variant_used(self):
        """Per layer: (lookup variant, True if lutnn_linear does both steps in one launch)."""
        lut, out = self.lut, {}
        for (w, layer, Xs, Ys, ws) in self.layers:
            if w.K > 256:
                out[w.name] = ("wide", False)
            elif self.variant == "fused":
                out[w.name] = ("fused", True)
            elif self.variant == "auto":  # what the library's AUTO rule picks at this shape
                if not w.conv and lut.linear_auto_variant(layer, w.N, ws) == "fused":
                    out[w.name] = ("fused", True)
                else:
                    out[w.name] = (lut.auto_variant(layer, w.N, ws), False)
            else:
                out[w.name] = (self.variant, False)
        return out

    def per_kernel_events(self, steps):
        """Per layer: event-timed durations of the encode and lookup launches, enqueued separately
        exactly as lutnn_linear enqueues them (or of the one launch that does both)."""
        torch, lut, np = self.torch, self.lut, self.np
        used, out = self.variant_used(), {}
        for (w, layer, Xs, Ys, ws) in self.layers:
            v, one_launch = used[w.name]
            e_all, l_all, f_all = [], [], []
            for i in range(steps):
                ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
                if one_launch:
                    ev[0].record()
                    self.run_layer(w, layer, Xs[i & 1], "fused", Ys[i & 1], ws)
                    ev[1].record()
                    ev[1].synchronize()
                    f_all.append(ev[0].elapsed_time(ev[1]))
                else:
                    ev[0].record()
                    self.run_encode(w, layer, Xs[i & 1], ws)
                    ev[1].record()
                    if v == "wide":
                        lut.lookup16(layer, ws, out=Ys[i & 1])
                    else:
                        lut.lookup(layer, ws, v, out=Ys[i & 1])
                    ev[2].record()
                    ev[2].synchronize()
                    e_all.append(ev[0].elapsed_time(ev[1]))
                    l_all.append(ev[1].elapsed_time(ev[2]))
            if one_launch:
                out[w.name] = {"fused_ms": round(float(np.mean(f_all)), 4), "fused_ms_min": round(min(f_all), 4)}
            else:
                out[w.name] = {"encode_ms": round(float(np.mean(e_all)), 4), "lookup_ms": round(float(np.mean(l_all)), 4),
                               "encode_ms_min": round(min(e_all), 4), "encode_ms_median": round(float(np.median(e_all)), 4),
                               "lookup_ms_min": round(min(l_all), 4), "lookup_ms_median": round(float(np.median(l_all)), 4),
                               "lookup_variant": v}
        return out

    def dominant_roofline(self, kernels):
        """Roofline record of the launch that takes the longest in a step, with the other kernel of
        the same layer attached when there is one."""
        cost, best = self.cost, None
        for (w, *_r) in self.layers:
            k = kernels[w.name]
            if "fused_ms" in k:
                cand = [(k["fused_ms"], "fused")]
            else:
                cand = [(k["encode_ms"], "encode_tree" if self.encoder == "tree" else "encode"),
                        (k["lookup_ms"], k["lookup_variant"])]
            for ms, kind in cand:
                if best is None or ms > best[0]:
                    best = (ms, kind, w, cand)
        ms, kind, w, cand = best
        r = kernel_roofline(cost, self.name, w, kind, ms)
        r["layer"] = w.name
        if w.conv and kind == "encode":  # the image is read instead of the kh*kw times larger matrix
            eb = 4 * w.conv["inp"].size + 4 * w.C * w.K * w.V + w.N * w.C
            r["hbm_frac"] = round(eb / (ms * 1e-3) / cost.PEAK_HBM_BYTES_PER_S, 4)
        for oms, okind in cand:
            if okind != kind:
                o = kernel_roofline(cost, self.name, w, okind, oms)
                o.pop("note", None)
                r["other_kernel_of_the_layer"] = o
        return r

    def describe(self):
        return "; ".join("%s N=%d D=%d M=%d V=%d C=%d K=%d %s table" %
                         (w.name, w.N, w.D, w.M, w.V, w.C, w.K,
                          "i4" if (self.int4 and w.table_dtype == "i8") else w.table_dtype)
                         for (w, *_r) in self.layers)

    def short_record(self, steps, warmup, settle_s):
        """A few steps of this workload, for the blocks that ride along with the headline."""
        n_settle = self.settle(settle_s)
        ms, _ = self.timed(steps, warmup)
        per = self.per_step_events(steps)
        kernels = self.per_kernel_events(steps)
        r = self.dominant_roofline(kernels)
        rows = sum(w.N for (w, *_r) in self.layers)
        flops = sum(self.cost.equivalent_flops(w.N, w.D, w.M) for (w, *_r) in self.layers)
        return {"workload": self.describe(), "ms_per_step": round(ms, 4),
                "ms_per_step_median": round(float(self.np.median(per)), 4), "ms_per_step_min": round(min(per), 4),
                "rows_per_s": round(rows / (ms * 1e-3), 1), "equiv_tflops": round(flops / (ms * 1e-3) / 1e12, 2),
                "steps": steps, "warmup": warmup, "settle_steps": n_settle,
                "variant_used": {k: v[0] for k, v in self.variant_used().items()},
                "dominant_kernel": r["kernel"], "dominant_layer": r["layer"], "kernel_ms": r["kernel_ms"],
                "bound": r["bound"], "frac": r["frac"], "hbm_frac": r.get("hbm_frac"),
                "kernels": kernels}


def bench_softpq_backward(args, w):
    """One step = one lutnn_softpq_backward call (both kernels) on the layer's activations and a
    seeded Z = dL/dY . W^T, everything resident in HBM."""
    import numpy as np
    import torch

    import paper_2302_03213_amd as lut
    from paper_2302_03213_amd import cost
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
        step(i)
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


def cpu_baseline(b, args):
    """The oracle, as it stands, on a bounded row sample of the same workload."""
    import numpy as np

    import oracle
    t_cpu, n_cpu = 0.0, 0
    for (w, layer, Xs, Ys, ws) in b.layers:
        n = min(w.N, len(w.X), args.cpu_sample_rows)
        Tf = oracle.build_table_f32(w.P, w.W)  # offline, untimed like on the GPU
        Xc = np.ascontiguousarray(w.X[:n])
        if w.table_dtype == "i8":
            q, s = oracle.quantize(Tf, 4 if args.int4 else 8)
        if args.encoder == "tree":
            _t, dims, thr = b.trees[w.name]
            c0 = time.perf_counter()
            idx = oracle.encode_tree(dims, thr, Xc, w.V)
            y = (oracle.lookup_i8(q, s, idx, w.bias) if w.table_dtype == "i8"
                 else oracle.lookup_f32(Tf, idx, w.bias))
        elif w.table_dtype == "i8":
            c0 = time.perf_counter()
            y = oracle.linear_i8(w.P, q, s, Xc, w.bias)
        else:
            c0 = time.perf_counter()
            y = oracle.linear_f32(w.P, Tf, Xc, w.bias)
        t_cpu += time.perf_counter() - c0
        n_cpu += n
        # cheap sanity link between the two sides on the sampled rows (not a parity test)
        b.run_layer(w, layer, Xs[0], b.variant, Ys[0], ws)
        got = Ys[0][:64].cpu().numpy()
        close = np.isclose(got, y[:64], rtol=1e-5, atol=1e-4).mean()
        assert close > 0.99, "GPU output disagrees with the oracle on %s" % w.name
    cpu = {"value": round(n_cpu / t_cpu, 1), "unit": "rows/s", "cores": oracle.threads(), "kind": "oracle",
           "sample": "first %d rows of each layer of %s, encode+lookup, tables prebuilt; %.2f s wall"
                     % (n_cpu // len(b.layers), args.workload, t_cpu)}
    # the same oracle on one core, on a 1024-row slice of the first layer (distance encoder)
    w = b.layers[0][0]
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
    return cpu


def stream_probe(torch, lut):
    """ns per v_smfmac_i32_32x32x64_i8 and SIMD in a loop of nothing else (lutnn_probe_smfmac_stream), by
    operand data; the random-INT8 figure is cost.SMFMAC_I8_STREAM_SECONDS_RANDOM_OPERANDS."""
    from paper_2302_03213_amd import cost
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    sink = torch.empty(256 * cus, dtype=torch.int32, device="cuda")
    iters, out = 40000, {}
    for name, operands in (("constant", 0), ("random_int8", 1), ("random_3bit", 2)):
        for _ in range(3):  # settle the clock on this kind of data
            lut.probe_smfmac_stream(operands, iters, sink)
        torch.cuda.synchronize()
        times = []
        for _ in range(5):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            lut.probe_smfmac_stream(operands, iters, sink)
            e1.record()
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e6 / (iters * 16.0))
        times.sort()
        out[name] = {"ns_per_instruction_median": round(times[2], 2), "ns_per_instruction_min": round(times[0], 2),
                     "clock_GHz_if_32.8_cycles": round(32.8 / times[2], 2)}
    print(json.dumps({"probe": "smfmac_stream", "compute_units": cus, "instructions_per_wave": iters * 16,
                      "operands": out,
                      "constant_in_cost_py_ns": cost.SMFMAC_I8_STREAM_SECONDS_RANDOM_OPERANDS * 1e9}))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="fc_large", choices=WORKLOADS)
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
    ap.add_argument("--settle-ms", type=float, default=400.0,
                    help="untimed settle phase before the warm-up: the same steps for this much wall time")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the short runs of the other configurations and variants that the default "
                         "workload's line carries")
    ap.add_argument("--cpu-sample-rows", type=int, default=16384)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run one 256 MiB device-to-device copy (untimed): the known-size kernel "
                         "against which rocprofv3 FETCH_SIZE / WRITE_SIZE readings are scaled")
    ap.add_argument("--stream-probe", action="store_true",
                    help="instead of the benchmark: time a stream of the lookup's matrix instruction alone "
                         "on constant, random INT8 and random 3-bit operands (the floor the roofline record "
                         "quotes as stream_floor_ms) and print one JSON line")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this build runs on ONE GPU only (the operator shards by rows with no "
              "communication; multi-GPU runs are not part of it). Use --gpus 1.", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import paper_2302_03213_amd as lut  # noqa: F401  (fails loudly if the HIP library is missing)
    if args.stream_probe:
        stream_probe(torch, lut)
        return
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
        return bench_softpq_backward(args, layers[0])

    b = Bench(args.workload, layers, args.variant, args.int4, args.encoder)
    if args.copy_calibration:
        src = torch.empty(256 * 2 ** 20, dtype=torch.uint8, device="cuda").fill_(1)
        dst = torch.empty_like(src)
        dst.copy_(src)  # reads 256 MiB, writes 256 MiB
        torch.cuda.synchronize()
        del src, dst

    settle_steps = b.settle(args.settle_ms * 1e-3)
    ms_per_step, args.steps = b.timed(args.steps, args.warmup, args.graph)
    per = b.per_step_events(args.steps)
    kernels = b.per_kernel_events(args.steps)
    roofline = b.dominant_roofline(kernels)
    for (w, *_r) in b.layers:  # the encoder against the HBM roofline, per layer
        k = kernels[w.name]
        if "encode_ms" in k:
            eb = cost.encode_bytes(w.N, w.C, w.V)
            if w.conv:  # the image is read instead of the kh*kw times larger matrix
                eb = 4 * w.conv["inp"].size + 4 * w.C * w.K * w.V + w.N * w.C
            k["encode_hbm_GBps"] = round(eb / (k["encode_ms"] * 1e-3) / 1e9, 1)
            k["encode_hbm_frac"] = round(eb / (k["encode_ms"] * 1e-3) / cost.PEAK_HBM_BYTES_PER_S, 4)

    rows = sum(w.N for (w, *_r) in b.layers)
    eq_flops = sum(cost.equivalent_flops(w.N, w.D, w.M) for (w, *_r) in b.layers)
    sec_per_step = ms_per_step * 1e-3
    w0 = b.layers[0][0]
    out = {
        "metric": "lut_linear_rows_per_s", "value": round(rows / sec_per_step, 1), "unit": "rows/s",
        "equiv_tflops": round(eq_flops / sec_per_step / 1e12, 2),
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "ms_per_step_median": round(float(np.median(per)), 4), "ms_per_step_min": round(min(per), 4),
        "higher_is_better": True, "scaling": "weak",
        "vs_baseline": None, "dtype": "i8" if w0.table_dtype == "i8" else "f32",
        "data": "synthetic",
        "config": {"workload": b.describe(), "variant": args.variant,
                   "variant_used": {k: v[0] for k, v in b.variant_used().items()},
                   "encoder": args.encoder, "settle_steps": settle_steps,
                   "step": ("lutnn_linear_tree per layer: hash encode + lookup" if args.encoder == "tree" else
                            "lutnn_linear (lutnn_conv2d for an image batch) per layer: encode fp32 + "
                            "lookup") + ", inputs resident in HBM, two rotating X/Y buffer sets",
                   "timing": "settle_steps untimed steps (%.0f ms of wall time), then warmup, then `steps` steps "
                             "between two synchronisations (value, ms_per_step); ms_per_step_median / _min from "
                             "a second pass with a HIP event between every two steps" % args.settle_ms,
                   "launch": ("replays of a HIP graph of %d steps" % args.graph) if args.graph > 0 else
                             "one host call per layer and step"},
        "roofline": roofline, "kernels": kernels,
        # (tables of 4096 rows per codebook take the plain-loop oracle minutes to build: no CPU leg there)
        "cpu_baseline": None if (args.no_cpu_baseline or any(w.K > 256 for (w, *_r) in b.layers))
        else cpu_baseline(b, args),
    }

    # ---- riding along with the headline (default workload only; outside its timed region, a few
    # steps each): the benchmark's other four configurations, and the other lookup variants of this one
    plain = (args.workload == "fc_large" and args.variant == "auto" and not args.int4 and not args.rows
             and args.encoder == "distance" and args.graph == 0)
    if plain and not args.no_extras:
        variants = {}
        for v, n in (("smfmac", 20), ("mfma", 20), ("lds", 8), ("fused", 8)):
            b.variant = v
            r = b.short_record(n, 2, 0.05)
            variants[v] = {k: r[k] for k in ("ms_per_step", "ms_per_step_median", "ms_per_step_min", "steps",
                                             "dominant_kernel", "kernel_ms", "bound", "frac", "hbm_frac")}
        b.variant = args.variant
        out["variants"] = {"note": "this workload with the lookup variant pinned (fused = the tile form of the "
                                   "one-kernel operator); a few steps each, after the headline's timed region",
                           **variants}
        del b
        torch.cuda.empty_cache()
        configs = {}
        for key, name in (("1_fc_small", "fc_small"), ("2_conv_resnet18", "conv_resnet18"),
                          ("3_bert_ffn_up", "bert_ffn_up"), ("4_bert_layer", "bert_layer")):
            ob = Bench(name, workload_by_name(name))
            configs[key] = ob.short_record(100, 10, 0.15)
            del ob
        out["configs"] = {"note": "the benchmark's other configurations, variant auto, 100 steps after 10 warm-up "
                                  "and a 150 ms settle phase each, after the headline's timed region; "
                                  "configuration 5 is the headline itself", **configs}
    print(json.dumps(out))


if __name__ == "__main__":
    main()
