#!/usr/bin/env python3
"""Benchmark of the quantized Winograd 3x3 convolution hot path on one MI355X.

Default workload = configuration 5: the thirteen 3x3 layers of a VGG-16-shaped network at
224x224, batch 16, F(2x2,3x3), 8 bits.  One "step" = the thirteen fused convolution calls
(range pass; range reduction and de-quantization constants; transform + quantize; int8 GEMM with
fused de-quantization and output transform) enqueued back to back on one stream, each layer on
its own seeded synthetic input and output buffers already resident in HBM (1.3 GB in all, so
every layer reads its input from HBM, not from the last-level cache).  The filter transforms are
done once beforehand (the method's off-line step) and timed separately; the ReLU / max-pool glue
between the layers is not part of the method and not run.

`value` = direct-convolution-equivalent TOPS = sum over layers of 2*N*K*C*Ho*Wo*9 / time.
The same JSON line carries `per_config`: configurations 1-4 and each of the thirteen layers with
ms, TOPS, per-kernel HIP-event times and the roofline of its longest kernel.

`--workload cfg1|cfg2|cfg3_m2|cfg3_m4|cfg4|probe` times a single layer instead.
`--pmc-pass` / `--ingest-pmc` produce and read rocprofv3 counter runs (HBM traffic per kernel).
Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import csv
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
I8_MFMA_PEAK_TOPS = 5000.0   # MI355X dense int8, published (5.0 POP/s)
LLC_BYTES = 256 << 20        # Infinity Cache: rotating buffers must exceed it
TRAFFIC_FILE = os.path.join(ROOT, "paper_2003_08646_amd", "measured_traffic.json")
SLOTS = ("range_pass", "range_reduce", "quantize_pass", "gemm_epilogue")
SEPARATOR_ELEMS = 64 << 20   # fp32 elements of the copy that separates workloads in a counter run


def source_digest() -> str:
    """Digest of the kernel sources and the header: stored with counter measurements so that a
    later build does not present them as its own."""
    h = hashlib.sha256()
    csrc = os.path.join(ROOT, "paper_2003_08646_amd", "csrc")
    for fn in sorted(os.listdir(csrc)) + ["../../include/lance.h"]:
        with open(os.path.join(csrc, fn), "rb") as f:
            h.update(fn.encode() + b"\0" + f.read())
    return h.hexdigest()[:16]


def slot_bytes(L, sz, names):
    """Algorithmic HBM bytes per launch of each kernel of the fused call (unit: one tile, all
    channels; per launch = P tiles): X is 4*m*m*C bytes per tile, V's codes E*Cp, their column
    sums 4*E, Y 4*m*m*K; the prepared filters are read once per launch."""
    x = L.N * L.C * L.H * L.W * 4
    vq = sz.E * sz.P * sz.Cp
    colsum = sz.E * sz.P * 4
    uq = sz.E * L.K * sz.Cp
    y = L.N * L.K * sz.Ho * sz.Wo * 4
    codes_on_chip = not names[2]      # the product kernel quantizes by itself
    return {"range_pass": x, "range_reduce": 0, "quantize_pass": x + vq + colsum,
            "gemm_epilogue": (x + uq + y) if codes_on_chip else (vq + colsum + uq + y)}


def load_traffic():
    try:
        with open(TRAFFIC_FILE) as f:
            rec = json.load(f)
    except (OSError, ValueError):
        return None
    return rec if rec.get("source_digest") == source_digest() else None


class LayerRun:
    """A layer with its buffers on the GPU: filters prepared, rotating (input, output) pairs."""

    def __init__(self, L, flags=0, min_pairs=1):
        import numpy as np
        import torch
        from paper_2003_08646_amd import binding as B
        from paper_2003_08646_amd import workloads as Wk
        from paper_2003_08646_amd.layer import LanceConv
        self.L = L
        X, Wt = Wk.make_inputs(L)
        self.X_host, self.W_host = X, Wt
        self.conv = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits, flags, bits_w=L.bits_w)
        if flags & B.LANCE_LAYOUT_NHWC:
            X = np.ascontiguousarray(X.transpose(0, 2, 3, 1))
        self.x = torch.from_numpy(X).cuda()
        self.w = torch.from_numpy(Wt).cuda()
        self.conv.prepare_filters(self.w)
        self.pair_bytes = self.x.numel() * 4 + self.conv.y.numel() * 4
        self.xs, self.ys = [self.x], [self.conv.y]
        for _ in range(min_pairs - 1):
            self.add_pair()

    def add_pair(self):
        import torch
        self.xs.append(self.x.clone())
        self.ys.append(torch.empty_like(self.conv.y))

    def rotate_beyond_llc(self):
        want = max(2, -(-(LLC_BYTES + (64 << 20)) // self.pair_bytes) + 1)
        while len(self.xs) < want:
            self.add_pair()

    def call(self, i=0):
        n = len(self.xs)
        self.conv.forward(self.xs[i % n], self.ys[i % n])

    def time_loop(self, steps, warmup, rotate):
        import torch
        n = len(self.xs) if rotate else 1
        for i in range(warmup):
            self.conv.forward(self.xs[i % n], self.ys[i % n])
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.conv.forward(self.xs[i % n], self.ys[i % n])
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) / steps * 1e3

    def kernel_times(self, repeats, rotate):
        """Per-kernel HIP-event times [ms] of back-to-back passes and the kernels' names."""
        from paper_2003_08646_amd import binding as B
        c = self.conv
        xs, ys = (self.xs, self.ys) if rotate else (self.xs[:1], self.ys[:1])
        for _ in range(2):  # the first batch brings the clocks up, the second is the measurement
            ms = B.lance_conv3x3_winograd_q8_profile_rotating(
                c.desc, xs, ys, c.uq, c.u_range, c.u_rowsum, c.v_range, c.workspace,
                repeats=repeats)
        names = [B.lance_profile_kernel_name(i) for i in range(len(SLOTS))]
        return ms, names


def layer_record(run, steps, warmup, traffic):
    """ms, TOPS, per-kernel times and the roofline of the longest kernel of one layer."""
    L, sz = run.L, run.conv.sz
    ms_resident = run.time_loop(steps, warmup, rotate=False)
    run.rotate_beyond_llc()
    ms_rot = run.time_loop(steps, warmup, rotate=True)
    reps = max(10, min(steps, 500))
    k_rot, names = run.kernel_times(reps, rotate=True)
    k_res, _ = run.kernel_times(reps, rotate=False)
    kb = slot_bytes(L, sz, names)
    # An event between two kernels costs a few microseconds of its own (the next kernel cannot be
    # launched under the tail of the previous one).  What the events added is known: the twin's
    # kernels sum to more than the plain call takes; each kernel's time is reduced by its share,
    # so that the kernels of a call add up to the call (launch gaps included).
    n_k = sum(1 for n in names if n)
    over_rot = max(0.0, sum(k_rot) - ms_rot) / n_k
    over_res = max(0.0, sum(k_res) - ms_resident) / n_k
    k_rot = [max(v - over_rot, 0.0) if names[i] else 0.0 for i, v in enumerate(k_rot)]
    k_res = [max(v - over_res, 0.0) if names[i] else 0.0 for i, v in enumerate(k_res)]
    kernels = []
    for i, slot in enumerate(SLOTS):
        if not names[i]:
            continue
        rec = {"slot": slot, "kernel": names[i], "ms": round(k_rot[i], 5),
               "ms_resident": round(k_res[i], 5), "algorithmic_bytes": kb[slot],
               "GBps": round(kb[slot] / (k_rot[i] * 1e-3) / 1e9, 1) if kb[slot] else None}
        t = (traffic or {}).get(L.name, {}).get(names[i])
        rec["traffic"] = None if t is None else int(t["fetch_bytes"] + t["write_bytes"])
        kernels.append(rec)
    dom = max(kernels, key=lambda k: k["ms"])
    gemm_ops = 2 * sz.E * L.K * L.C * sz.P
    prod = kernels[-1]
    fused_bytes = sz.E * sz.P * sz.Cp + sz.E * L.K * sz.Cp + L.N * L.K * sz.Ho * sz.Wo * 4
    i8 = gemm_ops / (prod["ms"] * 1e-3) / 1e12
    return {
        "name": L.name,
        "shape": f"N={L.N} C={L.C} K={L.K} H=W={L.H} pad={L.pad} F({L.m}x{L.m},3x3) {L.bits}-bit",
        "direct_GOP": round(L.direct_ops / 1e9, 4),
        "ms": round(ms_rot, 5), "TOPS": round(L.direct_ops / (ms_rot * 1e-3) / 1e12, 2),
        "ms_resident": round(ms_resident, 5),
        "TOPS_resident": round(L.direct_ops / (ms_resident * 1e-3) / 1e12, 2),
        "buffer_pairs": len(run.xs),
        "event_cost_removed_ms_per_kernel": round(over_rot, 5),
        "kernels": kernels,
        "roofline": {"kernel": dom["kernel"], "bound": "hbm", "achieved": dom["GBps"],
                     "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": round((dom["GBps"] or 0.0) / HBM_PEAK_GBS, 4),
                     "traffic": dom["traffic"], "avg_kernel_ms": dom["ms"],
                     "algorithmic_bytes": dom["algorithmic_bytes"]},
        "whole_call_hbm_frac": round((2 * L.N * L.C * L.H * L.W * 4 + sz.E * L.K * sz.Cp +
                                      L.N * L.K * sz.Ho * sz.Wo * 4) / (ms_rot * 1e-3) / 1e9 /
                                     HBM_PEAK_GBS, 4),
        "int8_mfma": {"kernel": prod["kernel"], "TOPS": round(i8, 1),
                      "frac_of_peak": round(i8 / I8_MFMA_PEAK_TOPS, 4),
                      # what the bytes of the fused product (codes in, Y out) allow at 8 TB/s
                      "cap_by_bytes": round(min(1.0, gemm_ops / fused_bytes * HBM_PEAK_GBS * 1e9 /
                                                (I8_MFMA_PEAK_TOPS * 1e12)), 4)},
    }


def compact(rec):
    """A per_config entry of the printed line: the figures, without the per-kernel detail."""
    r = rec["roofline"]
    return {"name": rec["name"], "ms": rec["ms"], "TOPS": rec["TOPS"],
            "ms_resident": rec["ms_resident"],
            **({"ms_in_sequence": rec["ms_in_sequence"]} if "ms_in_sequence" in rec else {}),
            "kernel_ms": {k["kernel"]: k["ms"] for k in rec["kernels"]},
            "roofline": {"kernel": r["kernel"], "achieved": r["achieved"], "frac": r["frac"],
                         "traffic": r["traffic"], "algorithmic_bytes": r["algorithmic_bytes"]},
            "whole_call_hbm_frac": rec["whole_call_hbm_frac"],
            "int8_mfma_frac": rec["int8_mfma"]["frac_of_peak"],
            "int8_mfma_cap_by_bytes": rec["int8_mfma"]["cap_by_bytes"],
            **({"bit_sweep": rec["bit_sweep"]} if "bit_sweep" in rec else {})}


def time_direct(run, reps=5):
    import torch
    from paper_2003_08646_amd import binding as B
    c = run.conv
    yd = torch.empty_like(c.y)
    for _ in range(2):
        B.lance_direct_conv3x3_f32(c.desc, run.x, run.w, yd)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        B.lance_direct_conv3x3_f32(c.desc, run.x, run.w, yd)
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / reps * 1e3
    y = c.forward(run.x)
    torch.cuda.synchronize()
    rel = float(torch.linalg.vector_norm(y - yd) / torch.linalg.vector_norm(yd))
    return ms, rel


def staged_entry_points(run, calls=100):
    """Each staged entry point on its own (every intermediate in HBM): microseconds per call
    (HIP events around a batch of calls, inputs resident), algorithmic bytes and their rate."""
    import torch
    from paper_2003_08646_amd import binding as B
    L, conv = run.L, run.conv
    s, d = conv.sz, conv.desc
    st = conv.alloc_staged()
    conv.forward_staged(run.x)
    rows = [
        ("lance_filter_transform_q8 (off-line)", lambda: conv.prepare_filters(run.w),
         4 * L.K * L.C * 9 + s.uq_bytes + 4 * s.E * L.K, 0),
        ("lance_input_transform_q8",
         lambda: B.lance_input_transform_q8(d, run.x, st["vq"], conv.v_range, st["v_colsum"],
                                            conv.workspace),
         2 * 4 * L.N * L.C * L.H * L.W + s.vq_bytes + 4 * s.E * s.P, 0),
        ("lance_winograd_gemm_i8", lambda: B.lance_winograd_gemm_i8(d, conv.uq, st["vq"], st["acc"]),
         s.uq_bytes + s.vq_bytes + 4 * s.E * L.K * s.P, 2.0 * s.E * L.K * s.Cp * s.P),
        ("lance_output_transform_dq",
         lambda: B.lance_output_transform_dq(d, st["acc"], conv.u_range, conv.u_rowsum,
                                             conv.v_range, st["v_colsum"], st["y"]),
         4 * s.E * L.K * s.P + 4 * s.E * s.P + 4 * L.N * L.K * s.Ho * s.Wo, 0),
    ]
    out = []
    for name, fn, nbytes, ops in rows:
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(calls):
            fn()
        b.record()
        torch.cuda.synchronize()
        dt = a.elapsed_time(b) * 1e-3 / calls
        rec = {"entry_point": name, "us": round(dt * 1e6, 2), "algorithmic_bytes": int(nbytes),
               "GBps": round(nbytes / dt / 1e9, 1), "frac_hbm": round(nbytes / dt / 1e9 / HBM_PEAK_GBS, 4)}
        if ops:
            rec["int8_TOPS"] = round(ops / dt / 1e12, 1)
            rec["frac_int8_mfma_peak"] = round(ops / dt / 1e12 / I8_MFMA_PEAK_TOPS, 4)
        out.append(rec)
    conv._staged = None
    return out


def width_sweep(L, widths, grid=False):
    """Relative L2 error against the fp32 direct convolution of the same library, and the time of
    the fused call, per code width (Sec. 4's weight / input width grid on a synthetic layer).
    grid: every (filter width, input width) pair, plus weight-only quantization and Algorithm 1
    with per-matrix ranges; else the diagonal only."""
    import torch
    from paper_2003_08646_amd import binding as B
    base = LayerRun(L)
    c0 = base.conv
    yd = torch.empty_like(c0.y)
    B.lance_direct_conv3x3_f32(c0.desc, base.x, base.w, yd)
    torch.cuda.synchronize()
    nd = float(torch.linalg.vector_norm(yd.double()))
    rel = lambda y: round(float(torch.linalg.vector_norm(y.double() - yd.double())) / nd, 5)
    out = []
    pairs = [(bw, bx) for bw in widths for bx in widths] if grid else [(b, b) for b in widths]
    for bw, bx in pairs:
        r = LayerRun(L.with_(bits=bx, bits_w=bw))
        rec = {"filter_bits": bw, "input_bits": bx, "ms": round(r.time_loop(50, 10, rotate=False), 5),
               "rel_l2_vs_fp32_direct": rel(r.conv.y)}
        if bw <= 4 and bx <= 4 and L.C > 16 and L.m == 2:
            rp = LayerRun(L.with_(bits=bx, bits_w=bw), flags=B.LANCE_CODES_PACKED4)
            rec["ms_packed_codes"] = round(rp.time_loop(50, 10, rotate=False), 5)
            rec["rel_l2_packed_codes"] = rel(rp.conv.y)
        out.append(rec)
    if grid:
        y = torch.empty_like(yd)
        for bw in widths:
            r = LayerRun(L.with_(bits_w=bw))
            B.lance_conv3x3_winograd_wq_f32(r.conv.desc, r.x, r.conv.uq, r.conv.u_range, y)
            torch.cuda.synchronize()
            out.append({"filter_bits": bw, "input_bits": 32, "mode": "weight-only",
                        "rel_l2_vs_fp32_direct": rel(y)})
        if L.direct_ops < 2e9:   # the literal form is O(K*P*C*E) vector work: small layers only
            for bw, bx in pairs:
                d = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, bx, B.LANCE_FILTER_BITS(bw))
                B.lance_alg1_literal_f32(d, base.x, base.w, y)
                torch.cuda.synchronize()
                out.append({"filter_bits": bw, "input_bits": bx, "mode": "Algorithm 1, per-matrix ranges",
                            "rel_l2_vs_fp32_direct": rel(y)})
    return out


def time_filter_transform(runs, reps=10):
    import torch
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        for r in runs:
            r.conv.prepare_filters(r.w)
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / reps * 1e3


def cpu_oracle(runs, min_seconds=0.0):
    """The oracle (stages 2-4, filters prepared) on the same layers, on the host cores."""
    from oracle import lance_oracle as O
    prepared = [O.prepare_filters(r.W_host, r.L.m, r.L.bits) for r in runs]
    passes, t_cpu = 0, 0.0
    while passes == 0 or (t_cpu < min_seconds and passes < 400):
        t0 = time.perf_counter()
        for r, f in zip(runs, prepared):
            O.lance_conv(r.X_host, r.W_host, r.L.pad, r.L.m, r.L.bits, filters=f)
        t_cpu += time.perf_counter() - t0
        passes += 1
    ops = sum(r.L.direct_ops for r in runs)
    return {"value": round(ops / (t_cpu / passes) / 1e12, 5), "unit": "TOPS", "cores": O.threads(),
            "kind": "oracle", "ms_per_step": round(t_cpu / passes * 1e3, 1), "passes": passes}


def run_single(args, L, traffic):
    import torch
    from paper_2003_08646_amd import binding as B
    lflags = B.LANCE_LAYOUT_NHWC if args.layout == "nhwc" else 0
    if args.ranges == "static":
        cal = LayerRun(L, flags=lflags)
        cal.call()
        torch.cuda.synchronize()
        v_range = cal.conv.v_range.clone()
        del cal
        run = LayerRun(L, flags=lflags | B.LANCE_INPUT_RANGE_STATIC)
        run.conv.v_range.copy_(v_range)
    else:
        run = LayerRun(L, flags=lflags)
    rec = layer_record(run, args.steps, args.warmup, traffic)
    ms_direct, rel = time_direct(run)
    st = LayerRun(L, flags=B.LANCE_INPUT_RANGE_STATIC | lflags)
    st.conv.v_range.copy_(run.conv.v_range)
    ms_static = st.time_loop(args.steps, args.warmup, rotate=False)
    same = bool(torch.equal(st.conv.y, run.conv.forward(run.x)))
    del st
    out = {
        "metric": "direct-conv-equivalent TOPS per 3x3 layer (1 MI355X)",
        "value": rec["TOPS"], "unit": "TOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": rec["ms"], "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "i8", "data": "synthetic",
        "config": {"workload": f"{L.name}: {rec['shape']}, fused stages 2-4, filters prepared, "
                               f"{rec['buffer_pairs']} rotating buffer pairs", "seed": L.seed,
                   "layout": args.layout, "input_ranges": args.ranges},
        "roofline": rec["roofline"], "kernels": rec["kernels"], "int8_mfma": rec["int8_mfma"],
        "resident_buffers": {"ms_per_step": rec["ms_resident"], "TOPS": rec["TOPS_resident"]},
        "whole_call_hbm_frac": rec["whole_call_hbm_frac"],
        "ms_filter_transform_offline": round(time_filter_transform([run]), 5),
        "fp32_direct_conv_gpu": {"ms": round(ms_direct, 5),
                                 "TFLOPS": round(L.direct_ops / (ms_direct * 1e-3) / 1e12, 2),
                                 "speedup_of_lance": round(ms_direct / rec["ms"], 2)},
        "rel_l2_vs_fp32_direct": round(rel, 5),
        "static_input_ranges": {"ms_per_step": round(ms_static, 5),
                                "TOPS": round(L.direct_ops / (ms_static * 1e-3) / 1e12, 2),
                                "same_output_as_dynamic": same},
        "traffic_source": traffic_note(traffic),
    }
    if args.staged:
        out["staged_entry_points"] = staged_entry_points(run)
    if args.width_grid:
        out["width_grid"] = width_sweep(L, [8, 6, 4, 3, 2], grid=True)
    if not args.no_cpu_baseline and L.name != "probe_n16_c2048_k2048_32":
        cb = cpu_oracle([run], min_seconds=10.0)
        cb["sample"] = f"the whole {L.name} layer, {cb['passes']} passes"
        out["cpu_baseline"] = cb
    return out


def traffic_note(traffic):
    if traffic is None:
        return ("none on file for this build of the kernels (see bench.py --pmc-pass / "
                "--ingest-pmc): traffic fields are null")
    return {"file": os.path.relpath(TRAFFIC_FILE, ROOT), "replayed": True,
            "measured_at_commit": traffic.get("commit"), "source_digest": traffic["source_digest"],
            "what": "FETCH_SIZE + WRITE_SIZE per launch from two rocprofv3 --pmc runs of "
                    "bench.py --pmc-pass, scaled by the same counters' readings for a 256 MiB copy"}


def run_cfg5(args, traffic):
    import torch
    from paper_2003_08646_amd import binding as B
    from paper_2003_08646_amd import workloads as Wk
    layers = Wk.vgg16_layers()
    runs = [LayerRun(L) for L in layers]
    total_ops = sum(L.direct_ops for L in layers)
    torch.cuda.synchronize()

    def sequence():
        for r in runs:
            r.conv.forward(r.x)

    # the timed region: W warm-up steps, then exactly K steps
    for _ in range(args.warmup):
        sequence()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        sequence()
    torch.cuda.synchronize()
    ms_step = (time.perf_counter() - t0) / args.steps * 1e3

    # per-layer times inside the same sequence (events between the layers; its own passes,
    # because an event between two calls keeps the second from starting under the first's tail)
    reps = max(3, min(args.steps, 50))
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(len(runs) + 1)] for _ in range(reps)]
    for rep in range(reps):
        ev[rep][0].record()
        for i, r in enumerate(runs):
            r.conv.forward(r.x)
            ev[rep][i + 1].record()
    torch.cuda.synchronize()
    in_seq_ms = [sum(ev[rep][i].elapsed_time(ev[rep][i + 1]) for rep in range(reps)) / reps
                 for i in range(len(runs))]

    # static (calibrated) ranges: the ranges each input produced are handed back, no range pass
    sruns = []
    for r in runs:
        s = LayerRun(r.L, flags=B.LANCE_INPUT_RANGE_STATIC)
        s.conv.v_range.copy_(r.conv.v_range)
        sruns.append(s)
    for _ in range(args.warmup):
        for s in sruns:
            s.conv.forward(s.x)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        for s in sruns:
            s.conv.forward(s.x)
    torch.cuda.synchronize()
    ms_static = (time.perf_counter() - t0) / args.steps * 1e3
    static_same = all(bool(torch.equal(s.conv.y, r.conv.y)) for s, r in zip(sruns, runs))
    del sruns

    # per-layer records (rotating buffers beyond the last-level cache, per-kernel event times)
    per_layer = []
    agg = {}
    for i, r in enumerate(runs):
        rec = layer_record(r, args.steps, args.warmup, traffic)
        rec["ms_in_sequence"] = round(in_seq_ms[i], 5)
        rec["TOPS_in_sequence"] = round(r.L.direct_ops / (in_seq_ms[i] * 1e-3) / 1e12, 2)
        per_layer.append(rec)
        for k in rec["kernels"]:
            a = agg.setdefault(k["kernel"], {"ms": 0.0, "bytes": 0, "launches": 0, "traffic": 0,
                                             "traffic_known": True})
            a["ms"] += k["ms"]; a["bytes"] += k["algorithmic_bytes"]; a["launches"] += 1
            if k["traffic"] is None:
                a["traffic_known"] = False
            else:
                a["traffic"] += k["traffic"]
    dom = max(agg, key=lambda n: agg[n]["ms"])
    a = agg[dom]
    achieved = a["bytes"] / (a["ms"] * 1e-3) / 1e9
    roofline = {"kernel": dom, "bound": "hbm", "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS,
                "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": int(a["traffic"] / a["launches"]) if a["traffic_known"] else None,
                "avg_kernel_ms": round(a["ms"] / a["launches"], 5),
                "algorithmic_bytes": int(a["bytes"] / a["launches"]),
                "launches_per_step": a["launches"],
                "share_of_step": round(a["ms"] / sum(v["ms"] for v in agg.values()), 3)}
    kernels = {n: {"ms_per_step": round(v["ms"], 5), "launches_per_step": v["launches"],
                   "GBps": round(v["bytes"] / (v["ms"] * 1e-3) / 1e9, 1) if v["bytes"] else None}
               for n, v in sorted(agg.items(), key=lambda kv: -kv[1]["ms"])}

    ms_direct, rels = 0.0, []
    for r in runs:
        md, rel = time_direct(r, reps=3)
        ms_direct += md
        rels.append(round(rel, 5))
    floor_bytes = sum(2 * r.L.N * r.L.C * r.L.H * r.L.W * 4 + r.conv.sz.E * r.L.K * r.conv.sz.Cp +
                      r.L.N * r.L.K * r.conv.sz.Ho * r.conv.sz.Wo * 4 for r in runs)
    out = {
        "metric": "direct-conv-equivalent TOPS per 3x3 layer (1 MI355X)",
        "value": round(total_ops / (ms_step * 1e-3) / 1e12, 2), "unit": "TOPS", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_step, 5),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "i8",
        "data": "synthetic",
        "config": {"workload": "cfg5: the thirteen 3x3 layers of a VGG-16-shaped network at 224x224, "
                               "N=16, pad 1, F(2x2,3x3) 8-bit, fused stages 2-4 back to back on "
                               "their own buffers, filters prepared, independent seeded inputs",
                   "direct_GOP": round(total_ops / 1e9, 1), "seeds": "501..513"},
        "roofline": roofline,
        "kernels": kernels,
        "whole_step_hbm_frac": round(floor_bytes / (ms_step * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "ms_filter_transform_offline": round(time_filter_transform(runs, reps=5), 5),
        "fp32_direct_conv_gpu": {"ms": round(ms_direct, 4),
                                 "TFLOPS": round(total_ops / (ms_direct * 1e-3) / 1e12, 2),
                                 "speedup_of_lance": round(ms_direct / ms_step, 2)},
        "rel_l2_vs_fp32_direct_per_layer": rels,
        "static_input_ranges": {"ms_per_step": round(ms_static, 5),
                                "TOPS": round(total_ops / (ms_static * 1e-3) / 1e12, 2),
                                "same_output_as_dynamic": static_same},
        "traffic_source": traffic_note(traffic),
    }
    per_config = []
    if not args.no_per_config:
        for L in (Wk.CFG1, Wk.CFG2, Wk.CFG3_M2, Wk.CFG3_M4, Wk.CFG4):
            r = LayerRun(L)
            per_config.append(layer_record(r, args.steps, args.warmup, traffic))
            del r
            torch.cuda.empty_cache()
        # configuration 4's width sweep: error against the fp32 direct convolution per width
        per_config[-1]["bit_sweep"] = width_sweep(Wk.CFG4, [8, 6, 4])
    full = per_config + per_layer
    out["per_config"] = [compact(r) for r in full]
    detail_dir = os.path.join(ROOT, "gpurun_out")
    if os.path.isdir(detail_dir):   # every field of every record, for the profile summaries
        with open(os.path.join(detail_dir, "bench_detail.json"), "w") as f:
            json.dump(dict(out, per_config=full), f, indent=1)
    if not args.no_cpu_baseline:
        cb = cpu_oracle(runs)
        cb["sample"] = (f"{cb['passes']} pass over the same thirteen layers at full size "
                        "(stages 2-4 of the oracle, filters prepared)")
        out["cpu_baseline"] = cb
    return out


# ---------------------------------------------------------------------------------------------
# HBM traffic from rocprofv3 counter runs
# ---------------------------------------------------------------------------------------------
def pmc_workloads():
    from paper_2003_08646_amd import workloads as Wk
    return [Wk.CFG1, Wk.CFG2, Wk.CFG3_M2, Wk.CFG3_M4, Wk.CFG4] + Wk.vgg16_layers()


def pmc_pass(order_path):
    """What a counter run executes: per workload one warm call, a 256 MiB copy (separator and
    scale), ONE fused call, the copy again.  Writes the workload order and kernel names."""
    import torch
    src = torch.ones(SEPARATOR_ELEMS, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    order = []
    for L in pmc_workloads():
        run = LayerRun(L)
        _, names = run.kernel_times(1, rotate=False)
        torch.cuda.synchronize()
        dst.copy_(src)
        run.call()
        torch.cuda.synchronize()
        order.append({"workload": L.name, "kernels": [n for n in names if n]})
        del run
        torch.cuda.empty_cache()
    dst.copy_(src)
    torch.cuda.synchronize()
    with open(order_path, "w") as f:
        json.dump({"order": order, "separator_bytes": SEPARATOR_ELEMS * 4,
                   "source_digest": source_digest()}, f, indent=1)
    print(json.dumps({"pmc_pass": "done", "workloads": len(order), "order_file": order_path}))


def _dispatches(path, counter):
    rows = {}
    with open(path) as f:
        for r in csv.DictReader(f):
            if r["Counter_Name"] == counter:
                rows[int(r["Dispatch_Id"])] = (r["Kernel_Name"], float(r["Counter_Value"]),
                                               int(r["Grid_Size"]))
    return [rows[k] for k in sorted(rows)]


def _segments(disp, order, counter_kib):
    """Splits the dispatches at the separator copies; returns per workload {kernel: KiB} and the
    separator's average reading."""
    # the runtime's copy kernel; its reading is the copy's size up to the counter's unit
    sep_idx = [i for i, d in enumerate(disp)
               if "copy" in d[0].lower() and "lance" not in d[0] and d[1] > 0.25 * counter_kib]
    if len(sep_idx) != len(order) + 1:
        raise SystemExit(f"expected {len(order) + 1} separator copies, found {len(sep_idx)}")
    sep_reading = sum(disp[i][1] for i in sep_idx) / len(sep_idx)
    out = []
    for w, (a, b) in zip(order, zip(sep_idx[:-1], sep_idx[1:])):
        # the fused call comes right after its separator (what follows it in the segment is the
        # next workload's preparation)
        seg = [d for d in disp[a + 1:b] if "lance" in d[0]][:len(w["kernels"])]
        got = {}
        for kern, d in zip(w["kernels"], seg):
            if not (kern + "<" in d[0] or kern + "(" in d[0]):
                raise SystemExit(f"{w['workload']}: expected {kern}, found {d[0]}")
            got[kern] = d[1]
        if len(got) != len(w["kernels"]):
            raise SystemExit(f"{w['workload']}: {len(seg)} kernels after the separator")
        out.append(got)
    return out, sep_reading


def ingest_pmc(fetch_csv, write_csv, order_path, commit):
    with open(order_path) as f:
        meta = json.load(f)
    order = meta["order"]
    sep_kib = meta["separator_bytes"] / 1024
    fetch, f_sep = _segments(_dispatches(fetch_csv, "FETCH_SIZE"), order, sep_kib)
    write, w_sep = _segments(_dispatches(write_csv, "WRITE_SIZE"), order, sep_kib)
    ff, wf = sep_kib / f_sep, sep_kib / w_sep
    rec = {"source_digest": meta["source_digest"], "commit": commit,
           "calibration": {"separator_kib": sep_kib, "fetch_reading_kib": f_sep,
                           "write_reading_kib": w_sep, "fetch_factor": ff, "write_factor": wf}}
    for w, fk, wk in zip(order, fetch, write):
        rec[w["workload"]] = {k: {"fetch_bytes": round(fk[k] * ff * 1024),
                                  "write_bytes": round(wk[k] * wf * 1024),
                                  "fetch_kib_raw": fk[k], "write_kib_raw": wk[k]}
                              for k in w["kernels"]}
    with open(TRAFFIC_FILE, "w") as f:
        json.dump(rec, f, indent=1, sort_keys=True)
    print(json.dumps({"ingested": len(order), "fetch_factor": ff, "write_factor": wf,
                      "file": TRAFFIC_FILE}))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="cfg5",
                    help="cfg5 (default: the thirteen VGG-16-shaped layers back to back) | cfg1 | "
                         "cfg2 | cfg3_m2 | cfg3_m4 | cfg4 | probe: a compute-bound layer "
                         "(C=K=2048) that shows the product kernel against the int8 matrix peak; "
                         "not a paper workload, no CPU baseline")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--ranges", choices=["dynamic", "static"], default="dynamic",
                    help="single-layer workloads: static = the timed calls take caller-supplied "
                         "input ranges (LANCE_INPUT_RANGE_STATIC), calibrated by one dynamic call")
    ap.add_argument("--layout", choices=["nchw", "nhwc"], default="nchw",
                    help="single workloads only: activations NCHW (default) or NHWC (Sec. 3.3's layout)")
    ap.add_argument("--staged", action="store_true",
                    help="single workloads only: also time the four staged entry points one by one")
    ap.add_argument("--width-grid", action="store_true",
                    help="single workloads only: error against the fp32 direct convolution over "
                         "filter x input code widths, weight-only quantization, packed 4-bit codes")
    ap.add_argument("--no-per-config", action="store_true",
                    help="cfg5 only: leave configurations 1-4 out of per_config")
    ap.add_argument("--pmc-pass", metavar="ORDER.json",
                    help="run what a rocprofv3 --pmc run should see and write the workload order")
    ap.add_argument("--ingest-pmc", nargs=3, metavar=("FETCH.csv", "WRITE.csv", "ORDER.json"),
                    help="turn two counter runs of --pmc-pass into measured_traffic.json (no GPU)")
    ap.add_argument("--commit", default=None, help="with --ingest-pmc: commit the runs were taken at")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (no multi-GPU path); use --gpus 1",
              file=sys.stderr)
        return 2
    if args.ingest_pmc:
        ingest_pmc(*args.ingest_pmc, commit=args.commit)
        return 0

    import torch
    from paper_2003_08646_amd import workloads as Wk
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    if args.pmc_pass:
        pmc_pass(args.pmc_pass)
        return 0
    traffic = load_traffic()
    if args.workload == "cfg5" and args.ranges == "static":
        print("bench.py: --ranges static times one layer (the cfg5 line reports its static-range "
              "time as static_input_ranges)", file=sys.stderr)
        return 2
    if args.workload == "cfg5":
        out = run_cfg5(args, traffic)
    else:
        layers = {"cfg1": Wk.CFG1, "cfg2": Wk.CFG2, "cfg3_m2": Wk.CFG3_M2, "cfg3_m4": Wk.CFG3_M4,
                  "cfg4": Wk.CFG4, "probe": Wk.PROBE}
        out = run_single(args, layers[args.workload], traffic)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
