"""Time the fused convolution and the fp32 direct comparator over the benchmark layer shapes.

    python -m paper_2003_08646_amd.sweep [--m 2|4] [--configs cfg2,cfg3,cfg4,cfg5]
                                         [--layer NAME] [--calls N] [--no-direct]
                                         [--static-ranges] [--nhwc]

Prints one line per layer (seeded synthetic inputs, filters prepared beforehand): microseconds per
fused call, direct-convolution-equivalent TOPS, microseconds of the fp32 direct convolution of the
same library, and their ratio.  cfg5 = the thirteen 3x3 layers of a VGG-16-shaped network.
--static-ranges times the inference mode instead: the ranges each layer's input produces in a
first call with dynamic ranges are handed back as caller-supplied ranges (LANCE_INPUT_RANGE_STATIC,
same codes and outputs, no range pass).
--nhwc times the calls on NHWC tensors (LANCE_LAYOUT_NHWC; the comparator too).
--layer restricts the run to one layer by name and --no-direct skips the comparator: the form to
put behind `rocprofv3 --kernel-trace --stats -- python3 -m paper_2003_08646_amd.sweep ...` for
the per-kernel durations of one layer.  When cfg5 is swept as a whole, a last line gives the
thirteen layers enqueued back to back (every layer on its own seeded input and output buffers;
no pooling or activation between them): the end-to-end time of the 3x3 convolutions of one pass.
"""
from __future__ import annotations

import argparse
import time


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--m", type=int, default=0, help="tile size override (2 or 4); 0: as configured")
    ap.add_argument("--configs", default="cfg2,cfg3,cfg4,cfg5")
    ap.add_argument("--layer", default="", help="only the layer of this name")
    ap.add_argument("--calls", type=int, default=20, help="timed fused calls per layer")
    ap.add_argument("--no-direct", action="store_true", help="skip the fp32 direct comparator")
    ap.add_argument("--static-ranges", action="store_true",
                    help="time the calls with caller-supplied input ranges (no range pass)")
    ap.add_argument("--nhwc", action="store_true",
                    help="X and Y in NHWC (LANCE_LAYOUT_NHWC); the same values, transposed")
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import workloads as Wk
    from .layer import LanceConv

    import numpy as np
    layout = B.LANCE_LAYOUT_NHWC if args.nhwc else 0

    def to_device(X):
        return torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1)) if args.nhwc else X).cuda()

    def make_conv(L, x, w):
        conv = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits, flags=layout)
        conv.prepare_filters(w)
        if not args.static_ranges:
            return conv
        conv.forward(x)  # dynamic ranges of this input ...
        torch.cuda.synchronize()
        st = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits, flags=B.LANCE_INPUT_RANGE_STATIC | layout)
        st.prepare_filters(w)
        st.v_range.copy_(conv.v_range)  # ... handed back as static ranges
        return st

    for cfg in args.configs.split(","):
        for L in Wk.CONFIGS[cfg]:
            if args.layer and L.name != args.layer:
                continue
            if args.m:
                L = L.with_(m=args.m)
            X, Wt = Wk.make_inputs(L)
            x, w = to_device(X), torch.from_numpy(Wt).cuda()
            conv = make_conv(L, x, w)
            for _ in range(3):
                conv.forward(x)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(args.calls):
                conv.forward(x)
            torch.cuda.synchronize()
            dt = (time.perf_counter() - t0) / args.calls
            if args.no_direct:
                print(f"{L.name:30s} m={L.m} N={L.N:3d} C={L.C:3d} K={L.K:3d} {L.H:3d}x{L.W:<3d} "
                      f"fused {dt * 1e6:8.1f} us {L.direct_ops / dt / 1e12:7.1f} TOPS", flush=True)
                del conv, x, w
                torch.cuda.empty_cache()
                continue
            yd = torch.empty_like(conv.y)
            for _ in range(2):
                B.lance_direct_conv3x3_f32(conv.desc, x, w, yd)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                B.lance_direct_conv3x3_f32(conv.desc, x, w, yd)
            torch.cuda.synchronize()
            dd = (time.perf_counter() - t0) / 5
            print(f"{L.name:30s} m={L.m} N={L.N:3d} C={L.C:3d} K={L.K:3d} {L.H:3d}x{L.W:<3d} "
                  f"fused {dt * 1e6:8.1f} us {L.direct_ops / dt / 1e12:7.1f} TOPS | "
                  f"fp32 direct {dd * 1e6:8.1f} us | x{dd / dt:5.2f}", flush=True)
            del conv, x, w, yd
            torch.cuda.empty_cache()
    if "cfg5" in args.configs.split(",") and not args.layer:
        layers = [L.with_(m=args.m) if args.m else L for L in Wk.CONFIGS["cfg5"]]
        convs, xs = [], []
        for L in layers:
            X, Wt = Wk.make_inputs(L)
            x, w = to_device(X), torch.from_numpy(Wt).cuda()
            convs.append(make_conv(L, x, w))
            xs.append(x)
            del w
        for _ in range(3):
            for conv, x in zip(convs, xs):
                conv.forward(x)
        torch.cuda.synchronize()
        passes = max(args.calls, 50)
        t0 = time.perf_counter()
        for _ in range(passes):
            for conv, x in zip(convs, xs):
                conv.forward(x)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / passes
        ops = sum(L.direct_ops for L in layers)
        print(f"cfg5 end to end: the {len(layers)} layers back to back {dt * 1e3:8.3f} ms per pass "
              f"{ops / dt / 1e12:7.1f} TOPS ({passes} passes)", flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
