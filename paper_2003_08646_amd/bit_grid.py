"""Relative L2 error of the fused convolution against the fp32 direct convolution of the same
library over a grid of filter and input code widths (the weight / input width grid of the
paper's Sec. 4, here on one seeded synthetic layer instead of a trained network).

    python -m paper_2003_08646_amd.bit_grid [--layer NAME] [--widths 8,6,4,3,2] [--m 2|4] [--literal]

Rows: width of the filter codes; columns: width of the input codes.  Both outputs come from the
GPU (`lance_conv3x3_winograd_q8` and `lance_direct_conv3x3_f32`); nothing here is a parity check.
--literal adds the same grid for Algorithm 1 taken literally (`lance_alg1_literal_f32`: every
transformed patch and filter quantized with the range of its own matrix, binary32 channel sum):
what the shared per-position ranges of the integer product cost, or gain, in accuracy.
"""
from __future__ import annotations

import argparse


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--layer", default="cfg4_n64_c512_k512_14")
    ap.add_argument("--widths", default="8,6,4,3,2")
    ap.add_argument("--m", type=int, default=0, help="tile size override (2 or 4); 0: as configured")
    ap.add_argument("--literal", action="store_true",
                    help="also the grid of Algorithm 1 with per-matrix ranges")
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import workloads as Wk
    from .layer import LanceConv
    L = [l for c in Wk.CONFIGS.values() for l in c if l.name == args.layer][0]
    if args.m:
        L = L.with_(m=args.m)
    widths = [int(v) for v in args.widths.split(",")]
    X, Wt = Wk.make_inputs(L)
    x, w = torch.from_numpy(X).cuda(), torch.from_numpy(Wt).cuda()
    ref = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, 8)
    yd = torch.empty_like(ref.y)
    B.lance_direct_conv3x3_f32(ref.desc, x, w, yd)
    torch.cuda.synchronize()
    nd = float(torch.linalg.vector_norm(yd.double()))
    print(f"{L.name} m={L.m}: relative L2 error of Y against the fp32 direct convolution")
    print("filter \\ input " + "".join(f"{'b=' + str(bx):>11s}" for bx in widths))
    for bw in widths:
        row = []
        for bx in widths:
            conv = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, bx, bits_w=bw)
            conv.prepare_filters(w)
            y = conv.forward(x)
            torch.cuda.synchronize()
            row.append(float(torch.linalg.vector_norm(y.double() - yd.double())) / nd)
            del conv
        print(f"{'b=' + str(bw):>14s} " + "".join(f"{v:11.4g}" for v in row), flush=True)
    if args.literal:
        print(f"{L.name} m={L.m}: the same for Algorithm 1 with per-matrix ranges (binary32 sums)")
        print("filter \\ input " + "".join(f"{'b=' + str(bx):>11s}" for bx in widths))
        y = torch.empty_like(yd)
        for bw in widths:
            row = []
            for bx in widths:
                d = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, bx, B.LANCE_FILTER_BITS(bw))
                B.lance_alg1_literal_f32(d, x, w, y)
                torch.cuda.synchronize()
                row.append(float(torch.linalg.vector_norm(y.double() - yd.double())) / nd)
            print(f"{'b=' + str(bw):>14s} " + "".join(f"{v:11.4g}" for v in row), flush=True)
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
