"""Time the staged entry points one by one (stages 1-4 with every intermediate in HBM).

    python -m paper_2003_08646_amd.stages [--configs cfg2,cfg3,cfg4] [--layer NAME] [--calls N]

For each layer and each of `lance_filter_transform_q8`, `lance_input_transform_q8`,
`lance_winograd_gemm_i8`, `lance_output_transform_dq`: microseconds per call (HIP events around a
batch of calls on the current stream, inputs resident), the algorithmic HBM bytes of the call and
the rate they give against 8 TB/s, and for the GEMM its int8 rate against 5.0 POP/s.  Algorithmic
bytes (b = 8, m the tile size, E = (m+2)^2 positions, P tiles, Cp padded channels):

    filter transform   4*K*C*9 read + E*K*Cp + 4*E*K written
    input transform    2 * 4*N*C*H*W read (range pass + quantize pass) + E*P*Cp + 4*E*P written
    GEMM               E*(K+P)*Cp read + 4*E*K*P written
    output transform   4*E*K*P + 4*E*P read + 4*N*K*Ho*Wo written

The form to put behind `rocprofv3 --kernel-trace --stats -- python3 -m paper_2003_08646_amd.stages`
for the durations of the individual kernels.
"""
from __future__ import annotations

import argparse

HBM_PEAK = 8.0e12
MFMA_I8_PEAK = 5.0e15


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--configs", default="cfg2,cfg3,cfg4")
    ap.add_argument("--layer", default="", help="only the layer of this name")
    ap.add_argument("--calls", type=int, default=200, help="timed calls per entry point")
    args = ap.parse_args()
    import torch
    from . import binding as B
    from . import workloads as Wk
    from .layer import LanceConv

    def timed(fn, calls):
        for _ in range(5):
            fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(calls):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) * 1e-3 / calls

    layers = [Wk.PROBE] if args.layer == Wk.PROBE.name else \
        [L for cfg in args.configs.split(",") for L in Wk.CONFIGS[cfg]]
    for L in layers:
        if args.layer and L.name != args.layer:
            continue
        X, Wt = Wk.make_inputs(L)
        x, w = torch.from_numpy(X).cuda(), torch.from_numpy(Wt).cuda()
        conv = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits)
        s, d = conv.sz, conv.desc
        st = conv.alloc_staged()
        conv.prepare_filters(w)
        conv.forward_staged(x)
        rows = [
            ("lance_filter_transform_q8 (off-line)",
             lambda: conv.prepare_filters(w),
             4 * L.K * L.C * 9 + s.E * L.K * s.Cp + 4 * s.E * L.K, 0),
            ("lance_input_transform_q8",
             lambda: B.lance_input_transform_q8(d, x, st["vq"], conv.v_range, st["v_colsum"],
                                                conv.workspace),
             2 * 4 * L.N * L.C * L.H * L.W + s.E * s.P * s.Cp + 4 * s.E * s.P, 0),
            ("lance_winograd_gemm_i8",
             lambda: B.lance_winograd_gemm_i8(d, conv.uq, st["vq"], st["acc"]),
             s.E * (L.K + s.P) * s.Cp + 4 * s.E * L.K * s.P, 2.0 * s.E * L.K * s.Cp * s.P),
            ("lance_output_transform_dq",
             lambda: B.lance_output_transform_dq(d, st["acc"], conv.u_range, conv.u_rowsum,
                                                 conv.v_range, st["v_colsum"], st["y"]),
             4 * s.E * L.K * s.P + 4 * s.E * s.P + 4 * L.N * L.K * s.Ho * s.Wo, 0),
        ]
        print(f"== {L.name} m={L.m} N={L.N} C={L.C} K={L.K} {L.H}x{L.W}  (P={s.P}, E={s.E}, Cp={s.Cp})",
              flush=True)
        total = 0.0
        for name, fn, nbytes, ops in rows:
            dt = timed(fn, args.calls)
            if "off-line" not in name:
                total += dt
            line = (f"   {name:38s} {dt * 1e6:9.1f} us  {nbytes / 1e6:9.1f} MB  "
                    f"{nbytes / dt / 1e9:7.0f} GB/s ({nbytes / dt / HBM_PEAK * 100:4.1f}% of 8 TB/s)")
            if ops:
                line += f"  {ops / dt / 1e12:7.1f} int8 TOPS ({ops / dt / MFMA_I8_PEAK * 100:4.1f}% of 5.0 POP/s)"
            print(line, flush=True)
        print(f"   stages 2-4 one by one: {total * 1e6:9.1f} us  "
              f"{L.direct_ops / total / 1e12:7.1f} direct-equivalent TOPS", flush=True)
        del conv, st, x, w
        torch.cuda.empty_cache()
    return 0


if __name__ == "__main__":
    raise SystemExit(main())
