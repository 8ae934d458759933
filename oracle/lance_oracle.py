"""ctypes front end of the CPU oracle (``lance_oracle.c``).

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only tests, the smoke check and the benchmark's
``cpu_baseline`` leg may import this module.  It never imports the HIP library's package.

The composition in :func:`lance_conv` follows Algorithm 1 of the paper in the GEMM form of
Sec. 3.3: filter transform -> Q, input transform -> Q, integer product, Q', output transform.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "lance_oracle.c")
_LIB = os.path.join(_HERE, "liblance_oracle.so")

CFLAGS = ["-O2", "-std=c99", "-fopenmp", "-ffp-contract=off", "-fno-fast-math", "-shared",
          "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, no intrinsics, no BLAS)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *CFLAGS, _SRC, "-o", _LIB, "-lm"])
    return _LIB


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.lance_oracle_dequantize_value.restype = ctypes.c_double
        _lib.lance_oracle_quantize_value.restype = ctypes.c_int
        _lib.lance_oracle_gemm_i8.restype = ctypes.c_int
        _lib.lance_oracle_threads.restype = ctypes.c_int
    return _lib


def _p(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _f32(a) -> np.ndarray:
    return np.ascontiguousarray(a, dtype=np.float32)


def threads() -> int:
    return int(lib().lance_oracle_threads())


# ------------------------------------------------------------------------------------------
# geometry
# ------------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Geometry:
    N: int
    C: int
    H: int
    W: int
    K: int
    pad: int
    m: int

    @property
    def alpha(self):
        return self.m + 2

    @property
    def E(self):
        return self.alpha * self.alpha

    @property
    def Ho(self):
        return self.H + 2 * self.pad - 2

    @property
    def Wo(self):
        return self.W + 2 * self.pad - 2

    @property
    def th(self):
        return -(-self.Ho // self.m)

    @property
    def tw(self):
        return -(-self.Wo // self.m)

    @property
    def P(self):
        return self.N * self.th * self.tw


def geometry(X: np.ndarray, W: np.ndarray, pad: int, m: int) -> Geometry:
    N, C, H, Wd = X.shape
    K, C2, R, S = W.shape
    assert C == C2 and R == 3 and S == 3
    return Geometry(N, C, H, Wd, K, pad, m)


# ------------------------------------------------------------------------------------------
# Part 1 and the unquantized Winograd form
# ------------------------------------------------------------------------------------------
def direct_conv_f64(X, W, pad: int) -> np.ndarray:
    X, W = _f32(X), _f32(W)
    g = geometry(X, W, pad, 2)
    Y = np.empty((g.N, g.K, g.Ho, g.Wo), dtype=np.float64)
    lib().lance_oracle_direct_conv_f64(_p(X), _p(W), _p(Y), g.N, g.C, g.H, g.W, g.K, pad)
    return Y


def winograd_conv_f64(X, W, pad: int, m: int) -> np.ndarray:
    X, W = _f32(X), _f32(W)
    g = geometry(X, W, pad, m)
    Y = np.empty((g.N, g.K, g.Ho, g.Wo), dtype=np.float64)
    lib().lance_oracle_winograd_conv_f64(_p(X), _p(W), _p(Y), g.N, g.C, g.H, g.W, g.K, pad, m)
    return Y


def matrices(m: int):
    a = m + 2
    bt = np.empty((a, a)); g = np.empty((a, 3)); at = np.empty((m, a))
    lib().lance_oracle_matrices(m, _p(bt), _p(g), _p(at))
    return bt, g, at


# ------------------------------------------------------------------------------------------
# Part 2, step by step
# ------------------------------------------------------------------------------------------
def input_tile_f32(d, m: int) -> np.ndarray:
    a = m + 2
    d = _f32(d).reshape(a, a)
    v = np.empty((a, a), dtype=np.float32)
    lib().lance_oracle_input_tile_f32(m, _p(d), _p(v))
    return v


def filter_tile_f32(g, m: int) -> np.ndarray:
    a = m + 2
    g = _f32(g).reshape(3, 3)
    u = np.empty((a, a), dtype=np.float32)
    lib().lance_oracle_filter_tile_f32(m, _p(g), _p(u))
    return u


def filter_transform_f32(W, m: int) -> np.ndarray:
    """U[e][k][c]."""
    W = _f32(W)
    K, C = W.shape[:2]
    E = (m + 2) ** 2
    U = np.empty((E, K, C), dtype=np.float32)
    lib().lance_oracle_filter_transform_f32(_p(W), _p(U), K, C, m)
    return U


def input_transform_f32(X, pad: int, m: int) -> np.ndarray:
    """V[e][p][c]."""
    X = _f32(X)
    N, C, H, Wd = X.shape
    g = Geometry(N, C, H, Wd, 1, pad, m)
    V = np.empty((g.E, g.P, C), dtype=np.float32)
    lib().lance_oracle_input_transform_f32(_p(X), _p(V), N, C, H, Wd, pad, m)
    return V


def ranges(T: np.ndarray, per_tensor: bool = False) -> np.ndarray:
    """(min,max) per leading index of T; float32 [E][2]."""
    T = _f32(T)
    E = T.shape[0]
    count = T.size // E
    r = np.empty((E, 2), dtype=np.float32)
    lib().lance_oracle_ranges(_p(T), E, ctypes.c_size_t(count), int(per_tensor), _p(r))
    return r


def quant_params(mn: float, mx: float, bits: int):
    inv = ctypes.c_float(); sc = ctypes.c_float()
    lib().lance_oracle_quant_params(ctypes.c_float(mn), ctypes.c_float(mx), bits,
                                    ctypes.byref(inv), ctypes.byref(sc))
    return np.float32(inv.value), np.float32(sc.value)


def quantize_value(x: float, mn: float, inv: float, bits: int) -> int:
    return int(lib().lance_oracle_quantize_value(ctypes.c_float(x), ctypes.c_float(mn),
                                                 ctypes.c_float(inv), bits))


def dequantize_value(code: int, mn: float, scale: float) -> float:
    return float(lib().lance_oracle_dequantize_value(int(code), ctypes.c_float(mn),
                                                     ctypes.c_float(scale)))


def quantize(T: np.ndarray, rng: np.ndarray, bits: int, Cp: int):
    """Signed codes [E][rows][Cp] (int8) and their sums over c<C [E][rows] (int32)."""
    T = _f32(T)
    E, rows, C = T.shape
    assert Cp >= C
    codes = np.empty((E, rows, Cp), dtype=np.int8)
    sums = np.empty((E, rows), dtype=np.int32)
    lib().lance_oracle_quantize(_p(T), _p(_f32(rng)), bits, E, ctypes.c_size_t(rows), C, Cp,
                                _p(codes), _p(sums))
    return codes, sums


def gemm_i8(Uq: np.ndarray, Vq: np.ndarray) -> np.ndarray:
    """ACC[e][k][p] = sum_c Uq[e][k][c] * Vq[e][p][c], exact."""
    E, K, Cp = Uq.shape
    E2, P, Cp2 = Vq.shape
    assert E == E2 and Cp == Cp2
    Uq = np.ascontiguousarray(Uq, dtype=np.int8); Vq = np.ascontiguousarray(Vq, dtype=np.int8)
    ACC = np.empty((E, K, P), dtype=np.int32)
    ovf = lib().lance_oracle_gemm_i8(_p(Uq), _p(Vq), _p(ACC), E, K, ctypes.c_size_t(P), Cp)
    if ovf:
        raise OverflowError("int32 accumulator overflow")
    return ACC


def gemm_i8_sampled(Uq: np.ndarray, Vq: np.ndarray, ekp: np.ndarray) -> np.ndarray:
    E, K, Cp = Uq.shape
    P = Vq.shape[1]
    Uq = np.ascontiguousarray(Uq, dtype=np.int8); Vq = np.ascontiguousarray(Vq, dtype=np.int8)
    ekp = np.ascontiguousarray(ekp, dtype=np.int64)
    out = np.empty(len(ekp), dtype=np.int32)
    lib().lance_oracle_gemm_i8_sampled(_p(Uq), _p(Vq), K, ctypes.c_size_t(P), Cp, _p(ekp),
                                       ctypes.c_size_t(len(ekp)), _p(out))
    return out


def dequant_output_f64(ACC, u_range, u_rowsum, v_range, v_colsum, g: Geometry, bits: int,
                       bits_w: int | None = None):
    """bits: width of the input codes; bits_w: of the filter codes (default: the same)."""
    ACC = np.ascontiguousarray(ACC, dtype=np.int32)
    Y = np.empty((g.N, g.K, g.Ho, g.Wo), dtype=np.float64)
    lib().lance_oracle_dequant_output_f64(
        _p(ACC), _p(_f32(u_range)), _p(np.ascontiguousarray(u_rowsum, dtype=np.int32)),
        _p(_f32(v_range)), _p(np.ascontiguousarray(v_colsum, dtype=np.int32)), _p(Y),
        g.N, g.C, g.H, g.W, g.K, g.pad, g.m, bits if bits_w is None else bits_w, bits)
    return Y


def alg1_literal_f64(X, W, pad: int, m: int, bits: int, u_range=None, v_range=None,
                     bits_w: int | None = None):
    """Algorithm 1 loop by loop.  Ranges: per (m+2)x(m+2) matrix unless both are given.
    bits: width of the input codes; bits_w: of the filter codes (default: the same)."""
    X, W = _f32(X), _f32(W)
    g = geometry(X, W, pad, m)
    Y = np.empty((g.N, g.K, g.Ho, g.Wo), dtype=np.float64)
    mode = 0 if u_range is None else 1
    ur = _f32(u_range) if mode else np.zeros((g.E, 2), np.float32)
    vr = _f32(v_range) if mode else np.zeros((g.E, 2), np.float32)
    lib().lance_oracle_alg1_literal_f64(_p(X), _p(W), _p(Y), g.N, g.C, g.H, g.W, g.K, pad, m,
                                        bits if bits_w is None else bits_w, bits, mode,
                                        _p(ur), _p(vr))
    return Y


def weight_only_conv_f64(X, W, pad: int, m: int, bits_w: int, per_tensor: bool = False,
                         filters: "Filters | None" = None) -> np.ndarray:
    """Weight-only quantization (Sec. 4, the 4-32 row of Table 2): quantized, de-quantized
    filters times the unquantized transformed input."""
    X, W = _f32(X), _f32(W)
    g = geometry(X, W, pad, m)
    f = filters if filters is not None else prepare_filters(W, m, bits_w, per_tensor)
    Uq = np.ascontiguousarray(f.Uq, dtype=np.int8)
    Y = np.empty((g.N, g.K, g.Ho, g.Wo), dtype=np.float64)
    lib().lance_oracle_weight_only_f64(_p(X), _p(Uq), _p(_f32(f.u_range)), _p(Y), g.N, g.C,
                                       Uq.shape[2], g.H, g.W, g.K, pad, m, bits_w)
    return Y


# ------------------------------------------------------------------------------------------
# the whole path
# ------------------------------------------------------------------------------------------
@dataclass
class Filters:
    Uq: np.ndarray        # int8  [E][K][C]
    u_range: np.ndarray   # f32   [E][2]
    u_rowsum: np.ndarray  # int32 [E][K]


@dataclass
class Result:
    geom: Geometry
    filters: Filters
    Vq: np.ndarray        # int8  [E][P][C]
    v_range: np.ndarray   # f32   [E][2]
    v_colsum: np.ndarray  # int32 [E][P]
    ACC: np.ndarray | None  # int32 [E][K][P]
    Y: np.ndarray | None    # f64   [N][K][Ho][Wo]


def prepare_filters(W, m: int, bits: int, per_tensor: bool = False) -> Filters:
    """Algorithm 1's u^ = Q(G g G^T) for every (k,c); done once off-line (Sec. 3.4)."""
    U = filter_transform_f32(W, m)
    r = ranges(U, per_tensor)
    Uq, rs = quantize(U, r, bits, U.shape[2])
    return Filters(Uq, r, rs)


def lance_conv(X, W, pad: int, m: int, bits: int, per_tensor: bool = False,
               static_v_range=None, filters: Filters | None = None,
               want_acc: bool = True, want_y: bool = True, bits_w: int | None = None) -> Result:
    """bits: width of the input codes; bits_w: of the filter codes (default: the same; Sec. 4
    evaluates weights and inputs at different widths)."""
    X, W = _f32(X), _f32(W)
    g = geometry(X, W, pad, m)
    bw = bits if bits_w is None else bits_w
    f = filters if filters is not None else prepare_filters(W, m, bw, per_tensor)
    V = input_transform_f32(X, pad, m)
    vr = ranges(V, per_tensor) if static_v_range is None else _f32(static_v_range)
    Vq, cs = quantize(V, vr, bits, g.C)
    del V
    ACC = gemm_i8(f.Uq, Vq) if (want_acc or want_y) else None
    Y = dequant_output_f64(ACC, f.u_range, f.u_rowsum, vr, cs, g, bits, bw) if want_y else None
    return Result(g, f, Vq, vr, cs, ACC, Y)
