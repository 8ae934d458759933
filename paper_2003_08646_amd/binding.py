"""Thin ctypes binding of liblance: argument marshalling only.  Every function has the name and
argument order of its C entry point in ``include/lance.h``; tensors are torch CUDA tensors (used
as device memory) or raw integer device pointers.  Nothing is computed here.

The library must have been built (``python -m paper_2003_08646_amd.build`` or
``__graft_entry__.build()``); loading fails loudly if it is missing -- there is no fallback.
"""
from __future__ import annotations

import ctypes
import os
from ctypes import POINTER, Structure, byref, c_char_p, c_int, c_int32, c_int64, c_size_t, c_uint32, c_void_p

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "liblance.so")

LANCE_OK = 0
LANCE_ERR_INVALID_ARG = -1
LANCE_ERR_UNSUPPORTED = -2
LANCE_ERR_WORKSPACE = -3
LANCE_ERR_HIP = -4

LANCE_RANGE_PER_POSITION = 0
LANCE_RANGE_PER_TENSOR = 1
LANCE_INPUT_RANGE_STATIC = 2
LANCE_PLAN_WIDE_TILES = 4
LANCE_LAYOUT_NHWC = 8
LANCE_CODES_PACKED4 = 16


def LANCE_FILTER_BITS(bw: int) -> int:
    """Flag field for filter codes of another width than the input codes (2..8)."""
    return (int(bw) << 8) & 0xFFFFFFFF   # unmasked: a width outside [2, 8] is rejected, not dropped

EXPORTS = ["lance_query_sizes", "lance_code_offset", "lance_code_shift", "lance_filter_transform_q8",
           "lance_input_transform_q8", "lance_winograd_gemm_i8", "lance_output_transform_dq",
           "lance_conv3x3_winograd_q8", "lance_conv3x3_winograd_q8_noalloc",
           "lance_conv3x3_winograd_q8_profile", "lance_conv3x3_winograd_q8_profile_rotating",
           "lance_profile_kernel_name",
           "lance_direct_conv3x3_f32", "lance_alg1_literal_f32", "lance_conv3x3_winograd_wq_f32", "lance_status_string",
           "lance_last_error_detail", "lance_version"]


class lance_conv_desc(Structure):
    _fields_ = [("N", c_int32), ("C", c_int32), ("H", c_int32), ("W", c_int32), ("K", c_int32),
                ("pad", c_int32), ("m", c_int32), ("bits", c_int32), ("flags", c_uint32)]


class lance_sizes(Structure):
    _fields_ = [(n, c_int32) for n in
                ("Ho", "Wo", "tiles_h", "tiles_w", "P", "E", "Cp", "CB", "NB")] + \
               [(n, c_size_t) for n in
                ("uq_bytes", "u_range_bytes", "u_rowsum_bytes", "vq_bytes", "v_range_bytes",
                 "v_colsum_bytes", "acc_bytes", "y_bytes", "input_workspace_bytes",
                 "conv_workspace_bytes")]


class LanceError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        detail = lib().lance_last_error_detail().decode() if status == LANCE_ERR_HIP else ""
        super().__init__(f"{where}: {status_string(status)} ({status}) {detail}".rstrip())


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: build it with "
                              "`python -m paper_2003_08646_amd.build` (no fallback exists)")
        # torch first: its wheel carries its own HIP runtime (same SONAME as the system one).
        # Loaded in this order, liblance binds to the runtime torch's allocator and streams
        # live in; the other way round the process would hold two runtimes.
        import torch  # noqa: F401
        L = ctypes.CDLL(LIB_PATH)
        D = POINTER(lance_conv_desc)
        L.lance_query_sizes.argtypes = [D, POINTER(lance_sizes)]
        L.lance_code_offset.argtypes = [D, c_int64, c_int32, c_int64, c_int32]
        L.lance_code_offset.restype = c_size_t
        L.lance_code_shift.argtypes = [D, c_int32]
        L.lance_code_shift.restype = c_int
        L.lance_filter_transform_q8.argtypes = [D] + [c_void_p] * 5
        L.lance_input_transform_q8.argtypes = [D] + [c_void_p] * 5 + [c_size_t, c_void_p]
        L.lance_winograd_gemm_i8.argtypes = [D] + [c_void_p] * 4
        L.lance_output_transform_dq.argtypes = [D] + [c_void_p] * 7
        L.lance_conv3x3_winograd_q8.argtypes = [D] + [c_void_p] * 7 + [c_size_t, c_void_p]
        L.lance_conv3x3_winograd_q8_noalloc.argtypes = [D] + [c_void_p] * 7
        L.lance_conv3x3_winograd_q8_profile.argtypes = ([D] + [c_void_p] * 7 +
                                                        [c_size_t, c_void_p, c_int, c_void_p])
        L.lance_conv3x3_winograd_q8_profile_rotating.argtypes = (
            [D, c_void_p, c_void_p, c_int] + [c_void_p] * 5 + [c_size_t, c_void_p, c_int, c_void_p])
        L.lance_profile_kernel_name.argtypes = [c_int]
        L.lance_profile_kernel_name.restype = c_char_p
        L.lance_direct_conv3x3_f32.argtypes = [D] + [c_void_p] * 4
        L.lance_alg1_literal_f32.argtypes = [D] + [c_void_p] * 4
        L.lance_conv3x3_winograd_wq_f32.argtypes = [D] + [c_void_p] * 5
        L.lance_status_string.argtypes = [c_int]
        L.lance_status_string.restype = c_char_p
        L.lance_version.restype = c_int
        L.lance_last_error_detail.restype = c_char_p
        _lib = L
    return _lib


def _ptr(t) -> c_void_p:
    """Device pointer of a torch tensor (or pass-through of an int / None)."""
    if t is None:
        return c_void_p(0)
    if isinstance(t, int):
        return c_void_p(t)
    if not t.is_contiguous():
        raise ValueError("liblance needs contiguous buffers")
    return c_void_p(t.data_ptr())


def _stream(stream) -> c_void_p:
    if stream is None:
        import torch
        return c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return c_void_p(stream)
    return c_void_p(stream.cuda_stream)


def _check(rc: int, where: str) -> None:
    if rc != LANCE_OK:
        raise LanceError(rc, where)


def make_desc(N, C, H, W, K, pad=1, m=2, bits=8, flags=0) -> lance_conv_desc:
    return lance_conv_desc(N, C, H, W, K, pad, m, bits, flags)


def status_string(status: int) -> str:
    return lib().lance_status_string(status).decode()


def lance_version() -> int:
    return int(lib().lance_version())


def lance_query_sizes(desc: lance_conv_desc) -> lance_sizes:
    out = lance_sizes()
    _check(lib().lance_query_sizes(byref(desc), byref(out)), "lance_query_sizes")
    return out


def lance_code_offset(desc, rows: int, e: int, row: int, c: int) -> int:
    return int(lib().lance_code_offset(byref(desc), rows, e, row, c))


def lance_code_shift(desc, c: int) -> int:
    return int(lib().lance_code_shift(byref(desc), c))


def lance_filter_transform_q8(desc, w, uq, u_range, u_rowsum, stream=None) -> None:
    _check(lib().lance_filter_transform_q8(byref(desc), _ptr(w), _ptr(uq), _ptr(u_range),
                                           _ptr(u_rowsum), _stream(stream)),
           "lance_filter_transform_q8")


def lance_input_transform_q8(desc, x, vq, v_range, v_colsum, workspace, workspace_bytes=None,
                             stream=None) -> None:
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    _check(lib().lance_input_transform_q8(byref(desc), _ptr(x), _ptr(vq), _ptr(v_range),
                                          _ptr(v_colsum), _ptr(workspace), nbytes,
                                          _stream(stream)), "lance_input_transform_q8")


def lance_winograd_gemm_i8(desc, uq, vq, acc, stream=None) -> None:
    _check(lib().lance_winograd_gemm_i8(byref(desc), _ptr(uq), _ptr(vq), _ptr(acc),
                                        _stream(stream)), "lance_winograd_gemm_i8")


def lance_output_transform_dq(desc, acc, u_range, u_rowsum, v_range, v_colsum, y,
                              stream=None) -> None:
    _check(lib().lance_output_transform_dq(byref(desc), _ptr(acc), _ptr(u_range), _ptr(u_rowsum),
                                           _ptr(v_range), _ptr(v_colsum), _ptr(y),
                                           _stream(stream)), "lance_output_transform_dq")


def lance_conv3x3_winograd_q8(desc, x, uq, u_range, u_rowsum, v_range, y, workspace,
                              workspace_bytes=None, stream=None) -> None:
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    _check(lib().lance_conv3x3_winograd_q8(byref(desc), _ptr(x), _ptr(uq), _ptr(u_range),
                                           _ptr(u_rowsum), _ptr(v_range), _ptr(y),
                                           _ptr(workspace), nbytes, _stream(stream)),
           "lance_conv3x3_winograd_q8")


LANCE_NOALLOC_SCRATCH_BYTES = 64 << 20


def lance_conv3x3_winograd_q8_noalloc(desc, x, uq, u_range, u_rowsum, v_range, y,
                                      stream=None) -> None:
    _check(lib().lance_conv3x3_winograd_q8_noalloc(byref(desc), _ptr(x), _ptr(uq), _ptr(u_range),
                                                   _ptr(u_rowsum), _ptr(v_range), _ptr(y),
                                                   _stream(stream)),
           "lance_conv3x3_winograd_q8_noalloc")


PROFILE_KERNELS = ("range_pass", "range_reduce", "quantize_pass", "gemm_epilogue")
LANCE_PROFILE_MAX_REPEATS = 4096


def lance_conv3x3_winograd_q8_profile(desc, x, uq, u_range, u_rowsum, v_range, y, workspace,
                                      workspace_bytes=None, stream=None, repeats=1) -> list:
    """Returns the per-kernel durations [ms], averaged over `repeats` passes enqueued back to
    back, in the order of PROFILE_KERNELS."""
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    ms = (ctypes.c_float * len(PROFILE_KERNELS))()
    _check(lib().lance_conv3x3_winograd_q8_profile(
        byref(desc), _ptr(x), _ptr(uq), _ptr(u_range), _ptr(u_rowsum), _ptr(v_range), _ptr(y),
        _ptr(workspace), nbytes, _stream(stream), int(repeats), ctypes.cast(ms, c_void_p)),
        "lance_conv3x3_winograd_q8_profile")
    return [float(v) for v in ms]


def lance_conv3x3_winograd_q8_profile_rotating(desc, xs, ys, uq, u_range, u_rowsum, v_range,
                                               workspace, workspace_bytes=None, stream=None,
                                               repeats=1) -> list:
    """The timing twin over the buffer pairs (xs[i], ys[i]), pass r on pair r % len(xs)."""
    if len(xs) != len(ys) or not xs:
        raise ValueError("need as many outputs as inputs, at least one")
    nbytes = workspace_bytes if workspace_bytes is not None else (
        0 if workspace is None else workspace.numel() * workspace.element_size())
    xp = (c_void_p * len(xs))(*[_ptr(t).value for t in xs])
    yp = (c_void_p * len(ys))(*[_ptr(t).value for t in ys])
    ms = (ctypes.c_float * len(PROFILE_KERNELS))()
    _check(lib().lance_conv3x3_winograd_q8_profile_rotating(
        byref(desc), ctypes.cast(xp, c_void_p), ctypes.cast(yp, c_void_p), len(xs), _ptr(uq),
        _ptr(u_range), _ptr(u_rowsum), _ptr(v_range), _ptr(workspace), nbytes, _stream(stream),
        int(repeats), ctypes.cast(ms, c_void_p)), "lance_conv3x3_winograd_q8_profile_rotating")
    return [float(v) for v in ms]


def lance_profile_kernel_name(slot: int) -> str:
    return lib().lance_profile_kernel_name(int(slot)).decode()


def lance_alg1_literal_f32(desc, x, w, y, stream=None) -> None:
    _check(lib().lance_alg1_literal_f32(byref(desc), _ptr(x), _ptr(w), _ptr(y),
                                        _stream(stream)), "lance_alg1_literal_f32")


def lance_conv3x3_winograd_wq_f32(desc, x, uq, u_range, y, stream=None) -> None:
    _check(lib().lance_conv3x3_winograd_wq_f32(byref(desc), _ptr(x), _ptr(uq), _ptr(u_range),
                                               _ptr(y), _stream(stream)),
           "lance_conv3x3_winograd_wq_f32")


def lance_direct_conv3x3_f32(desc, x, w, y, stream=None) -> None:
    _check(lib().lance_direct_conv3x3_f32(byref(desc), _ptr(x), _ptr(w), _ptr(y),
                                          _stream(stream)), "lance_direct_conv3x3_f32")
