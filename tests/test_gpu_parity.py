"""GPU parity: the HIP path (through the C ABI) against the CPU oracle, element by element.

Bar: codes, code sums and int32 accumulators bit-exact; ranges equal as numbers; fp32 outputs
within 1e-4 * (max Y - min Y) of the oracle's fp64 result (max-abs).  The relative L2 error
against the fp64 direct convolution is printed for information.
"""
import sys

import numpy as np
import pytest

from oracle import lance_oracle as O
from paper_2003_08646_amd import workloads as Wk

pytestmark = pytest.mark.gpu

torch = pytest.importorskip("torch")


def _say(*a):
    print(*a, flush=True)
    sys.stdout.flush()


def _gpu_layer(L, flags=0):
    from paper_2003_08646_amd.layer import LanceConv
    return LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits, flags, bits_w=L.bits_w)


def _assert_codes(logical, ref_codes, what):
    """The library's codes [E][rows][Cp] against the oracle's [E][rows][C]: the real channels
    bit for bit, and every padding channel holds code 0."""
    C = ref_codes.shape[2]
    np.testing.assert_array_equal(logical[:, :, :C], ref_codes, err_msg=what)
    assert not logical[:, :, C:].any(), f"{what}: padding channels must hold code 0"


def _check_layer(L, X=None, Wt=None, flags=0, static_v_range=None, check_direct=False,
                 staged=True):
    """Runs stage by stage and fused on the GPU, compares everything with the oracle."""
    from paper_2003_08646_amd import binding as B
    if X is None:
        X, Wt = Wk.make_inputs(L)
    per_tensor = bool(flags & B.LANCE_RANGE_PER_TENSOR)
    # NHWC calls get the transposed tensors and must give the transposed result: the oracle
    # works on NCHW throughout, the codes are the same
    nhwc = bool(flags & B.LANCE_LAYOUT_NHWC)
    to_nchw = (lambda a: a.transpose(0, 3, 1, 2)) if nhwc else (lambda a: a)
    _say(f"[case] {L.name} N{L.N} C{L.C} K{L.K} {L.H}x{L.W} pad{L.pad} m{L.m} b{L.bits} "
         f"bw{L.bits_w} flags{flags}")
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits, per_tensor=per_tensor,
                       static_v_range=static_v_range, bits_w=L.bits_w)
    conv = _gpu_layer(L, flags)
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1)) if nhwc else X).cuda()
    w = torch.from_numpy(Wt).cuda()
    _say("  gpu: filter transform")
    conv.prepare_filters(w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(conv.u_range.cpu().numpy(), ref.filters.u_range)
    _assert_codes(conv.codes_to_logical(conv.uq, L.K), ref.filters.Uq, "filter codes")
    np.testing.assert_array_equal(conv.u_rowsum.cpu().numpy(), ref.filters.u_rowsum)
    if static_v_range is not None:
        conv.v_range.copy_(torch.from_numpy(np.ascontiguousarray(static_v_range, np.float32)))
    tol = 1e-4 * float(ref.Y.max() - ref.Y.min())
    if staged:
        _say("  gpu: staged path")
        st = conv.forward_staged(x)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(conv.v_range.cpu().numpy(), ref.v_range)
        _assert_codes(conv.codes_to_logical(st["vq"], conv.sz.P), ref.Vq, "input codes")
        np.testing.assert_array_equal(st["v_colsum"].cpu().numpy(), ref.v_colsum)
        np.testing.assert_array_equal(st["acc"].cpu().numpy(), ref.ACC)
        ys = to_nchw(st["y"].cpu().numpy().astype(np.float64))
        err = float(np.abs(ys - ref.Y).max())
        assert err <= tol, ("staged Y", err, tol)
        del st
        conv._staged = None
    _say("  gpu: fused path")
    if static_v_range is None:
        conv.v_range.fill_(float("nan"))
    conv.y.fill_(float("nan"))
    yf = conv.forward(x)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(conv.v_range.cpu().numpy(), ref.v_range)
    yf = to_nchw(yf.cpu().numpy().astype(np.float64))
    err = float(np.abs(yf - ref.Y).max())
    assert err <= tol, ("fused Y", err, tol)
    msg = f"  ok: max|Y-oracle| = {err:.3g} (tol {tol:.3g})"
    if check_direct:
        Yd = O.direct_conv_f64(X, Wt, L.pad)
        rel = float(np.linalg.norm(yf - Yd) / np.linalg.norm(Yd))
        msg += f", rel-L2 vs fp64 direct convolution = {rel:.4g}"
    _say(msg)
    return conv, ref


SMALL = [
    Wk.Layer("tiny_one_tile", 1, 1, 1, 4, 4, pad=0, m=2, seed=11),
    Wk.Layer("ragged_m2_pad1", 2, 3, 5, 7, 9, pad=1, m=2, seed=12),
    Wk.Layer("ragged_m2_pad0", 2, 5, 3, 9, 6, pad=0, m=2, seed=13),
    Wk.Layer("ragged_m4_pad1", 2, 3, 5, 7, 9, pad=1, m=4, seed=14),
    Wk.Layer("ragged_m4_pad0", 1, 6, 4, 11, 13, pad=0, m=4, seed=15),
    Wk.Layer("pad2_m2", 1, 4, 4, 5, 5, pad=2, m=2, seed=16),
    Wk.Layer("c17_k33_m2", 3, 17, 33, 12, 10, pad=1, m=2, seed=17),
    Wk.Layer("c48_k40_m2", 2, 48, 40, 14, 14, pad=1, m=2, seed=18),
    Wk.Layer("c48_k40_m4", 2, 48, 40, 14, 14, pad=1, m=4, seed=19),
    Wk.Layer("c130_k70_m2", 2, 130, 70, 10, 18, pad=1, m=2, seed=20),
    Wk.Layer("c130_k70_m4", 2, 130, 70, 10, 18, pad=1, m=4, seed=21),
    Wk.Layer("wide_m2", 1, 8, 8, 6, 150, pad=1, m=2, seed=22),
    Wk.Layer("tall_m4", 1, 8, 8, 150, 6, pad=1, m=4, seed=23),
    Wk.Layer("many_tiles_m2", 5, 64, 64, 20, 20, pad=1, m=2, seed=24),
    Wk.Layer("normal_input_m2", 2, 16, 16, 16, 16, pad=1, m=2, seed=25, x_dist="normal"),
]


@pytest.mark.parametrize("L", SMALL, ids=[l.name for l in SMALL])
def test_small_and_ragged_layers(L):
    _check_layer(L, check_direct=True)


@pytest.mark.parametrize("bits", [2, 3, 4, 5, 6, 7, 8])
@pytest.mark.parametrize("m", [2, 4])
def test_bit_widths(bits, m):
    _check_layer(Wk.Layer(f"bits{bits}_m{m}", 2, 24, 20, 12, 12, pad=1, m=m, bits=bits, seed=30 + bits))


@pytest.mark.parametrize("m", [2, 4])
def test_per_tensor_ranges(m):
    from paper_2003_08646_amd import binding as B
    _check_layer(Wk.Layer(f"per_tensor_m{m}", 2, 20, 12, 10, 10, m=m, seed=40), flags=B.LANCE_RANGE_PER_TENSOR)


@pytest.mark.parametrize("C", [20, 130])
def test_static_input_ranges_clamp(C):
    """Caller-supplied ranges narrower than the data: out-of-range values clamp to end codes."""
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer(f"static_c{C}", 2, C, 12, 10, 10, m=2, seed=41)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)


@pytest.mark.parametrize("bits", [8, 4])
@pytest.mark.parametrize("m", [2, 4])
def test_rounding_ties_and_both_clamps(bits, m):
    """Integer-valued inputs and a static range [0, 2*L] make inv = 0.5 exactly: every odd
    transformed value lands on an exact .5 tie (round-half-to-even decides the code), negative
    values clamp to code 0 and values above 2*L clamp to code L."""
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer(f"ties_b{bits}_m{m}", 2, 20, 8, 12, 12, m=m, bits=bits, seed=43)
    _, Wt = Wk.make_inputs(L)
    levels = 2 ** bits - 1
    rng = np.random.default_rng(44)
    X = rng.integers(0, levels + 1, size=(L.N, L.C, L.H, L.W)).astype(np.float32)
    E = (m + 2) ** 2
    static = np.tile(np.array([0.0, 2.0 * levels], np.float32), (E, 1))
    V = O.input_transform_f32(X, L.pad, L.m)
    half = V * 0.5
    assert (np.abs(half - np.floor(half) - 0.5) < 1e-6).sum() > 100   # ties do occur
    assert (V < 0).any() and (V > 2 * levels).any()                  # both clamps are live
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=static)


# Layers whose plan quantizes inside the product kernel (m = 2, 17 <= C <= 64): the fused Y is the
# only output of that kernel, so every feature of the path gets a case of its own here.
ONE_KERNEL = [
    Wk.Layer("c64_pad0_odd", 3, 64, 40, 9, 11, pad=0, m=2, seed=60),
    Wk.Layer("c50_pad1", 2, 50, 64, 13, 10, pad=1, m=2, seed=61),
    Wk.Layer("c64_pad2", 1, 64, 16, 6, 6, pad=2, m=2, seed=62),
    Wk.Layer("c60_k70_bits5", 2, 60, 70, 12, 12, pad=1, m=2, bits=5, seed=63),
    Wk.Layer("c64_tiny_images", 40, 64, 8, 4, 4, pad=1, m=2, seed=64),
    Wk.Layer("c64_k130", 2, 64, 130, 16, 16, pad=1, m=2, seed=65),
    Wk.Layer("c49_one_tile", 1, 49, 3, 2, 2, pad=1, m=2, seed=66),
    Wk.Layer("c64_bits2", 2, 64, 33, 10, 14, pad=1, m=2, bits=2, seed=67),
    Wk.Layer("c63_wide", 1, 63, 32, 4, 300, pad=1, m=2, seed=68),
]


@pytest.mark.parametrize("L", ONE_KERNEL, ids=[l.name for l in ONE_KERNEL])
def test_one_kernel_plan_layers(L):
    _check_layer(L, check_direct=True)


def test_one_kernel_plan_static_and_per_tensor_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("c64_static", 2, 64, 24, 10, 10, m=2, seed=69)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)
    _check_layer(L.with_(name="c64_per_tensor"), X, Wt, flags=B.LANCE_RANGE_PER_TENSOR)


@pytest.mark.parametrize("bits", [8, 4])
def test_one_kernel_plan_rounding_ties(bits):
    """The tie/clamp construction of test_rounding_ties_and_both_clamps at C = 64."""
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer(f"ties64_b{bits}", 2, 64, 8, 12, 12, m=2, bits=bits, seed=70)
    _, Wt = Wk.make_inputs(L)
    levels = 2 ** bits - 1
    X = np.random.default_rng(71).integers(0, levels + 1, size=(L.N, L.C, L.H, L.W)).astype(np.float32)
    static = np.tile(np.array([0.0, 2.0 * levels], np.float32), (16, 1))
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=static)


# Layers of the general plan with 64-channel code blocks: patch-loader quantize pass (both tile
# sizes, every load mode) and the fused GEMMs of layers with C > 64 (partial filter tiles, odd
# and even numbers of channel blocks, tile counts that are not multiples of the block sizes).
# F(2x2,3x3) layers of this size multiply with one wave per row of the position grid; the
# second test sends them through the 128 x 64 workgroup tiles that only large layers get by
# default.
TILED = [
    Wk.Layer("c128_k200_m2", 2, 128, 200, 12, 12, pad=1, m=2, seed=80),
    Wk.Layer("c256_k130_m2_pad0", 1, 256, 130, 11, 13, pad=0, m=2, seed=81),
    Wk.Layer("c192_k64_m2_pad2", 1, 192, 64, 6, 6, pad=2, m=2, seed=82),
    Wk.Layer("c100_k16_m2_odd", 3, 100, 16, 9, 7, pad=1, m=2, seed=83),
    Wk.Layer("c128_k130_m4", 2, 128, 130, 16, 16, pad=1, m=4, seed=84),
    Wk.Layer("c64_k64_m4", 3, 64, 64, 12, 12, pad=1, m=4, seed=85),
    Wk.Layer("c200_k40_m4_pad0_odd", 1, 200, 40, 13, 11, pad=0, m=4, seed=86),
    Wk.Layer("c128_k64_m4_bits6", 2, 128, 64, 8, 8, pad=1, m=4, bits=6, seed=87),
    Wk.Layer("c70_k33_m4_tiny_images", 20, 70, 33, 4, 4, pad=1, m=4, seed=88),
    Wk.Layer("c128_k64_m2_bits3", 2, 128, 64, 8, 8, pad=1, m=2, bits=3, seed=89),
    Wk.Layer("c384_k20_m4_six_blocks", 1, 384, 20, 8, 8, pad=1, m=4, seed=92),
    Wk.Layer("c768_k16_m4_twelve_blocks", 1, 768, 16, 8, 8, pad=1, m=4, seed=93),
    Wk.Layer("c300_k70_m4_five_blocks", 2, 300, 70, 12, 10, pad=1, m=4, seed=94),
    Wk.Layer("c448_k33_m4_seven_blocks", 1, 448, 33, 9, 13, pad=0, m=4, seed=95),
    Wk.Layer("c576_k40_m4_nine_blocks", 1, 576, 40, 8, 12, pad=1, m=4, seed=96),
]


@pytest.mark.parametrize("L", TILED, ids=[l.name for l in TILED])
def test_tiled_plan_layers(L):
    _check_layer(L, check_direct=True)


WIDE = [l for l in TILED if l.m == 2] + [
    Wk.Layer("c320_k129_m2_wide", 2, 320, 129, 10, 14, pad=1, m=2, seed=90),
    Wk.Layer("c384_k40_m2_wide", 1, 384, 40, 8, 8, pad=1, m=2, seed=91),
]


@pytest.mark.parametrize("L", WIDE, ids=[l.name for l in WIDE])
def test_wide_tile_plan_layers(L):
    from paper_2003_08646_amd import binding as B
    _check_layer(L, flags=B.LANCE_PLAN_WIDE_TILES)


# Filter codes of another width than the input codes (the weight / input width grid of Sec. 4):
# one layer per plan of the fused call, staged path included.
MIXED = [
    Wk.Layer("mixed_two_kernels_w4_x8", 2, 64, 40, 12, 12, m=2, bits=8, bits_w=4, seed=140),
    Wk.Layer("mixed_two_blocks_w8_x4", 2, 128, 40, 12, 12, m=2, bits=4, bits_w=8, seed=141),
    Wk.Layer("mixed_small_channels_w6_x3", 2, 3, 40, 12, 12, m=2, bits=3, bits_w=6, seed=142),
    Wk.Layer("mixed_general_m2_w5_x8", 2, 200, 40, 12, 12, m=2, bits=8, bits_w=5, seed=143),
    Wk.Layer("mixed_general_m4_w8_x6", 2, 130, 40, 12, 12, m=4, bits=6, bits_w=8, seed=144),
    Wk.Layer("mixed_fallback_m2_w2_x8", 2, 20, 12, 10, 10, m=2, bits=8, bits_w=2, seed=145),
    Wk.Layer("mixed_fallback_m4_w7_x5", 2, 10, 12, 10, 10, m=4, bits=5, bits_w=7, seed=146),
]


@pytest.mark.parametrize("L", MIXED, ids=[l.name for l in MIXED])
def test_filter_and_input_codes_of_different_widths(L):
    _check_layer(L, check_direct=True)


def test_mixed_widths_with_wide_tiles_and_static_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("mixed_wide_w4_x7", 2, 128, 40, 12, 12, m=2, bits=7, bits_w=4, seed=147)
    _check_layer(L, flags=B.LANCE_PLAN_WIDE_TILES)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)


# F(2x2,3x3) layers with two 64-channel blocks: the one-kernel plan that keeps 128 KB of codes in
# LDS (several filter blocks, partial blocks, every padding and load mode, narrow codes, one
# range for all positions, caller-supplied ranges).
TWO_BLOCKS = [
    Wk.Layer("c96_k40_m2_pad0", 2, 96, 40, 11, 13, pad=0, m=2, seed=130),
    Wk.Layer("c128_k24_m2_pad2", 1, 128, 24, 6, 6, pad=2, m=2, seed=131),
    Wk.Layer("c65_k300_m2", 1, 65, 300, 12, 12, pad=1, m=2, seed=132),
    Wk.Layer("c128_k130_m2_bits5", 3, 128, 130, 10, 10, pad=1, m=2, bits=5, seed=133),
    Wk.Layer("c120_k64_m2_many_images", 30, 120, 64, 4, 4, pad=1, m=2, seed=134),
]


@pytest.mark.parametrize("L", TWO_BLOCKS, ids=[l.name for l in TWO_BLOCKS])
def test_two_block_one_kernel_plan_layers(L):
    _check_layer(L, check_direct=True)


def test_two_block_one_kernel_plan_static_and_per_tensor_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("c100_k20_ranges", 2, 100, 20, 10, 10, m=2, seed=135)
    _check_layer(L, flags=B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)


# F(4x4,3x3) layers with one or two 64-channel blocks: the plan whose last kernel quantizes into
# LDS, multiplies and transforms back (16-tile workgroups; several filter blocks, partial channel
# blocks, every padding and load mode, tiles that span many images, narrow and mixed codes).
FUSED_M4 = [
    Wk.Layer("m4f_c64_k64", 2, 64, 64, 16, 16, pad=1, m=4, seed=140),
    Wk.Layer("m4f_c17_k5_pad0_odd", 2, 17, 5, 11, 13, pad=0, m=4, seed=141),
    Wk.Layer("m4f_c128_k130", 1, 128, 130, 12, 12, pad=1, m=4, seed=142),
    Wk.Layer("m4f_c65_k70_pad2", 2, 65, 70, 9, 10, pad=2, m=4, seed=143),
    Wk.Layer("m4f_c100_k40_bits5", 3, 100, 40, 10, 10, pad=1, m=4, bits=5, seed=144),
    Wk.Layer("m4f_c128_k24_many_images", 37, 128, 24, 4, 4, pad=1, m=4, seed=145),
    Wk.Layer("m4f_c48_k200_wide", 1, 48, 200, 6, 150, pad=1, m=4, seed=146),
    Wk.Layer("m4f_c64_k8_bits2_w4", 2, 64, 8, 12, 12, pad=1, m=4, bits=2, bits_w=4, seed=147),
    Wk.Layer("m4f_c127_k33_odd_width", 2, 127, 33, 13, 15, pad=1, m=4, seed=148),
]


@pytest.mark.parametrize("L", FUSED_M4, ids=[l.name for l in FUSED_M4])
def test_fused_m4_plan_layers(L):
    _check_layer(L, check_direct=True)


def test_fused_m4_plan_static_and_per_tensor_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("m4f_c100_k20_ranges", 2, 100, 20, 10, 10, m=4, seed=149)
    _check_layer(L, flags=B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)


def test_fused_m4_plan_with_reduction_kernel():
    """Enough workgroups and range records that the reduction kernel runs between the passes."""
    _check_layer(Wk.Layer("m4f_c64_k16_many_records", 32, 64, 16, 64, 64, pad=1, m=4, seed=139),
                 staged=False)


# Layers with 64-channel code blocks whose quantize pass reduces the range pass's records itself
# (no reduction kernel between the passes): one range for all positions, caller-supplied ranges
# with F(4x4,3x3), and a record count that takes more than one batch of loads per thread.
@pytest.mark.parametrize("m", [2, 4])
def test_general_plan_per_tensor_ranges(m):
    from paper_2003_08646_amd import binding as B
    _check_layer(Wk.Layer(f"per_tensor_c130_m{m}", 2, 130, 12, 10, 10, m=m, seed=110),
                 flags=B.LANCE_RANGE_PER_TENSOR)


def test_general_plan_static_ranges_m4():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("static_c130_m4", 2, 130, 12, 10, 10, m=4, seed=111)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)


def test_general_plan_many_range_records_m4():
    _check_layer(Wk.Layer("c128_k16_m4_240_records", 10, 128, 16, 64, 64, pad=1, m=4, seed=112))


# Layers with at most 16 channels (F(2x2,3x3)): the one-kernel plan whose waves keep the codes in
# registers.  Several filter tiles, filter counts that are not multiples of 32, tile counts that
# are not multiples of 64 and span images, every load mode, narrow codes, all channel counts
# that change the packing (1..16).
NARROW = [
    Wk.Layer("c3_k64_40x40", 2, 3, 64, 40, 40, pad=1, m=2, seed=100),
    Wk.Layer("c3_k70_pad0_odd", 3, 3, 70, 13, 11, pad=0, m=2, seed=101),
    Wk.Layer("c16_k33_tiny_images", 37, 16, 33, 4, 4, pad=1, m=2, seed=102),
    Wk.Layer("c7_k5_pad2", 2, 7, 5, 9, 10, pad=2, m=2, seed=103),
    Wk.Layer("c12_k96_bits5", 1, 12, 96, 18, 22, pad=1, m=2, bits=5, seed=104),
    Wk.Layer("c1_k40_wide", 1, 1, 40, 6, 300, pad=1, m=2, seed=105),
    Wk.Layer("c9_k8_bits2", 2, 9, 8, 12, 12, pad=1, m=2, bits=2, seed=106),
]


@pytest.mark.parametrize("L", NARROW, ids=[l.name for l in NARROW])
def test_narrow_layers_one_kernel_plan(L):
    _check_layer(L, check_direct=True)


@pytest.mark.parametrize("C", [2, 4, 5, 8, 11, 13, 15])
def test_narrow_layers_every_packing(C):
    _check_layer(Wk.Layer(f"c{C}_k20_packing", 2, C, 20, 10, 14, pad=1, m=2, seed=110 + C))


def test_narrow_layers_static_and_per_tensor_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("c3_static", 2, 3, 24, 16, 16, pad=1, m=2, seed=120)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow)
    _check_layer(L.with_(name="c3_per_tensor"), X, Wt, flags=B.LANCE_RANGE_PER_TENSOR)


def _random_layers(count, seed):
    """Seeded random small layers: every plan of the fused call, both tile sizes, odd shapes."""
    rng = np.random.default_rng(seed)
    out = []
    for i in range(count):
        m = int(rng.choice([2, 2, 4]))
        C = int(rng.choice([rng.integers(1, 17), rng.integers(17, 65), rng.integers(65, 129),
                            rng.integers(129, 400)]))
        K = int(rng.integers(1, 150))
        pad = int(rng.choice([0, 1, 1, 1, 2]))
        H, W = int(rng.integers(3, 21)), int(rng.integers(3, 21))
        if H + 2 * pad < 3 or W + 2 * pad < 3:
            continue
        N = int(rng.integers(1, 5))
        bits = int(rng.choice([8, 8, 8, 7, 5, 4, 2]))
        bits_w = int(rng.choice([0, 0, 8, 6, 3]))
        out.append(Wk.Layer(f"rand{i}_m{m}_c{C}_k{K}_{H}x{W}_p{pad}_b{bits}_w{bits_w}", N, C, K, H, W,
                            pad=pad, m=m, bits=bits, seed=1000 + i,
                            bits_w=bits_w if bits_w else None))
    return out


RANDOM = _random_layers(48, 2024)


@pytest.mark.parametrize("L", RANDOM, ids=[l.name for l in RANDOM])
def test_random_small_layers(L):
    from paper_2003_08646_amd import binding as B
    flags = [0, B.LANCE_RANGE_PER_TENSOR, B.LANCE_PLAN_WIDE_TILES][L.seed % 3]
    _check_layer(L, flags=flags)


RANDOM_NHWC = _random_layers(40, 2025)


@pytest.mark.parametrize("L", RANDOM_NHWC, ids=[l.name for l in RANDOM_NHWC])
def test_random_small_layers_nhwc(L):
    """The same net of random shapes over the NHWC plans (channel counts that are and are not
    multiples of 4, every block count, both tile sizes)."""
    from paper_2003_08646_amd import binding as B
    flags = [0, B.LANCE_RANGE_PER_TENSOR, B.LANCE_PLAN_WIDE_TILES][L.seed % 3]
    _check_layer(L, flags=flags | B.LANCE_LAYOUT_NHWC)


NHWC = [
    Wk.Layer("nhwc_tiny_one_tile", 1, 1, 1, 4, 4, pad=0, m=2, seed=311),
    Wk.Layer("nhwc_ragged_m2_pad1", 2, 3, 5, 7, 9, pad=1, m=2, seed=312),
    Wk.Layer("nhwc_ragged_m4_pad0", 1, 6, 4, 11, 13, pad=0, m=4, seed=313),
    Wk.Layer("nhwc_pad2_m4", 1, 4, 4, 5, 5, pad=2, m=4, seed=314),
    Wk.Layer("nhwc_c17_k33_m2", 3, 17, 33, 12, 10, pad=1, m=2, seed=315),
    Wk.Layer("nhwc_c48_k40_m4", 2, 48, 40, 14, 14, pad=1, m=4, seed=316),
    Wk.Layer("nhwc_c64_k64_m2", 3, 64, 64, 20, 20, pad=1, m=2, seed=317),
    Wk.Layer("nhwc_c130_k70_m2", 2, 130, 70, 10, 18, pad=1, m=2, seed=318),
    Wk.Layer("nhwc_c130_k70_m4", 2, 130, 70, 10, 18, pad=1, m=4, seed=319),
    Wk.Layer("nhwc_c256_k96_m2", 2, 256, 96, 14, 14, pad=1, m=2, seed=320),
    Wk.Layer("nhwc_c128_k128_m4", 4, 128, 128, 28, 28, pad=1, m=4, seed=321),
    Wk.Layer("nhwc_c128_k256_m2", 8, 128, 256, 28, 28, pad=1, m=2, seed=322),
    Wk.Layer("nhwc_c64_k50_odd_m2", 2, 64, 50, 13, 11, pad=0, m=2, seed=325),
    Wk.Layer("nhwc_c512_k64_m2", 2, 512, 64, 14, 14, pad=1, m=2, seed=326),
    Wk.Layer("nhwc_c192_k66_m4", 3, 192, 66, 15, 13, pad=1, m=4, seed=327),
    Wk.Layer("nhwc_c512_k128_m4", 2, 512, 128, 14, 14, pad=1, m=4, seed=328),
    Wk.Layer("nhwc_c192_k256_m2", 16, 192, 256, 28, 28, pad=1, m=2, seed=329),
    Wk.Layer("nhwc_c52_k64_m2", 3, 52, 64, 18, 14, pad=1, m=2, seed=332),
    Wk.Layer("nhwc_c50_k64_m2", 3, 50, 64, 18, 14, pad=1, m=2, seed=333),
    Wk.Layer("nhwc_c64_k130_b5_m2", 2, 64, 130, 17, 9, pad=1, m=2, bits=5, seed=334),
    Wk.Layer("nhwc_c60_k64_many_tiles", 6, 60, 64, 32, 32, pad=1, m=2, seed=335),
    Wk.Layer("nhwc_c3_k64_m2", 2, 3, 64, 30, 26, pad=1, m=2, seed=337),
    Wk.Layer("nhwc_c2_k24_m2", 2, 2, 24, 17, 21, pad=1, m=2, seed=348),
    Wk.Layer("nhwc_c4_k24_pad0_m2", 3, 4, 24, 16, 18, pad=0, m=2, seed=349),
    Wk.Layer("nhwc_c1_k40_b6_m2", 2, 1, 40, 19, 9, pad=2, m=2, bits=6, seed=350),
    Wk.Layer("nhwc_c5_k24_m2", 2, 5, 24, 17, 21, pad=1, m=2, seed=351),
    Wk.Layer("nhwc_c9_k70_pad0_m2", 3, 9, 70, 15, 17, pad=0, m=2, seed=338),
    Wk.Layer("nhwc_c16_k33_pad2_b5_m2", 2, 16, 33, 9, 12, pad=2, m=2, bits=5, seed=339),
    Wk.Layer("nhwc_c3_k32_m4", 2, 3, 32, 22, 18, pad=1, m=4, seed=340),
    Wk.Layer("nhwc_c13_k20_many_tiles", 5, 13, 20, 40, 36, pad=1, m=2, seed=341),
    Wk.Layer("nhwc_c100_k64_m2", 3, 100, 64, 18, 14, pad=1, m=2, seed=343),
    Wk.Layer("nhwc_c72_k70_odd_b6_m2", 2, 72, 70, 13, 11, pad=0, m=2, bits=6, seed=344),
    Wk.Layer("nhwc_c128_k200_many_tiles", 5, 128, 200, 24, 24, pad=1, m=2, seed=345),
    Wk.Layer("nhwc_b4_bw6_m2", 2, 40, 24, 12, 12, pad=1, m=2, bits=4, bits_w=6, seed=323),
    Wk.Layer("nhwc_b5_m4", 2, 70, 24, 12, 12, pad=1, m=4, bits=5, seed=324),
]


@pytest.mark.parametrize("L", NHWC, ids=[l.name for l in NHWC])
def test_nhwc_layers(L):
    """X [N][H][W][C] in, Y [N][Ho][Wo][K] out (the layout of Sec. 3.3): same codes, same Y."""
    from paper_2003_08646_amd import binding as B
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC, check_direct=True)


def test_nhwc_static_and_per_tensor_ranges():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("nhwc_ranges", 2, 70, 33, 12, 10, pad=1, m=2, seed=330)
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits)
    narrow = np.stack([ref.v_range[:, 0] * 0.5, ref.v_range[:, 1] * 0.5], axis=1).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_INPUT_RANGE_STATIC,
                 static_v_range=narrow)
    # the two-block one-kernel plan
    L = Wk.Layer("nhwc_ranges_c96", 2, 96, 40, 12, 10, pad=1, m=2, seed=346)
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits)
    narrow = np.stack([ref.v_range[:, 0] * 0.5, ref.v_range[:, 1] * 0.5], axis=1).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_INPUT_RANGE_STATIC,
                 static_v_range=narrow)
    # two blocks with the wide-tile flag: the general plan instead of the one-kernel plan
    L = Wk.Layer("nhwc_wide_c128", 4, 128, 130, 16, 16, pad=1, m=2, seed=347)
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_PLAN_WIDE_TILES)
    # the small-channel one-kernel plan
    L = Wk.Layer("nhwc_ranges_c5", 2, 5, 24, 14, 12, pad=1, m=2, seed=342)
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits)
    narrow = np.stack([ref.v_range[:, 0] * 0.5, ref.v_range[:, 1] * 0.5], axis=1).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_INPUT_RANGE_STATIC,
                 static_v_range=narrow)
    # the same on a one-block layer (range reduction inside the fused kernel)
    L = Wk.Layer("nhwc_ranges_c64", 2, 64, 40, 12, 10, pad=1, m=2, seed=336)
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits)
    narrow = np.stack([ref.v_range[:, 0] * 0.5, ref.v_range[:, 1] * 0.5], axis=1).astype(np.float32)
    _check_layer(L, X, Wt, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_INPUT_RANGE_STATIC,
                 static_v_range=narrow)


def test_nhwc_direct_conv_comparator():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("nhwc_direct", 2, 19, 40, 9, 11, pad=1, seed=331)
    X, Wt = Wk.make_inputs(L)
    Yd = O.direct_conv_f64(X, Wt, L.pad)
    d = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.pad, 2, 8, B.LANCE_LAYOUT_NHWC)
    y = torch.empty((L.N, Yd.shape[2], Yd.shape[3], L.K), dtype=torch.float32, device="cuda")
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1))).cuda()
    B.lance_direct_conv3x3_f32(d, x, torch.from_numpy(Wt).cuda(), y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64).transpose(0, 3, 1, 2)
    assert np.abs(got - Yd).max() <= 1e-5 * np.abs(Yd).max()


LITERAL = [
    Wk.Layer("literal_m2", 2, 5, 7, 9, 11, pad=1, m=2, seed=401),
    Wk.Layer("literal_m4", 2, 6, 5, 11, 13, pad=1, m=4, seed=402),
    Wk.Layer("literal_m2_b4_pad0", 1, 20, 9, 12, 10, pad=0, m=2, bits=4, seed=403),
    Wk.Layer("literal_m4_b5_pad2", 1, 3, 6, 7, 6, pad=2, m=4, bits=5, seed=404),
    Wk.Layer("literal_one_channel", 3, 1, 2, 6, 6, pad=1, m=2, seed=405),
    Wk.Layer("literal_many_tiles", 3, 12, 10, 40, 36, pad=1, m=2, seed=406),
    Wk.Layer("literal_mixed_w4_x8_m2", 2, 6, 5, 10, 12, pad=1, m=2, bits=8, bits_w=4, seed=407),
    Wk.Layer("literal_mixed_w7_x3_m4", 1, 4, 6, 11, 9, pad=1, m=4, bits=3, bits_w=7, seed=408),
]


@pytest.mark.parametrize("nhwc", [False, True], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("L", LITERAL, ids=[l.name for l in LITERAL])
def test_alg1_literal_ablation(L, nhwc):
    """Algorithm 1 loop by loop with the range of every single matrix (Eq. 7's T = the matrix
    itself): the GPU's binary32 result against the oracle's binary64 one.  The codes on both
    sides come from the same binary32 operations, so the difference is rounding of the
    de-quantized products and their sum only."""
    from paper_2003_08646_amd import binding as B
    _say(f"[case] {L.name} nhwc={nhwc}")
    X, Wt = Wk.make_inputs(L)
    ref = O.alg1_literal_f64(X, Wt, L.pad, L.m, L.bits, bits_w=L.bits_w)
    d = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits,
                    (B.LANCE_LAYOUT_NHWC if nhwc else 0) |
                    (B.LANCE_FILTER_BITS(L.bits_w) if L.bits_w else 0))
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1)) if nhwc else X).cuda()
    Ho, Wo = ref.shape[2], ref.shape[3]
    y = torch.full((L.N, Ho, Wo, L.K) if nhwc else (L.N, L.K, Ho, Wo), float("nan"),
                   dtype=torch.float32, device="cuda")
    B.lance_alg1_literal_f32(d, x, torch.from_numpy(Wt).cuda(), y)
    torch.cuda.synchronize()
    got = y.cpu().numpy().astype(np.float64)
    if nhwc:
        got = got.transpose(0, 3, 1, 2)
    tol = 1e-4 * float(ref.max() - ref.min())
    err = float(np.abs(got - ref).max())
    assert err <= tol, (err, tol)
    Yd = O.direct_conv_f64(X, Wt, L.pad)
    _say(f"  ok: max|Y-oracle| = {err:.3g} (tol {tol:.3g}), rel-L2 vs fp64 direct convolution = "
         f"{np.linalg.norm(got - Yd) / np.linalg.norm(Yd):.4g}")


WEIGHT_ONLY = [
    Wk.Layer("wo_m2_w4", 2, 5, 7, 9, 11, pad=1, m=2, bits_w=4, seed=421),
    Wk.Layer("wo_m4_w4", 2, 6, 5, 11, 13, pad=1, m=4, bits_w=4, seed=422),
    Wk.Layer("wo_m2_w8_c70_pad0", 1, 70, 19, 12, 10, pad=0, m=2, bits_w=8, seed=423),
    Wk.Layer("wo_m4_w2_pad2", 1, 3, 6, 7, 6, pad=2, m=4, bits_w=2, seed=424),
    Wk.Layer("wo_m2_w4_c130_many_tiles", 3, 130, 10, 40, 36, pad=1, m=2, bits_w=4, seed=425),
    Wk.Layer("wo_m4_w6_c64", 2, 64, 9, 16, 16, pad=1, m=4, bits_w=6, seed=426),
]


@pytest.mark.parametrize("nhwc", [False, True], ids=["nchw", "nhwc"])
@pytest.mark.parametrize("L", WEIGHT_ONLY, ids=[l.name for l in WEIGHT_ONLY])
def test_weight_only_quantization(L, nhwc):
    """Quantized filters, full-precision inputs (Sec. 4's weight-only rows): filter codes bit for
    bit, Y within 1e-4 of the output range of the oracle's binary64 sum (the GPU sums the same
    binary32 operands in binary32)."""
    from paper_2003_08646_amd import binding as B
    from paper_2003_08646_amd.layer import LanceConv
    _say(f"[case] {L.name} nhwc={nhwc}")
    X, Wt = Wk.make_inputs(L)
    f = O.prepare_filters(Wt, L.m, L.bits_w)
    ref = O.weight_only_conv_f64(X, Wt, L.pad, L.m, L.bits_w, filters=f)
    conv = LanceConv(L.N, L.C, L.H, L.W, L.K, L.pad, L.m, L.bits,
                     B.LANCE_LAYOUT_NHWC if nhwc else 0, bits_w=L.bits_w)
    conv.prepare_filters(torch.from_numpy(Wt).cuda())
    _assert_codes(conv.codes_to_logical(conv.uq, L.K), f.Uq, "filter codes")
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1)) if nhwc else X).cuda()
    conv.y.fill_(float("nan"))
    B.lance_conv3x3_winograd_wq_f32(conv.desc, x, conv.uq, conv.u_range, conv.y)
    torch.cuda.synchronize()
    got = conv.y.cpu().numpy().astype(np.float64)
    if nhwc:
        got = got.transpose(0, 3, 1, 2)
    tol = 1e-4 * float(ref.max() - ref.min())
    err = float(np.abs(got - ref).max())
    assert err <= tol, (err, tol)
    Yd = O.direct_conv_f64(X, Wt, L.pad)
    _say(f"  ok: max|Y-oracle| = {err:.3g} (tol {tol:.3g}), rel-L2 vs fp64 direct convolution = "
         f"{np.linalg.norm(got - Yd) / np.linalg.norm(Yd):.4g}")


PACKED = [
    Wk.Layer("packed_c130_k70_b4", 2, 130, 70, 10, 18, pad=1, m=2, bits=4, seed=441),
    Wk.Layer("packed_c64_k40_b4", 3, 64, 40, 12, 12, pad=1, m=2, bits=4, seed=442),
    Wk.Layer("packed_c17_k33_b3_w4", 3, 17, 33, 12, 10, pad=1, m=2, bits=3, bits_w=4, seed=443),
    Wk.Layer("packed_c256_k130_b4_pad0", 1, 256, 130, 11, 13, pad=0, m=2, bits=4, seed=444),
    Wk.Layer("packed_c320_k129_b2_w3", 2, 320, 129, 10, 14, pad=1, m=2, bits=2, bits_w=3, seed=445),
    Wk.Layer("packed_c512_k64_b4_many_tiles", 6, 512, 64, 28, 28, pad=1, m=2, bits=4, seed=446),
    Wk.Layer("packed_c192_k64_b4_pad2", 1, 192, 64, 6, 6, pad=2, m=2, bits=4, seed=447),
    Wk.Layer("packed_c100_k16_b4_w2_odd", 3, 100, 16, 9, 7, pad=1, m=2, bits=4, bits_w=2, seed=448),
    Wk.Layer("packed_m4_c130_k70_b4", 2, 130, 70, 10, 18, pad=1, m=4, bits=4, seed=451),
    Wk.Layer("packed_m4_c64_k64_b4", 3, 64, 64, 12, 12, pad=1, m=4, bits=4, seed=452),
    Wk.Layer("packed_m4_c128_k130_b3", 2, 128, 130, 16, 16, pad=1, m=4, bits=3, seed=453),
    Wk.Layer("packed_m4_c200_k40_b4_pad0_odd", 1, 200, 40, 13, 11, pad=0, m=4, bits=4, seed=454),
    Wk.Layer("packed_m4_c512_k33_b4_w2", 2, 512, 33, 14, 14, pad=1, m=4, bits=4, bits_w=2, seed=455),
    Wk.Layer("packed_m4_c384_k20_b2", 1, 384, 20, 8, 8, pad=2, m=4, bits=2, seed=456),
]


def _check_packed(L, flags=0, static_v_range=None, X=None, Wt=None):
    from paper_2003_08646_amd import binding as B
    nhwc = bool(flags & B.LANCE_LAYOUT_NHWC)
    return _check_packed_impl(L, flags, static_v_range, X, Wt, nhwc)


def _check_packed_impl(L, flags, static_v_range, X, Wt, nhwc):
    """Two 4-bit codes per byte: the codes, sums and ranges of the unpacked method bit for bit
    (filter transform and input transform), the fused Y within the usual tolerance."""
    from paper_2003_08646_amd import binding as B
    _say(f"[case] packed {L.name} N{L.N} C{L.C} K{L.K} {L.H}x{L.W} pad{L.pad} b{L.bits} "
         f"bw{L.bits_w} flags{flags}")
    if X is None:
        X, Wt = Wk.make_inputs(L)
    ref = O.lance_conv(X, Wt, L.pad, L.m, L.bits, bits_w=L.bits_w,
                       per_tensor=bool(flags & B.LANCE_RANGE_PER_TENSOR),
                       static_v_range=static_v_range)
    conv = _gpu_layer(L, flags | B.LANCE_CODES_PACKED4)
    assert conv.sz.uq_bytes * 2 == conv.sz.E * L.K * conv.sz.Cp
    x = torch.from_numpy(np.ascontiguousarray(X.transpose(0, 2, 3, 1)) if nhwc else X).cuda()
    w = torch.from_numpy(Wt).cuda()
    conv.uq.fill_(0x55)
    conv.prepare_filters(w)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(conv.u_range.cpu().numpy(), ref.filters.u_range)
    _assert_codes(conv.codes_to_logical(conv.uq, L.K), ref.filters.Uq, "packed filter codes")
    np.testing.assert_array_equal(conv.u_rowsum.cpu().numpy(), ref.filters.u_rowsum)
    if static_v_range is not None:
        conv.v_range.copy_(torch.from_numpy(np.ascontiguousarray(static_v_range, np.float32)))
    tol = 1e-4 * float(ref.Y.max() - ref.Y.min())
    st = conv.alloc_staged()
    st["vq"].fill_(0x55)
    st = conv.forward_staged(x)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(conv.v_range.cpu().numpy(), ref.v_range)
    _assert_codes(conv.codes_to_logical(st["vq"], conv.sz.P), ref.Vq, "packed input codes")
    np.testing.assert_array_equal(st["v_colsum"].cpu().numpy(), ref.v_colsum)
    np.testing.assert_array_equal(st["acc"].cpu().numpy(), ref.ACC)
    ys = st["y"].cpu().numpy().astype(np.float64)
    if nhwc:
        ys = ys.transpose(0, 3, 1, 2)
    err = float(np.abs(ys - ref.Y).max())
    assert err <= tol, ("packed staged Y", err, tol)
    del st
    conv._staged = None
    if static_v_range is None:
        conv.v_range.fill_(float("nan"))
    conv.y.fill_(float("nan"))
    y = conv.forward(x).cpu().numpy().astype(np.float64)
    if nhwc:
        y = y.transpose(0, 3, 1, 2)
    np.testing.assert_array_equal(conv.v_range.cpu().numpy(), ref.v_range)
    err = float(np.abs(y - ref.Y).max())
    assert err <= tol, ("packed fused Y", err, tol)
    _say(f"  ok: max|Y-oracle| = {err:.3g} (tol {tol:.3g})")


@pytest.mark.parametrize("L", PACKED, ids=[l.name for l in PACKED])
def test_packed_four_bit_codes(L):
    _check_packed(L)


PACKED_NHWC = [l for l in PACKED if l.name in (
    "packed_c130_k70_b4", "packed_c64_k40_b4", "packed_c17_k33_b3_w4", "packed_c256_k130_b4_pad0",
    "packed_c512_k64_b4_many_tiles", "packed_m4_c130_k70_b4", "packed_m4_c128_k130_b3",
    "packed_m4_c200_k40_b4_pad0_odd", "packed_m4_c384_k20_b2")]


@pytest.mark.parametrize("L", PACKED_NHWC, ids=[l.name for l in PACKED_NHWC])
def test_packed_four_bit_codes_nhwc(L):
    from paper_2003_08646_amd import binding as B
    _check_packed(L, flags=B.LANCE_LAYOUT_NHWC)


def test_packed_four_bit_codes_with_range_flags():
    from paper_2003_08646_amd import binding as B
    L = Wk.Layer("packed_ranges_c130", 2, 130, 24, 10, 10, m=2, bits=4, seed=449)
    _check_packed(L, flags=B.LANCE_RANGE_PER_TENSOR)
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    _check_packed(L, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=narrow, X=X, Wt=Wt)


def test_packed_four_bit_codes_full_size_cfg4():
    """Configuration 4 at 4 bits, packed: the layer whose code traffic packing halves."""
    _check_packed(Wk.CFG4.with_(bits=4, name="cfg4_b4_packed"))


def test_packed_four_bit_codes_full_size_cfg3_m4():
    _check_packed(Wk.CFG3_M4.with_(bits=4, name="cfg3_m4_b4_packed"))


def test_degenerate_constant_and_zero_inputs():
    """max(T) == min(T) at some or all positions: every code 0, Q' returns min exactly."""
    L = Wk.Layer("const_input", 1, 4, 4, 8, 8, pad=0, m=2, seed=42)
    _, Wt = Wk.make_inputs(L)
    X = np.full((1, 4, 8, 8), 0.5, np.float32)     # interior-only tiles: V is constant per e
    _check_layer(L, X, Wt)
    L0 = L.with_(name="zero_input", pad=1)
    _check_layer(L0, np.zeros((1, 4, 8, 8), np.float32), Wt)
    Lw = L.with_(name="zero_filters", pad=1)
    Xr, _ = Wk.make_inputs(Lw)
    _check_layer(Lw, Xr, np.zeros_like(Wt))


def test_gemm_extreme_codes_through_the_abi():
    """All-(-128) and all-127 codes at C = 512 exercise the int32 range of the accumulators."""
    from paper_2003_08646_amd import binding as B
    C, K, P = 512, 40, 100
    d = B.make_desc(1, C, 22, 22, K, pad=0, m=2)   # Ho=Wo=20, th=tw=10 -> P=100
    s = B.lance_query_sizes(d)
    assert s.P == P
    for a, b in [(-128, -128), (127, 127), (-128, 127)]:
        _say(f"[case] gemm extremes {a} {b}")
        uq = torch.full((s.uq_bytes,), a, dtype=torch.int8, device="cuda")
        vq = torch.full((s.vq_bytes,), b, dtype=torch.int8, device="cuda")
        acc = torch.empty((s.E, K, P), dtype=torch.int32, device="cuda")
        B.lance_winograd_gemm_i8(d, uq, vq, acc)
        torch.cuda.synchronize()
        assert bool((acc == a * b * C).all())
    # packed 4-bit rows: every code -8 (nibble 0) or 7 (nibble 15)
    dp = B.make_desc(1, C, 22, 22, K, pad=0, m=2, bits=4, flags=B.LANCE_CODES_PACKED4)
    sp = B.lance_query_sizes(dp)
    assert sp.uq_bytes * 2 == s.uq_bytes
    for a, b in [(-8, -8), (7, 7), (-8, 7)]:
        _say(f"[case] packed gemm extremes {a} {b}")
        uq = torch.full((sp.uq_bytes,), 0 if a < 0 else -1, dtype=torch.int8, device="cuda")
        vq = torch.full((sp.vq_bytes,), 0 if b < 0 else -1, dtype=torch.int8, device="cuda")
        acc = torch.empty((sp.E, K, P), dtype=torch.int32, device="cuda")
        B.lance_winograd_gemm_i8(dp, uq, vq, acc)
        torch.cuda.synchronize()
        assert bool((acc == a * b * C).all())


def test_gemm_random_codes_equal_oracle_product():
    from paper_2003_08646_amd import binding as B
    from paper_2003_08646_amd.layer import LanceConv
    rng = np.random.default_rng(50)
    for C, K, hw, m in [(64, 64, 18, 2), (200, 37, 11, 2), (16, 16, 9, 4), (48, 70, 10, 4)]:
        conv = LanceConv(3, C, hw, hw, K, 1, m, 8)
        s = conv.sz
        _say(f"[case] gemm random C{C} K{K} P{s.P} m{m}")
        Uq = rng.integers(-128, 128, size=(s.E, K, s.Cp), dtype=np.int8)
        Vq = rng.integers(-128, 128, size=(s.E, s.P, s.Cp), dtype=np.int8)
        ref = O.gemm_i8(Uq, Vq)

        def to_blocked(a, rows):     # logical [E][rows][Cp] -> device layout (index permutation)
            Q = s.CB // 4
            r = np.arange(s.CB)
            pos = 4 * (r % Q) + r // Q
            b = a.reshape(s.E, rows, s.NB, s.CB).transpose(0, 2, 1, 3)
            out = np.empty_like(b)
            out[:, :, :, pos] = b
            return np.ascontiguousarray(out).reshape(-1)

        uq = torch.from_numpy(to_blocked(Uq, K)).cuda()
        vq = torch.from_numpy(to_blocked(Vq, s.P)).cuda()
        np.testing.assert_array_equal(conv.codes_to_logical(uq, K), Uq)
        acc = torch.empty((s.E, K, s.P), dtype=torch.int32, device="cuda")
        B.lance_winograd_gemm_i8(conv.desc, uq, vq, acc)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(acc.cpu().numpy(), ref)


@pytest.mark.parametrize("L", [
    Wk.Layer("twin_two_kernels", 2, 64, 32, 12, 12, m=2, seed=120),
    Wk.Layer("twin_small_channels", 2, 3, 32, 12, 12, m=2, seed=121),
    Wk.Layer("twin_general_m2", 2, 130, 32, 12, 12, m=2, seed=122),
    Wk.Layer("twin_two_blocks", 2, 128, 32, 12, 12, m=2, seed=125),
    Wk.Layer("twin_general_m4", 2, 130, 32, 12, 12, m=4, seed=123),
    Wk.Layer("twin_padded_block", 2, 20, 32, 12, 12, m=2, seed=124),
    Wk.Layer("twin_fallback", 2, 10, 32, 12, 12, m=4, seed=126),
    Wk.Layer("twin_fused_m4", 2, 64, 32, 12, 12, m=4, seed=118),
    Wk.Layer("twin_fused_m4_two_blocks", 2, 128, 32, 12, 12, m=4, seed=119),
    Wk.Layer("twin_nhwc_two_kernels", 2, 64, 32, 12, 12, m=2, seed=127),
    Wk.Layer("twin_nhwc_general_m4", 2, 130, 32, 12, 12, m=4, seed=128),
    Wk.Layer("twin_nhwc_small_channels", 2, 3, 32, 12, 12, m=2, seed=129),
], ids=lambda l: l.name)
def test_timing_twin_runs_the_same_kernels(L):
    """The per-kernel timing twin of the fused call: same output bits, plausible durations."""
    from paper_2003_08646_amd import binding as B
    X, Wt = Wk.make_inputs(L)
    nhwc = "nhwc" in L.name
    conv = _gpu_layer(L, B.LANCE_LAYOUT_NHWC if nhwc else 0)
    if nhwc:
        X = np.ascontiguousarray(X.transpose(0, 2, 3, 1))
    x, w = torch.from_numpy(X).cuda(), torch.from_numpy(Wt).cuda()
    conv.prepare_filters(w)
    y0 = conv.forward(x).clone()
    r0 = conv.v_range.clone()
    conv.y.fill_(float("nan"))
    conv.v_range.fill_(float("nan"))
    _say(f"[case] timing twin {L.name}")
    ms = B.lance_conv3x3_winograd_q8_profile(conv.desc, x, conv.uq, conv.u_range, conv.u_rowsum,
                                             conv.v_range, conv.y, conv.workspace, repeats=7)
    torch.cuda.synchronize()
    assert torch.equal(conv.y, y0) and torch.equal(conv.v_range, r0)
    assert len(ms) == len(B.PROFILE_KERNELS)
    assert all(0.0 <= v < 50.0 for v in ms), ms
    assert ms[0] > 0.0 and ms[3] > 0.0, ms


@pytest.mark.parametrize("L", [
    Wk.Layer("graph_two_kernels", 4, 64, 48, 16, 16, m=2, seed=150),
    Wk.Layer("graph_general_m2", 2, 200, 48, 12, 12, m=2, seed=151),
    Wk.Layer("graph_general_m4", 2, 130, 48, 12, 12, m=4, seed=152),
    Wk.Layer("graph_small_channels", 2, 3, 48, 16, 16, m=2, seed=153),
    Wk.Layer("graph_fused_m4", 2, 100, 48, 12, 12, m=4, seed=158),
    Wk.Layer("graph_nhwc_two_kernels", 4, 64, 48, 16, 16, m=2, seed=154),
    Wk.Layer("graph_nhwc_general_m2", 2, 256, 48, 12, 12, m=2, seed=155),
    Wk.Layer("graph_nhwc_three_blocks_m4", 2, 130, 48, 12, 12, m=4, seed=156),
    Wk.Layer("graph_nhwc_small_channels", 2, 3, 48, 16, 16, m=2, seed=157),
], ids=lambda l: l.name)
def test_fused_call_replays_from_a_hip_graph(L):
    """The fused call only launches kernels (no memset nodes), so a caller may capture it.  Every
    replay, with eager calls on other inputs in between, gives the bits of the eager call."""
    from paper_2003_08646_amd import binding as B
    X, Wt = Wk.make_inputs(L)
    nhwc = "nhwc" in L.name
    conv = _gpu_layer(L, B.LANCE_LAYOUT_NHWC if nhwc else 0)
    w = torch.from_numpy(Wt).cuda()
    if nhwc:
        X = np.ascontiguousarray(X.transpose(0, 2, 3, 1))
    xs = [torch.from_numpy(X).cuda(), torch.from_numpy(np.ascontiguousarray(X[::-1] * 0.5)).cuda()]
    conv.prepare_filters(w)
    eager = []
    for x in xs:
        eager.append((conv.forward(x).clone(), conv.v_range.clone()))
    torch.cuda.synchronize()
    s = torch.cuda.Stream()
    x_in = xs[0].clone()
    with torch.cuda.stream(s):
        conv.forward(x_in, stream=s)  # warm-up on the capture stream
        s.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            conv.forward(x_in, stream=s)
        for rep in range(4):
            which = rep % 2
            x_in.copy_(xs[which])
            conv.y.fill_(float("nan"))
            g.replay()
            s.synchronize()
            assert torch.equal(conv.y, eager[which][0]), f"replay {rep}"
            assert torch.equal(conv.v_range, eager[which][1]), f"replay {rep}"
            # eager work of the program between the replays
            other = conv.forward(xs[1 - which], stream=s).clone()
            s.synchronize()
            assert torch.equal(other, eager[1 - which][0])


def test_deterministic_across_runs():
    L = Wk.Layer("determinism", 4, 96, 64, 14, 14, m=2, seed=60)
    X, Wt = Wk.make_inputs(L)
    conv = _gpu_layer(L)
    conv.prepare_filters(torch.from_numpy(Wt).cuda())
    x = torch.from_numpy(X).cuda()
    a = conv.forward_staged(x)
    a = {k: v.clone() for k, v in a.items()}
    y1 = conv.forward(x).clone()
    b = conv.forward_staged(x)
    y2 = conv.forward(x)
    torch.cuda.synchronize()
    for k in a:
        assert torch.equal(a[k], b[k]), k
    assert torch.equal(y1, y2)


def test_direct_conv_comparator_matches_eq1():
    from paper_2003_08646_amd import binding as B
    for L in [Wk.Layer("direct_small", 2, 5, 7, 9, 11, pad=1, seed=70),
              Wk.Layer("direct_pad0", 1, 19, 40, 20, 17, pad=0, seed=71),
              Wk.CFG1]:
        _say(f"[case] direct conv {L.name}")
        X, Wt = Wk.make_inputs(L)
        Yd = O.direct_conv_f64(X, Wt, L.pad)
        d = B.make_desc(L.N, L.C, L.H, L.W, L.K, L.pad)
        y = torch.empty(Yd.shape, dtype=torch.float32, device="cuda")
        B.lance_direct_conv3x3_f32(d, torch.from_numpy(X).cuda(), torch.from_numpy(Wt).cuda(), y)
        torch.cuda.synchronize()
        err = np.abs(y.cpu().numpy() - Yd).max()
        assert err <= 1e-5 * max(1.0, np.abs(Yd).max()) * np.sqrt(9 * L.C), err


# ------------------------------------------------------------------ the five configurations
def test_config1_full():
    _check_layer(Wk.CFG1, check_direct=True)


def test_config2_full_size():
    _check_layer(Wk.CFG2, check_direct=True)


@pytest.mark.parametrize("L", [Wk.CFG3_M2, Wk.CFG3_M4], ids=["m2", "m4"])
def test_config3_full_size(L):
    _check_layer(L, check_direct=True)


@pytest.mark.parametrize("bits", [8, 6, 4])
def test_config4_full_size_bit_sweep(bits):
    _check_layer(Wk.CFG4.with_(bits=bits, name=f"cfg4_b{bits}"), check_direct=True)


@pytest.mark.parametrize("L", Wk.vgg16_layers(), ids=[l.name for l in Wk.vgg16_layers()])
def test_config5_vgg16_layers(L):
    _check_layer(L)


# ------------------------------------------------------------------ the same, NHWC, full size
# Layers large enough (at least 4096 strips of four tile rows) that the NHWC range pass takes its
# rolling-window kernel: the configurations themselves, and ragged layers whose tile rows are not
# a multiple of the strip length, with pad 0 and pad 2 and two or three channel blocks.
NHWC_FULL = [
    Wk.CFG2, Wk.CFG3_M2, Wk.CFG4,
    Wk.Layer("nhwc_roll_ragged_c72_pad0", 48, 72, 40, 27, 27, pad=0, m=2, seed=360),
    Wk.Layer("nhwc_roll_ragged_c136_pad2", 24, 136, 24, 25, 27, pad=2, m=2, seed=361),
    Wk.Layer("nhwc_roll_c64_th5", 110, 64, 16, 10, 38, pad=1, m=2, seed=362),
    Wk.vgg16_layers()[1].with_(N=4, name="nhwc_roll_vgg_c64_224"),
]


@pytest.mark.parametrize("L", NHWC_FULL, ids=[l.name for l in NHWC_FULL])
def test_nhwc_full_size_layers_take_the_rolling_range_pass(L):
    from paper_2003_08646_amd import binding as B
    th, tw = -(-(L.H + 2 * L.pad - 2) // 2), -(-(L.W + 2 * L.pad - 2) // 2)
    nb = -(-L.C // 64)
    assert L.C % 4 == 0 and L.N * tw * nb * -(-th // 4) >= 4096   # the kernel's dispatch rule
    _check_layer(L, flags=B.LANCE_LAYOUT_NHWC)


def test_nhwc_full_size_static_ranges():
    """Calibrated ranges (narrower than the data, so both clamps are live) on cfg2 in NHWC."""
    from paper_2003_08646_amd import binding as B
    L = Wk.CFG2
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    narrow = (O.ranges(V) * np.float32(0.5)).astype(np.float32)
    del V
    _check_layer(L, X, Wt, flags=B.LANCE_LAYOUT_NHWC | B.LANCE_INPUT_RANGE_STATIC,
                 static_v_range=narrow)


# ------------------------------------------------------------------ calibrated ranges, full size
# bench.py also times every configuration with caller-supplied ranges (Sec. 3.4's inference mode,
# no range pass): the same layers at full size, with the ranges the data has (same codes as the
# dynamic call) -- one layer per plan of the fused call.
STATIC_FULL = [Wk.CFG2, Wk.CFG3_M2, Wk.CFG3_M4, Wk.CFG4, Wk.vgg16_layers()[0], Wk.vgg16_layers()[5],
               Wk.vgg16_layers()[11]]


@pytest.mark.parametrize("L", STATIC_FULL, ids=[l.name for l in STATIC_FULL])
def test_full_size_layers_with_calibrated_ranges(L):
    from paper_2003_08646_amd import binding as B
    X, Wt = Wk.make_inputs(L)
    V = O.input_transform_f32(X, L.pad, L.m)
    vr = O.ranges(V)
    del V
    _check_layer(L, X, Wt, flags=B.LANCE_INPUT_RANGE_STATIC, static_v_range=vr, staged=False)
