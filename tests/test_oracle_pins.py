"""Pins for the CPU oracle: each part is checked against something other than itself --
values the paper prints, library routines, closed forms, brute force on tiny inputs.
CPU only.
"""
import itertools
import os

import numpy as np
import pytest
from scipy.signal import correlate2d

from oracle import lance_oracle as O

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def _rand_layer(rng, N, C, K, H, W):
    X = rng.standard_normal((N, C, H, W)).astype(np.float32)
    Wt = rng.standard_normal((K, C, 3, 3)).astype(np.float32)
    return X, Wt


# ---------------------------------------------------------------- Part 1: Eq. 1 ----------
@pytest.mark.parametrize("pad", [0, 1, 2])
def test_direct_conv_equals_library_correlation(pad):
    """Eq. 1 / Eq. 2: Y[n,k] = sum_c X[n,c] (2-D correlation) W[k,c]; scipy is the library."""
    rng = np.random.default_rng(10 + pad)
    X, Wt = _rand_layer(rng, 2, 3, 4, 7, 9)
    Y = O.direct_conv_f64(X, Wt, pad)
    Xp = np.pad(X.astype(np.float64), ((0, 0), (0, 0), (pad, pad), (pad, pad)))
    ref = np.zeros_like(Y)
    for n, k, c in itertools.product(range(2), range(4), range(3)):
        ref[n, k] += correlate2d(Xp[n, c], Wt[k, c].astype(np.float64), mode="valid")
    assert Y.shape == (2, 4, 7 + 2 * pad - 2, 9 + 2 * pad - 2)
    np.testing.assert_allclose(Y, ref, rtol=0, atol=1e-12)


def test_direct_conv_hand_case():
    """One channel, all-ones 3x3 filter on a 3x3 ramp, pad 1: box sums computed by hand."""
    X = np.arange(9, dtype=np.float32).reshape(1, 1, 3, 3)
    Wt = np.ones((1, 1, 3, 3), np.float32)
    Y = O.direct_conv_f64(X, Wt, 1)[0, 0]
    hand = np.array([[8, 15, 12], [21, 36, 27], [20, 33, 24]], dtype=np.float64)
    np.testing.assert_array_equal(Y, hand)


def test_direct_conv_is_correlation_not_flipped():
    """A filter with a single tap at (r,s)=(0,2) must pick X[i+0-pad, j+2-pad]."""
    rng = np.random.default_rng(3)
    X = rng.standard_normal((1, 1, 5, 5)).astype(np.float32)
    Wt = np.zeros((1, 1, 3, 3), np.float32)
    Wt[0, 0, 0, 2] = 1
    Y = O.direct_conv_f64(X, Wt, 0)[0, 0]
    np.testing.assert_array_equal(Y, X[0, 0, 0:3, 2:5].astype(np.float64))


# ------------------------------------------------- Eq. 4 == Eq. 1 (matrices, tiling) ------
@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("pad", [0, 1])
@pytest.mark.parametrize("hw", [(4, 4), (6, 6), (7, 5), (9, 11), (8, 13)])
def test_unquantized_winograd_equals_direct(m, pad, hw):
    H, W = hw
    if H + 2 * pad - 2 < 1 or W + 2 * pad - 2 < 1:
        pytest.skip("empty output")
    rng = np.random.default_rng(100 * m + 10 * pad + H)
    X, Wt = _rand_layer(rng, 2, 3, 2, H, W)
    Yd = O.direct_conv_f64(X, Wt, pad)
    Yw = O.winograd_conv_f64(X, Wt, pad, m)
    np.testing.assert_allclose(Yw, Yd, rtol=0, atol=1e-9)


# ------------------------------------------------- values printed in Eq. 6 ----------------
def test_eq6_printed_bt_and_transform():
    bt_printed = np.loadtxt(os.path.join(GOLD, "eq6_bt.txt"))
    dhat = np.loadtxt(os.path.join(GOLD, "eq5_codes.txt"))
    printed = np.loadtxt(os.path.join(GOLD, "eq6_result.txt"))
    bt, _, _ = O.matrices(2)
    np.testing.assert_array_equal(bt, bt_printed)
    v = O.input_tile_f32(dhat, 2)  # B^T d^ B through the binary32 expression tree
    np.testing.assert_array_equal(v.astype(np.float64), printed)
    # orientation: the transposed order (B d^ B^T) would not give the printed matrix
    assert not np.array_equal(bt_printed.T @ dhat @ bt_printed, printed)


def test_eq5_printed_codes_follow_ceil_not_eq7():
    """Eq. 5 is introduced as a 'naive' quantizer before Eq. 7 is defined.  Its printed codes
    equal ceil(x*3/15), not Eq. 7's round().  Eq. 7 is the authority; this records the
    mismatch so that nobody changes the quantizer to chase the illustration."""
    d = np.loadtxt(os.path.join(GOLD, "eq5_d.txt"))
    printed = np.loadtxt(os.path.join(GOLD, "eq5_codes.txt"))
    np.testing.assert_array_equal(np.ceil(d * 3 / 15), printed)
    inv, scale = O.quant_params(0.0, 15.0, 2)
    ours = np.array([[O.quantize_value(x, 0.0, inv, 2) for x in row] for row in d])
    hand = np.array([[0, 0, 0, 1], [1, 1, 1, 1], [2, 2, 2, 2], [2, 3, 3, 3]])  # round(x/5)
    np.testing.assert_array_equal(ours, hand)
    assert not np.array_equal(ours, printed)


# ------------------------------------------------- binary32 expression trees --------------
@pytest.mark.parametrize("m", [2, 4])
def test_transform_trees_exact_on_small_integers(m):
    """On small integers every intermediate is exact in binary32, so the tree must equal the
    matrix products B^T d B and G g G^T (G scaled to integers) exactly."""
    rng = np.random.default_rng(m)
    bt, g, _ = O.matrices(m)
    a = m + 2
    for _ in range(50):
        d = rng.integers(-8, 9, size=(a, a)).astype(np.float64)
        np.testing.assert_array_equal(O.input_tile_f32(d, m).astype(np.float64), bt @ d @ bt.T)
    den = 2 if m == 2 else 24
    for _ in range(50):
        # multiples of den^2 make G g G^T integral; the tree's own factors (1/6, 1/24 in
        # binary32) are inexact for m = 4, so compare within a few ulp there
        gg = rng.integers(-4, 5, size=(3, 3)).astype(np.float64) * den * den
        u = O.filter_tile_f32(gg, m).astype(np.float64)
        ref = g @ gg @ g.T
        if m == 2:
            np.testing.assert_array_equal(u, ref)
        else:
            bound = np.abs(g) @ np.abs(gg) @ np.abs(g.T)
            assert np.all(np.abs(u - ref) <= 4e-7 * bound)


@pytest.mark.parametrize("m", [2, 4])
def test_transform_trees_close_to_fp64_products(m):
    rng = np.random.default_rng(20 + m)
    bt, g, _ = O.matrices(m)
    a = m + 2
    eps = np.finfo(np.float32).eps
    for _ in range(100):
        d = rng.standard_normal((a, a)).astype(np.float32)
        ref = bt @ d.astype(np.float64) @ bt.T
        bound = np.abs(bt) @ np.abs(d.astype(np.float64)) @ np.abs(bt.T)
        assert np.all(np.abs(O.input_tile_f32(d, m) - ref) <= 8 * eps * bound + 1e-30)
        gg = rng.standard_normal((3, 3)).astype(np.float32)
        ref = g @ gg.astype(np.float64) @ g.T
        bound = np.abs(g) @ np.abs(gg.astype(np.float64)) @ np.abs(g.T)
        assert np.all(np.abs(O.filter_tile_f32(gg, m) - ref) <= 8 * eps * bound + 1e-30)


def test_transform_layout_e_p_c_and_tile_order():
    """U[e][k][c], V[e][p][c] with e = i*(m+2)+j and p = (n*th+ty)*tw+tx."""
    rng = np.random.default_rng(5)
    X, Wt = _rand_layer(rng, 2, 3, 2, 6, 8)
    m, pad = 2, 1
    V = O.input_transform_f32(X, pad, m)
    U = O.filter_transform_f32(Wt, m)
    th, tw = 3, 4
    assert V.shape == (16, 2 * th * tw, 3) and U.shape == (16, 2, 3)
    Xp = np.pad(X, ((0, 0), (0, 0), (1, 1), (1, 1)))
    n, ty, tx, c = 1, 2, 3, 1
    tile = Xp[n, c, ty * 2:ty * 2 + 4, tx * 2:tx * 2 + 4]
    np.testing.assert_array_equal(V[:, (n * th + ty) * tw + tx, c].reshape(4, 4),
                                  O.input_tile_f32(tile, m))
    np.testing.assert_array_equal(U[:, 1, 2].reshape(4, 4), O.filter_tile_f32(Wt[1, 2], m))


# ------------------------------------------------- ranges ---------------------------------
def test_ranges_match_numpy_min_max():
    rng = np.random.default_rng(6)
    T = rng.standard_normal((16, 37, 5)).astype(np.float32)
    r = O.ranges(T)
    np.testing.assert_array_equal(r[:, 0], T.reshape(16, -1).min(axis=1))
    np.testing.assert_array_equal(r[:, 1], T.reshape(16, -1).max(axis=1))
    rt = O.ranges(T, per_tensor=True)
    assert np.all(rt[:, 0] == T.min()) and np.all(rt[:, 1] == T.max())


# ------------------------------------------------- the quantizer, Eq. 7 / Eq. 8 -----------
@pytest.mark.parametrize("bits", [2, 4, 6, 8])
def test_quantizer_invariants(bits):
    rng = np.random.default_rng(bits)
    L = 2 ** bits - 1
    for _ in range(20):
        mn, mx = np.sort(rng.standard_normal(2).astype(np.float32) * 10)
        if mn == mx:
            continue
        inv, scale = O.quant_params(mn, mx, bits)
        xs = np.sort(np.concatenate([[mn, mx], rng.uniform(mn, mx, 300)]).astype(np.float32))
        codes = np.array([O.quantize_value(x, mn, inv, bits) for x in xs])
        assert codes[0] == 0 and codes[-1] == L          # Q(min)=0, Q(max)=2^b-1
        assert codes.min() >= 0 and codes.max() <= L
        assert np.all(np.diff(codes) >= 0)               # monotone
        back = np.array([O.dequantize_value(c, mn, scale) for c in codes])
        err = np.abs(back - xs.astype(np.float64))
        # |x - Q'(Q(x))| <= half a step (plus binary32 rounding of x-min, inv and scale)
        assert err.max() <= 0.5 * float(scale) * (1 + 1e-5) + 4 * np.finfo(np.float32).eps * max(abs(mn), abs(mx))
        # scale is (max-min)/(2^b-1)
        assert scale == np.float32((float(mx) - float(mn)) / L)


def test_quantizer_hand_vectors_and_ties():
    # 8 bits, range [0, 510]: inv = 0.5 exactly, so odd x land on exact .5 ties -> half-to-even
    inv, scale = O.quant_params(0.0, 510.0, 8)
    assert inv == np.float32(0.5) and scale == np.float32(2.0)
    got = [O.quantize_value(x, 0.0, inv, 8) for x in [0, 1, 2, 3, 5, 7, 9, 509, 510]]
    assert got == [0, 0, 1, 2, 2, 4, 4, 254, 255]
    # 2 bits, range [-1.5, 1.5]: step 1 -> codes of -1.5,-1.0,-0.4,0.49,0.5,0.51,1.5
    inv, scale = O.quant_params(-1.5, 1.5, 2)
    assert inv == np.float32(1.0) and scale == np.float32(1.0)
    got = [O.quantize_value(x, -1.5, inv, 2) for x in [-1.5, -1.0, -0.4, 0.49, 0.5, 0.51, 1.5]]
    assert got == [0, 0, 1, 2, 2, 2, 3]   # (x+1.5): 0,.5->0,1.1,1.99,2.0,2.01,3.0
    # values outside a given (static) range are clamped
    assert O.quantize_value(9.0, -1.5, inv, 2) == 3 and O.quantize_value(-9.0, -1.5, inv, 2) == 0


def test_quantizer_constant_matrix():
    """max(T) == min(T): every code is 0 and Q' returns min exactly."""
    inv, scale = O.quant_params(0.75, 0.75, 8)
    assert inv == 0 and scale == 0
    assert O.quantize_value(0.75, 0.75, inv, 8) == 0
    assert O.dequantize_value(0, 0.75, scale) == 0.75
    T = np.full((4, 3, 5), 0.75, np.float32)
    codes, sums = O.quantize(T, O.ranges(T), 8, 16)
    assert np.all(codes[:, :, :5] == -128) and np.all(codes[:, :, 5:] == 0)
    assert np.all(sums == -128 * 5)


@pytest.mark.parametrize("bits", [4, 8])
def test_quantize_array_layout_padding_and_sums(bits):
    rng = np.random.default_rng(7)
    T = rng.standard_normal((4, 9, 5)).astype(np.float32)
    r = O.ranges(T)
    codes, sums = O.quantize(T, r, bits, 16)
    h = 2 ** (bits - 1)
    assert codes.shape == (4, 9, 16) and np.all(codes[:, :, 5:] == 0)
    for e in range(4):
        inv, _ = O.quant_params(r[e, 0], r[e, 1], bits)
        for row in range(9):
            for c in range(5):
                assert codes[e, row, c] == O.quantize_value(T[e, row, c], r[e, 0], inv, bits) - h
    np.testing.assert_array_equal(sums, codes[:, :, :5].astype(np.int64).sum(axis=2))
    assert codes.min() >= -h and codes.max() <= h - 1


# ------------------------------------------------- integer product ------------------------
def test_gemm_equals_exact_integer_matmul():
    rng = np.random.default_rng(8)
    Uq = rng.integers(-128, 128, size=(16, 7, 48), dtype=np.int8)
    Vq = rng.integers(-128, 128, size=(16, 11, 48), dtype=np.int8)
    ACC = O.gemm_i8(Uq, Vq)
    ref = np.einsum("ekc,epc->ekp", Uq.astype(np.int64), Vq.astype(np.int64))
    np.testing.assert_array_equal(ACC.astype(np.int64), ref)
    ekp = np.array([[0, 0, 0], [15, 6, 10], [3, 2, 7]])
    np.testing.assert_array_equal(O.gemm_i8_sampled(Uq, Vq, ekp), ref[ekp[:, 0], ekp[:, 1], ekp[:, 2]])


def test_gemm_extreme_codes():
    C = 512
    for a, b in [(-128, -128), (127, 127), (-128, 127)]:
        Uq = np.full((1, 2, C), a, np.int8)
        Vq = np.full((1, 3, C), b, np.int8)
        assert np.all(O.gemm_i8(Uq, Vq) == a * b * C)


# ------------------------------------------------- de-quantization algebra ----------------
@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("bits,bits_w", [(4, 4), (8, 8), (8, 4), (5, 8), (2, 7)])
def test_dequant_expansion_equals_elementwise_eq8(m, bits, bits_w):
    """The 4-term expansion used after the integer product equals sum_c Q'(u^) * Q'(v^) with
    Q' of Eq. 8 applied to each unsigned code, followed by A^T M A (numpy, fp64); filter and
    input codes of the same or of different widths (each shifted by its own 2^(b-1))."""
    rng = np.random.default_rng(30 + m + bits + 7 * bits_w)
    X, Wt = _rand_layer(rng, 1, 5, 3, 5, 7)
    X = np.maximum(X, 0)
    res = O.lance_conv(X, Wt, 1, m, bits, bits_w=bits_w)
    g = res.geom
    hv, hu = 2 ** (bits - 1), 2 ** (bits_w - 1)
    _, _, at = O.matrices(m)
    a = m + 2
    uq = res.filters.Uq[:, :, :g.C].astype(np.float64) + hu   # unsigned codes of Eq. 7
    vq = res.Vq[:, :, :g.C].astype(np.float64) + hv
    assert uq.min() >= 0 and uq.max() <= 2 ** bits_w - 1 and vq.min() >= 0 and vq.max() <= 2 ** bits - 1
    su = np.array([O.quant_params(*res.filters.u_range[e], bits_w)[1] for e in range(g.E)], np.float64)
    sv = np.array([O.quant_params(*res.v_range[e], bits)[1] for e in range(g.E)], np.float64)
    ut = uq * su[:, None, None] + res.filters.u_range[:, 0].astype(np.float64)[:, None, None]
    vt = vq * sv[:, None, None] + res.v_range[:, 0].astype(np.float64)[:, None, None]
    M = np.einsum("ekc,epc->ekp", ut, vt).reshape(a, a, g.K, g.P)
    S = np.einsum("xi,ijkp,yj->kpxy", at, M, at)          # [K][P][m][m]
    Y = np.zeros((g.N, g.K, g.th * m, g.tw * m))
    S = S.reshape(g.K, g.N, g.th, g.tw, m, m)
    for n, ty, tx in itertools.product(range(g.N), range(g.th), range(g.tw)):
        Y[n, :, ty * m:(ty + 1) * m, tx * m:(tx + 1) * m] = S[:, n, ty, tx]
    Y = Y[:, :, :g.Ho, :g.Wo]
    scale = np.abs(Y).max()
    np.testing.assert_allclose(res.Y, Y, rtol=0, atol=1e-11 * scale)


# ------------------------------------------------- Algorithm 1 literally ------------------
@pytest.mark.parametrize("m", [2, 4])
def test_alg1_literal_with_shared_ranges_equals_gemm_form(m):
    """Algorithm 1 (per-channel quantize, multiply, de-quantize, float channel sum) with the
    ranges held constant over channels is the GEMM form re-associated."""
    rng = np.random.default_rng(40 + m)
    X, Wt = _rand_layer(rng, 2, 4, 3, 6, 5)
    res = O.lance_conv(X, Wt, 1, m, 8)
    lit = O.alg1_literal_f64(X, Wt, 1, m, 8, res.filters.u_range, res.v_range)
    np.testing.assert_allclose(lit, res.Y, rtol=0, atol=1e-11 * np.abs(res.Y).max())


@pytest.mark.parametrize("m", [2, 4])
def test_alg1_literal_16_bits_converges_to_direct(m):
    """With 16-bit codes the whole pipeline (transform, Q, product, Q', A^T . A, merge) must
    reproduce the direct convolution to about 2^-15 of the operand ranges."""
    rng = np.random.default_rng(50 + m)
    X, Wt = _rand_layer(rng, 1, 4, 3, 8, 8)
    X = np.maximum(X, 0)
    Yd = O.direct_conv_f64(X, Wt, 1)
    U = O.filter_transform_f32(Wt, m)
    V = O.input_transform_f32(X, 1, m)
    lit = O.alg1_literal_f64(X, Wt, 1, m, 16, O.ranges(U), O.ranges(V))
    rel = np.linalg.norm(lit - Yd) / np.linalg.norm(Yd)
    assert rel < (2e-4 if m == 2 else 2e-3), rel
    # per-matrix ranges (the most literal reading of T in Eq. 7) converge as well
    lit0 = O.alg1_literal_f64(X, Wt, 1, m, 16)
    rel0 = np.linalg.norm(lit0 - Yd) / np.linalg.norm(Yd)
    assert rel0 < (2e-4 if m == 2 else 2e-3), rel0


@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("bits,bits_w", [(4, 4), (8, 8), (6, 6), (8, 4), (5, 7)])
def test_alg1_literal_per_matrix_ranges_equal_numpy_recomputation(m, bits, bits_w):
    """Algorithm 1 with T = the single (m+2)x(m+2) matrix (Eq. 7 read literally), at working
    widths: two filters, two channels, two tiles, recomputed in numpy from the matrices of
    Eq. 4 (plain matrix products), Eq. 7 and Eq. 8 -- none of the oracle's transform or
    quantizer functions.  The data are integers (filters scaled by the common denominator of G)
    so that both transforms are exact in binary32 whatever the order of operations, and the
    two sides can agree to rounding of the final fp64 sums."""
    rng = np.random.default_rng(600 + 10 * m + bits + 3 * bits_w)
    a = m + 2
    bt, g, at = O.matrices(m)
    gs = 2 if m == 2 else 24                      # G = (integer matrix) / gs, exactly
    gi = np.rint(g * gs)
    np.testing.assert_allclose(gi / gs, g, rtol=0, atol=1e-15)
    den = gs * gs
    X = rng.integers(0, 16, size=(1, 2, a, a + m)).astype(np.float32)       # pad 0: 1 x 2 tiles
    Wt = (rng.integers(-8, 9, size=(2, 2, 3, 3)) * den).astype(np.float32)

    def q_then_dq(T, b):
        """Eq. 7 then Eq. 8 with min(T), max(T) of this very matrix."""
        T = T.astype(np.float32)
        mn, mx = T.min(), T.max()
        L = 2 ** b - 1
        rg = float(mx) - float(mn)
        if rg == 0.0:
            return np.full(T.shape, float(mn))
        inv, scale = np.float32(L / rg), np.float32(rg / L)
        code = np.clip(np.rint((T - mn) * inv), 0, L)        # binary32, ties to even
        assert code.min() == 0 and code.max() == L
        return code.astype(np.float64) * float(scale) + float(mn)

    Y = np.zeros((1, 2, m, 2 * m))
    for k in range(2):
        for tx in range(2):
            M = np.zeros((a, a))
            for c in range(2):
                U = gi @ Wt[k, c].astype(np.float64) @ gi.T / den      # = G g G^T, exact
                V = bt @ X[0, c, :, tx * m:tx * m + a].astype(np.float64) @ bt.T
                # the premise: these are integers, so the oracle's binary32 trees are exact on them
                assert np.array_equal(U, np.rint(U)) and np.array_equal(V, np.rint(V))
                M += q_then_dq(U, bits_w) * q_then_dq(V, bits)
            Y[0, k, :, tx * m:(tx + 1) * m] = at @ M @ at.T
    lit = O.alg1_literal_f64(X, Wt, 0, m, bits, bits_w=bits_w)
    np.testing.assert_allclose(lit, Y, rtol=0, atol=1e-12 * np.abs(Y).max())
    # and it is not the shared-range form: ranges over a whole position differ from these
    shared = O.lance_conv(X, Wt, 0, m, bits, bits_w=bits_w).Y
    assert np.abs(shared - Y).max() > 1e-6 * np.abs(Y).max()


# ------------------------------------------------- weight-only quantization ---------------
@pytest.mark.parametrize("m", [2, 4])
@pytest.mark.parametrize("bits_w", [4, 8, 2])
def test_weight_only_equals_elementwise_numpy_sum(m, bits_w):
    """Sec. 4's weight-only rows: M = sum_c Q'(u^) v with v the unquantized transform, then
    A^T M A -- recomputed in numpy from the filter codes, Eq. 8 and the transformed input."""
    rng = np.random.default_rng(700 + m + bits_w)
    X, Wt = _rand_layer(rng, 2, 5, 3, 7, 9)
    f = O.prepare_filters(Wt, m, bits_w)
    Y = O.weight_only_conv_f64(X, Wt, 1, m, bits_w, filters=f)
    g = O.geometry(X, Wt, 1, m)
    a = m + 2
    _, _, at = O.matrices(m)
    L = 2 ** bits_w - 1
    scale = np.array([np.float32((float(hi) - float(lo)) / L) if hi != lo else np.float32(0)
                      for lo, hi in f.u_range], np.float64)
    ut = (f.Uq.astype(np.float64) + 2 ** (bits_w - 1)) * scale[:, None, None] + \
        f.u_range[:, 0].astype(np.float64)[:, None, None]
    V = O.input_transform_f32(X, 1, m).astype(np.float64)
    M = np.einsum("ekc,epc->ekp", ut, V).reshape(a, a, g.K, g.P)
    S = np.einsum("xi,ijkp,yj->kpxy", at, M, at).reshape(g.K, g.N, g.th, g.tw, m, m)
    ref = np.zeros((g.N, g.K, g.th * m, g.tw * m))
    for n, ty, tx in itertools.product(range(g.N), range(g.th), range(g.tw)):
        ref[n, :, ty * m:(ty + 1) * m, tx * m:(tx + 1) * m] = S[:, n, ty, tx]
    ref = ref[:, :, :g.Ho, :g.Wo]
    np.testing.assert_allclose(Y, ref, rtol=0, atol=1e-11 * np.abs(ref).max())


@pytest.mark.parametrize("m", [2, 4])
def test_weight_only_is_the_limit_of_the_two_sided_method(m):
    """With 16-bit input codes the two-sided method (int64 products) must agree with the
    weight-only form to about 2^-15 of the input range per term; and with 8-bit filters both
    are close to the direct convolution."""
    rng = np.random.default_rng(720 + m)
    X, Wt = _rand_layer(rng, 1, 4, 3, 8, 8)
    X = np.maximum(X, 0)
    f = O.prepare_filters(Wt, m, 4)
    wo = O.weight_only_conv_f64(X, Wt, 1, m, 4, filters=f)
    V = O.input_transform_f32(X, 1, m)
    two = O.alg1_literal_f64(X, Wt, 1, m, 16, f.u_range, O.ranges(V), bits_w=4)
    assert np.abs(two - wo).max() < 1e-3 * np.abs(wo).max()
    Yd = O.direct_conv_f64(X, Wt, 1)
    wo8 = O.weight_only_conv_f64(X, Wt, 1, m, 8)
    assert np.linalg.norm(wo8 - Yd) / np.linalg.norm(Yd) < (0.01 if m == 2 else 0.05)
    assert np.linalg.norm(wo - Yd) / np.linalg.norm(Yd) > np.linalg.norm(wo8 - Yd) / np.linalg.norm(Yd)


# ------------------------------------------------- the method as an approximation ---------
def test_error_halves_per_bit_and_respects_apriori_bound():
    rng = np.random.default_rng(60)
    X, Wt = _rand_layer(rng, 2, 16, 8, 12, 12)
    X = np.maximum(X, 0)
    Wt *= np.float32(np.sqrt(2.0 / (9 * 16)))
    Yd = O.direct_conv_f64(X, Wt, 1)
    rels = {}
    for bits in [4, 5, 6, 7, 8]:
        res = O.lance_conv(X, Wt, 1, 2, bits)
        rels[bits] = np.linalg.norm(res.Y - Yd) / np.linalg.norm(Yd)
        # a-priori bound per Winograd-domain element:
        #   |sum_c (u v - u~ v~)| <= sum_c (|u| sv/2 + |v| su/2 + su sv/4), through ||A^T||_1^2 = 9
        U = O.filter_transform_f32(Wt, 2).astype(np.float64)
        V = O.input_transform_f32(X, 1, 2).astype(np.float64)
        su = np.array([O.quant_params(*res.filters.u_range[e], bits)[1] for e in range(16)], np.float64)
        sv = np.array([O.quant_params(*res.v_range[e], bits)[1] for e in range(16)], np.float64)
        bound_e = (np.abs(U).sum(axis=2).max(axis=1) * sv / 2 * 1.001
                   + np.abs(V).sum(axis=2).max(axis=1) * su / 2 * 1.001 + 16 * su * sv / 4)
        assert np.abs(res.Y - Yd).max() <= bound_e.sum() * 1.001
    for b in [4, 5, 6, 7]:
        ratio = rels[b] / rels[b + 1]
        assert 1.5 < ratio < 2.7, (b, ratio, rels)
    assert rels[8] < 0.02


def test_special_cases_delta_filter_and_single_tile():
    rng = np.random.default_rng(70)
    # centre-tap delta filter: Y ~= X (pad 1), within the quantization error
    X = np.maximum(rng.standard_normal((1, 1, 8, 8)).astype(np.float32), 0)
    Wt = np.zeros((1, 1, 3, 3), np.float32)
    Wt[0, 0, 1, 1] = 1
    for m in (2, 4):
        res = O.lance_conv(X, Wt, 1, m, 8)
        assert np.abs(res.Y[0, 0] - X[0, 0]).max() < 0.05 * X.max()
    # K = C = 1, one 4x4 tile, pad 0: the 2x2 valid correlation computed by hand
    d = np.arange(16, dtype=np.float32).reshape(1, 1, 4, 4)
    g = np.array([[1, 0, -1], [2, 0, -2], [1, 0, -1]], np.float32).reshape(1, 1, 3, 3)
    hand = np.array([[-8.0, -8.0], [-8.0, -8.0]])
    np.testing.assert_array_equal(O.direct_conv_f64(d, g, 0)[0, 0], hand)
    res = O.lance_conv(d, g, 0, 2, 8)
    assert res.geom.P == 1
    np.testing.assert_allclose(res.Y[0, 0], hand, rtol=0, atol=0.25)


def test_batch_shares_one_range_per_position():
    """Tiles of all N images form one P axis and share the per-position range."""
    rng = np.random.default_rng(80)
    X, Wt = _rand_layer(rng, 3, 2, 2, 6, 6)
    res = O.lance_conv(X, Wt, 1, 2, 8)
    V = O.input_transform_f32(X, 1, 2)
    np.testing.assert_array_equal(res.v_range[:, 1], V.reshape(16, -1).max(axis=1))
    assert res.Vq.shape == (16, 3 * 3 * 3, 2)


def test_static_range_and_per_tensor_modes():
    rng = np.random.default_rng(90)
    X, Wt = _rand_layer(rng, 1, 3, 2, 6, 6)
    Yd = O.direct_conv_f64(X, Wt, 1)
    base = O.lance_conv(X, Wt, 1, 2, 8)
    pt = O.lance_conv(X, Wt, 1, 2, 8, per_tensor=True)
    assert np.all(pt.v_range == pt.v_range[0]) and np.all(pt.filters.u_range == pt.filters.u_range[0])
    wide = base.v_range * np.float32(2)
    st = O.lance_conv(X, Wt, 1, 2, 8, static_v_range=wide)
    np.testing.assert_array_equal(st.v_range, wide)
    for r in (base, pt, st):
        assert np.linalg.norm(r.Y - Yd) / np.linalg.norm(Yd) < 0.05
