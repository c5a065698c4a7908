"""Pins for the oracle's quantizers, packing and column statistic (CPU only)."""
import math

import numpy as np
import pytest

from oracle import perq_oracle as orc


def _rng(seed):
    return np.random.default_rng(seed)


# ---- INT4 symmetric per token (Section 3; Eq. 4 with z = 0) ----------------------------
def test_int4_error_bounds_and_extremes():
    Y = _rng(1).standard_t(3, size=(50, 256))
    c, s = orc.quant_int4_sym_token(Y)
    assert c.min() >= -7 and c.max() <= 7
    dq = orc.dequant_int4(c, s)
    assert np.all(np.abs(Y - dq) <= s[:, None] / 2 * (1 + 1e-12))
    # Section 3: ||X - Q(X)||_2 <= sqrt(d)/(2^q - 2) ||X||_inf, q = 4
    assert np.all(np.linalg.norm(Y - dq, axis=1)
                  <= math.sqrt(256) / 14.0 * np.abs(Y).max(axis=1) * (1 + 1e-12))
    # the element that sets the scale gets +-7 and s = ||Y||_inf / 7
    arg = np.abs(Y).argmax(axis=1)
    assert np.all(np.abs(c[np.arange(50), arg]) == 7)
    assert np.allclose(s, np.abs(Y).max(axis=1) / 7.0, rtol=1e-16)


def test_int4_ties_go_to_even_and_zero_row():
    Y = np.array([[7.0, 0.5, 1.5, 2.5, 3.5, -0.5, -1.5, -2.5, 6.5, -6.5, 0.49999, 0.50001],
                  [0.0] * 12])
    c, s = orc.quant_int4_sym_token(Y)
    assert s[0] == 1.0 and s[1] == 0.0
    assert c[0].tolist() == [7, 0, 2, 2, 4, 0, -2, -2, 6, -6, 0, 1]
    assert np.all(c[1] == 0)


def test_int4_scale_and_sign_equivariance():
    Y = _rng(2).standard_normal((8, 64))
    c, s = orc.quant_int4_sym_token(Y)
    for k in (-140, -9, 3, 20, 100):         # down to magnitudes below the smallest normal fp32
        c2, s2 = orc.quant_int4_sym_token(np.ldexp(Y, k))
        assert np.array_equal(c, c2) and np.array_equal(np.ldexp(s, k), s2)
    c3, s3 = orc.quant_int4_sym_token(-Y)
    assert np.array_equal(c3, -c) and np.array_equal(s3, s)


def test_pack_nibbles_layout():
    codes = np.array([[1, -1, 7, -7, 0, 3, -8 + 1, 2]], dtype=np.int8)
    assert orc.pack_nibbles(codes).tolist() == [[0xF1, 0x97, 0x30, 0x29]]
    u = np.array([[0x0, 0xF, 0x8, 0x7]], dtype=np.uint8)
    assert orc.pack_nibbles(u).tolist() == [[0xF0, 0x78]]


# ---- MXFP4 (Appendix B: e = 2, m = 1, one power-of-two scale per 32) --------------------
def _e2m1_value_from_bits(code):
    """The e2m1 definition: 1 sign, 2 exponent bits with bias 1, 1 mantissa bit; exponent
    field 0 is subnormal."""
    s, e, m = (code >> 3) & 1, (code >> 1) & 3, code & 1
    mag = m * 0.5 if e == 0 else (1 + m / 2) * 2.0 ** (e - 1)
    return -mag if s else mag


def test_e2m1_table_matches_format_definition():
    for code in range(16):
        mag = orc.E2M1_GRID[code & 7]
        assert _e2m1_value_from_bits(code) == (-mag if code & 8 else mag)
    assert orc.E2M1_GRID.max() == 6.0


def _group(vals):
    g = np.zeros(32)
    g[:len(vals)] = vals
    return g[None, :]


def test_mxfp4_grid_points_and_tie_points():
    # group maximum 6 -> floor(log2 6) = 2 -> scale 2^(2-2) = 1, E = 127
    vals = [6, 0, 0.5, 1, 1.5, 2, 3, 4,              # grid points
            0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5,     # midpoints: even code wins
            -0.25, -0.75, -5, -6, -0.1,
            0.2499, 0.2501, 4.99, 5.01]
    want = [7, 0, 1, 2, 3, 4, 5, 6,
            0, 2, 2, 4, 4, 6, 6,
            0, 8 | 2, 8 | 6, 8 | 7, 0,
            0, 1, 6, 7]
    c, E = orc.quant_mxfp4(_group(vals))
    assert E.tolist() == [[127]]
    assert c[0, :len(vals)].tolist() == want


def test_mxfp4_scale_is_group_max_rounded_down_to_power_of_two():
    rng = _rng(3)
    Y = rng.standard_t(3, size=(40, 128)) * np.exp(rng.uniform(-20, 20, size=(40, 1)))
    c, E = orc.quant_mxfp4(Y)
    amax = np.abs(Y).reshape(40, 4, 32).max(axis=2)
    sc = np.ldexp(1.0, E.astype(int) - 127)
    assert np.all(4 * sc <= amax) and np.all(amax < 8 * sc)
    # saturation region (6, 8) * scale -> +-6
    c2, E2 = orc.quant_mxfp4(_group([7.9, -7.0, 6.01]))
    assert E2.tolist() == [[127]] and c2[0, :3].tolist() == [7, 15, 7]
    # exact powers of two at the boundary
    c3, E3 = orc.quant_mxfp4(_group([8.0, 4.0]))
    assert E3.tolist() == [[128]] and c3[0, :2].tolist() == [6, 4]       # 8/2 = 4, 4/2 = 2
    c4, E4 = orc.quant_mxfp4(_group([]))
    assert E4.tolist() == [[0]] and np.all(c4 == 0)


def test_mxfp4_error_bound_and_roundtrip():
    rng = _rng(4)
    Y = rng.standard_normal((30, 256)) * 3
    c, E = orc.quant_mxfp4(Y)
    dq = orc.dequant_mxfp4(c, E)
    sc = np.repeat(np.ldexp(1.0, E.astype(int) - 127), 32, axis=1)
    v = np.abs(Y) / sc
    spacing = np.where(v < 2, 0.5, np.where(v < 4, 1.0, 2.0))
    ok_in = (v <= 6) & (np.abs(Y - dq) <= spacing / 2 * sc * (1 + 1e-12))
    ok_sat = (v > 6) & (np.abs(Y - dq) < 2 * sc)
    assert np.all(ok_in | ok_sat)
    # values already on the grid come back exactly
    grid_vals = rng.choice(orc.E2M1_GRID, size=(10, 64)) * rng.choice([-1, 1], size=(10, 64))
    grid_vals[:, 0] = 6; grid_vals[:, 32] = -6
    g = grid_vals * 2.0 ** -5
    cg, Eg = orc.quant_mxfp4(g)
    assert np.array_equal(orc.dequant_mxfp4(cg, Eg), g)
    # power-of-two equivariance
    for k in (-30, 7):
        c2, E2 = orc.quant_mxfp4(np.ldexp(Y, k))
        assert np.array_equal(c2, c) and np.array_equal(E2.astype(int), E.astype(int) + k)


def test_mxfp4_rounding_agrees_with_piecewise_rint():
    """Independent formulation: the e2m1 grid is uniform with step 0.5 on [0,2), 1 on [2,4),
    2 on [4,6]; round-half-even on the step count equals ties-to-even-code."""
    a = np.abs(_rng(5).standard_normal(200000)) * 2.5
    a = np.concatenate([a, np.arange(0, 6.01, 0.125)])
    code = orc._round_to_e2m1_codes(a)
    sat = np.minimum(a, 6.0)
    val = np.where(sat < 2, np.rint(sat / 0.5) * 0.5,
                   np.where(sat < 4, np.rint(sat), np.rint(sat / 2) * 2))
    assert np.array_equal(orc.E2M1_GRID[code], val)


def test_mxfp4_group_is_32_contiguous_positions():
    Y = np.zeros((1, 64)); Y[0, 31] = 6.0; Y[0, 32] = 96.0; Y[0, 0] = 1.0; Y[0, 63] = 16.0
    c, E = orc.quant_mxfp4(Y)
    assert E.tolist() == [[127, 131]]
    assert c[0, [0, 31, 32, 63]].tolist() == [2, 7, 7, 2]


def test_mxfp4_exponent_clamp():
    c, E = orc.quant_mxfp4(_group([2.0 ** -140, 2.0 ** -141]))
    assert E.tolist() == [[0]]          # floor(log2) - 2 + 127 < 0 -> clamped
    assert c[0, 0] == 0


# ---- a_i (Algorithm 1, sort key) ---------------------------------------------------------
def test_colabs_mean_closed_forms():
    X = np.array([[1.0, -2.0, 0.0], [-3.0, 2.0, 0.5], [1.0, -2.0, -0.5], [-1.0, 2.0, 0.0]])
    assert orc.colabs_mean(X).tolist() == [1.5, 2.0, 0.25]
    R = _rng(6).standard_normal((100, 37))
    a = orc.colabs_mean(R)
    assert math.isclose(a.sum(), np.abs(R).sum(axis=1).mean(), rel_tol=1e-13)
    s = np.array([math.fsum(np.abs(R[:, i])) / 100 for i in range(37)])
    assert np.allclose(a, s, rtol=1e-14)
    C = np.sign(R) * np.arange(1, 38)
    assert np.allclose(orc.colabs_mean(C), np.arange(1, 38), rtol=1e-15)


# ---- whole path ---------------------------------------------------------------------------
@pytest.mark.parametrize("fmt", ["int4", "mxfp4"])
def test_end_to_end_reconstruction(fmt):
    """dequantised codes, rotated back and un-permuted, reproduce x within the format's bound."""
    from paper_2601_22347_amd import synth
    rng = _rng(7)
    d, b, T = 256, 32, 16
    bits = synth.f64_to_bf16_bits(rng.standard_normal((T, d)) * 2)
    perm = rng.permutation(d).astype(np.int32)
    out = orc.perq_apply(bits, perm, b, fmt)
    X = orc.bf16_bits_to_f64(bits)
    if fmt == "int4":
        dq = orc.dequant_int4(out["codes"], out["s64"])
        tol = out["s64"][:, None] / 2 * math.sqrt(d)
    else:
        dq = orc.dequant_mxfp4(out["codes"], out["scales"])
        tol = np.abs(out["y"]).max() * math.sqrt(d)
    back = orc.block_hadamard(dq, b)                # R~ is an involution
    rec = np.empty_like(back); rec[:, perm] = back
    assert np.all(np.linalg.norm(rec - X, axis=1) <= np.ravel(tol.max(axis=1) if tol.ndim > 1 else tol))
    assert np.allclose(np.linalg.norm(out["y"], axis=1), np.linalg.norm(X, axis=1), rtol=1e-12)
    assert out["packed"].shape == (T, d // 2)


# ---- INT4 asymmetric per token (Appendix B, INT4 paragraph) -----------------------------------
def _rint_fraction(q):
    """Round a Fraction to the nearest integer, ties to even (independent of numpy.rint)."""
    from fractions import Fraction
    fl = q.numerator // q.denominator
    r = q - fl
    if r > Fraction(1, 2) or (r == Fraction(1, 2) and fl % 2 == 1):
        return fl + 1
    return fl


def test_int4_asym_exact_rational_small_rows():
    """Integer-valued rows worked in exact rational arithmetic: step, zero point, codes."""
    from fractions import Fraction
    rng = _rng(11)
    for _ in range(40):
        row = rng.integers(-40, 60, size=12)
        if row.max() == row.min():
            continue
        lo, hi = int(row.min()), int(row.max())
        s = Fraction(hi - lo, 15)
        z = _rint_fraction(Fraction(lo) / s)
        want = [min(15, max(0, _rint_fraction(Fraction(int(v)) / s) - z)) for v in row]
        c, s64, z64 = orc.quant_int4_asym_token(row[None, :].astype(np.float64))
        assert z64[0] == z and abs(s64[0] - float(s)) <= 1e-15 * float(s)
        # a value whose quotient is an exact tie in rationals may sit a hair off it in floating
        # point; everything else must agree
        ties = [(Fraction(int(v)) / s - Fraction(1, 2)).denominator == 1 for v in row]
        for k in range(12):
            if not ties[k]:
                assert c[0, k] == want[k], (row, k)


def test_int4_asym_error_bound_end_codes_and_constant_row():
    Y = _rng(12).standard_t(3, size=(60, 128)) + _rng(13).uniform(-3, 3, size=(60, 1))
    c, s, z = orc.quant_int4_asym_token(Y)
    assert c.min() >= 0 and c.max() <= 15 and np.all(z == np.rint(z))
    assert np.allclose(s, (Y.max(axis=1) - Y.min(axis=1)) / 15.0, rtol=1e-16)
    dq = orc.dequant_int4_asym(c, s, z)
    assert np.all(np.abs(Y - dq) <= s[:, None] / 2 * (1 + 1e-9))
    rows = np.arange(60)
    assert np.all(c[rows, Y.argmin(axis=1)] == 0)
    assert np.all(c[rows, Y.argmax(axis=1)] >= 14)         # 15 unless min/s and max/s round apart
    # constant rows: no step, no information
    c0, s0, z0 = orc.quant_int4_asym_token(np.full((2, 8), 3.25))
    assert np.all(c0 == 0) and np.all(s0 == 0) and np.all(z0 == 0)


def test_int4_asym_offset_rows_with_a_small_spread():
    """Rows that are a large offset plus a small spread (zero points up to 15 * 2^24 in magnitude, the
    most an fp32 row allows): the quotients are large integers plus a fraction; the half-step error
    bound, the end codes and exact rational arithmetic still hold."""
    from fractions import Fraction
    rng = _rng(21)
    for offset, spread in ((1024.0, 2.0 ** -9), (-3.0e4, 2.0 ** -7), (1.0, 2.0 ** -20), (-7.0, 2.0 ** -18)):
        # dyadic values, so every quotient below is an exact rational of small height
        Y = offset + spread * np.rint(rng.uniform(-1, 1, size=(6, 64)) * 256) / 256
        c, s, z = orc.quant_int4_asym_token(Y)
        assert np.all(np.abs(z) > 1e5) and np.all(z == np.rint(z))
        dq = orc.dequant_int4_asym(c, s, z)
        assert np.all(np.abs(Y - dq) <= s[:, None] / 2 * (1 + 1e-6))
        rows = np.arange(6)
        assert np.all(c[rows, Y.argmin(axis=1)] == 0) and np.all(c[rows, Y.argmax(axis=1)] >= 14)
        for r in range(2):
            lo, hi = Fraction(float(Y[r].min())), Fraction(float(Y[r].max()))
            step = (hi - lo) / 15
            def rne(q):
                f = q.numerator // q.denominator
                rem = q - f
                return f + (1 if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and f % 2) else 0)
            zq = rne(lo / step)
            near_tie = False
            want = []
            for v in Y[r]:
                q = Fraction(float(v)) / step
                near_tie |= abs(abs(q - (q.numerator // q.denominator)) - Fraction(1, 2)) < Fraction(1, 10 ** 6)
                want.append(min(15, max(0, rne(q) - zq)))
            if not near_tie:           # fp64 decides a quotient of this size to about 1e-9 of a step
                assert int(z[r]) == zq and c[r].tolist() == want


def test_int4_asym_scale_shift_and_reflection():
    Y = _rng(14).standard_normal((10, 64))
    c, s, z = orc.quant_int4_asym_token(Y)
    for k in (-7, 5):
        c2, s2, z2 = orc.quant_int4_asym_token(np.ldexp(Y, k))
        assert np.array_equal(c, c2) and np.array_equal(np.ldexp(s, k), s2) and np.array_equal(z, z2)
    # moving a row by a whole number of steps moves the zero point, not the codes, wherever no
    # quotient is within rounding error of a tie
    Yq = np.rint(Y * 8) / 8                                   # dyadic values: shifts are exact
    cq, sq, zq = orc.quant_int4_asym_token(Yq)
    frac = np.abs((Yq / sq[:, None]) % 1.0 - 0.5)
    shift = 4 * sq
    cs, ss, zs = orc.quant_int4_asym_token(Yq + shift[:, None])
    ok = frac.min(axis=1) > 1e-9
    assert ok.sum() >= 5
    assert np.allclose(ss, sq, rtol=1e-12)
    assert np.array_equal(cs[ok], cq[ok]) and np.array_equal(zs[ok], zq[ok] + 4)
    # reflection: codes run the other way round when the two ends round to 15 steps apart
    cn, sn, zn = orc.quant_int4_asym_token(-Y)
    span = np.rint(Y.max(axis=1) / s) - np.rint(Y.min(axis=1) / s)
    good = span == 15
    assert good.sum() >= 5 and np.array_equal(cn[good], 15 - c[good])


def test_int4_asym_given_zero_point():
    Y = _rng(15).standard_normal((3, 32))
    c, s, z = orc.quant_int4_asym_token(Y)
    c1, _, z1 = orc.quant_int4_asym_token(Y, z_given=z + 1)
    assert np.array_equal(z1, z + 1)
    assert np.array_equal(c1, np.clip(c.astype(int) - 1, 0, 15))


# ---- FP4 with one scale per token (Appendix B, (MX)FP4 paragraph) -----------------------------
def test_fp4_token_reduces_to_mxfp4_when_max_is_6_times_power_of_two():
    rng = _rng(21)
    for k in (-5, 0, 9):
        Y = rng.uniform(-6, 6, size=(20, 32))
        Y[:, 3] = 6.0 * rng.choice([-1.0, 1.0], size=20)        # the row maximum, exactly 6
        Y = np.ldexp(Y, k)
        c, s = orc.quant_fp4_token(Y)
        cm, E = orc.quant_mxfp4(Y)
        assert np.all(s == 2.0 ** k) and np.all(E.astype(int) - 127 == k)
        assert np.array_equal(c, cm)


def test_fp4_token_grid_round_trip_error_bound_and_signs():
    rng = _rng(22)
    grid = orc.E2M1_GRID
    # rows made of grid values times a per-row constant, maximum 6: reproduced exactly
    idx = rng.integers(0, 8, size=(30, 64)); idx[:, 0] = 7
    sgn = rng.choice([-1.0, 1.0], size=(30, 64))
    cst = rng.uniform(0.1, 10, size=(30, 1))
    Y = grid[idx] * sgn * cst
    c, s = orc.quant_fp4_token(Y)
    assert np.allclose(s[:, None], cst, rtol=1e-15)
    assert np.allclose(orc.dequant_fp4_token(c, s), Y, rtol=1e-14, atol=0)
    assert np.all((c & 7)[idx == 0] == 0) and np.all((c & 8)[idx == 0] == 0)     # +0 only
    # generic rows: nothing saturates, the maximum takes the top code, error <= half the local spacing
    Y = rng.standard_t(3, size=(40, 96))
    c, s = orc.quant_fp4_token(Y)
    V = np.abs(Y) / s[:, None]
    assert V.max() <= 6 * (1 + 1e-15)
    assert np.all((c & 7)[np.arange(40), np.abs(Y).argmax(axis=1)] == 7)
    lo = grid[np.searchsorted(grid, np.minimum(V, 6.0), side="right") - 1]
    hi = grid[np.minimum(np.searchsorted(grid, np.minimum(V, 6.0), side="left"), 7)]
    half = np.where(hi > lo, (hi - lo) / 2, 0.0)
    err = np.abs(orc.dequant_fp4_token(c, s) - Y) / s[:, None]
    assert np.all(err <= half + 1e-12)
    # sign flip flips the sign bit of every non-zero code; power-of-two scaling keeps the codes
    c2, s2 = orc.quant_fp4_token(-Y)
    nz = (c & 7) != 0
    assert np.array_equal(c2[nz], c[nz] ^ 8) and np.array_equal(c2[~nz], c[~nz]) and np.array_equal(s, s2)
    c3, s3 = orc.quant_fp4_token(np.ldexp(Y, 6))
    assert np.array_equal(c3, c) and np.array_equal(s3, np.ldexp(s, 6))
    c0, s0 = orc.quant_fp4_token(np.zeros((1, 32)))
    assert np.all(c0 == 0) and s0[0] == 0


def test_apply_new_formats_shapes():
    x = np.random.default_rng(5).integers(0, 2 ** 16, size=(4, 64), dtype=np.uint16)
    x = np.where((x & 0x7F80) == 0x7F80, 0, x).astype(np.uint16)        # no inf / nan patterns
    r = orc.perq_apply(x, None, 16, "int4_asym")
    assert r["scales"].shape == (4, 2) and r["packed"].shape == (4, 32) and r["codes"].max() <= 15
    r = orc.perq_apply(x, None, 16, "fp4_token")
    assert r["scales"].shape == (4,) and r["packed"].shape == (4, 32)


# ---- merged weights and the W4A4 product (Remark "Merging Permutations", Section 4) -----------
def test_merged_weights_reproduce_the_unrotated_product():
    rng = _rng(31)
    d, N, b = 128, 24, 32
    X = rng.standard_normal((10, d))
    W = rng.standard_normal((d, N))
    perm = rng.permutation(d)
    Y = orc.block_hadamard(orc.permute_channels(X, perm), b)            # X P R~
    Wt = orc.merge_into_weights(W, perm, b)                             # (R~^T P^T W)^T
    assert np.allclose(Y @ Wt.T, X @ W, rtol=1e-12, atol=1e-12)
    # without the permutation on the weight side the product is a different one
    assert not np.allclose(Y @ orc.merge_into_weights(W, None, b).T, X @ W, atol=1e-3)


def test_w4a4_matmul_is_the_product_of_the_dequantised_operands():
    rng = _rng(32)
    ca = rng.integers(-7, 8, size=(9, 64)).astype(np.int8)
    cw = rng.integers(-7, 8, size=(5, 64)).astype(np.int8)
    sa, sw = rng.uniform(0.01, 2, size=9), rng.uniform(0.01, 2, size=5)
    acc, out = orc.w4a4_matmul(ca, sa, cw, sw)
    brute = [[sum(int(ca[t, i]) * int(cw[n, i]) for i in range(64)) for n in range(5)] for t in range(9)]
    assert acc.tolist() == brute
    assert np.allclose(out, orc.dequant_int4(ca, sa) @ orc.dequant_int4(cw, sw).T, rtol=1e-13)


def test_w4a4_end_to_end_error_is_quantisation_error_only():
    """Q(X P R~) Q(R~^T P^T W) stays within the product of the two INT4 error bounds of X W."""
    rng = _rng(33)
    d, N, b = 256, 16, 64
    X, W = rng.standard_normal((12, d)), rng.standard_normal((d, N))
    perm = rng.permutation(d)
    Y = orc.block_hadamard(orc.permute_channels(X, perm), b)
    Wt = orc.merge_into_weights(W, perm, b)
    ca, sa = orc.quant_int4_sym_token(Y)
    cw, sw = orc.quant_int4_sym_token(Wt)
    _, out = orc.w4a4_matmul(ca, sa, cw, sw)
    # |y~ w~ - y w| <= |dy||w| + |y||dw| + |dy||dw| with |dy|_2 <= sqrt(d) s_a / 2 etc.
    ey, ew = math.sqrt(d) * sa / 2, math.sqrt(d) * sw / 2
    ny, nw = np.linalg.norm(Y, axis=1), np.linalg.norm(Wt, axis=1)
    bound = ey[:, None] * nw[None, :] + ny[:, None] * ew[None, :] + ey[:, None] * ew[None, :]
    assert np.all(np.abs(out - X @ W) <= bound * (1 + 1e-12))


def test_mxfp4_product_of_hand_decoded_operands():
    # two rows of 32 against one: codes decoded by hand from the e2m1 definition (sign, 2-bit exponent
    # with bias 1, 1 mantissa bit; exponent field 0 is subnormal: 0 or 0.5), group scales 2^(E-127)
    def e2m1(c):
        s, e, m = (c >> 3) & 1, (c >> 1) & 3, c & 1
        v = (0.5 * m) if e == 0 else (1.0 + 0.5 * m) * 2.0 ** (e - 1)
        return -v if s else v
    rng = np.random.default_rng(4)
    ca, cw = rng.integers(0, 16, size=(2, 64)), rng.integers(0, 16, size=(1, 64))
    Ea, Ew = np.array([[120, 131], [127, 125]]), np.array([[126, 129]])
    want = np.zeros((2, 1))
    for t in range(2):
        for i in range(64):
            want[t, 0] += e2m1(int(ca[t, i])) * 2.0 ** (int(Ea[t, i // 32]) - 127) * \
                          e2m1(int(cw[0, i])) * 2.0 ** (int(Ew[0, i // 32]) - 127)
    got = orc.w4a4_mxfp4_matmul(ca.astype(np.uint8), Ea.astype(np.uint8), cw.astype(np.uint8), Ew.astype(np.uint8))
    assert np.array_equal(got, want)


# ---- per-token quantization error and the worst-case bound of Section 3 ----------------------------
def test_quant_error_hand_case_bound_and_tightness():
    # hand case, symmetric INT4: maximum 7 -> step 1; 0.25 -> 0, 2.6 -> 3, -1.5 -> -2 (tie to even), 7 -> 7
    Y = np.array([[0.25, 2.6, -1.5, 7.0]])
    e = orc.quant_error(Y, "int4")
    assert np.allclose(e[0], [math.sqrt(0.25 ** 2 + 0.4 ** 2 + 0.5 ** 2), math.sqrt((Y ** 2).sum()), 7.0], rtol=1e-14)
    # Section 3: ||Y - Q(Y)||_2 <= sqrt(d) / (2^q - 2) ||Y||_inf, q = 4, on heavy-tailed rows
    R = _rng(31).standard_t(3, size=(200, 96))
    e = orc.quant_error(R, "int4")
    assert np.all(e[:, 0] <= math.sqrt(96) / 14.0 * e[:, 2] * (1 + 1e-12))
    assert np.allclose(e[:, 1], np.linalg.norm(R, axis=1)) and np.array_equal(e[:, 2], np.abs(R).max(axis=1))
    # the bound is attained: every element half a step from its code (one element carries the maximum,
    # itself a tie: 7.5 steps would leave the alphabet, so it sits at 6.5 with another element at 7)
    d = 64
    T = np.full((1, d), 2.5); T[0, 0] = 7.0; T[0, 1::2] = -3.5
    e = orc.quant_error(T, "int4")[0]
    assert math.isclose(e[0], math.sqrt(d - 1) * 0.5, rel_tol=1e-14)           # all but the maximum are off by s/2
    assert e[0] <= math.sqrt(d) / 14.0 * 7.0 and e[0] >= 0.99 * math.sqrt(d) / 14.0 * 7.0
    # scale equivariance and the other quantizers: the error is that of the dequantized codes
    for fmt in ("int4", "mxfp4", "int4_asym", "fp4_token"):
        e1, e2 = orc.quant_error(R, fmt), orc.quant_error(R * 8.0, fmt)
        assert np.allclose(e2, 8.0 * e1, rtol=1e-13)
    c, E = orc.quant_mxfp4(R[:, :64])
    want = np.linalg.norm(R[:, :64] - orc.dequant_mxfp4(c, E), axis=1)
    assert np.allclose(orc.quant_error(R[:, :64], "mxfp4")[:, 0], want, rtol=1e-14)
    # asymmetric INT4 has 16 levels over the range: half a step of (max - min)/15 per element
    ea = orc.quant_error(R, "int4_asym")
    rng_ = R.max(axis=1) - R.min(axis=1)
    assert np.all(ea[:, 0] <= math.sqrt(96) * rng_ / 30.0 * (1 + 1e-9))
    # a row that is exactly representable has no error
    G = np.array([[7.0, -3.0, 0.0, 1.0, 2.0, -7.0, 5.0, 4.0]])
    assert orc.quant_error(G, "int4")[0, 0] == 0.0




def test_fp4_token_with_the_printed_constant_saturates_the_top_of_the_row():
    """Appendix B prints s = ||Y||_inf / (2^(q-1) - 1) for FP4 as well: the row maximum then sits at 7
    steps, past the largest e2m1 magnitude, and saturates together with everything above 6.5."""
    Y = np.array([[7.0, -6.6, 6.4, 5.0, 0.2, -0.26, 3.5, 2.5]])
    c, s = orc.quant_fp4_token(Y, 7.0)
    assert s[0] == 1.0
    # 7 -> 6 (saturated), -6.6 -> -6, 6.4 -> 6, 5 -> 4 (tie to even), 0.2 -> 0, -0.26 -> -0.5, 3.5 -> 4, 2.5 -> 2
    assert [float(orc.dequant_fp4_token(c, s)[0, i]) for i in range(8)] == [6.0, -6.0, 6.0, 4.0, 0.0, -0.5, 4.0, 2.0]
    R = _rng(33).standard_t(3, size=(50, 64))
    c7, s7 = orc.quant_fp4_token(R, 7.0)
    assert np.allclose(s7 * 7.0, np.abs(R).max(axis=1), rtol=1e-15)
    arg = np.abs(R).argmax(axis=1)
    assert np.all((c7[np.arange(50), arg] & 7) == 7)                   # the maximum saturates to +-6
    dq = orc.dequant_fp4_token(c7, s7)
    assert np.all(np.abs(R - dq) <= s7[:, None] * (1 + 1e-12))           # at most one step (the saturated top)
    e7 = orc.quant_error(R, "fp4_token7")
    assert np.allclose(e7[:, 0], np.linalg.norm(R - dq, axis=1), rtol=1e-14)
