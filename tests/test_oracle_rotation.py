"""Pins for the oracle's permutation and block Hadamard rotation (CPU only).

Each test ties the oracle to something the paper or the mathematics fixes, not to itself.
"""
import math
import os

import numpy as np
import pytest
import scipy.linalg

from oracle import perq_oracle as orc

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _rng(seed):
    return np.random.default_rng(seed)


# ---- R: normalised Hadamard matrix (Notation, Section 1) --------------------------------
@pytest.mark.parametrize("k", [1, 2, 4, 16, 32, 128, 1024])
def test_hadamard_matrix_properties(k):
    H = orc.sylvester_hadamard(k)
    assert H.shape == (k, k)
    assert set(np.unique(H).tolist()) <= {-1, 1}
    assert np.array_equal(H @ H.T, k * np.eye(k, dtype=np.int64))     # orthogonal, exactly
    assert np.array_equal(H, H.T)
    assert np.all(H[0] == 1) and np.all(H[:, 0] == 1)
    # columns of R = H/sqrt(k): unit l2 norm, l_inf norm 1/sqrt(k)
    R = H / math.sqrt(k)
    assert np.allclose(np.linalg.norm(R, axis=0), 1.0, rtol=0, atol=1e-15)
    assert np.allclose(np.abs(R).max(axis=0), 1 / math.sqrt(k), rtol=0, atol=1e-17)
    # library construction and the closed form (-1)^popcount(i & j)
    assert np.array_equal(H, scipy.linalg.hadamard(k))
    if k <= 128:
        i, j = np.meshgrid(np.arange(k), np.arange(k), indexing="ij")
        pc = np.vectorize(lambda v: bin(v).count("1"))(i & j)
        assert np.array_equal(H, 1 - 2 * (pc % 2))


def test_hadamard_rejects_non_power_of_two():
    with pytest.raises(ValueError):
        orc.sylvester_hadamard(12)


# ---- P: (XP)_i = X_pi(i) with P e_i = e_pi(i) ------------------------------------------
def test_permutation_matches_matrix_definition():
    d = 12
    perm = _rng(1).permutation(d)
    P = np.zeros((d, d))
    for i in range(d):
        P[perm[i], i] = 1.0                 # column i of P is e_{pi(i)}
    X = _rng(2).standard_normal((5, d))
    assert np.array_equal(orc.permute_channels(X, perm), X @ P)
    assert np.array_equal(orc.permute_channels(np.array([[10., 20., 30.]]), [2, 0, 1]),
                          np.array([[30., 10., 20.]]))
    assert orc.permute_channels(X, None) is X
    inv = np.argsort(perm)
    assert np.array_equal(orc.permute_channels(orc.permute_channels(X, perm), inv), X)


# ---- R~ = I_n (x) R -----------------------------------------------------------------------
@pytest.mark.parametrize("d,b", [(64, 16), (256, 32), (256, 256), (1024, 128)])
def test_block_rotation_equals_kronecker_matrix(d, b):
    X = _rng(3).standard_normal((7, d))
    Rt = np.kron(np.eye(d // b), orc.sylvester_hadamard(b) / math.sqrt(b))
    assert np.allclose(orc.block_hadamard(X, b), X @ Rt, rtol=0, atol=1e-12)


@pytest.mark.parametrize("d,b", [(256, 16), (512, 64), (2048, 2048)])
def test_block_l2_preserved_and_involution(d, b):
    X = _rng(4).standard_t(3, size=(9, d))
    Y = orc.block_hadamard(X, b)
    nx = np.linalg.norm(X.reshape(9, d // b, b), axis=2)
    ny = np.linalg.norm(Y.reshape(9, d // b, b), axis=2)
    assert np.allclose(nx, ny, rtol=1e-12, atol=0)
    assert np.allclose(orc.block_hadamard(Y, b), X, rtol=0, atol=1e-11 * np.abs(X).max())


def test_one_hot_and_all_ones_closed_forms():
    d, b = 128, 32
    for pos, c in [(0, 3.0), (37, -2.5), (127, 7.0)]:
        X = np.zeros((1, d)); X[0, pos] = c
        Y = orc.block_hadamard(X, b)[0]
        j, r = divmod(pos, b)
        blk = Y[j * b:(j + 1) * b]
        assert np.allclose(np.abs(blk), abs(c) / math.sqrt(b), rtol=1e-15)
        # sign pattern is row r of the Sylvester matrix: (-1)^popcount(r & i)
        sgn = np.array([(-1) ** bin(r & i).count("1") for i in range(b)])
        assert np.array_equal(np.sign(blk), np.sign(c) * sgn)
        rest = np.delete(Y, np.s_[j * b:(j + 1) * b])
        assert np.all(rest == 0)
    Y = orc.block_hadamard(np.ones((1, d)), b)[0].reshape(d // b, b)
    assert np.allclose(Y[:, 0], math.sqrt(b)) and np.all(Y[:, 1:] == 0)


def test_full_vector_is_single_block():
    X = _rng(5).standard_normal((3, 512))
    H = orc.sylvester_hadamard(512) / math.sqrt(512)
    assert np.allclose(orc.block_hadamard(X, 512), X @ H, atol=1e-12)


# ---- Propositions 1, 2; Corollary 3.3 ----------------------------------------------------
def test_prop1_prop2_cor33_bounds():
    rng = _rng(6)
    d = 1024
    X = rng.standard_t(3, size=(64, d))
    X[:, [3, 99, 640]] *= 50
    Z = {}
    for b in [16, 32, 64, 128, 256, 512, 1024]:
        Y = orc.block_hadamard(X, b)
        l1 = np.abs(X).reshape(64, d // b, b).sum(axis=2)
        bound = l1.max(axis=1) / math.sqrt(b)                 # Prop. 2 right-hand side
        assert np.all(np.abs(Y).max(axis=1) <= bound * (1 + 1e-12))
        # ||X R~||_inf = max_j ||X_j R||_inf
        per_block = np.abs(Y).reshape(64, d // b, b).max(axis=2).max(axis=1)
        assert np.array_equal(per_block, np.abs(Y).max(axis=1))
        Z[b] = bound
        amax = np.abs(X).reshape(64, d // b, b).max(axis=2)
        delta_j = l1 / (b * amax)
        assert np.all(delta_j >= 1 / b - 1e-15) and np.all(delta_j <= 1 + 1e-15)
    # Prop. 1: b = d
    assert np.all(np.abs(orc.block_hadamard(X, d)).max(axis=1)
                  <= np.abs(X).sum(axis=1) / math.sqrt(d) * (1 + 1e-12))
    # Cor. 3.3: Z(b) <= sqrt(k) Z(b') for b = k b'
    for bp in [16, 32, 64]:
        for k in [2, 4, 8]:
            assert np.all(Z[bp * k] <= math.sqrt(k) * Z[bp] * (1 + 1e-12))


def test_prop4_random_signs_bound_holds_with_stated_probability():
    rng = _rng(7)
    d, b, eps = 512, 32, 0.05
    Yabs = np.abs(rng.standard_t(3, size=d)); Yabs[[5, 77]] *= 40
    S = rng.choice([-1.0, 1.0], size=(4000, d))
    X = S * Yabs
    out = np.abs(orc.block_hadamard(X, b)).max(axis=1)
    bound = math.sqrt(2.0 / b * math.log(2 * d / eps) * (Yabs ** 2).sum())
    tight = math.sqrt(2.0 / b * math.log(2 * d / eps) * (Yabs ** 2).reshape(-1, b).sum(axis=1).max())
    assert tight <= bound
    assert (out > tight).mean() <= eps
    assert (out > bound).mean() <= eps


# ---- butterfly cross-check and Table 3 ---------------------------------------------------
@pytest.mark.parametrize("d,b", [(256, 16), (512, 128), (4096, 4096), (14336 // 7, 2048)])
def test_butterfly_agrees_with_matrix_definition(d, b):
    X = _rng(8).standard_t(4, size=(4, d))
    A = orc.block_hadamard(X, b)
    B = orc.fwht_f64(X, b)
    assert np.allclose(A, B, rtol=0, atol=1e-12 * np.linalg.norm(X, axis=1).max())


def test_table3_addsub_counts():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table3_addsub_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 16
    for d, b, count in rows:
        d, b, count = int(d), int(b), int(count)
        assert d * int(math.log2(b)) == count
        ctr = [0]
        orc.fwht_f64(np.zeros((1, d)), b, counter=ctr)
        assert ctr[0] == count


# ---- non-power-of-two rotation (Appendix A.1) -------------------------------------------------
@pytest.mark.parametrize("m", [12, 28, 76])
def test_paley_base_is_hadamard(m):
    H = orc.paley_hadamard(m)
    assert H.shape == (m, m) and set(np.unique(H).tolist()) == {-1, 1}
    assert np.array_equal(H @ H.T, m * np.eye(m, dtype=np.int64))
    assert np.array_equal(H.T @ H, m * np.eye(m, dtype=np.int64))
    # type II matrices are symmetric; the type I matrix is the identity plus a skew matrix
    # whose first row is all ones
    if m == 12:
        assert np.array_equal(H + H.T, 2 * np.eye(m, dtype=np.int64))
        assert np.all(H[0] == 1) and np.all(H[1:, 0] == -1)
    else:
        assert np.array_equal(H, H.T)


def test_paley_residues_by_euler_criterion():
    # chi(x) = x^((q-1)/2) mod q, computed here with modular powers rather than a table of squares
    for m, q, two in [(12, 11, False), (28, 13, True), (76, 37, True)]:
        H = orc.paley_hadamard(m)
        for i in range(q):
            for j in range(q):
                if i == j:
                    continue
                chi = 1 if pow((i - j) % q, (q - 1) // 2, q) == 1 else -1
                got = H[2 * (1 + i), 2 * (1 + j)] if two else H[1 + i, 1 + j]
                assert got == chi


@pytest.mark.parametrize("b", [48, 96, 112, 224, 152])
def test_kronecker_rotation_equals_explicit_matrix(b):
    kp, m = orc.hadamard_factors(b)
    assert (1 << kp) * m == b
    H = orc.hadamard_matrix(b)
    assert np.array_equal(H @ H.T, b * np.eye(b, dtype=np.int64))
    base = orc.paley_hadamard(m)
    assert np.array_equal(H[:m, :m], base) and np.array_equal(H[m:2 * m, m:2 * m], -base if kp else base)
    X = _rng(b).standard_t(4, size=(5, 3 * b))
    want = (X.reshape(15, b) @ H.astype(np.float64) / math.sqrt(b)).reshape(5, 3 * b)
    got = orc.block_hadamard(X, b)
    assert np.allclose(got, want, rtol=0, atol=1e-12 * np.abs(X).sum(axis=1).max())
    # rotation: l2 norm of every block preserved, |y|_inf <= |x|_1 / sqrt(b) (Proposition 1)
    assert np.allclose((got.reshape(-1, b) ** 2).sum(1), (X.reshape(-1, b) ** 2).sum(1), rtol=1e-12)
    assert np.all(np.abs(got).reshape(-1, b).max(1) <= np.abs(X).reshape(-1, b).sum(1) / math.sqrt(b) * (1 + 1e-12))


def test_nonpo2_one_hot():
    # c e_i -> c times row i of H_b / sqrt(b): every output of the block has magnitude |c| / sqrt(b)
    b = 224
    H = orc.hadamard_matrix(b)
    for i in (0, 5, 27, 28, 223):
        x = np.zeros((1, 2 * b)); x[0, b + i] = 3.0
        y = orc.block_hadamard(x, b)
        assert np.all(y[0, :b] == 0)
        assert np.allclose(y[0, b:], 3.0 * H[i] / math.sqrt(b), rtol=0, atol=1e-15)
        assert np.allclose(np.abs(y[0, b:]), 3.0 / math.sqrt(b), rtol=1e-15)


def _printed(count, unit):
    return f"{count / (1e6 if unit == 'M' else 1e3):.2f}{unit}"


def test_appendix_a1_operation_counts():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "table4_nonpo2_counts.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 5
    for d, pieces, base, matmul, bfly_mm, ours, full in rows:
        d, pieces, base = int(d), int(pieces), int(base)
        kp, m = orc.hadamard_factors(d)
        assert (1 << kp, m) == (pieces, base)
        x = _rng(d).standard_normal(d)
        want = orc.block_hadamard(x[None, :], d)[0] * math.sqrt(d)
        tol = 1e-12 * np.abs(x).sum()
        ctr = [0]
        got = orc.nonpo2_rotation_counted(x, d, ctr)
        assert np.allclose(got, want, rtol=0, atol=tol)
        assert _printed(ctr[0], "K") == ours
        assert ctr[0] == d * (kp + m // 4 + 2)
        if full != "-":
            assert ctr[0] == int(full)
        ctr = [0]
        got = orc.nonpo2_rotation_counted(x, d, ctr, dense_base=True)
        assert np.allclose(got, want, rtol=0, atol=tol)
        assert _printed(ctr[0], "K") == bfly_mm
        assert _printed(d * (d - 1), "M") == matmul      # a dense product: d - 1 add/sub per output


def test_bf16_decode():
    bits = np.array([0x3F80, 0xBF80, 0x0000, 0x8000, 0x4049, 0x7F7F, 0x0001], dtype=np.uint16)
    want = [1.0, -1.0, 0.0, -0.0, 3.140625, 3.3895313892515355e38, 2.0 ** -133]
    got = orc.bf16_bits_to_f64(bits)
    assert np.array_equal(got, np.array(want))
    assert np.signbit(got[3])
