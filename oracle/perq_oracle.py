"""CPU oracle for PeRQ's online activation path.  TEST INFRASTRUCTURE ONLY.

This file is the checker, not the product: only the test-suite, the smoke check and the
benchmark's CPU-baseline leg may import it.  It shares no code, table or constant with the
HIP library, and it never receives a value that the HIP library produced.

What it computes, in the paper's order and notation (row-vector activations X in R^d,
d = n*b, Notation paragraph of Section 1):

    X  --P-->  XP  --R~ = I_n (x) R-->  XP R~  --Q-->  codes, scales

  * P   : channel permutation, (XP)_i = X_{pi(i)}            (Notation, Section 1)
  * R   : normalised b x b Hadamard matrix, entries +-1/sqrt(b) (Notation, Section 1;
          butterfly form for powers of two in Remark A.1 -- here the plain matrix)
  * Q   : INT4, symmetric, step s = ||.||_inf / (2^(q-1) - 1), q = 4   (Section 3, Eq. 4
          with z = 0), one step per token;  or MXFP4: e2m1 elements (e = 2, m = 1) with one
          power-of-two scale per group of 32, rounded down             (Appendix B, Eq. 5)
  * calibration: a_i = (1/m) sum_k |X_i^(k)| and the greedy mass-diffusion permutation
          (Algorithm 1)

Everything is float64 NumPy.  The rotation is the *definition* (an explicit Sylvester matrix
product), not a fast transform; rounding is half-to-even (numpy.rint).  Readings of points
the paper leaves open are listed next to each function and collected in the design notes.

Pins (tests/test_oracle_*.py, run without a GPU): Hadamard orthogonality and SciPy's
construction, per-block l2 preservation, one-hot / all-ones closed forms, involution,
Propositions 1, 2 and 4 and Corollary 3.3, Table 3's add/sub counts via an instrumented
butterfly, the Section 3 worst-case INT-q error bound, the e2m1 grid/tie table by brute
force, scale equivariance, closed forms and brute-force optimum for the greedy; for the two
per-token quantizers of Appendix B (asymmetric INT4, FP4) exact rational arithmetic on small
rows, the half-step error bound, end codes, and the reduction of FP4 to the MXFP4 routine
when the row maximum is 6 * 2^k; for the non-power-of-two rotation of Appendix A.1 (base
matrix by Paley's constructions, a stated reading) orthogonality, the quadratic character by
Euler's criterion, the Kronecker form against the written-out matrix, and the operation counts
that the appendix's second table and Table 3's "Full" column print, reproduced by a staged
evaluation that counts its additions and subtractions.
"""
from __future__ import annotations

import itertools
import math

import numpy as np

__all__ = [
    "bf16_bits_to_f64", "sylvester_hadamard", "permute_channels", "block_hadamard",
    "paley_hadamard", "hadamard_factors", "hadamard_matrix", "nonpo2_rotation_counted",
    "quant_int4_sym_token", "quant_mxfp4", "pack_nibbles", "E2M1_GRID",
    "quant_int4_asym_token", "dequant_int4_asym", "quant_fp4_token", "dequant_fp4_token",
    "merge_into_weights", "w4a4_matmul", "w4a4_mxfp4_matmul", "colabs_max", "perm_sorted_desc", "perm_zigzag", "block_diagnostics", "quant_error", "splitmix64", "perm_random",
    "dequant_int4", "dequant_mxfp4", "colabs_mean", "massdiff_greedy",
    "block_masses", "brute_force_min_max_block_mass", "fwht_f64", "perq_apply",
]


# ----------------------------------------------------------------------------------------
# input decoding
# ----------------------------------------------------------------------------------------
def bf16_bits_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 bit patterns (uint16) -> float64, exactly.

    bfloat16 is the upper half of an IEEE binary32, so the value is obtained by placing the
    16 bits in the high half of a 32-bit word; binary32 -> binary64 is exact.
    """
    bits = np.ascontiguousarray(bits, dtype=np.uint16)
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32).astype(np.float64)


# ----------------------------------------------------------------------------------------
# P and R~   (Notation paragraph, Section 1)
# ----------------------------------------------------------------------------------------
def sylvester_hadamard(k: int) -> np.ndarray:
    """Unnormalised k x k Hadamard matrix of +-1 (int64), k a power of two.

    Sylvester's recursion H_1 = [1], H_2k = [[H_k, H_k], [H_k, -H_k]].  The paper only says
    "normalized Hadamard matrix" with columns of unit l2 norm and l_inf norm 1/sqrt(k); the
    reading taken is the Sylvester matrix in natural order with no random sign diagonal.
    """
    if k < 1 or (k & (k - 1)) != 0:
        raise ValueError("k must be a power of two")
    H = np.array([[1]], dtype=np.int64)
    while H.shape[0] < k:
        H = np.block([[H, H], [H, -H]])
    return H


def permute_channels(X: np.ndarray, perm) -> np.ndarray:
    """XP with (XP)_i = X_{perm[i]}  (P e_i = e_{pi(i)} acting on a row vector).

    `perm` is the concatenation [B_1, ..., B_n] that Algorithm 1 returns: perm[j*b + k] is
    the k-th channel placed in block j.  None means P = I.
    """
    if perm is None:
        return X
    perm = np.asarray(perm)
    return X[:, perm]


def _quadratic_character(q: int) -> np.ndarray:
    """chi(x) for x in Z_q, q an odd prime: 0 at 0, +1 on non-zero squares, -1 otherwise."""
    if q < 3 or any(q % p == 0 for p in range(2, int(math.isqrt(q)) + 1)):
        raise ValueError("q must be an odd prime")
    chi = -np.ones(q, dtype=np.int64)
    chi[0] = 0
    for x in range(1, q):
        chi[(x * x) % q] = 1
    return chi


def paley_hadamard(m: int) -> np.ndarray:
    """Unnormalised m x m Hadamard matrix (+-1, int64) for the non-power-of-two base, m = 4t.

    Appendix A.1 builds the full rotation from a 4t-dimensional base matrix but does not
    print one (the Llama3-8B example needs 28, the Qwen3 widths 12 and 76).  The reading
    taken: Paley's constructions over the prime field Z_q, with the Jacobsthal matrix
    Q[i][j] = chi(i - j):
      * type I  when q = m - 1 is a prime with q = 3 (mod 4):  H = I + S,
                S = [[0, 1^T], [-1, Q]]  (S is skew, S S^T = q I);            m = 12 (q = 11)
      * type II when q = m/2 - 1 is a prime with q = 1 (mod 4): S = [[0, 1^T], [1, Q]]
                (symmetric), every 0 of S becomes [[1, -1], [-1, -1]] and every entry
                e = +-1 becomes e * [[1, 1], [1, -1]];                m = 28 (q = 13), 76 (q = 37)
    Type I is tried first.  Any Hadamard matrix satisfies what the paper proves about the
    rotation (Propositions 1 and 2 use only that entries are +-1/sqrt(d) and rows orthogonal).
    """
    def is_prime(q):
        return q >= 2 and all(q % p for p in range(2, int(math.isqrt(q)) + 1))

    if m % 4 != 0 or m < 8:
        raise ValueError("m must be a multiple of four, at least 8")
    if is_prime(m - 1) and (m - 1) % 4 == 3:
        q = m - 1
        chi = _quadratic_character(q)
        S = np.zeros((m, m), dtype=np.int64)
        S[0, 1:] = 1
        S[1:, 0] = -1
        for i in range(q):
            for j in range(q):
                S[1 + i, 1 + j] = chi[(i - j) % q]
        return np.eye(m, dtype=np.int64) + S
    if is_prime(m // 2 - 1) and (m // 2 - 1) % 4 == 1:
        q = m // 2 - 1
        chi = _quadratic_character(q)
        S = np.zeros((q + 1, q + 1), dtype=np.int64)
        S[0, 1:] = 1
        S[1:, 0] = 1
        for i in range(q):
            for j in range(q):
                S[1 + i, 1 + j] = chi[(i - j) % q]
        zero_cell = np.array([[1, -1], [-1, -1]], dtype=np.int64)
        unit_cell = np.array([[1, 1], [1, -1]], dtype=np.int64)
        H = np.zeros((m, m), dtype=np.int64)
        for i in range(q + 1):
            for j in range(q + 1):
                H[2 * i:2 * i + 2, 2 * j:2 * j + 2] = zero_cell if S[i, j] == 0 else S[i, j] * unit_cell
        return H
    raise ValueError(f"no Paley construction over a prime field for order {m}")


def hadamard_factors(b: int):
    """b -> (k', m): R_b is k' Sylvester doublings of an m x m base (Appendix A.1).

    b = k * t with t the odd part; t = 1 gives the pure Sylvester matrix (returned as
    (log2 b, 1)); otherwise the base has m = 4t rows and k' = log2(k) - 2.
    """
    if b < 1:
        raise ValueError("b must be positive")
    t = b
    while t % 2 == 0:
        t //= 2
    k = b // t
    if t == 1:
        return int(math.log2(b)), 1
    if k < 4:
        raise ValueError("a Hadamard order above 2 is a multiple of four")
    return int(math.log2(k)) - 2, 4 * t


def hadamard_matrix(b: int) -> np.ndarray:
    """Unnormalised b x b matrix H_{2^k'} (x) H_m written out (int64); for small b."""
    kp, m = hadamard_factors(b)
    H = np.array([[1]], dtype=np.int64) if m == 1 else paley_hadamard(m)
    for _ in range(kp):
        H = np.block([[H, H], [H, -H]])
    return H


def block_hadamard(X: np.ndarray, b: int) -> np.ndarray:
    """X R~ with R~ = I_n (x) R, R = H_b / sqrt(b); X is [T, d], d = n*b, float64.

    Written as the definition: each b-wide block of each row is multiplied by the explicit
    matrix, then scaled by 1/sqrt(b) (the normalisation is applied after the +-1 sums).
    When b is not a power of two, H_b = H_{2^k'} (x) H_m (Appendix A.1: k' doublings of the
    4t-dimensional base) and the product is taken one Kronecker factor at a time -- with the
    block viewed as a [2^k', m] array Z, that is H_{2^k'} Z H_m (the Sylvester factor is
    symmetric); `hadamard_matrix` writes the same matrix out for the sizes a test can hold.
    """
    T, d = X.shape
    if d % b != 0:
        raise ValueError("b must divide d")
    kp, m = hadamard_factors(b)
    if m == 1:
        H = sylvester_hadamard(b).astype(np.float64)
        Y = (X.reshape(T * (d // b), b) @ H) / math.sqrt(b)
        return Y.reshape(T, d)
    A = 1 << kp
    HA = sylvester_hadamard(A).astype(np.float64)
    Hm = paley_hadamard(m).astype(np.float64)
    Z = X.reshape(T * (d // b), A, m)
    Y = np.matmul(HA, np.matmul(Z, Hm)) / math.sqrt(b)
    return Y.reshape(T, d)


def nonpo2_rotation_counted(x: np.ndarray, b: int, counter: list, dense_base: bool = False) -> np.ndarray:
    """One row through the staged non-power-of-two rotation of Appendix A.1, counting add/sub.

    x is one b-dimensional vector (float64), b = 2^k' * 4t.  Steps, in the appendix's order:
    k' radix-2 butterfly stages over the index that counts the 4t-wide pieces, then one
    4t-dimensional rotation per piece.  With dense_base the piece is multiplied by the base
    matrix directly (4t - 1 add/sub per output: the "butterfly + matmul" column of the
    appendix's second table).  Otherwise every group of four adjacent inputs first yields
    its sums and differences -- two stages, (a+-b, c+-d) then the eight combinations
    (a+-b)+-(c+-d), which are all sign patterns of four terms up to a common sign -- and
    each output then adds or subtracts one of these per group, t terms.  counter[0]
    accumulates the number of additions and subtractions.  Returns x H_b (unnormalised).
    """
    kp, m = hadamard_factors(b)
    if m == 1:
        raise ValueError("power-of-two sizes use the plain butterfly")
    t = m // 4
    H = paley_hadamard(m)
    v = np.array(x, dtype=np.float64).reshape(1 << kp, m)
    h = 1
    while h < (1 << kp):
        w = v.reshape((1 << kp) // (2 * h), 2, h, m)
        v = np.stack([w[:, 0] + w[:, 1], w[:, 0] - w[:, 1]], axis=1).reshape(1 << kp, m)
        counter[0] += b
        h *= 2
    out = np.empty_like(v)
    for piece in range(1 << kp):
        z = v[piece]
        if dense_base:
            for i in range(m):
                acc = H[0, i] * z[0]
                for r in range(1, m):
                    acc = acc + z[r] if H[r, i] > 0 else acc - z[r]
                    counter[0] += 1
                out[piece, i] = acc
            continue
        combos = []
        for g in range(t):
            a_, b_, c_, d_ = z[4 * g:4 * g + 4]
            p, q_, r_, s_ = a_ + b_, a_ - b_, c_ + d_, c_ - d_
            counter[0] += 4
            # keyed by the signs of (b, c, d) relative to a
            table = {(1, 1, 1): p + r_, (1, -1, -1): p - r_, (1, 1, -1): p + s_, (1, -1, 1): p - s_,
                     (-1, 1, 1): q_ + r_, (-1, -1, -1): q_ - r_, (-1, 1, -1): q_ + s_, (-1, -1, 1): q_ - s_}
            counter[0] += 8
            combos.append(table)
        for i in range(m):
            acc = None
            for g in range(t):
                col = H[4 * g:4 * g + 4, i]
                lead = int(col[0])
                term = combos[g][(int(col[1]) * lead, int(col[2]) * lead, int(col[3]) * lead)]
                if acc is None:
                    acc = term if lead > 0 else -term      # a sign on the first term is not an add/sub
                else:
                    acc = acc + term if lead > 0 else acc - term
                    counter[0] += 1
            out[piece, i] = acc
    return out.reshape(b)


def fwht_f64(X: np.ndarray, b: int, counter: list | None = None) -> np.ndarray:
    """Second, independent evaluation of X R~: radix-2 butterflies in float64 (Remark A.1).

    Used only (i) as a cross-check of `block_hadamard` and (ii) where the explicit product
    is too slow (b >= 2048 on all rows), after being validated against it on a subset.
    `counter`, if given, is a one-element list that accumulates the number of additions and
    subtractions performed per row -- the quantity tabulated in Table 3.
    """
    T, d = X.shape
    Y = np.array(X, dtype=np.float64, copy=True).reshape(T, d // b, b)
    h = 1
    while h < b:
        Z = Y.reshape(T, d // b, b // (2 * h), 2, h)
        lo = Z[:, :, :, 0, :] + Z[:, :, :, 1, :]
        hi = Z[:, :, :, 0, :] - Z[:, :, :, 1, :]
        Y = np.stack([lo, hi], axis=3).reshape(T, d // b, b)
        if counter is not None:
            counter[0] += d          # d/2 additions + d/2 subtractions per row per stage
        h *= 2
    return (Y / math.sqrt(b)).reshape(T, d)


# ----------------------------------------------------------------------------------------
# Q: INT4, symmetric, one step size per token   (Section 3; Appendix B, Eq. 4 with z = 0)
# ----------------------------------------------------------------------------------------
def quant_int4_sym_token(Y: np.ndarray):
    """Returns (codes int8 [T,d] in [-7, 7], s float64 [T]).

    s = ||Y_t||_inf / (2^(q-1) - 1) with q = 4; code = clip(round_half_even(Y / s), -7, 7).
    An all-zero row has s = 0 and all codes 0 (the paper is silent; 0/0 is read as 0).
    The scale handed to a consumer is float32(s).
    """
    amax = np.abs(Y).max(axis=1)
    s = amax / 7.0
    safe = np.where(s > 0.0, s, 1.0)
    V = Y / safe[:, None]
    codes = np.clip(np.rint(V), -7, 7).astype(np.int8)
    codes[s == 0.0, :] = 0
    return codes, s


def dequant_int4(codes: np.ndarray, s: np.ndarray) -> np.ndarray:
    return codes.astype(np.float64) * np.asarray(s, dtype=np.float64)[:, None]


# ----------------------------------------------------------------------------------------
# Q: MXFP4   (Appendix B, Eq. 5: e = 2, m = 1; one power-of-two scale per 32, rounded down)
# ----------------------------------------------------------------------------------------
# e2m1 magnitudes by 3-bit code: 1 sign bit, 2 exponent bits (bias 1), 1 mantissa bit,
# exponent field 0 is subnormal (0 and 0.5).
E2M1_GRID = np.array([0.0, 0.5, 1.0, 1.5, 2.0, 3.0, 4.0, 6.0], dtype=np.float64)
_E2M1_EMAX = 2          # 6 = 1.5 * 2^2
_E8M0_BIAS = 127


def _round_to_e2m1_codes(A: np.ndarray) -> np.ndarray:
    """Nearest e2m1 magnitude code for non-negative A; ties go to the even code (mantissa
    bit 0); anything above 6 saturates to 6 (it is its nearest grid point)."""
    dist = np.abs(A[..., None] - E2M1_GRID)                  # [..., 8]
    best = dist.min(axis=-1, keepdims=True)
    is_best = dist == best
    even = (np.arange(8) % 2 == 0)
    # prefer an even code among the (at most two) nearest ones
    pick_even = is_best & even
    has_even = pick_even.any(axis=-1)
    code = np.where(has_even, pick_even.argmax(axis=-1), is_best.argmax(axis=-1))
    return code.astype(np.uint8)


def quant_mxfp4(Y: np.ndarray, E_given: np.ndarray | None = None):
    """Returns (codes uint8 [T,d], 4-bit sign|exp|mant; E uint8 [T, d/32], biased e8m0).

    Per group of 32 contiguous outputs of the (permuted, rotated) row:
      shared scale 2^(E-127) with E-127 = floor(log2 ||group||_inf) - 2, i.e. the group maximum
      rounded down to a power of two and divided by the largest e2m1 power of two (2^2);
      E is clamped to [0, 254]; an all-zero group has E = 0.
      element code = round-to-nearest-even of y / 2^(E-127) on the e2m1 grid, saturating at 6;
      zero is always emitted as +0.
    Reading: the appendix's printed scale formula is inconsistent with its own sentence before
    it (the group maximum goes down to the next power of two) and with the OCP format it says it
    follows; the sentence and the format are taken.

    `E_given` (uint8 [T, d/32]) replaces the computed exponents; the parity tests use it to
    check the codes of a group whose maximum sits on a power-of-two boundary.
    """
    T, d = Y.shape
    if d % 32 != 0:
        raise ValueError("MXFP4 needs d % 32 == 0")
    G = Y.reshape(T, d // 32, 32)
    amax = np.abs(G).max(axis=2)
    mant, expo = np.frexp(amax)                      # amax = mant * 2^expo, mant in [0.5, 1)
    floor_log2 = expo.astype(np.int64) - 1
    E = floor_log2 - _E2M1_EMAX + _E8M0_BIAS
    E = np.where(amax > 0.0, E, 0)
    E = np.clip(E, 0, 254).astype(np.int64)
    if E_given is not None:
        E = np.asarray(E_given).astype(np.int64).reshape(T, d // 32)
    V = np.ldexp(G, -(E - _E8M0_BIAS)[:, :, None].astype(np.int64))
    mag = _round_to_e2m1_codes(np.abs(V))
    sign = ((V < 0.0) & (mag != 0)).astype(np.uint8)
    codes = (sign << 3) | mag
    return codes.reshape(T, d), E.astype(np.uint8)


def dequant_mxfp4(codes: np.ndarray, E: np.ndarray) -> np.ndarray:
    T, d = codes.shape
    mag = E2M1_GRID[codes & 7]
    val = np.where((codes & 8) != 0, -mag, mag).reshape(T, d // 32, 32)
    return np.ldexp(val, (E.astype(np.int64) - _E8M0_BIAS)[:, :, None]).reshape(T, d)


# ----------------------------------------------------------------------------------------
# Q: INT4, asymmetric, one step size and zero point per token   (Appendix B, INT4 paragraph)
# ----------------------------------------------------------------------------------------
def quant_int4_asym_token(Y: np.ndarray, z_given: np.ndarray | None = None):
    """Returns (codes uint8 [T,d] in [0, 15], s float64 [T], z float64 [T], integer valued).

    Appendix B: s = (max(Y_t) - min(Y_t)) / (2^q - 1), zero point z = min(Y_t) / s, q = 4, and
    Eq. 4 rounds Y/s before it subtracts z, so the alphabet is met only with an integer z.
    Reading: z = round_half_even(min / s); code = clip(round_half_even(Y / s) - z, 0, 15);
    the value a code stands for is s * (code + z)  (Eq. 4 with its last term read as s * z).
    A constant row has s = 0; then z = 0 and all codes are 0 (the paper is silent).

    `z_given` replaces the computed zero points; the parity tests use it for a row whose
    min / s sits on a rounding boundary.
    """
    lo = Y.min(axis=1)
    hi = Y.max(axis=1)
    s = (hi - lo) / 15.0
    safe = np.where(s > 0.0, s, 1.0)
    z = np.where(s > 0.0, np.rint(lo / safe), 0.0)
    if z_given is not None:
        z = np.asarray(z_given, dtype=np.float64)
    codes = np.clip(np.rint(Y / safe[:, None]) - z[:, None], 0, 15)
    codes[s == 0.0, :] = 0
    return codes.astype(np.uint8), s, z


def dequant_int4_asym(codes: np.ndarray, s: np.ndarray, z: np.ndarray) -> np.ndarray:
    return (codes.astype(np.float64) + np.asarray(z, dtype=np.float64)[:, None]) * np.asarray(s, dtype=np.float64)[:, None]


# ----------------------------------------------------------------------------------------
# Q: FP4 (e2m1) with one real-valued scale per token   (Appendix B, (MX)FP4 paragraph)
# ----------------------------------------------------------------------------------------
def quant_fp4_token(Y: np.ndarray, c: float = 6.0):
    """Returns (codes uint8 [T,d], 4-bit sign|exp|mant; s float64 [T]).

    Appendix B: FP4 activations take one scale per token, s = ||Y_t||_inf / c, z = 0, and the
    elements are rounded (nearest, ties to the even code) onto the e2m1 grid.
    Reading of c: the appendix prints c = 2^(q-1) - 1 = 7, the integer quantizer's constant,
    which is not an e2m1 value; with it the row maximum lands on 7 and saturates to 6, as does
    everything above 6.5.  The default takes the largest magnitude of the alphabet, c = 6, so the
    row maximum maps onto the largest code; c = 7 is the formula as printed (format "fp4_token7").
    An all-zero row has s = 0 and all codes 0; zero is always emitted as +0.
    """
    amax = np.abs(Y).max(axis=1)
    s = amax / c
    safe = np.where(s > 0.0, s, 1.0)
    V = Y / safe[:, None]
    mag = _round_to_e2m1_codes(np.abs(V))
    sign = ((V < 0.0) & (mag != 0)).astype(np.uint8)
    codes = (sign << 3) | mag
    codes[s == 0.0, :] = 0
    return codes.astype(np.uint8), s


def dequant_fp4_token(codes: np.ndarray, s: np.ndarray) -> np.ndarray:
    mag = E2M1_GRID[codes & 7]
    return np.where((codes & 8) != 0, -mag, mag) * np.asarray(s, dtype=np.float64)[:, None]



def pack_nibbles(codes: np.ndarray) -> np.ndarray:
    """[T, d] 4-bit codes -> [T, d/2] bytes; element 2k in the low nibble, 2k+1 in the high.

    Signed INT4 codes are stored in two's complement (code & 0xF).  The paper never packs
    (it fake-quantises); this is the storage convention of the library under test.
    """
    u = (codes.astype(np.int16) & 0xF).astype(np.uint8)
    return (u[:, 0::2] | (u[:, 1::2] << 4)).astype(np.uint8)


# ----------------------------------------------------------------------------------------
# calibration   (Algorithm 1)
# ----------------------------------------------------------------------------------------
def colabs_mean(X: np.ndarray) -> np.ndarray:
    """a_i = (1/m) sum_k |X_i^(k)|  -- the sort key of Algorithm 1, X is [m, d] float64."""
    return np.abs(X).sum(axis=0) / X.shape[0]


def massdiff_greedy(a, b: int) -> np.ndarray:
    """Algorithm 1 (mass diffusion) on the per-channel means `a`; returns perm int32[d].

    Channels are visited in descending order of a (equal values: lower channel first) and each
    goes to the block, among those not yet full, whose accumulated mass is smallest (equal
    masses: lowest block index).  The candidate-dependent term |X_i| in the algorithm's argmin
    is the same for every block, and the mean of block l1 norms is the sum of the block's
    a-values, so the data enter only through a.  Blocks keep insertion order and are
    concatenated in block order.
    """
    a = np.asarray(a, dtype=np.float64)
    d = a.shape[0]
    if d % b != 0:
        raise ValueError("b must divide d")
    n = d // b
    order = np.argsort(-a, kind="stable")
    mass = [0.0] * n
    blocks = [[] for _ in range(n)]
    for i in order:
        j_star = -1
        for j in range(n):
            if len(blocks[j]) == b:
                continue
            if j_star < 0 or mass[j] < mass[j_star]:
                j_star = j
        blocks[j_star].append(int(i))
        mass[j_star] += float(a[i])
    return np.array([i for blk in blocks for i in blk], dtype=np.int32)


def block_masses(a, perm, b: int) -> np.ndarray:
    """L_j = sum_{i in B_j} a_i for the blocks of `perm` (None = identity)."""
    a = np.asarray(a, dtype=np.float64)
    ap = a if perm is None else a[np.asarray(perm)]
    return ap.reshape(-1, b).sum(axis=1)


def brute_force_min_max_block_mass(a, b: int) -> float:
    """min over all partitions of the channels into d/b blocks of size b of max_j L_j.
    Exhaustive; tiny d only."""
    a = [float(v) for v in a]
    d = len(a)
    best = [math.inf]

    def rec(remaining, cur_max):
        if not remaining:
            best[0] = min(best[0], cur_max)
            return
        first, rest = remaining[0], remaining[1:]
        for others in itertools.combinations(rest, b - 1):
            m = a[first] + sum(a[i] for i in others)
            if max(m, cur_max) >= best[0]:
                continue
            left = [i for i in rest if i not in others]
            rec(left, max(m, cur_max))

    rec(list(range(d)), 0.0)
    return best[0]


# ----------------------------------------------------------------------------------------
# alternative permutations of the ablation (Appendix C, "Permutations") and the quantities of
# Propositions 1, 2 and Corollary 3.3 per token
# ----------------------------------------------------------------------------------------
def colabs_max(X: np.ndarray) -> np.ndarray:
    """Per-channel l_inf over the calibration tokens: the statistic of "absmax" and ZigZag."""
    return np.abs(X).max(axis=0)


def perm_sorted_desc(stat) -> np.ndarray:
    """"absmax": coordinates in descending order of the statistic (stable: lower channel first)."""
    stat = np.asarray(stat, dtype=np.float64)
    return np.argsort(-stat, kind="stable").astype(np.int32)


def perm_zigzag(stat, b: int) -> np.ndarray:
    """ZigZag.  The paper only names the strategy (coordinates sorted by their l_inf and dealt to
    the blocks in a zigzag) and cites it; reading: rank r of the stable descending order goes to
    block r mod n on even rounds floor(r / n) and to block n - 1 - (r mod n) on odd rounds; blocks
    are concatenated in index order, each in the order its coordinates arrived."""
    stat = np.asarray(stat, dtype=np.float64)
    d = stat.size
    n = d // b
    order = np.argsort(-stat, kind="stable")
    blocks = [[] for _ in range(n)]
    for r, ch in enumerate(order):
        rnd, pos = divmod(r, n)
        blocks[pos if rnd % 2 == 0 else n - 1 - pos].append(int(ch))
    return np.array([i for blk in blocks for i in blk], dtype=np.int32)


def splitmix64(seed: int, k: int) -> int:
    """k-th output (k = 0, 1, ...) of the SplitMix64 generator started at `seed` (Steele, Lea and
    Flood, "Fast splittable pseudorandom number generators", 2014): the state advances by the
    golden-ratio constant, the output is the state through two xor-shift-multiply rounds."""
    mask = (1 << 64) - 1
    z = (seed + (k + 1) * 0x9E3779B97F4A7C15) & mask
    z = ((z ^ (z >> 30)) * 0xBF58476D1CE4E5B9) & mask
    z = ((z ^ (z >> 27)) * 0x94D049BB133111EB) & mask
    return z ^ (z >> 31)


def perm_random(d: int, seed: int) -> np.ndarray:
    """The ablation's random permutation, made reproducible.  The paper draws it with an unnamed
    generator; reading: a Fisher-Yates shuffle of the identity from the top down, i = d-1 .. 1,
    swapping position i with position floor(u * (i + 1) / 2^64), u the (d-1-i)-th SplitMix64 output
    for the seed.  Every channel is equally likely at every position up to 2^-64 * d."""
    perm = np.arange(d, dtype=np.int64)
    for i in range(d - 1, 0, -1):
        j = (splitmix64(seed, d - 1 - i) * (i + 1)) >> 64
        perm[i], perm[j] = perm[j], perm[i]
    return perm.astype(np.int32)


def block_diagnostics(x_bits: np.ndarray, perm, b: int) -> np.ndarray:
    """float64 [T, 4] per token: ||X||_inf, ||X||_1, max_j ||(XP)_{j}||_1, ||XP R~||_inf.

    From these: delta = ||X||_1 / (d ||X||_inf) (Proposition 1); the bound of Proposition 2,
    max_j delta_j sqrt(b) ||X_j||_inf = max_j ||X_j||_1 / sqrt(b) = Z(b; XP) of Corollary 3.3;
    the suppression ratio ||XP R~||_inf / ||X||_inf."""
    X = bf16_bits_to_f64(x_bits)
    Xp = permute_channels(X, perm)
    T, d = X.shape
    l1b = np.abs(Xp).reshape(T, d // b, b).sum(axis=2).max(axis=1)
    y = block_hadamard(Xp, b)
    return np.stack([np.abs(X).max(axis=1), np.abs(X).sum(axis=1), l1b, np.abs(y).max(axis=1)], axis=1)


def quant_error(Y: np.ndarray, fmt: str) -> np.ndarray:
    """float64 [T, 3] per token: ||Y - Q(Y)||_2, ||Y||_2, ||Y||_inf for the rotated row Y = XP R~ and
    the quantizer `fmt` ("int4", "mxfp4", "int4_asym", "fp4_token"), Q(Y) being the value the codes
    stand for.  Section 3: with the symmetric q-bit step s = ||Y||_inf / (2^(q-1) - 1) every element
    is off by at most s/2, so ||Y - Q(Y)||_2 <= sqrt(d) / (2^q - 2) ||Y||_inf (q = 4: sqrt(d)/14)."""
    if fmt == "int4":
        c, s = quant_int4_sym_token(Y)
        Q = dequant_int4(c, s)
    elif fmt == "mxfp4":
        c, E = quant_mxfp4(Y)
        Q = dequant_mxfp4(c, E)
    elif fmt == "int4_asym":
        c, s, z = quant_int4_asym_token(Y)
        Q = dequant_int4_asym(c, s, z)
    elif fmt in ("fp4_token", "fp4_token7"):
        c, s = quant_fp4_token(Y, 7.0 if fmt == "fp4_token7" else 6.0)
        Q = dequant_fp4_token(c, s)
    else:
        raise ValueError("fmt must be 'int4', 'mxfp4', 'int4_asym', 'fp4_token' or 'fp4_token7'")
    return np.stack([np.sqrt(((Y - Q) ** 2).sum(axis=1)), np.sqrt((Y ** 2).sum(axis=1)), np.abs(Y).max(axis=1)], axis=1)


# ----------------------------------------------------------------------------------------
# consumer of the codes: W4A4 product with P and R~ merged into the weights
# (Remark "Merging Permutations", Section 4;  R~ R~^T = I, Notation of Section 1)
# ----------------------------------------------------------------------------------------
def merge_into_weights(W: np.ndarray, perm, b: int) -> np.ndarray:
    """W~ = R~^T P^T W for W in R^{d x N} (row i = input channel i), returned transposed as
    [N, d]: row n is column n of W gathered through perm and block-rotated -- the same P, R~ the
    activations go through, since (X P R~)(R~^T P^T W) = X W."""
    return block_hadamard(permute_channels(np.ascontiguousarray(W.T, dtype=np.float64), perm), b)


def w4a4_matmul(codes_a: np.ndarray, s_a: np.ndarray, codes_w: np.ndarray, s_w: np.ndarray):
    """out[t, n] = s_a[t] * s_w[n] * sum_i codes_a[t, i] * codes_w[n, i] for symmetric INT4 codes
    (Eq. 4 with z = 0 on both operands).  Returns (integer sums int64 [T, N], out float64)."""
    acc = codes_a.astype(np.int64) @ codes_w.astype(np.int64).T
    return acc, acc.astype(np.float64) * np.asarray(s_a, np.float64)[:, None] * np.asarray(s_w, np.float64)[None, :]


def w4a4_mxfp4_matmul(codes_a: np.ndarray, E_a: np.ndarray, codes_w: np.ndarray, E_w: np.ndarray) -> np.ndarray:
    """out[t, n] = sum_i a[t, i] w[n, i] with both operands decoded from MXFP4 (Eq. 5: e2m1 element
    times 2^(E - 127) of its 32-group); float64 [T, N].  Every product and every partial sum of a
    realistic size is exact in float64, so this is the value itself."""
    return dequant_mxfp4(codes_a, E_a) @ dequant_mxfp4(codes_w, E_w).T


# ----------------------------------------------------------------------------------------
# the whole path
# ----------------------------------------------------------------------------------------
def perq_apply(x_bits: np.ndarray, perm, b: int, fmt: str, rotate=block_hadamard):
    """bf16 bits [T,d] -> dict(y, codes, packed, scales[, s64]) following P, R~, Q in order.

    fmt is "int4" (scales: float32 [T]), "mxfp4" (scales: uint8 [T, d/32]), "int4_asym"
    (scales: float32 [T, 2] = step, zero point), "fp4_token" or "fp4_token7" (scales: float32 [T]).
    """
    X = bf16_bits_to_f64(x_bits)
    Y = rotate(permute_channels(X, perm), b)
    if fmt == "int4":
        codes, s = quant_int4_sym_token(Y)
        return {"y": Y, "codes": codes, "packed": pack_nibbles(codes),
                "scales": s.astype(np.float32), "s64": s}
    if fmt == "mxfp4":
        codes, E = quant_mxfp4(Y)
        return {"y": Y, "codes": codes, "packed": pack_nibbles(codes), "scales": E}
    if fmt == "int4_asym":
        codes, s, z = quant_int4_asym_token(Y)
        return {"y": Y, "codes": codes, "packed": pack_nibbles(codes),
                "scales": np.stack([s, z], axis=1).astype(np.float32), "s64": s, "z": z}
    if fmt in ("fp4_token", "fp4_token7"):
        codes, s = quant_fp4_token(Y, 7.0 if fmt == "fp4_token7" else 6.0)
        return {"y": Y, "codes": codes, "packed": pack_nibbles(codes),
                "scales": s.astype(np.float32), "s64": s}
    raise ValueError("fmt must be 'int4', 'mxfp4', 'int4_asym', 'fp4_token' or 'fp4_token7'")
