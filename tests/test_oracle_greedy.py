"""Pins for the oracle's mass-diffusion permutation (Algorithm 1), CPU only."""
import math

import numpy as np
import pytest

from oracle import perq_oracle as orc
from paper_2601_22347_amd import synth


def _rng(seed):
    return np.random.default_rng(seed)


def _check_structure(perm, d):
    assert perm.dtype == np.int32 and perm.shape == (d,)
    assert np.array_equal(np.sort(perm), np.arange(d))


@pytest.mark.parametrize("d,b", [(64, 16), (256, 32), (96, 8), (128, 128)])
def test_greedy_is_a_bijection_with_full_blocks(d, b):
    a = np.abs(_rng(1).standard_t(3, size=d))
    perm = orc.massdiff_greedy(a, b)
    _check_structure(perm, d)
    n = d // b
    order = np.argsort(-a, kind="stable")
    # the first n picks meet n empty blocks (all masses 0): lowest index wins each time
    assert np.array_equal(perm[0::b][:n], order[:n])
    # inside a block channels appear in the order they were placed: descending a
    blocks = a[perm].reshape(n, b)
    assert np.all(np.diff(blocks, axis=1) <= 0)
    L = orc.block_masses(a, perm, b)
    assert L.max() >= a.sum() / n - 1e-12 and L.max() >= a.max()
    assert math.isclose(L.sum(), a.sum(), rel_tol=1e-13)


def test_greedy_closed_forms():
    # all channels equal: round-robin, perm[j*b + k] = k*n + j
    d, b = 48, 8
    n = d // b
    perm = orc.massdiff_greedy(np.full(d, 0.75), b)
    want = np.array([k * n + j for j in range(n) for k in range(b)])
    assert np.array_equal(perm, want)
    # a single block: stable descending argsort
    a = np.array([1.0, 3.0, 3.0, 0.5, 2.0, 3.0, 0.0, 1.0])
    assert orc.massdiff_greedy(a, 8).tolist() == [1, 2, 5, 4, 0, 7, 3, 6]
    # hand-worked example, d = 6, b = 3 (n = 2): a sorted desc = 9(ch2) 7(ch0) 4(ch5) 3(ch1) 2(ch4) 1(ch3)
    # 9->B0 (9,0); 7->B1 (9,7); 4->B1 (9,11); 3->B0 (12,11); 2->B1 (12,13) full; 1->B0 (13,13)
    a = np.array([7.0, 3.0, 9.0, 1.0, 2.0, 4.0])
    assert orc.massdiff_greedy(a, 3).tolist() == [2, 1, 3, 0, 5, 4]
    assert orc.block_masses(a, [2, 1, 3, 0, 5, 4], 3).tolist() == [13.0, 13.0]


def test_full_blocks_are_dropped_from_the_candidate_set():
    # one huge channel then many small ones: block 0 must still end with exactly b members
    a = np.array([100.0] + [1.0] * 7)
    perm = orc.massdiff_greedy(a, 4)
    _check_structure(perm, 8)
    # B0 gets ch0, then B1 fills (1,2,3,4) while lighter, then the rest must go to B0
    assert perm.tolist() == [0, 5, 6, 7, 1, 2, 3, 4]


@pytest.mark.parametrize("d,b", [(8, 4), (8, 2), (12, 4), (12, 3), (16, 8)])
def test_greedy_against_brute_force_optimum(d, b):
    worst = 1.0
    for seed in range(6):
        a = np.abs(_rng(100 + seed).standard_t(3, size=d))
        if seed % 2:
            a[_rng(seed).integers(d)] *= 20
        perm = orc.massdiff_greedy(a, b)
        g = orc.block_masses(a, perm, b).max()
        opt = orc.brute_force_min_max_block_mass(a, b)
        assert opt <= g * (1 + 1e-12)
        assert opt >= max(a.sum() / (d // b), a.max()) * (1 - 1e-12)
        worst = max(worst, g / opt)
    # a greedy heuristic of the longest-processing-time kind; it stays within 4/3 of optimal here
    assert worst <= 4.0 / 3.0 + 1e-9


def test_brute_force_on_known_instance():
    # {8,1} {7,2} {6,3}: every block 9
    assert orc.brute_force_min_max_block_mass([8, 7, 6, 3, 2, 1], 2) == 9
    assert orc.brute_force_min_max_block_mass([5, 5, 5, 5], 4) == 20


def test_greedy_beats_identity_on_outlier_workloads():
    for wl, b in [(synth.tiny(), 16)]:
        X = orc.bf16_bits_to_f64(wl.calib_rows())
        a = orc.colabs_mean(X)
        perm = orc.massdiff_greedy(a, b)
        Lg, Li = orc.block_masses(a, perm, b), orc.block_masses(a, None, b)
        assert Lg.max() < Li.max()
        assert Lg.max() - Lg.min() < Li.max() - Li.min()
        # and the rotated apply-time rows have a smaller worst-case bound (Prop. 2) on average
        Xa = orc.bf16_bits_to_f64(wl.apply_rows())
        bound_g = np.abs(Xa[:, perm]).reshape(wl.T, -1, b).sum(axis=2).max(axis=1)
        bound_i = np.abs(Xa).reshape(wl.T, -1, b).sum(axis=2).max(axis=1)
        assert bound_g.mean() < bound_i.mean()


# ---- alternative permutations (Appendix C) and the per-token quantities of Section 3 ----------
def test_sorted_and_zigzag_permutations_closed_forms():
    stat = np.array([5.0, 1.0, 7.0, 3.0, 8.0, 2.0, 6.0, 4.0])
    assert orc.perm_sorted_desc(stat).tolist() == [4, 2, 6, 0, 7, 3, 5, 1]
    # n = 4 blocks of 2: ranks 0..3 go to blocks 0..3, ranks 4..7 to blocks 3..0
    assert orc.perm_zigzag(stat, 2).tolist() == [4, 1, 2, 5, 6, 3, 0, 7]
    # n = 2 blocks of 4: rounds alternate direction
    assert orc.perm_zigzag(stat, 4).tolist() == [4, 0, 7, 1, 2, 6, 3, 5]
    # one block: the sorted order; equal statistics: stable
    assert orc.perm_zigzag(stat, 8).tolist() == orc.perm_sorted_desc(stat).tolist()
    assert orc.perm_sorted_desc(np.ones(6)).tolist() == list(range(6))
    rng = np.random.default_rng(5)
    for d, b in ((64, 16), (96, 32), (128, 128)):
        p = orc.perm_zigzag(rng.random(d), b)
        assert sorted(p.tolist()) == list(range(d))
    # on a geometric sequence the serpentine beats the sorted order by construction
    g = 2.0 ** -np.arange(16.0)
    assert orc.block_masses(g, orc.perm_zigzag(g, 4), 4).max() < orc.block_masses(g, orc.perm_sorted_desc(g), 4).max()


def test_colabs_max_hand_case_and_relations():
    """Per-channel l_inf over the tokens (the statistic of the ablation's absmax / ZigZag rows,
    Appendix C): a hand-worked case, then what any maximum of magnitudes must satisfy."""
    # channel 0: the largest magnitude is negative; 1: +2 and -2 tie; 2: all zero; 3: a maximum in the
    # last row, smaller negative entries before it
    X = np.array([[-5.0, 2.0, 0.0, -0.25],
                  [3.0, -2.0, -0.0, -0.5],
                  [-1.0, 1.0, 0.0, 0.75]])
    assert orc.colabs_max(X).tolist() == [5.0, 2.0, 0.0, 0.75]
    # a transposed reading (maximum per token instead of per channel) gives another shape and values
    assert orc.colabs_max(X).shape == (4,)
    R = np.random.default_rng(8).standard_t(3, size=(257, 41))
    m = orc.colabs_max(R)
    a = orc.colabs_mean(R)
    assert np.all(m >= a) and np.all(m <= 257 * a * (1 + 1e-12))        # mean <= max <= sum
    # entry by entry against plain Python, and the maximum is attained by some token
    for i in range(41):
        col = [abs(float(v)) for v in R[:, i]]
        assert m[i] == max(col) and m[i] in col
    # invariances: sign flips and a reordering of the tokens change nothing; one row: |x|
    assert np.array_equal(orc.colabs_max(-R), m) and np.array_equal(orc.colabs_max(R[::-1]), m)
    assert np.array_equal(orc.colabs_max(R[:1]), np.abs(R[0]))
    # scaling one channel scales its statistic only
    S = R.copy(); S[:, 7] *= -3.0
    want = m.copy(); want[7] *= 3.0
    assert np.array_equal(orc.colabs_max(S), want)


def test_block_diagnostics_bounds_and_special_cases():
    from paper_2601_22347_amd import synth
    rng = np.random.default_rng(6)
    T, d = 40, 256
    x = rng.standard_t(3, size=(T, d))
    x[:, [3, 4, 5]] *= 40
    bits = synth.f64_to_bf16_bits(x)
    X = orc.bf16_bits_to_f64(bits)
    perm = orc.massdiff_greedy(orc.colabs_mean(X), 32)
    for pm in (None, perm):
        for b in (16, 32, 256):
            if pm is not None and b != 32:
                continue
            D = orc.block_diagnostics(bits, pm, b)
            amax, l1, l1b, ymax = D.T
            assert np.allclose(amax, np.abs(X).max(axis=1)) and np.allclose(l1, np.abs(X).sum(axis=1))
            assert np.all(ymax <= l1b / np.sqrt(b) * (1 + 1e-12))               # Proposition 2
            assert np.all(l1b >= l1 / (d // b) * (1 - 1e-12)) and np.all(l1b <= l1 * (1 + 1e-12))
            if b == d:
                assert np.allclose(l1b, l1)                                      # Proposition 1 is the case b = d
    # Corollary 3.3: Z(b) <= sqrt(k) Z(b') for b = k b'
    Z = {b: orc.block_diagnostics(bits, None, b)[:, 2] / np.sqrt(b) for b in (16, 32, 64, 256)}
    for b, bp in ((32, 16), (64, 16), (256, 64), (256, 32)):
        assert np.all(Z[b] <= np.sqrt(b / bp) * Z[bp] * (1 + 1e-12))
    # the calibrated permutation lowers the mean bound on data with the calibrated outlier channels
    assert orc.block_diagnostics(bits, perm, 32)[:, 2].mean() < orc.block_diagnostics(bits, None, 32)[:, 2].mean()
    # one-hot row: every quantity in closed form
    r = np.zeros((1, 64)); r[0, 10] = -2.0
    D = orc.block_diagnostics(synth.f64_to_bf16_bits(r), None, 16)
    assert np.allclose(D[0], [2.0, 2.0, 2.0, 0.5])


# ---- reproducible random permutation (the ablation's "Random" row) ---------------------------------
def test_splitmix64_reference_outputs():
    # first outputs of the published reference implementation for seed 0
    assert [orc.splitmix64(0, k) for k in range(3)] == [0xE220A8397B1DCDAF, 0x6E789E6AA1B965F4, 0x06C45D188009454F]


def test_random_permutation_is_a_uniform_looking_bijection():
    for d, seed in [(1, 5), (2, 0), (17, 1), (256, 2), (4096, 3)]:
        p = orc.perm_random(d, seed)
        assert p.dtype == np.int32 and np.array_equal(np.sort(p), np.arange(d))
        assert np.array_equal(p, orc.perm_random(d, seed))
    # d = 2: position 1 is swapped with floor(u * 2 / 2^64), i.e. kept iff the top bit of u is set
    for seed in range(20):
        kept = orc.splitmix64(seed, 0) >> 63
        assert list(orc.perm_random(2, seed)) == ([0, 1] if kept else [1, 0])
    # over many seeds every channel lands on every position about equally often (d = 8: 64 cells,
    # 4000 shuffles, expected 500 each; chi-square with 49 degrees of freedom stays far below 120)
    counts = np.zeros((8, 8))
    for seed in range(4000):
        p = orc.perm_random(8, seed)
        counts[np.arange(8), p] += 1
    chi2 = ((counts - 500.0) ** 2 / 500.0).sum()
    assert chi2 < 120.0, chi2
