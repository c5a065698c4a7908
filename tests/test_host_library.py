"""Host-side checks that need no GPU: the C-ABI library loads, exports what the header
declares, rejects bad arguments before touching the device, and its greedy matches the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest

from oracle import perq_oracle as orc
from paper_2601_22347_amd import binding, synth
import prepared_form

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def test_library_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "perq.h")).read()
    header = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(perq_[a-z0-9_]+)\s*\(", header))
    assert declared == set(binding.EXPORTS)
    for name in declared:
        assert getattr(lib, name) is not None
    assert binding.status_string(0) == "PERQ_OK"
    assert binding.status_string(1) == "PERQ_ERR_INVALID_ARG"
    assert binding.status_string(2) == "PERQ_ERR_UNSUPPORTED"
    assert binding.status_string(3) == "PERQ_ERR_LAUNCH"


@pytest.mark.parametrize("d,b,seed", [(256, 16, 0), (256, 32, 1), (8192, 16, 2), (8192, 128, 3),
                                      (14336, 2048, 4), (4096, 4096, 5), (96, 8, 6)])
def test_greedy_matches_oracle_bit_exactly(d, b, seed):
    rng = np.random.default_rng(seed)
    a = np.abs(rng.standard_t(3, size=d)).astype(np.float32)
    a[rng.choice(d, size=max(1, d // 100), replace=False)] *= 50
    if seed % 2:
        a[rng.choice(d, size=d // 4, replace=False)] = a[0]          # plenty of ties
    got = binding.perq_massdiff_perm(a, b)
    want = orc.massdiff_greedy(a.astype(np.float64), b)
    assert np.array_equal(got, want)
    assert binding.perq_perm_validate(got)


def test_greedy_on_calibration_statistic_of_tiny_workload():
    wl = synth.tiny()
    a = orc.colabs_mean(orc.bf16_bits_to_f64(wl.calib_rows())).astype(np.float32)
    assert np.array_equal(binding.perq_massdiff_perm(a, 16), orc.massdiff_greedy(a.astype(np.float64), 16))


def test_greedy_rejects_bad_arguments(lib):
    a = np.ones(64, dtype=np.float32)
    perm = np.empty(64, dtype=np.int32)
    pa, pp = a.ctypes.data_as(ctypes.c_void_p), perm.ctypes.data_as(ctypes.c_void_p)
    assert lib.perq_massdiff_perm(None, 64, 16, pp) == binding.PERQ_ERR_INVALID_ARG
    assert lib.perq_massdiff_perm(pa, 64, 16, None) == binding.PERQ_ERR_INVALID_ARG
    assert lib.perq_massdiff_perm(pa, 64, 24, pp) == binding.PERQ_ERR_INVALID_ARG
    assert lib.perq_massdiff_perm(pa, 0, 16, pp) == binding.PERQ_ERR_INVALID_ARG
    a[3] = np.nan
    assert lib.perq_massdiff_perm(pa, 64, 16, pp) == binding.PERQ_ERR_INVALID_ARG
    a[3] = -1.0
    assert lib.perq_massdiff_perm(pa, 64, 16, pp) == binding.PERQ_ERR_INVALID_ARG


def test_perm_validate():
    assert binding.perq_perm_validate(np.arange(100)[::-1])
    assert not binding.perq_perm_validate(np.array([0, 1, 1, 3]))
    assert not binding.perq_perm_validate(np.array([0, 1, 2, 4]))
    assert not binding.perq_perm_validate(np.array([0, -1, 2, 3]))


def test_apply_argument_checks_happen_before_any_launch(lib):
    """Bad shapes are refused on the host; the fake non-null pointers are never dereferenced."""
    fake = ctypes.c_void_p(0x1000)
    bad16 = ctypes.c_void_p(0x1008)
    INV, UNS = binding.PERQ_ERR_INVALID_ARG, binding.PERQ_ERR_UNSUPPORTED

    def q(x=fake, T=4, d=256, ldx=256, perm=None, b=16, fmt=0, codes=fake, scales=fake):
        return lib.perq_permute_rotate_quant(x, T, d, ldx, perm, b, fmt, codes, scales, None)

    assert q(x=None) == INV and q(codes=None) == INV and q(scales=None) == INV
    assert q(T=-1) == INV and q(d=0) == INV and q(ldx=128) == INV
    assert q(b=8) == INV and q(b=24) == INV and q(b=512) == INV and q(d=96, ldx=96, b=64) == INV
    assert q(d=48, ldx=48, b=16) == INV          # d % 32
    assert q(fmt=7) == INV
    assert q(d=65536, ldx=65536, b=16) == UNS
    assert q(x=bad16) == UNS and q(ldx=260) == UNS and q(codes=bad16) == UNS
    assert q(T=0) == binding.PERQ_OK
    assert lib.perq_permute_rotate_quant_algo(fake, 4, 256, 256, None, 16, 0, 9, fake, fake, None) == INV
    assert lib.perq_permute_rotate_f32(fake, 4, 256, 256, None, 16, 0, None, None) == INV
    assert lib.perq_permute_rotate_f32(fake, 4, 256, 256, None, 16, 5, fake, None) == INV
    assert lib.perq_permute_rotate_f32(None, 0, 256, 256, None, 16, 0, None, None) == binding.PERQ_OK
    assert q(x=None, T=0, codes=None, scales=None) == binding.PERQ_OK
    assert q(x=None, T=0, b=24) == INV            # shape errors are still reported for T == 0
    # colabs
    assert lib.perq_colabs_mean(None, 4, 256, 256, fake, fake, 1 << 20, None) == INV
    assert lib.perq_colabs_mean(fake, 0, 256, 256, fake, fake, 1 << 20, None) == INV
    assert lib.perq_colabs_mean(fake, 4, 256, 256, fake, fake, 16, None) == INV      # workspace too small
    assert lib.perq_colabs_mean(fake, 4, 256, 256, fake, None, 0, None) == INV
    assert lib.perq_colabs_mean_workspace_bytes(4096, 8192) >= 8192 * 4
    assert lib.perq_colabs_mean_workspace_bytes(0, 8192) == 0


def test_sorted_and_zigzag_match_oracle():
    rng = np.random.default_rng(77)
    for d, b in ((256, 16), (4096, 128), (96, 32), (64, 64)):
        stat = rng.gamma(0.5, size=d).astype(np.float32)
        stat[rng.choice(d, size=d // 8, replace=False)] = stat[0]          # ties
        assert np.array_equal(binding.perq_perm_sorted(stat), orc.perm_sorted_desc(stat))
        z = binding.perq_perm_zigzag(stat, b)
        assert np.array_equal(z, orc.perm_zigzag(stat, b)) and binding.perq_perm_validate(z)
    with pytest.raises(binding.PerqError):
        binding.perq_perm_zigzag(np.ones(10, np.float32), 4)
    with pytest.raises(binding.PerqError):
        binding.perq_perm_sorted(np.array([1.0, np.nan], np.float32))


@pytest.mark.parametrize("m", [12, 20, 28, 36, 44, 76])
def test_hadamard_base_matches_oracle_construction(m):
    H = binding.perq_hadamard_base(m).astype(np.int64)
    assert np.array_equal(H @ H.T, m * np.eye(m, dtype=np.int64))
    assert np.array_equal(H, orc.paley_hadamard(m))


def test_hadamard_base_rejects_orders_without_a_construction():
    for m in (4, 10, 16, 24, 32, 92, 0, -12):   # 24 = 2 * 12 and 32 are not 4t with t odd; 92: 91 = 7 * 13, 45 = 9 * 5
        with pytest.raises(binding.PerqError) as ei:
            binding.perq_hadamard_base(m)
        assert ei.value.status == binding.PERQ_ERR_INVALID_ARG


def test_random_permutation_matches_oracle_generator():
    for d, seed in [(1, 0), (2, 7), (33, 1), (4096, 123456789), (14336, 2 ** 63 + 5)]:
        got = binding.perq_perm_random(d, seed)
        assert np.array_equal(got, orc.perm_random(d, seed))
        assert binding.perq_perm_validate(got)
    with pytest.raises(binding.PerqError) as ei:
        binding.perq_perm_random(0, 1)
    assert ei.value.status == binding.PERQ_ERR_INVALID_ARG


# ---- perq_perm_arrange: same blocks, an order that suits the kernel's LDS gather -----------------
@pytest.mark.parametrize("d,b", [(4096, 128), (4096, 16), (4096, 4096), (8192, 32), (14336, 128), (14336, 2048),
                                 (12288, 1024), (32768, 512)])
def test_perm_arrange_keeps_every_block_and_lowers_the_gather_cost(d, b):
    rng = np.random.default_rng(d + b)
    a = np.exp(rng.normal(0, 1.5, d)).astype(np.float32)
    for perm in (rng.permutation(d).astype(np.int32), binding.perq_massdiff_perm(a, b)):
        out = binding.perq_perm_arrange(perm, b)
        assert binding.perq_perm_validate(out)
        # what is unique: the channel set of every block (and so every block mass of Algorithm 1)
        # (blocks may also change places inside the row)
        def blocks(p):
            rows = np.sort(p.reshape(-1, b), axis=1)
            return rows[np.lexsort(rows.T[::-1])]
        assert np.array_equal(blocks(out), blocks(perm))
        assert np.array_equal(binding.perq_perm_arrange(perm, b), out)          # deterministic
        p0, r0 = binding.perq_perm_gather_cost(perm, b)
        p1, r1 = binding.perq_perm_gather_cost(out, b)
        assert r0 == r1 and r0 <= 128 * ((d + 4095) // 4096)
        assert p1 >= r1 and p0 >= r0
        assert p1 <= 0.65 * p0, (p0, p1, r1)       # a random order costs about 3.4 passes per read
        if b >= 128:        # (from b = 512 on, 64 positions per block stay where they are)
            assert p1 <= (1.65 if b >= 512 else 1.4) * r1, (p1, r1)


def test_perm_arrange_keeps_the_head_of_every_block():
    """The first `head` positions of a block stay as Algorithm 1 filled them (heaviest channels first)."""
    rng = np.random.default_rng(12)
    for d, b, head in [(4096, 1024, -1), (8192, 512, -1), (14336, 2048, 32), (4096, 4096, 128), (4096, 128, 16)]:
        a = np.exp(rng.normal(0, 1.5, d)).astype(np.float32)
        perm = binding.perq_massdiff_perm(a, b)
        out = binding.perq_perm_arrange(perm, b, head)
        h = 64 if head < 0 else head
        given = {tuple(sorted(blk)): blk for blk in perm.reshape(-1, b)}
        for blk in out.reshape(-1, b):
            src = given[tuple(sorted(blk))]
            assert np.array_equal(blk[:h], src[:h])
        assert not np.array_equal(out, perm)
    with pytest.raises(binding.PerqError):
        binding.perq_perm_arrange(np.arange(4096, dtype=np.int32), 128, 129)


def test_order_inside_large_blocks_matters_for_int4_and_the_default_head_keeps_it():
    """On blocks with several outlier channels the per-token INT4 error (oracle) is lower in
    Algorithm 1's order than in an order that moves the heavy channels; with the default head the
    arranged permutation quantizes as well as the given one."""
    from oracle import perq_oracle as orc
    from paper_2601_22347_amd import synth
    wl = synth.ALL["llama8b_d4096"]()
    a = orc.colabs_mean(orc.bf16_bits_to_f64(wl.calib_rows()))
    x = wl.apply_rows(0, 96)

    def err(p, b):
        r = orc.perq_apply(x, p, b, "int4")
        return np.linalg.norm(r["y"] - orc.dequant_int4(r["codes"], r["scales"])) / np.linalg.norm(r["y"])
    for b in (2048,):
        g = orc.massdiff_greedy(a, b)
        e_given, e_default, e_all = err(g, b), err(binding.perq_perm_arrange(g, b), b), err(binding.perq_perm_arrange(g, b, 0), b)
        assert abs(e_default / e_given - 1) < 0.02, (e_given, e_default)
        assert e_all > 1.05 * e_given, (e_given, e_all)
    g = orc.massdiff_greedy(a, 128)
    assert abs(err(binding.perq_perm_arrange(g, 128), 128) / err(g, 128) - 1) < 0.01     # small blocks: no difference


def test_perm_arrange_gather_cost_model_on_known_orders():
    d, b = 4096, 128
    ident = np.arange(d, dtype=np.int32)
    # the identity read element by element: the 32 lanes of a half-wave are 128 channels apart,
    # eight granule slots four banks apart each -> four lanes per bank
    assert binding.perq_perm_gather_cost(ident, b) == (512, 128)
    # all lanes on the same word: one pass
    with pytest.raises(binding.PerqError):
        binding.perq_perm_gather_cost(np.zeros(d, dtype=np.int32), b)          # not a permutation


def test_perm_arrange_leaves_other_shapes_alone_and_checks_arguments():
    rng = np.random.default_rng(9)
    for d, b in [(2048, 128), (3584, 3584), (4096 + 32, 32), (8192, 8192), (512, 64)]:
        perm = rng.permutation(d).astype(np.int32)
        assert np.array_equal(binding.perq_perm_arrange(perm, b), perm)
        with pytest.raises(binding.PerqError) as ei:
            binding.perq_perm_gather_cost(perm, b)
        assert ei.value.status == binding.PERQ_ERR_UNSUPPORTED
    bad = np.arange(4096, dtype=np.int32); bad[5] = 6
    with pytest.raises(binding.PerqError):
        binding.perq_perm_arrange(bad, 128)
    with pytest.raises(binding.PerqError):
        binding.perq_perm_arrange(np.arange(4096, dtype=np.int32), 100)        # b does not divide d


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    res = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True,
                         text=True, timeout=120, cwd=root)
    assert res.returncode != 0 and "one GPU" in res.stderr


def test_perm_arrange_is_never_worse_than_the_given_order_on_regular_permutations():
    """Blocks of consecutive channels, strides, a bank-sorted order: heads that stay in place can all
    meet in one bank there, and the routine then hands back what it was given."""
    for d, b in [(4096, 128), (8192, 512), (14336, 2048), (8192, 16)]:
        ar = np.arange(d)
        for p in (ar, ar[::-1], ar.reshape(b, d // b).T.reshape(-1), np.r_[ar[0::2], ar[1::2]],
                  np.argsort((ar >> 1) & 31, kind="stable")):
            p = np.ascontiguousarray(p, dtype=np.int32)
            for head in (-1, 0):
                q = binding.perq_perm_arrange(p, b, head)
                assert binding.perq_perm_validate(q)
                assert sorted(map(tuple, np.sort(q.reshape(-1, b), axis=1))) == sorted(map(tuple, np.sort(p.reshape(-1, b), axis=1)))
                assert binding.perq_perm_gather_cost(q, b)[0] <= binding.perq_perm_gather_cost(p, b)[0]


# ---- run-time row schedule of the matrix-core kernel: the host model on the kernel's own arithmetic ----
@pytest.mark.parametrize("n_units,n_blocks,per_block", [
    (4096, 512, 4),        # d = 4096: a wave per row, T = 4096 is the first size on the queues (nothing left to draw)
    (4097, 512, 4), (4160, 512, 4), (32768, 512, 4), (9999, 512, 4),
    (1024, 512, 1),        # a workgroup per unit, exactly two units each
    (1025, 512, 1), (8192, 512, 1), (32768, 256, 1), (700, 256, 1),
])
def test_schedule_model_takes_every_unit_once_and_leaves_the_counters_at_zero(n_units, n_blocks, per_block):
    for seed in range(4):
        # three launches on the same counters: a counter left non-zero would skew the next launch
        assert binding.perq_schedule_selftest(n_units, n_blocks, per_block, seed, 3) == binding.PERQ_OK


def test_schedule_model_rejects_shapes_off_the_queues():
    UNS, INV = binding.PERQ_ERR_UNSUPPORTED, binding.PERQ_ERR_INVALID_ARG
    assert binding.perq_schedule_selftest(4095, 512, 4, 0, 1) == UNS       # fewer than two units per worker
    assert binding.perq_schedule_selftest(8192, 500, 1, 0, 1) == UNS       # queues would not fill evenly
    assert binding.perq_schedule_selftest(0, 512, 4, 0, 1) == INV
    assert binding.perq_schedule_selftest(8192, 512, 0, 0, 1) == INV
    assert binding.status_string(4) == "PERQ_ERR_INTERNAL"


# ---- placement of a row's pieces in LDS for a permutation (perq_perm_prepare) ---------------------------
@pytest.mark.parametrize("d,b", [(4096, 128), (4096, 4096), (8192, 32), (14336, 128), (14336, 2048), (20480, 1024)])
def test_prepared_placement_is_a_line_bijection_and_never_worse(d, b):
    rng = np.random.default_rng(d + b)
    perm = rng.permutation(d).astype(np.int32)
    table, before, after, reads = binding.perq_perm_prepare(perm, b)
    tiles = (d + 4095) // 4096
    assert table.dtype == np.uint8 and table.size == 4 * d + d // 4 + 2 * tiles * 8192
    G = d // 8
    place, granule_of, lanes = binding.prepared_parts(table, d)
    granule_of = granule_of.astype(np.int64)
    assert np.array_equal(np.sort(granule_of), np.arange(G))                   # every slot takes one piece
    assert np.array_equal(granule_of // 8, np.arange(G) // 8)                  # inside the 128-byte lines of the row
    slot_of = np.empty(G, dtype=np.int64); slot_of[granule_of] = np.arange(G)
    # a position's place: the slot of its channel's piece, and the channel's place inside the piece
    assert np.array_equal(place, slot_of[perm >> 3] * 8 + (perm & 7))
    assert binding.perq_perm_prepared_validate(table, perm)
    # the operand offsets in lane order, rebuilt from the description of the form: both modes, every tile,
    # the ragged end marked; and the whole form byte for byte
    assert np.array_equal(lanes, prepared_form.lane_tables(perm, slot_of))
    assert np.array_equal(table, prepared_form.assemble(perm, slot_of))
    in_row = lanes[lanes != 0xFFFF]
    assert in_row.size == 2 * d and in_row.max() < 2 * d and not (in_row & 1).any()
    for mode in range(2):           # every channel of the row is read exactly once per mode
        assert np.array_equal(np.sort(lanes[mode][lanes[mode] != 0xFFFF].astype(np.int64)), 2 * np.arange(d))
    # the count for the fixed layout is the one perq_perm_gather_cost reports; the table lowers it
    assert (before, reads) == binding.perq_perm_gather_cost(perm, b)
    assert after <= before and after < 0.8 * before                            # 3.2 - 3.5 -> about 2.3 passes per read
    assert after >= reads
    # recount with plain NumPy what the table gives: per read the largest number of distinct words per bank
    # (bank = 4 * (slot % 8) + (channel % 8) // 2), for the low-K reads of the first tile
    if b < 1024:
        total = 0
        for f in range(8):
            for e in range(8):
                for h in range(2):
                    pos = np.array([(l * 4 + (f >> 1)) * 32 + 16 * (f & 1) + 8 * h + e for l in range(32)])
                    words = np.unique(perm[pos] >> 1)
                    bank = 4 * (slot_of[words >> 2] % 8) + (words & 3)
                    total += np.bincount(bank, minlength=32).max()
        # the first tile's 128 reads: the whole count for a row of one tile, a part of it otherwise
        assert 128 <= total and (total == after if d == 4096 else total < after)
    again = binding.perq_perm_prepare(perm, b)
    assert np.array_equal(again[0], table) and again[1:] == (before, after, reads)     # deterministic
    # a form that belongs to another permutation, or a broken one, is told apart
    other = perm.copy(); other[[0, 9]] = other[[9, 0]]
    assert not binding.perq_perm_prepared_validate(table, other)
    bad = table.copy(); bad[4 * d], bad[4 * d + 2] = bad[4 * d + 2], bad[4 * d]
    assert not binding.perq_perm_prepared_validate(bad, perm)
    bad = table.copy(); bad[-2] ^= 2                       # one operand offset of the last table
    assert not binding.perq_perm_prepared_validate(bad, perm)


def test_prepare_on_regular_and_unsupported_shapes(lib):
    # the identity is served without conflicts by the fixed layout: nothing to gain, nothing lost
    ident = np.arange(4096, dtype=np.int32)
    table, before, after, reads = binding.perq_perm_prepare(ident, 128)
    assert after <= before and binding.perq_perm_prepared_validate(table, ident)
    perm = np.arange(2048, dtype=np.int32)
    buf = np.zeros(2048 * 5 + 16384, dtype=np.uint8)
    pp, pt = perm.ctypes.data_as(ctypes.c_void_p), buf.ctypes.data_as(ctypes.c_void_p)
    assert lib.perq_perm_prepare(pp, 2048, 128, pt, None, None, None) == binding.PERQ_ERR_UNSUPPORTED     # d < 4096
    assert lib.perq_perm_prepare(None, 4096, 128, pt, None, None, None) == binding.PERQ_ERR_INVALID_ARG
    assert lib.perq_perm_prepare(pp, 2048, 128, None, None, None, None) == binding.PERQ_ERR_INVALID_ARG
    perm[3] = 4
    assert lib.perq_perm_prepare(pp, 2048, 128, pt, None, None, None) == binding.PERQ_ERR_INVALID_ARG      # not a bijection
    assert lib.perq_perm_prepared_bytes(14336) == 14336 * 4 + 14336 // 4 + 2 * 4 * 8192 and lib.perq_perm_prepared_bytes(7) == 0
    fake = ctypes.c_void_p(0x10000)
    odd = ctypes.c_void_p(0x10004)
    assert lib.perq_permute_rotate_quant_prepared(fake, 4, 4096, 4096, fake, odd, 128, 0, fake, fake, None) == binding.PERQ_ERR_UNSUPPORTED
    assert lib.perq_permute_rotate_quant_prepared(fake, 4, 4096, 4096, fake, fake, 100, 0, fake, fake, None) == binding.PERQ_ERR_INVALID_ARG
