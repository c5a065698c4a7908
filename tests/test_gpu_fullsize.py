"""Full-size runs of the BASELINE configurations in the launch configuration bench.py times: every
row against the oracle (the explicit matrix product for b <= 128; for power-of-two b >= 2048 the
oracle's fp64 butterfly evaluation, which the CPU tests pin to the explicit product up to b = 4096, on
every row and the explicit product on sampled rows), plus properties that hold at any size."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402
from oracle import perq_oracle as orc  # noqa: E402
from paper_2601_22347_amd import binding, synth  # noqa: E402

pytestmark = pytest.mark.gpu

CASES = [
    # workload, b list, rows sampled for the explicit-matrix oracle
    ("llama1b_down", (16, 32, 64, 128), 2048),
    ("block_vs_full", (32, 2048), 640),
    ("llama8b_d4096", (128, 4096), 192),
    ("llama8b_d14336", (128, 2048, 14336), 96),       # 14336 = 2^9 * 28: the full-vector rotation
    ("calib_apply", (16, 32), 256),
    ("qwen3_d12288", (12288, 3072), 96),              # 2^10 * 12
    ("qwen3_d9728", (9728,), 96),                     # 2^7 * 76
]


# the BASELINE configurations: every row is compared, not only the sample
ALL_ROWS = ("llama1b_down", "block_vs_full", "llama8b_d4096", "llama8b_d14336", "calib_apply")


def _sample_rows(wl, count):
    rng = np.random.default_rng(7)
    head = np.arange(min(count // 4, wl.T))
    tail = wl.T - 1 - np.arange(min(count // 4, wl.T))
    mid = rng.choice(wl.T, size=min(count, wl.T), replace=False)
    rows = np.unique(np.concatenate([head, tail, mid, wl.massive_rows]))
    return rows[:max(count, wl.massive_rows.size + count // 2)] if rows.size > 2 * count else rows


@pytest.mark.parametrize("name,bs,count", CASES)
def test_full_size_config(name, bs, count):
    import torch
    wl = synth.ALL[name]()
    print(f"[full] {name}: generating T={wl.T} d={wl.d}", flush=True)
    x_bits = wl.apply_rows_parallel()
    x = binding.bits_to_device(x_bits)
    rows = _sample_rows(wl, count) if count < wl.T else np.arange(wl.T)
    rows_t = torch.from_numpy(rows).cuda()
    a_dev = None
    if wl.calib_tokens:
        a_dev = binding.perq_colabs_mean(binding.bits_to_device(wl.calib_rows())).cpu().numpy()
        a_orc = orc.colabs_mean(orc.bf16_bits_to_f64(wl.calib_rows()))
        assert np.all(np.abs(a_dev - a_orc) <= 2e-6 * a_orc)
    for b in bs:
        perm = perm_t = None
        if a_dev is not None:
            perm = binding.perq_massdiff_perm(a_dev, b)
            assert np.array_equal(perm, orc.massdiff_greedy(a_dev.astype(np.float64), b))
            perm_t = torch.from_numpy(perm).cuda()
        print(f"[full] {name} b={b} fmt={wl.fmt} rows checked={rows.size}", flush=True)
        codes, scales = binding.perq_permute_rotate_quant(x, perm_t, b, wl.fmt)
        codes2, scales2 = binding.perq_permute_rotate_quant(x, perm_t, b, wl.fmt)
        torch.cuda.synchronize()
        assert torch.equal(codes, codes2) and torch.equal(scales, scales2)      # deterministic
        # properties at full size
        if wl.fmt == "int4":
            assert bool(torch.isfinite(scales).all()) and bool((scales >= 0).all())
            lo, hi = codes & 0xF, codes >> 4
            assert not bool(((lo == 8) | (hi == 8)).any())                      # -8 is never produced
        else:
            lo, hi = codes & 0xF, codes >> 4
            assert not bool(((lo == 8) | (hi == 8)).any())                      # zero is always +0
            assert int(scales.max()) < 255
        rep = parity.compare_apply(x_bits[rows], perm, b, wl.fmt, codes[rows_t].cpu().numpy(),
                                   scales[rows_t].cpu().numpy())
        print("       ", rep.summary(), flush=True)
        assert rep.ok(), (rep.summary(), rep.notes[:5])
        if name in ALL_ROWS and b & (b - 1) == 0 and rows.size < wl.T:
            rot = orc.fwht_f64 if b >= 2048 else None
            rep = parity.compare_apply_all_rows(x_bits, perm, b, wl.fmt, codes.cpu().numpy(), scales.cpu().numpy(), rotate=rot)
            print(f"[full] {name} b={b} every row ({'fp64 butterflies' if rot else 'explicit product'}):",
                  rep.summary(), flush=True)
            assert rep.ok() and rep.elements == wl.T * wl.d, (rep.summary(), rep.notes[:5])
        del codes, scales, codes2, scales2
        if perm is not None and b == 128 and name.startswith("llama8b"):
            # the same launch with the permutation's blocks arranged for the LDS gather
            arranged = binding.perq_perm_arrange(perm, b)
            assert binding.perq_perm_gather_cost(arranged, b)[0] < binding.perq_perm_gather_cost(perm, b)[0]
            codes, scales = binding.perq_permute_rotate_quant(x, torch.from_numpy(arranged).cuda(), b, wl.fmt)
            torch.cuda.synchronize()
            rep = parity.compare_apply(x_bits[rows], arranged, b, wl.fmt, codes[rows_t].cpu().numpy(),
                                       scales[rows_t].cpu().numpy())
            print("        arranged:", rep.summary(), flush=True)
            assert rep.ok(), (rep.summary(), rep.notes[:5])
            del codes, scales


def test_calibration_equalises_block_mass_and_lowers_the_rotated_maximum():
    """configs[4]: blockwise l1 spread and post-rotation maximum, greedy permutation vs identity."""
    import torch
    wl = synth.calib_apply()
    a = binding.perq_colabs_mean(binding.bits_to_device(wl.calib_rows())).cpu().numpy()
    x_bits = wl.apply_rows(0, 512)
    X = orc.bf16_bits_to_f64(x_bits)
    x = binding.bits_to_device(x_bits)
    for b in wl.block_sizes:
        perm = binding.perq_massdiff_perm(a, b)
        # block masses of the library's own statistic under its own permutation (plain sums here: the
        # oracle is not handed values that the library produced)
        a64 = a.astype(np.float64)
        Lg, Li = a64[perm].reshape(-1, b).sum(axis=1), a64.reshape(-1, b).sum(axis=1)
        # one outlier channel alone outweighs an average block, so max_j L_j cannot go below a_max;
        # the greedy reaches that floor (the heaviest channel is joined by the b-1 lightest ones)
        assert Lg.max() - Lg.min() < Li.max() - Li.min()
        assert Lg.max() / Lg.mean() < Li.max() / Li.mean()
        assert Lg.max() <= max(a.max() + (b - 1) * np.median(a), 1.01 * a.sum() / Lg.size)
        yg = binding.perq_permute_rotate_f32(x, torch.from_numpy(perm).cuda(), b).cpu().numpy()
        yi = binding.perq_permute_rotate_f32(x, None, b).cpu().numpy()
        bound_g = np.abs(X[:, perm]).reshape(512, -1, b).sum(axis=2).max(axis=1) / np.sqrt(b)
        bound_i = np.abs(X).reshape(512, -1, b).sum(axis=2).max(axis=1) / np.sqrt(b)
        # Proposition 2 on the device output, and the permutation lowers both bound and maximum
        assert np.all(np.abs(yg).max(axis=1) <= bound_g * (1 + 1e-5))
        assert np.all(np.abs(yi).max(axis=1) <= bound_i * (1 + 1e-5))
        assert bound_g.mean() < bound_i.mean()
        assert np.abs(yg).max(axis=1).mean() < np.abs(yi).max(axis=1).mean()
        print(f"[calib] b={b}: block-mass spread {Li.max()-Li.min():.3f} -> {Lg.max()-Lg.min():.5f}; "
              f"mean bound {bound_i.mean():.2f} -> {bound_g.mean():.2f}; "
              f"mean |y|max {np.abs(yi).max(axis=1).mean():.2f} -> {np.abs(yg).max(axis=1).mean():.2f}", flush=True)
