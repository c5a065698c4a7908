"""Inputs and outputs beyond 2^31 elements / 4 GiB: every kernel family on rows whose byte offsets
do not fit 32 bits, checked on sampled rows against the oracle (the first and last rows, the rows
on either side of the 2 GiB and 4 GiB offsets of the input and of the output, and random ones)."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402
from oracle import perq_oracle as orc  # noqa: E402
from paper_2601_22347_amd import binding, synth  # noqa: E402

pytestmark = pytest.mark.gpu


def _rows_to_check(T, row_bytes_list, seed, extra=12):
    rows = {0, 1, T - 2, T - 1}
    for rb in row_bytes_list:
        for edge in (1 << 31, 1 << 32):
            r = edge // rb
            rows.update(q for q in (r - 1, r, r + 1) if 0 <= q < T)
    rng = np.random.default_rng(seed)
    rows.update(int(q) for q in rng.integers(0, T, size=extra))
    return np.array(sorted(rows), dtype=np.int64)


def _bits(t):
    import torch
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


# T, d, b, fmt, permutation, algo: T * d just above 2^31 elements (the input is 4 GiB + a few rows)
LARGE = [
    (524291, 4096, 128, "int4", True, "auto"),          # mfma_kernel, wave-local rows, run-time schedule
    (524291, 4096, 64, "mxfp4", True, "butterfly"),     # shuffle butterflies
    (262147, 8192, 32, "mxfp4", False, "mfma"),         # rows over two waves
    (149800, 14336, 14336, "int4", False, "auto"),      # chunked kernel, base 28
    (262147, 8192, 8192, "int4_asym", True, "auto"),    # chunked kernel, Sylvester base
    (4194309, 512, 128, "fp4_token", True, "auto"),     # eight rows folded into one, five left over
]


@pytest.mark.parametrize("T,d,b,fmt,with_perm,algo", LARGE)
def test_rows_past_4_gib(T, d, b, fmt, with_perm, algo):
    import torch
    print(f"[large] T={T} d={d} b={b} {fmt} perm={with_perm} algo={algo}", flush=True)
    x = synth.device_rows(T, d, seed=T % 1000 + d)
    perm = perm_t = None
    if with_perm:
        perm = orc.perm_random(d, 11)
        perm_t = torch.from_numpy(perm.astype(np.int32)).cuda()
    codes, scales = binding.perq_permute_rotate_quant(x, perm_t, b, fmt, algo=algo)
    torch.cuda.synchronize()
    scale_bytes = scales.element_size() * (scales.numel() // T)
    rows = _rows_to_check(T, [2 * d, d // 2, scale_bytes], seed=d + b)
    rows_t = torch.from_numpy(rows).cuda()
    rep = parity.compare_apply(_bits(x[rows_t]), perm, b, fmt, codes[rows_t].cpu().numpy(),
                               scales[rows_t].cpu().numpy())
    print("       ", rep.summary(), flush=True)
    assert rep.ok(), (rep.summary(), rep.notes[:5])


@pytest.mark.parametrize("T,d,b,algo", [(262147, 4096, 128, "mfma"), (262147, 4096, 4096, "butterfly"),
                                         (87400, 12288, 3072, "auto")])
def test_fp32_output_past_4_gib(T, d, b, algo):
    """The pre-quantization output is 4 bytes per element: past 4 GiB from 2^30 elements on."""
    import torch
    print(f"[large] f32 T={T} d={d} b={b} algo={algo}", flush=True)
    x = synth.device_rows(T, d, seed=3 + b)
    y = binding.perq_permute_rotate_f32(x, None, b, algo=algo)
    torch.cuda.synchronize()
    rows = _rows_to_check(T, [2 * d, 4 * d], seed=b)
    rows_t = torch.from_numpy(rows).cuda()
    x_bits = _bits(x[rows_t])
    rep = parity.ParityReport()
    parity.check_prequant(y[rows_t].cpu().numpy(), orc.block_hadamard(orc.bf16_bits_to_f64(x_bits), b), x_bits, rep)
    print("       ", rep.summary(), flush=True)
    assert rep.ok(), (rep.summary(), rep.notes[:5])


def test_statistics_past_4_gib():
    """perq_colabs_mean and perq_block_diagnostics on 2^31 + elements.  The oracle's channel means are
    taken slice by slice (65536 rows at a time) and combined with the slices' row counts."""
    import torch
    T, d, b = 524291, 4096, 128
    x = synth.device_rows(T, d, seed=77)
    a = binding.perq_colabs_mean(x).cpu().numpy()
    total = np.zeros(d, dtype=np.float64)
    for r0 in range(0, T, 65536):
        part = orc.bf16_bits_to_f64(_bits(x[r0:r0 + 65536]))
        total += orc.colabs_mean(part) * part.shape[0]
    a_orc = total / T
    # fp32 partial sums of 1024+ rows per slice: the worst case is (rows per slice + 1) * 2^-24, the
    # rounding errors of random data stay far below it; 33 * 2^-24 is about the weight 1/T of one row,
    # so a row left out or counted twice fails
    assert np.all(np.abs(a - a_orc) <= 33 * 2.0 ** -24 * a_orc)
    perm = orc.massdiff_greedy(a_orc, b)
    diag = binding.perq_block_diagnostics(x, torch.from_numpy(perm.astype(np.int32)).cuda(), b)
    torch.cuda.synchronize()
    rows = _rows_to_check(T, [2 * d], seed=5)
    rows_t = torch.from_numpy(rows).cuda()
    bits = _bits(x[rows_t])
    want = orc.block_diagnostics(bits, perm, b)
    got = diag[rows_t].cpu().numpy().astype(np.float64)
    l2 = np.linalg.norm(orc.bf16_bits_to_f64(bits), axis=1)
    assert np.array_equal(got[:, 0], want[:, 0])
    assert np.allclose(got[:, 1], want[:, 1], rtol=2e-6) and np.allclose(got[:, 2], want[:, 2], rtol=2e-6)
    assert np.all(np.abs(got[:, 3] - want[:, 3]) <= 1e-5 * l2)
