"""perq_colabs_mean_static, the entry point that allocates nothing, against perq_colabs_mean (same
kernels, the partial sums in the library's own array instead of a caller's workspace) and against
the oracle; two calls in a row, the second on a smaller input."""
import ctypes

import numpy as np
import pytest

from oracle import perq_oracle as orc
from paper_2601_22347_amd import binding, synth

pytestmark = pytest.mark.gpu


def _rows(seed, M, d):
    rng = np.random.default_rng(seed)
    x = rng.standard_t(4, size=(M, d)) * np.exp(rng.uniform(-1.0, 1.0, size=(1, d)))
    return synth.f64_to_bf16_bits(x)


def test_static_scratch_entry_point_matches_the_workspace_one():
    import torch
    lib = binding.load()
    stream = torch.cuda.current_stream()
    sp = ctypes.c_void_p(stream.cuda_stream)
    # the second input is smaller in both directions: fewer slices, narrower rows; the third is the
    # largest the array holds for its width (32 slices of 32768 columns = 4 MiB)
    for seed, (M, d) in enumerate([(4096, 8192), (777, 2048), (260, 32768)]):
        print(f"[case] perq_colabs_mean_static M={M} d={d}", flush=True)
        bits = _rows(seed, M, d)
        x = binding.bits_to_device(bits)
        want = binding.perq_colabs_mean(x)
        got = torch.full((d,), -1.0, dtype=torch.float32, device="cuda")
        st = lib.perq_colabs_mean_static(ctypes.c_void_p(x.data_ptr()), M, d, d, ctypes.c_void_p(got.data_ptr()), sp)
        assert st == binding.PERQ_OK
        torch.cuda.synchronize()
        assert torch.equal(got, want)                                   # bit for bit
        a = orc.colabs_mean(orc.bf16_bits_to_f64(bits))
        r = max(8, -(-M // (512 // -(-d // 2048))))                      # rows per slice of the first pass
        assert np.all(np.abs(got.cpu().numpy() - a) <= (r + 1) * 2.0 ** -24 * a)
    # strided rows, the same call again on the first size (the array holds the last call's partials)
    bits = _rows(9, 1000, 4096)
    wide = torch.zeros((1000, 4096 + 64), dtype=torch.bfloat16, device="cuda")
    wide[:, :4096] = binding.bits_to_device(bits)
    got = torch.empty(4096, dtype=torch.float32, device="cuda")
    binding.perq_colabs_mean_static(wide[:, :4096], got)
    torch.cuda.synchronize()
    assert torch.equal(got, binding.perq_colabs_mean(binding.bits_to_device(bits)))


def test_static_scratch_entry_point_rejects_what_it_cannot_hold():
    import torch
    lib = binding.load()
    fake = ctypes.c_void_p(0x10000)
    INV, UNS = binding.PERQ_ERR_INVALID_ARG, binding.PERQ_ERR_UNSUPPORTED
    assert lib.perq_colabs_mean_static(None, 4, 256, 256, fake, None) == INV
    assert lib.perq_colabs_mean_static(fake, 0, 256, 256, fake, None) == INV
    assert lib.perq_colabs_mean_static(fake, 4, 256, 128, fake, None) == INV
    assert lib.perq_colabs_mean_static(fake, 4, 252, 256, fake, None) == UNS
    # wider than the array's limit (one slice of 2^21 columns needs 8 MiB of partial sums)
    assert lib.perq_colabs_mean_workspace_bytes(16, 1 << 21) > (4 << 20)
    assert lib.perq_colabs_mean_static(fake, 16, 1 << 21, 1 << 21, fake, None) == UNS
    assert torch.cuda.is_available()
