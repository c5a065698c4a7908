"""The input generators: bf16 rounding, chunk independence, outlier structure (CPU only)."""
import numpy as np

from paper_2601_22347_amd import synth


def test_bf16_round_to_nearest_even():
    # 1 + 2^-8 is exactly half-way between bf16 neighbours 1.0 and 1 + 2^-7: ties to even -> 1.0
    x = np.array([1.0, 1.0 + 2.0 ** -8, 1.0 + 2.0 ** -7 + 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -3.140625, 0.0])
    bits = synth.f64_to_bf16_bits(x)
    assert bits.tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0xC049, 0x0000]


def test_row_ranges_are_reproducible_and_chunk_independent():
    wl = synth.block_vs_full()
    a = wl.apply_rows(1000, 1100)
    b = wl.apply_rows(0, 2048)[1000:1100]
    assert np.array_equal(a, b)
    assert np.array_equal(wl.apply_rows(5, 9), wl.apply_rows(5, 9))


def test_outlier_structure():
    wl = synth.tiny()
    x = (wl.apply_rows().astype(np.uint32) << 16).view(np.float32)
    col = np.abs(x).mean(axis=0)
    assert set(np.argsort(-col)[:4].tolist()) == {4, 5, 6, 200}
    wl2 = synth.block_vs_full()
    r = int(wl2.massive_rows[0])
    seg = (wl2.apply_rows(r - 1, r + 1).astype(np.uint32) << 16).view(np.float32)
    assert np.abs(seg[1]).mean() > 50 * np.abs(seg[0]).mean()
    assert np.isfinite((synth.llama8b(4096).apply_rows(0, 64).astype(np.uint32) << 16)
                       .view(np.float32)).all()
