"""Seeded synthetic activations for tests and benchmarks.

This module only draws random numbers and rounds them to bfloat16 bit patterns.  It holds none
of the method's arithmetic (no rotation, no quantizer, no permutation search) and imports
neither the HIP binding nor the CPU checker; both are fed the same uint16 arrays from here.

The workloads stand in for the down-projection input activations the paper measures on
(Llama3 widths d = 8192 and 14336 from Table 3, a 2048-token calibration sequence from
Appendix B, channel-concentrated outliers as in Figure 1, signs close to i.i.d. +-1 as checked
in Appendix D).  The text corpora and checkpoints themselves are not used.

Rows are generated in independent chunks of CHUNK rows, chunk c of a stream being seeded with
(seed, c), so any row range of a large workload can be produced without the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

CHUNK = 1024
CLAMP = 1.0e4      # Student-t(3) has unbounded kurtosis; keep every draw finite in bf16


def f64_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float64 -> float32 -> bfloat16 (round to nearest, ties to even) -> uint16 bit pattern."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


@dataclass
class Workload:
    """One synthetic activation law: base distribution, outlier channels, massive rows."""
    name: str
    T: int
    d: int
    law: str                      # "normal" or "student_t"
    nu: float = 0.0
    data_seed: int = 0
    calib_seed: int = 0
    calib_tokens: int = 0
    outlier_channels: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    outlier_factors: np.ndarray = field(default_factory=lambda: np.zeros(0, np.float64))
    massive_rows: np.ndarray = field(default_factory=lambda: np.zeros(0, np.int64))
    massive_factor: float = 1.0
    block_sizes: tuple = ()
    fmt: str = "int4"

    def _chunk(self, seed: int, c: int, rows: int) -> np.ndarray:
        rng = np.random.default_rng([seed, c])
        if self.law == "normal":
            x = rng.standard_normal((rows, self.d))
        elif self.law == "student_t":
            x = rng.standard_t(self.nu, size=(rows, self.d))
        else:
            raise ValueError(self.law)
        if self.outlier_channels.size:
            x[:, self.outlier_channels] *= self.outlier_factors
        return x

    def _rows(self, seed: int, r0: int, r1: int, total: int, massive: bool) -> np.ndarray:
        if not (0 <= r0 <= r1 <= total):
            raise ValueError("row range out of bounds")
        out = np.empty((r1 - r0, self.d), dtype=np.uint16)
        c = r0 // CHUNK
        while c * CHUNK < r1:
            lo, hi = c * CHUNK, min((c + 1) * CHUNK, total)
            x = self._chunk(seed, c, hi - lo)
            if massive and self.massive_rows.size:
                sel = self.massive_rows[(self.massive_rows >= lo) & (self.massive_rows < hi)]
                x[sel - lo, :] *= self.massive_factor
            np.clip(x, -CLAMP, CLAMP, out=x)
            a, b_ = max(lo, r0), min(hi, r1)
            out[a - r0:b_ - r0] = f64_to_bf16_bits(x[a - lo:b_ - lo])
            c += 1
        return out

    def apply_rows(self, r0: int = 0, r1: int | None = None) -> np.ndarray:
        """bf16 bits [r1-r0, d] of the apply-time token stream."""
        r1 = self.T if r1 is None else r1
        return self._rows(self.data_seed, r0, r1, self.T, massive=True)

    def apply_rows_parallel(self, r0: int = 0, r1: int | None = None, threads: int = 8) -> np.ndarray:
        """Same rows as apply_rows, generated chunk by chunk on a few threads (NumPy's generators
        release the GIL); for the full-size workloads."""
        from concurrent.futures import ThreadPoolExecutor
        r1 = self.T if r1 is None else r1
        out = np.empty((r1 - r0, self.d), dtype=np.uint16)
        spans = [(max(e, r0), min(e + CHUNK, r1)) for e in range(r0 - r0 % CHUNK, r1, CHUNK)]

        def work(span):
            a, b_ = span
            out[a - r0:b_ - r0] = self.apply_rows(a, b_)

        with ThreadPoolExecutor(max_workers=threads) as ex:
            list(ex.map(work, spans))
        return out

    def calib_rows(self) -> np.ndarray:
        """bf16 bits [calib_tokens, d] of the calibration stream (same outlier channels)."""
        return self._rows(self.calib_seed, 0, self.calib_tokens, self.calib_tokens, massive=False)


def _channels(d: int, count: int, seed: int, lo: float, hi: float):
    rng = np.random.default_rng(seed)
    ch = np.sort(rng.choice(d, size=count, replace=False))
    fac = np.full(count, lo) if lo == hi else rng.uniform(lo, hi, size=count)
    return ch.astype(np.int64), fac.astype(np.float64)


def tiny() -> Workload:
    """T=64, d=256, N(0,1), four fixed outlier channels x50 (three of them in block 0 at b=16)."""
    return Workload("tiny", 64, 256, "normal", data_seed=100, calib_seed=101, calib_tokens=256,
                    outlier_channels=np.array([4, 5, 6, 200]), outlier_factors=np.full(4, 50.0),
                    block_sizes=(16,), fmt="int4")


def llama1b_down() -> Workload:
    """T=2048, d=8192, Student-t(4), 1% of channels scaled by U[20,100]."""
    ch, fac = _channels(8192, 82, 112, 20.0, 100.0)
    return Workload("llama1b_down", 2048, 8192, "student_t", nu=4.0, data_seed=110, calib_seed=111,
                    calib_tokens=2048, outlier_channels=ch, outlier_factors=fac,
                    block_sizes=(16, 32, 64, 128), fmt="int4")


def block_vs_full() -> Workload:
    """T=16384, d=2048, N(0,1), 0.5% channels x50, 0.1% whole rows x200; MXFP4; identity perm."""
    ch, fac = _channels(2048, 10, 122, 50.0, 50.0)
    rows = np.sort(np.random.default_rng(123).choice(16384, size=16, replace=False)).astype(np.int64)
    return Workload("block_vs_full", 16384, 2048, "normal", data_seed=120,
                    outlier_channels=ch, outlier_factors=fac, massive_rows=rows,
                    massive_factor=200.0, block_sizes=(32, 2048), fmt="mxfp4")


def llama8b(d: int) -> Workload:
    """T=32768, d in {4096, 14336}, Student-t(3), 1% channels x50; INT4 with the gather fused."""
    if d == 4096:
        ch, fac = _channels(4096, 41, 134, 50.0, 50.0)
        return Workload("llama8b_d4096", 32768, 4096, "student_t", nu=3.0, data_seed=130,
                        calib_seed=132, calib_tokens=2048, outlier_channels=ch, outlier_factors=fac,
                        block_sizes=(128, 4096), fmt="int4")
    if d == 14336:
        ch, fac = _channels(14336, 143, 135, 50.0, 50.0)
        return Workload("llama8b_d14336", 32768, 14336, "student_t", nu=3.0, data_seed=131,
                        calib_seed=133, calib_tokens=2048, outlier_channels=ch, outlier_factors=fac,
                        block_sizes=(128, 2048), fmt="int4")
    raise ValueError("d must be 4096 or 14336")


def qwen3(d: int) -> Workload:
    """T=32768, d in {9728, 12288} (Qwen3 4B / 8B down-projection inputs, widths 2^7*76 and 2^10*12),
    Student-t(3), 1% channels x50; INT4; for the full-vector rotation of non-power-of-two width."""
    if d not in (9728, 12288):
        raise ValueError("d must be 9728 or 12288")
    ch, fac = _channels(d, d // 100, 154 if d == 9728 else 155, 50.0, 50.0)
    return Workload(f"qwen3_d{d}", 32768, d, "student_t", nu=3.0, data_seed=150 if d == 9728 else 151,
                    calib_seed=152 if d == 9728 else 153, calib_tokens=2048, outlier_channels=ch,
                    outlier_factors=fac, block_sizes=(d,), fmt="int4")


def calib_apply() -> Workload:
    """Calibrate on 4096 tokens of d=8192, apply to T=65536; Student-t(3) + 1% channels xU[20,100]."""
    ch, fac = _channels(8192, 82, 142, 20.0, 100.0)
    return Workload("calib_apply", 65536, 8192, "student_t", nu=3.0, data_seed=140, calib_seed=141,
                    calib_tokens=4096, outlier_channels=ch, outlier_factors=fac,
                    block_sizes=(16, 32), fmt="mxfp4")


ALL = {"tiny": tiny, "llama1b_down": llama1b_down, "block_vs_full": block_vs_full,
       "llama8b_d4096": lambda: llama8b(4096), "llama8b_d14336": lambda: llama8b(14336),
       "calib_apply": calib_apply, "qwen3_d9728": lambda: qwen3(9728), "qwen3_d12288": lambda: qwen3(12288)}


def device_rows(T: int, d: int, seed: int, device="cuda", rows_per_draw: int = 65536):
    """T x d bfloat16 rows drawn on the device, for inputs too large to draw on the host (several
    GiB): N(0, 1) entries, every 97th channel scaled by 24 (channel-concentrated outliers).
    Seeded: draw k of rows_per_draw rows uses torch's device generator seeded with (seed, k)."""
    import torch
    x = torch.empty((T, d), dtype=torch.bfloat16, device=device)
    scale = torch.ones(d, dtype=torch.float32, device=device)
    scale[5::97] = 24.0
    gen = torch.Generator(device=device)
    for k, r0 in enumerate(range(0, T, rows_per_draw)):
        r1 = min(T, r0 + rows_per_draw)
        gen.manual_seed(seed * 1000003 + k)
        block = torch.randn((r1 - r0, d), generator=gen, device=device, dtype=torch.float32)
        x[r0:r1] = (block * scale).to(torch.bfloat16)
    return x
