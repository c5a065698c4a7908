"""Comparison rules between the HIP library and the CPU oracle (shared by the GPU tests,
the smoke check and the benchmark's self-check).

Pre-quantization values: per token row, max_i |y_gpu - y_orc| <= 1e-5 * ||x_row||_2.
Codes / scales: bit-exact, except where the oracle's pre-rounding value lies within the
pre-quantization tolerance of a rounding boundary:
   (A) |v - boundary| <= 1e-5 code units             (strict)
   (B) |v - boundary| <= 1e-5 * ||x_row||_2 / scale  (the tolerance above, in code units)
A mismatch outside (B), or by more than one code, is a failure; mismatches inside are counted.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

from oracle import perq_oracle as orc

REL_TOL = 1e-5
E2M1_BOUNDARIES = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])


@dataclass
class ParityReport:
    elements: int = 0
    code_mismatch_A: int = 0        # within 1e-5 code units of a boundary
    code_mismatch_B: int = 0        # within the pre-quant tolerance but not (A)
    code_mismatch_fail: int = 0
    scale_exceptions: int = 0       # MXFP4 groups whose maximum sits on a power-of-two boundary
    scale_fail: int = 0
    neg_zero_seen: int = 0
    max_prequant_rel: float = 0.0
    notes: list = field(default_factory=list)

    def ok(self) -> bool:
        return self.code_mismatch_fail == 0 and self.scale_fail == 0 and self.max_prequant_rel <= REL_TOL

    def summary(self) -> dict:
        return {"elements": self.elements, "mismatch_A": self.code_mismatch_A,
                "mismatch_B_only": self.code_mismatch_B, "mismatch_fail": self.code_mismatch_fail,
                "scale_exceptions": self.scale_exceptions, "scale_fail": self.scale_fail,
                "neg_zero": self.neg_zero_seen, "max_prequant_rel": self.max_prequant_rel}


def row_l2(x_bits: np.ndarray) -> np.ndarray:
    return np.linalg.norm(orc.bf16_bits_to_f64(x_bits), axis=1)


def unpack_nibbles(packed: np.ndarray) -> np.ndarray:
    T, h = packed.shape
    out = np.empty((T, 2 * h), dtype=np.uint8)
    out[:, 0::2] = packed & 0xF
    out[:, 1::2] = packed >> 4
    return out


def check_prequant(y_gpu: np.ndarray, y_orc: np.ndarray, x_bits: np.ndarray, rep: ParityReport) -> None:
    l2 = row_l2(x_bits)
    err = np.abs(y_gpu.astype(np.float64) - y_orc).max(axis=1)
    rel = np.where(l2 > 0, err / np.where(l2 > 0, l2, 1.0), np.where(err == 0, 0.0, np.inf))
    rep.max_prequant_rel = max(rep.max_prequant_rel, float(rel.max()) if rel.size else 0.0)


def check_int4(packed_gpu: np.ndarray, scales_gpu: np.ndarray, ref: dict, x_bits: np.ndarray,
               rep: ParityReport) -> None:
    l2 = row_l2(x_bits)
    nib = unpack_nibbles(packed_gpu).astype(np.int16)
    c_gpu = np.where(nib >= 8, nib - 16, nib).astype(np.int16)
    c_orc = ref["codes"].astype(np.int16)
    rep.elements += c_orc.size
    s = ref["s64"]
    # scale: float32, within the pre-quant tolerance / 7
    sd = np.abs(scales_gpu.astype(np.float64) - s)
    bad_scale = sd > REL_TOL * l2 / 7.0
    rep.scale_fail += int(bad_scale.sum())
    if bad_scale.any():
        i = int(np.argmax(bad_scale))
        rep.notes.append(f"int4 scale row {i}: gpu {scales_gpu[i]!r} oracle {s[i]!r}")
    mis = c_gpu != c_orc
    if mis.any():
        rows, cols = np.nonzero(mis)
        v = ref["y"][rows, cols] / s[rows]
        bnd = np.floor(v) + 0.5
        dist = np.abs(v - bnd)
        adjacent = np.abs(c_gpu[rows, cols] - c_orc[rows, cols]) == 1
        # the two codes must be the ones on either side of that boundary
        sides = np.minimum(c_gpu[rows, cols], c_orc[rows, cols]) == np.floor(v)
        inA = adjacent & sides & (dist <= REL_TOL)
        inB = adjacent & sides & (dist <= REL_TOL * l2[rows] / s[rows]) & ~inA
        fail = ~(inA | inB)
        rep.code_mismatch_A += int(inA.sum())
        rep.code_mismatch_B += int(inB.sum())
        rep.code_mismatch_fail += int(fail.sum())
        if fail.any():
            k = int(np.argmax(fail))
            rep.notes.append(f"int4 code row {rows[k]} col {cols[k]}: gpu {c_gpu[rows[k], cols[k]]} "
                             f"oracle {c_orc[rows[k], cols[k]]} v {v[k]!r}")


def check_mxfp4(packed_gpu: np.ndarray, E_gpu: np.ndarray, ref: dict, x_bits: np.ndarray,
                rep: ParityReport) -> None:
    l2 = row_l2(x_bits)
    T, d = ref["codes"].shape
    c_gpu = unpack_nibbles(packed_gpu)
    rep.neg_zero_seen += int((c_gpu == 8).sum())
    c_gpu = np.where(c_gpu == 8, 0, c_gpu).astype(np.uint8)
    E_orc = ref["scales"].astype(np.int64)
    E_g = E_gpu.astype(np.int64)
    rep.elements += T * d
    c_orc = ref["codes"]
    Ediff = E_g != E_orc
    if Ediff.any():
        # allowed only when the group's maximum is within tolerance of a power of two and the
        # exponents are neighbours; the codes are then checked against the oracle re-quantised
        # with the GPU's exponent
        amax = np.abs(ref["y"]).reshape(T, d // 32, 32).max(axis=2)
        rows, grps = np.nonzero(Ediff)
        a = amax[rows, grps]
        pow2 = np.ldexp(1.0, np.round(np.log2(np.where(a > 0, a, 1.0))).astype(np.int64))
        near = (np.abs(a - pow2) <= REL_TOL * l2[rows]) & (np.abs(E_g[rows, grps] - E_orc[rows, grps]) == 1)
        rep.scale_exceptions += int(near.sum())
        rep.scale_fail += int((~near).sum())
        if (~near).any():
            k = int(np.argmax(~near))
            rep.notes.append(f"mxfp4 E row {rows[k]} group {grps[k]}: gpu {E_g[rows[k], grps[k]]} "
                             f"oracle {E_orc[rows[k], grps[k]]} amax {a[k]!r}")
        c_orc, _ = orc.quant_mxfp4(ref["y"], E_given=np.clip(E_g, 0, 254))
    mis = c_gpu != c_orc
    if mis.any():
        rows, cols = np.nonzero(mis)
        sc = np.ldexp(1.0, E_g[rows, cols // 32] - 127)
        v = np.abs(ref["y"][rows, cols]) / sc
        k = np.abs(v[:, None] - E2M1_BOUNDARIES[None, :]).argmin(axis=1)
        dist = np.abs(v - E2M1_BOUNDARIES[k])
        g, o = c_gpu[rows, cols].astype(np.int16), c_orc[rows, cols].astype(np.int16)
        # neighbours on the magnitude grid with equal sign (or one of them is zero)
        same_sign = ((g & 8) == (o & 8)) | ((g & 7) == 0) | ((o & 7) == 0)
        adjacent = (np.abs((g & 7) - (o & 7)) == 1) & same_sign & (np.minimum(g & 7, o & 7) == k)
        inA = adjacent & (dist <= REL_TOL)
        inB = adjacent & (dist <= REL_TOL * l2[rows] / sc) & ~inA
        fail = ~(inA | inB)
        rep.code_mismatch_A += int(inA.sum())
        rep.code_mismatch_B += int(inB.sum())
        rep.code_mismatch_fail += int(fail.sum())
        if fail.any():
            j = int(np.argmax(fail))
            rep.notes.append(f"mxfp4 code row {rows[j]} col {cols[j]}: gpu {g[j]:#x} oracle {o[j]:#x} v {v[j]!r}")


def check_int4_asym(packed_gpu: np.ndarray, scales_gpu: np.ndarray, ref: dict, x_bits: np.ndarray,
                    rep: ParityReport) -> None:
    """Asymmetric per-token INT4: step within the tolerance of (max - min)/15; the integer zero
    point exact unless min/s is within tolerance of a tie (then the oracle is re-quantised with
    the library's zero point, counted as a scale exception); codes as for the symmetric case.
    The quotient y/s inherits the error of y and of s: tolerance (1 + 2|v|/15) * 1e-5*||x||/s.
    On a row that is a large offset plus a small spread that tolerance exceeds a whole step; the
    rule is therefore written for any size of it: acceptable is the rounding of any quotient
    within tolerance of the oracle's."""
    l2 = row_l2(x_bits)
    c_gpu = unpack_nibbles(packed_gpu).astype(np.int16)
    rep.elements += c_gpu.size
    s, z = ref["s64"], ref["z"]
    s_g, z_g = scales_gpu[:, 0].astype(np.float64), scales_gpu[:, 1].astype(np.float64)
    bad_scale = np.abs(s_g - s) > 2.0 * REL_TOL * l2 / 15.0
    rep.scale_fail += int(bad_scale.sum())
    if bad_scale.any():
        i = int(np.argmax(bad_scale))
        rep.notes.append(f"int4_asym step row {i}: gpu {s_g[i]!r} oracle {s[i]!r}")
    safe = np.where(s > 0, s, 1.0)
    lo_q = ref["y"].min(axis=1) / safe

    def qtol(v, rows):
        # how far the library's quotient y/s may lie from the oracle's, in code units
        return (1.0 + 2.0 * np.abs(v) / 15.0) * REL_TOL * l2[rows] / safe[rows]
    every = np.arange(s.size)
    zd = z_g != z
    if zd.any():
        # acceptable zero points: the roundings of every quotient within tolerance of the oracle's
        # (for a tolerance below half a step: the other side of a tie, as for the codes)
        tz = qtol(lo_q, every)
        near = (z_g >= np.rint(lo_q - tz)) & (z_g <= np.rint(lo_q + tz)) & (s > 0)
        ok_rows = zd & near
        rep.scale_exceptions += int(ok_rows.sum())
        rep.scale_fail += int((zd & ~near).sum())
        if (zd & ~near).any():
            i = int(np.argmax(zd & ~near))
            rep.notes.append(f"int4_asym zero point row {i}: gpu {z_g[i]!r} oracle {z[i]!r} min/s {lo_q[i]!r}")
        c_orc, _, _ = orc.quant_int4_asym_token(ref["y"], z_given=np.where(ok_rows, z_g, z))
        z = np.where(ok_rows, z_g, z)
    else:
        c_orc = ref["codes"]
    c_orc = c_orc.astype(np.int16)
    mis = c_gpu != c_orc
    if mis.any():
        rows, cols = np.nonzero(mis)
        v = ref["y"][rows, cols] / safe[rows]
        bnd = np.floor(v) + 0.5
        dist = np.abs(v - bnd)
        g = c_gpu[rows, cols]
        adjacent = np.abs(g - c_orc[rows, cols]) == 1
        sides = np.minimum(g, c_orc[rows, cols]) + z[rows] == np.floor(v)
        inA = adjacent & sides & (dist <= REL_TOL)
        # (B): the code of some quotient within tolerance of the oracle's (below half a step that is
        # the neighbouring code across a boundary no further away than the tolerance)
        tv = qtol(v, rows)
        c_lo = np.clip(np.rint(v - tv) - z[rows], 0, 15)
        c_hi = np.clip(np.rint(v + tv) - z[rows], 0, 15)
        inB = (g >= c_lo) & (g <= c_hi) & ~inA
        fail = ~(inA | inB)
        rep.code_mismatch_A += int(inA.sum())
        rep.code_mismatch_B += int(inB.sum())
        rep.code_mismatch_fail += int(fail.sum())
        if fail.any():
            k = int(np.argmax(fail))
            rep.notes.append(f"int4_asym code row {rows[k]} col {cols[k]}: gpu {c_gpu[rows[k], cols[k]]} "
                             f"oracle {c_orc[rows[k], cols[k]]} v {v[k]!r} z {z[rows[k]]!r}")


def check_fp4_token(packed_gpu: np.ndarray, scales_gpu: np.ndarray, ref: dict, x_bits: np.ndarray,
                    rep: ParityReport, qmax: float = 6.0) -> None:
    """FP4 with one scale per token: scale within tolerance / 6, codes as for MXFP4 with the
    quotient tolerance (1 + |v|/c) * 1e-5*||x||/s, c = 6 (7 for the step as Appendix B prints it)."""
    l2 = row_l2(x_bits)
    c_gpu = unpack_nibbles(packed_gpu)
    rep.neg_zero_seen += int((c_gpu == 8).sum())
    c_gpu = np.where(c_gpu == 8, 0, c_gpu).astype(np.uint8)
    c_orc = ref["codes"]
    rep.elements += c_orc.size
    s = ref["s64"]
    bad_scale = np.abs(scales_gpu.astype(np.float64) - s) > REL_TOL * l2 / qmax
    rep.scale_fail += int(bad_scale.sum())
    if bad_scale.any():
        i = int(np.argmax(bad_scale))
        rep.notes.append(f"fp4 scale row {i}: gpu {scales_gpu[i]!r} oracle {s[i]!r}")
    safe = np.where(s > 0, s, 1.0)
    mis = c_gpu != c_orc
    if mis.any():
        rows, cols = np.nonzero(mis)
        v = np.abs(ref["y"][rows, cols]) / safe[rows]
        k = np.abs(v[:, None] - E2M1_BOUNDARIES[None, :]).argmin(axis=1)
        dist = np.abs(v - E2M1_BOUNDARIES[k])
        g, o = c_gpu[rows, cols].astype(np.int16), c_orc[rows, cols].astype(np.int16)
        same_sign = ((g & 8) == (o & 8)) | ((g & 7) == 0) | ((o & 7) == 0)
        adjacent = (np.abs((g & 7) - (o & 7)) == 1) & same_sign & (np.minimum(g & 7, o & 7) == k)
        inA = adjacent & (dist <= REL_TOL)
        inB = adjacent & (dist <= (1.0 + v / qmax) * REL_TOL * l2[rows] / safe[rows]) & ~inA
        fail = ~(inA | inB)
        rep.code_mismatch_A += int(inA.sum())
        rep.code_mismatch_B += int(inB.sum())
        rep.code_mismatch_fail += int(fail.sum())
        if fail.any():
            j = int(np.argmax(fail))
            rep.notes.append(f"fp4 code row {rows[j]} col {cols[j]}: gpu {g[j]:#x} oracle {o[j]:#x} v {v[j]!r}")


def compare_apply(x_bits, perm, b, fmt, packed_gpu, scales_gpu, y_gpu=None, rotate=None) -> ParityReport:
    """Run the oracle on x_bits and compare a GPU result (NumPy arrays) with it."""
    rep = ParityReport()
    ref = orc.perq_apply(x_bits, perm, b, fmt, rotate=rotate or orc.block_hadamard)
    if y_gpu is not None:
        check_prequant(y_gpu, ref["y"], x_bits, rep)
    if fmt == "int4":
        check_int4(packed_gpu, scales_gpu, ref, x_bits, rep)
    elif fmt == "mxfp4":
        check_mxfp4(packed_gpu, scales_gpu, ref, x_bits, rep)
    elif fmt == "int4_asym":
        check_int4_asym(packed_gpu, scales_gpu, ref, x_bits, rep)
    else:
        check_fp4_token(packed_gpu, scales_gpu, ref, x_bits, rep, 7.0 if fmt == "fp4_token7" else 6.0)
    return rep


def merge_reports(reports) -> ParityReport:
    out = ParityReport()
    for r in reports:
        out.elements += r.elements
        out.code_mismatch_A += r.code_mismatch_A
        out.code_mismatch_B += r.code_mismatch_B
        out.code_mismatch_fail += r.code_mismatch_fail
        out.scale_exceptions += r.scale_exceptions
        out.scale_fail += r.scale_fail
        out.neg_zero_seen += r.neg_zero_seen
        out.max_prequant_rel = max(out.max_prequant_rel, r.max_prequant_rel)
        out.notes += r.notes[:3]
    return out


def compare_apply_all_rows(x_bits, perm, b, fmt, packed_gpu, scales_gpu, rotate=None, chunk=512, threads=None) -> ParityReport:
    """compare_apply over every row of a full-size result, in chunks of rows on a few threads (NumPy
    releases the interpreter lock in its array loops).  The matrix products of the oracle run on one
    BLAS thread each while several chunks are in flight: concurrent calls into a multi-threaded BLAS
    from several Python threads gave wrong products on this image."""
    import os
    from concurrent.futures import ThreadPoolExecutor
    from threadpoolctl import threadpool_limits
    T = x_bits.shape[0]
    threads = threads or min(16, os.cpu_count() or 1)

    def work(s):
        e = min(T, s + chunk)
        return compare_apply(x_bits[s:e], perm, b, fmt, packed_gpu[s:e], scales_gpu[s:e], None, rotate=rotate)
    with threadpool_limits(limits=1):
        with ThreadPoolExecutor(max_workers=threads) as ex:
            reports = list(ex.map(work, range(0, T, chunk)))
    return merge_reports(reports)

