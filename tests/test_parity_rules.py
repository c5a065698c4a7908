"""The comparison rules themselves, on the CPU: the oracle's own output passes, planted mistakes fail."""
import os
import sys

import numpy as np
import pytest

sys.path.insert(0, os.path.dirname(os.path.abspath(__file__)))
import parity  # noqa: E402
from oracle import perq_oracle as orc  # noqa: E402
from paper_2601_22347_amd import synth  # noqa: E402


def _case(fmt, b=32, T=24, d=256, seed=0):
    rng = np.random.default_rng(seed)
    x = synth.f64_to_bf16_bits(rng.standard_t(4, size=(T, d)) + (0.3 if fmt == "int4_asym" else 0.0))
    perm = rng.permutation(d).astype(np.int32)
    ref = orc.perq_apply(x, perm, b, fmt)
    return x, perm, ref


@pytest.mark.parametrize("fmt", ["int4", "mxfp4", "int4_asym", "fp4_token"])
def test_oracle_output_passes_and_planted_mistakes_fail(fmt):
    x, perm, ref = _case(fmt)
    rep = parity.compare_apply(x, perm, 32, fmt, ref["packed"], ref["scales"], ref["y"].astype(np.float32))
    assert rep.ok() and rep.code_mismatch_A == 0 and rep.code_mismatch_B == 0, rep.summary()
    # a wrong code in one place
    bad = ref["packed"].copy()
    bad[3, 7] ^= 0x02
    assert not parity.compare_apply(x, perm, 32, fmt, bad, ref["scales"]).ok()
    # nibbles of a byte swapped
    bad = ref["packed"].copy()
    bad[5, :] = (bad[5, :] >> 4) | ((bad[5, :] & 0xF) << 4)
    assert not parity.compare_apply(x, perm, 32, fmt, bad, ref["scales"]).ok()
    # a wrong scale
    sc = ref["scales"].copy()
    if fmt == "mxfp4":
        sc[2, 1] += 1
    elif fmt == "int4_asym":
        sc[2, 0] *= 1.01
    else:
        sc[2] *= 1.01
    assert not parity.compare_apply(x, perm, 32, fmt, ref["packed"], sc).ok()
    # the permutation ignored
    ref_id = orc.perq_apply(x, None, 32, fmt)
    assert not parity.compare_apply(x, perm, 32, fmt, ref_id["packed"], ref_id["scales"]).ok()


def test_asym_zero_point_off_by_one_is_a_failure_away_from_a_tie():
    x, perm, ref = _case("int4_asym", seed=3)
    sc = ref["scales"].copy()
    lo_q = ref["y"].min(axis=1) / ref["s64"]
    row = int(np.argmax(np.abs(lo_q - np.floor(lo_q) - 0.5)))       # the row farthest from a tie
    sc[row, 1] += 1
    assert not parity.compare_apply(x, perm, 32, "int4_asym", ref["packed"], sc).ok()
