"""Pins for the oracle's bfloat16 rounding of scores (Section 6 of the paper names lower-precision
scores as a direction; the reading taken is round-to-nearest-even of the fp32 score).  None of
these re-evaluates the oracle's own formula: hand-worked values, the format's invariants, and
PyTorch's CPU conversion as an independent library routine."""
import numpy as np
import torch

import oracle


def test_hand_worked_values():
    # 8-bit significand: neighbours of 1.0 are 1 - 2^-8 and 1 + 2^-7
    cases = {
        1.0: 1.0,
        1.0 + 2.0 ** -8: 1.0,                    # tie -> even significand (1.0000000b)
        1.0 + 3.0 * 2.0 ** -8: 1.0 + 2.0 ** -6,  # tie between 1+2^-7 (odd) and 1+2^-6 (even)
        1.0 + 2.0 ** -8 + 2.0 ** -20: 1.0 + 2.0 ** -7,   # just above the tie
        1.0 - 2.0 ** -10: 1.0,                   # rounds up across the power of two
        0.1: 0.10009765625,                      # 0x3DCD
        0.3333333432674408: 0.333984375,         # 0x3EAB
        0.0: 0.0,
        2.0 ** -126: 2.0 ** -126,
        2.0 ** -133: 2.0 ** -133,                # smallest subnormal is kept
        2.0 ** -135: 0.0,                        # below half of it: flushed by rounding
    }
    for x, want in cases.items():
        got = float(oracle.to_bfloat16(np.array([x]))[0])
        assert got == want, (x, got, want)


def test_matches_the_library_conversion_on_scores_and_small_values():
    rng = np.random.default_rng(11)
    x = np.concatenate([rng.random(200000), rng.random(50000) * 1e-6, np.exp(-rng.random(50000) * 60)])
    ours = oracle.to_bfloat16(x)
    lib = torch.from_numpy(x.astype(np.float32)).to(torch.bfloat16).to(torch.float64).numpy()
    assert np.array_equal(ours, lib)


def test_format_invariants():
    rng = np.random.default_rng(12)
    x = rng.random(100000)
    y = oracle.to_bfloat16(x)
    assert np.array_equal(oracle.to_bfloat16(y), y)                      # idempotent
    assert np.all(np.abs(y - x.astype(np.float32)) <= np.abs(x) * 2.0 ** -8)   # half an ulp is 2^(e-8) <= |x| 2^-8
    order = np.argsort(x)
    assert np.all(np.diff(y[order]) >= 0)                                # monotone
    # every result has at most 8 significant bits: scaled to [128, 256) it is an integer
    nz = y[y > 2.0 ** -120]
    scaled = nz / np.exp2(np.floor(np.log2(nz)) - 7)
    assert np.array_equal(scaled, np.rint(scaled))
