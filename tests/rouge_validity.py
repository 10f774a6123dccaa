"""Comparison of a ROUGE-N result of the GPU path with the oracle's (shared by the GPU tests).

The oracle picks the best reference in exact rational arithmetic; the kernel picks it on a
single-precision quotient proportional to F (one fused multiply-add and one division, each
rounded once: relative error at most 2 * 2^-24 per quotient).  Two references whose exact F
differ by less than 4 * 2^-24 relative may therefore be ordered differently by the kernel, and
either is a valid answer.  What is checked: overlap counts bit-exactly; the kernel's choice has an
exact F within that bound of the best exact F; precision, recall and F equal the oracle's numbers
FOR THE REFERENCE THE KERNEL CHOSE within the score tolerance.
"""
import numpy as np

CHOICE_EPS = 4.0 * 2.0 ** -24


def check_rouge(ref, overlap, best, prf, tol=1e-5, ref_count=None):
    overlap, best = np.asarray(overlap), np.asarray(best)
    prf = np.asarray(prf, dtype=np.float64)
    np.testing.assert_array_equal(overlap, ref.overlap)
    B, R = ref.overlap.shape
    used = np.full(B, R) if ref_count is None else np.asarray(ref_count)
    assert ((best >= 0) & (best < used)).all(), "chosen reference outside the candidate's references"
    rows = np.arange(B)
    chosen = ref.prf_all[rows, best]
    f_best = ref.prf[:, 2]
    assert (chosen[:, 2] >= f_best * (1.0 - CHOICE_EPS)).all(), "chosen reference is not the best"
    if B:
        assert np.abs(prf - chosen).max() <= tol
    return int((best != ref.best).sum())      # how many (near-)ties went to another reference
