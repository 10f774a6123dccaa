"""CPU oracle for token-ID BLEU -- TEST INFRASTRUCTURE, not part of the product path.

`bleu_oracle.cpp` is the plain per-sentence dictionary-count definition (fp64, std::map);
`paper_pipeline.py` walks the paper's own tensor-op steps (Sections 3.1-3.4) with numpy.
Only tests, the smoke check and the benchmark's CPU-baseline leg may import this package; it
imports nothing from the HIP package and the HIP package imports nothing from here.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional, Sequence

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "bleu_oracle.cpp")
_LIB = os.path.join(_HERE, "libbleu_oracle.so")

SMOOTHING = {"none": 0, "floor": 1, "add-k": 2, "exp": 3}


def build(force: bool = False) -> str:
    """Compile the C++ oracle with the host compiler (no GPU code involved)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + f".tmp{os.getpid()}"
        subprocess.check_call(["g++", "-O2", "-std=c++17", "-shared", "-fPIC", "-pthread",
                               "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        lib = ctypes.CDLL(build())
        i32p, i64p, f64p = (ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int64),
                            ctypes.POINTER(ctypes.c_double))
        lib.oracle_bleu.restype = ctypes.c_int
        lib.oracle_bleu.argtypes = [i32p, ctypes.c_int64, i32p, i32p, ctypes.c_int64, i32p,
                                    ctypes.c_int, ctypes.c_int, ctypes.c_int, f64p, ctypes.c_int,
                                    ctypes.c_double, ctypes.c_int, i32p, i32p, i32p, i32p, i32p,
                                    f64p, i64p, f64p, i32p]
        lib.oracle_bleu_from_stats.restype = ctypes.c_double
        lib.oracle_bleu_from_stats.argtypes = [i64p, i64p, ctypes.c_int64, ctypes.c_int64,
                                               ctypes.c_int, f64p, ctypes.c_int, ctypes.c_double]
        lib.oracle_group_counts.restype = ctypes.c_int
        lib.oracle_group_counts.argtypes = [i32p, ctypes.c_int, i32p, ctypes.c_int64, i32p,
                                            ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p, i32p,
                                            i32p]
        lib.oracle_rouge_overlap.restype = ctypes.c_int
        lib.oracle_rouge_overlap.argtypes = [i32p, ctypes.c_int64, i32p, i32p, ctypes.c_int64,
                                             i32p, ctypes.c_int, ctypes.c_int, ctypes.c_int, i32p,
                                             i32p]
        _lib = lib
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def expand_reference_lists(refs: np.ndarray, ref_len: np.ndarray, ref_offsets: np.ndarray):
    """Reference lists in CSR form -> the padded fixed-R form plus a per-candidate count.

    refs [rows, Lr], ref_len [rows]; candidate i owns the rows ref_offsets[i] .. ref_offsets[i+1]-1
    in order.  Returns refs [B, R, Lr], ref_len [B, R] (R = the largest list, at least 1), the
    counts [B] and a mask [B] of candidates without any reference.  Such a candidate is given one
    EMPTY reference: nothing can match it, so its statistics and score are 0 and its closest
    reference length is 0 -- the reading taken for a candidate that has nothing to be compared
    with.  Pure rearrangement of the inputs; all arithmetic stays in the routines that follow."""
    refs = np.ascontiguousarray(refs, dtype=np.int32)
    ref_len = np.ascontiguousarray(ref_len, dtype=np.int32)
    off = np.asarray(ref_offsets, dtype=np.int64)
    assert refs.ndim == 2 and ref_len.shape == (refs.shape[0],) and off.ndim == 1
    assert off[0] >= 0 and (np.diff(off) >= 0).all() and off[-1] <= refs.shape[0]
    B = off.size - 1
    counts = np.diff(off).astype(np.int32)
    R = max(int(counts.max()) if B else 1, 1)
    out = np.zeros((B, R, refs.shape[1]), np.int32)
    out_len = np.zeros((B, R), np.int32)
    for i in range(B):
        k = int(counts[i])
        out[i, :k] = refs[off[i]:off[i] + k]
        out_len[i, :k] = ref_len[off[i]:off[i] + k]
    return out, out_len, np.maximum(counts, 1).astype(np.int32), counts == 0


@dataclass
class OracleResult:
    clipped: np.ndarray         # [B, N] int32
    total: np.ndarray           # [B, N] int32
    closest_ref_len: np.ndarray  # [B] int32
    group_distinct: np.ndarray  # [B, N] int32  distinct n-grams over candidate + references
    cand_distinct: np.ndarray   # [B, N] int32  distinct n-grams of the candidate alone
    bleu: np.ndarray            # [B] float64
    corpus_stats: np.ndarray    # [2N+2] int64
    corpus_bleu: float


def bleu(cand: np.ndarray, cand_len: np.ndarray, refs: np.ndarray, ref_len: np.ndarray,
         max_n: int = 4, weights: Optional[Sequence[float]] = None, smoothing: str = "none",
         smooth_param: float = 0.0, threads: int = 1,
         ref_count: Optional[np.ndarray] = None,
         ref_offsets: Optional[np.ndarray] = None) -> OracleResult:
    """Per-sentence and corpus BLEU of a padded batch (see bleu_oracle.cpp for the definition).

    ref_count [B] (optional): candidate i has only its first ref_count[i] references.
    ref_offsets [B + 1] (optional): reference lists in CSR form, refs [rows, Lr], ref_len [rows]
    (see expand_reference_lists)."""
    if ref_offsets is not None:
        assert ref_count is None
        refs, ref_len, ref_count, _ = expand_reference_lists(refs, ref_len, ref_offsets)
    lib = _load()
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    refs = np.ascontiguousarray(refs, dtype=np.int32)
    cand_len = np.ascontiguousarray(cand_len, dtype=np.int32)
    ref_len = np.ascontiguousarray(ref_len, dtype=np.int32)
    B = cand.shape[0]
    assert refs.ndim == 3 and refs.shape[0] == B and ref_len.shape == refs.shape[:2]
    R = refs.shape[1]
    assert (cand_len <= cand.shape[1]).all() and (ref_len <= refs.shape[2]).all()
    assert (cand_len >= 0).all() and (ref_len >= 0).all()
    N = int(max_n)
    w = np.full(N, 1.0 / N) if weights is None else np.asarray(weights, dtype=np.float64)[:N]
    w = np.ascontiguousarray(w, dtype=np.float64)
    clipped = np.zeros((B, N), np.int32)
    total = np.zeros((B, N), np.int32)
    closest = np.zeros(B, np.int32)
    gd = np.zeros((B, N), np.int32)
    cd = np.zeros((B, N), np.int32)
    out = np.zeros(B, np.float64)
    cstats = np.zeros(2 * N + 2, np.int64)
    cb = np.zeros(1, np.float64)
    rcnt = None
    if ref_count is not None:
        rcnt = np.ascontiguousarray(ref_count, dtype=np.int32)
        assert rcnt.shape == (B,)
    rc = lib.oracle_bleu(_p(cand, ctypes.c_int32), cand.shape[1], _p(cand_len, ctypes.c_int32),
                         _p(refs, ctypes.c_int32), refs.shape[2], _p(ref_len, ctypes.c_int32),
                         B, R, N, _p(w, ctypes.c_double), SMOOTHING[smoothing],
                         float(smooth_param), int(threads), _p(clipped, ctypes.c_int32),
                         _p(total, ctypes.c_int32), _p(closest, ctypes.c_int32),
                         _p(gd, ctypes.c_int32), _p(cd, ctypes.c_int32),
                         _p(out, ctypes.c_double), _p(cstats, ctypes.c_int64),
                         _p(cb, ctypes.c_double),
                         _p(rcnt, ctypes.c_int32) if rcnt is not None else None)
    if rc != 0:
        raise ValueError("oracle_bleu: invalid arguments")
    return OracleResult(clipped, total, closest, gd, cd, out, cstats, float(cb[0]))


def bleu_from_stats(clipped, total, c: int, r: int, weights, smoothing: str = "none",
                    smooth_param: float = 0.0) -> float:
    lib = _load()
    cl = np.ascontiguousarray(clipped, dtype=np.int64)
    to = np.ascontiguousarray(total, dtype=np.int64)
    w = np.ascontiguousarray(weights, dtype=np.float64)
    return float(lib.oracle_bleu_from_stats(_p(cl, ctypes.c_int64), _p(to, ctypes.c_int64),
                                            int(c), int(r), len(cl), _p(w, ctypes.c_double),
                                            SMOOTHING[smoothing], float(smooth_param)))


def group_counts(cand_row: np.ndarray, cand_len: int, ref_rows: np.ndarray, ref_len: np.ndarray,
                 n: int):
    """Distinct n-grams of one sentence group with candidate count and max reference count."""
    lib = _load()
    cand_row = np.ascontiguousarray(cand_row, dtype=np.int32)
    ref_rows = np.ascontiguousarray(ref_rows, dtype=np.int32)
    ref_len = np.ascontiguousarray(ref_len, dtype=np.int32)
    R = ref_rows.shape[0]
    cap = int(max(cand_len, 0) + int(np.maximum(ref_len, 0).sum()) + 1)
    grams = np.zeros((cap, n), np.int32)
    cc = np.zeros(cap, np.int32)
    rm = np.zeros(cap, np.int32)
    k = lib.oracle_group_counts(_p(cand_row, ctypes.c_int32), int(cand_len),
                                _p(ref_rows, ctypes.c_int32), ref_rows.shape[1],
                                _p(ref_len, ctypes.c_int32), R, n, cap,
                                _p(grams, ctypes.c_int32), _p(cc, ctypes.c_int32),
                                _p(rm, ctypes.c_int32))
    return grams[:k], cc[:k], rm[:k]


@dataclass
class RougeResult:
    overlap: np.ndarray      # [B, R] int32: sum over n-grams of min(candidate count, reference count)
    prf: np.ndarray          # [B, 3] float64: precision, recall, F of the best reference
    best: np.ndarray         # [B] int32: index of that reference (highest F, lowest index on ties)
    prf_all: np.ndarray      # [B, R, 3] float64: precision, recall, F against every reference
                             # (zeros for references beyond ref_count)


def rouge_n(cand: np.ndarray, cand_len: np.ndarray, refs: np.ndarray, ref_len: np.ndarray,
            n: int = 2, beta: float = 1.0, ref_count: Optional[np.ndarray] = None,
            ref_offsets: Optional[np.ndarray] = None) -> RougeResult:
    """ROUGE-N of every candidate against its references (Lin 2004; the paper's Section 6 names
    ROUGE as the first metric its counting method extends to).

    For one order n and every candidate i, reference j: precision = overlap / candidate n-grams,
    recall = overlap / reference n-grams (each 0 when its denominator is 0),
    F = (1 + beta^2) P R / (R + beta^2 P), 0 when P + R = 0.  The candidate is credited with the
    reference of the highest F, the lowest index among equal ones.  The choice is made in exact
    rational arithmetic (beta is taken as the exact value of the given double), so it does not
    depend on any rounding; the reported numbers are those fractions rounded to float64."""
    from fractions import Fraction
    if ref_offsets is not None:     # CSR reference lists (see expand_reference_lists)
        assert ref_count is None
        refs, ref_len, ref_count, _ = expand_reference_lists(refs, ref_len, ref_offsets)
    lib = _load()
    cand = np.ascontiguousarray(cand, dtype=np.int32)
    refs = np.ascontiguousarray(refs, dtype=np.int32)
    cand_len = np.ascontiguousarray(cand_len, dtype=np.int32)
    ref_len = np.ascontiguousarray(ref_len, dtype=np.int32)
    B, R = cand.shape[0], refs.shape[1]
    assert refs.ndim == 3 and refs.shape[0] == B and ref_len.shape == (B, R)
    assert (cand_len <= cand.shape[1]).all() and (ref_len <= refs.shape[2]).all()
    assert (cand_len >= 0).all() and (ref_len >= 0).all()
    if not float(beta) > 0.0:
        raise ValueError("rouge_n: beta must be positive")
    rcnt = None
    if ref_count is not None:
        rcnt = np.ascontiguousarray(ref_count, dtype=np.int32)
        assert rcnt.shape == (B,)
    overlap = np.zeros((B, R), np.int32)
    rc = lib.oracle_rouge_overlap(_p(cand, ctypes.c_int32), cand.shape[1],
                                  _p(cand_len, ctypes.c_int32), _p(refs, ctypes.c_int32),
                                  refs.shape[2], _p(ref_len, ctypes.c_int32), B, R, int(n),
                                  _p(rcnt, ctypes.c_int32) if rcnt is not None else None,
                                  _p(overlap, ctypes.c_int32))
    if rc != 0:
        raise ValueError("oracle_rouge_overlap: invalid arguments")
    b2 = Fraction(float(beta)) ** 2
    prf = np.zeros((B, 3), np.float64)
    prf_all = np.zeros((B, R, 3), np.float64)
    best = np.zeros(B, np.int32)
    zero = Fraction(0)
    for i in range(B):
        ct = max(int(cand_len[i]) - n + 1, 0)
        top = None
        for j in range(int(rcnt[i]) if rcnt is not None else R):
            rt = max(int(ref_len[i, j]) - n + 1, 0)
            ov = int(overlap[i, j])
            P = Fraction(ov, ct) if ct else zero
            Rc = Fraction(ov, rt) if rt else zero
            F = (1 + b2) * P * Rc / (Rc + b2 * P) if P + Rc > 0 else zero
            prf_all[i, j] = (float(P), float(Rc), float(F))
            if top is None or F > top:          # strict: the lowest index wins ties
                top = F
                best[i] = j
        prf[i] = prf_all[i, best[i]]
    return RougeResult(overlap, prf, best, prf_all)


def to_bfloat16(x) -> np.ndarray:
    """The stored value of a bfloat16 score (Section 6: lower-precision scores), as float64.

    The paper fixes no rounding; the reading taken: the fp32 score (the precision the scores are
    formed in) rounded to the nearest number with an 8-bit significand, ties to the even one.
    Written from that definition: a finite x with 2^e <= |x| < 2^(e+1) lies on a grid of spacing
    2^(e-7) (2^-133 below the smallest normal, 2^-126), and is moved to the nearest grid point.
    """
    x32 = np.asarray(x, dtype=np.float64).astype(np.float32).astype(np.float64)
    out = np.array(x32, copy=True)
    finite = np.isfinite(x32) & (x32 != 0.0)
    if finite.any():
        v = x32[finite]
        e = np.maximum(np.floor(np.log2(np.abs(v))), -126.0)
        spacing = np.exp2(e - 7.0)
        out[finite] = np.rint(v / spacing) * spacing          # rint: ties to even
    return out
