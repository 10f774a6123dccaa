"""Seeded synthetic workloads for batched token-ID BLEU.

This module only *draws inputs*: token-ID matrices, explicit length arrays and the list of
smoothing runs of each benchmark configuration.  It holds none of the metric's arithmetic and is
the one piece of code that both the CPU oracle's tests and the HIP path's tests / benchmark share.

The paper times batches of 256- and 1024-token sequences at batch sizes 16..512 (Section 4.2) but
never says how the tokens were drawn, how many references each candidate had, or which vocabulary
was used; the five configurations below stand in for that unspecified data.

Randomness is a counter-based generator written out here (a splitmix64-style finaliser applied to
(seed, sentence, stream, position)), so a batch is a pure function of its seed, independent of the
numpy version and of the order in which sentences are generated.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import List, Tuple

import numpy as np

_U64 = np.uint64
_GOLDEN = _U64(0x9E3779B97F4A7C15)
_M1 = _U64(0xBF58476D1CE4E5B9)
_M2 = _U64(0x94D049BB133111EB)
BASE_SEED = 0x7B1E0000

# streams: one independent substream per purpose inside a sentence
_S_BASE, _S_SUB_MASK, _S_SUB_DRAW, _S_DEL, _S_INS, _S_INS_DRAW, _S_LEN, _S_EXT = range(8)
_STREAMS_PER_SEQ = 16


def _mix(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, dtype=_U64)
    with np.errstate(over="ignore"):
        z = (z ^ (z >> _U64(30))) * _M1
        z = (z ^ (z >> _U64(27))) * _M2
        return z ^ (z >> _U64(31))


def uniforms(seed: int, sentence: int, stream: int, count: int) -> np.ndarray:
    """`count` doubles in [0, 1), a pure function of (seed, sentence, stream, position)."""
    with np.errstate(over="ignore"):
        key = _mix(np.array([seed], dtype=_U64) * _GOLDEN
                   + _mix(np.array([sentence * 1024 + stream + 1], dtype=_U64)))
        ctr = np.arange(1, count + 1, dtype=_U64) * _GOLDEN
        bits = _mix(key + ctr)
    return (bits >> _U64(11)).astype(np.float64) * (1.0 / 9007199254740992.0)


class TokenSampler:
    """Inverse-CDF sampler over a finite vocabulary; token id = rank - 1."""

    def __init__(self, vocab: int, zipf_s: float | None):
        self.vocab = int(vocab)
        if zipf_s is None:  # uniform ids
            self.cdf = None
        else:
            w = np.arange(1, vocab + 1, dtype=np.float64) ** (-float(zipf_s))
            cdf = np.cumsum(w)
            self.cdf = cdf / cdf[-1]

    def draw(self, u: np.ndarray) -> np.ndarray:
        if self.cdf is None:
            t = np.floor(u * self.vocab).astype(np.int64)
        else:
            t = np.searchsorted(self.cdf, u, side="right")
        return np.minimum(t, self.vocab - 1).astype(np.int32)


@dataclass
class Run:
    """One scoring run over a workload: smoothing mode + parameter (+ corpus flag)."""
    smoothing: str          # "none" | "floor" | "add-k" | "exp"
    smooth_param: float = 0.0
    corpus: bool = False


@dataclass
class Workload:
    name: str
    vocab: int
    cand: np.ndarray        # [B, cand_stride] int32, right-padded with 0
    cand_len: np.ndarray    # [B] int32
    refs: np.ndarray        # [B, R, ref_stride] int32, right-padded with 0
    ref_len: np.ndarray     # [B, R] int32
    max_n: int = 4
    weights: Tuple[float, ...] = (0.25, 0.25, 0.25, 0.25)
    runs: List[Run] = field(default_factory=list)

    @property
    def B(self) -> int:
        return int(self.cand.shape[0])

    @property
    def R(self) -> int:
        return int(self.refs.shape[1])

    @property
    def tokens(self) -> int:
        return int(self.cand_len.sum() + self.ref_len.sum())

    def ngrams(self, n: int) -> int:
        return int(np.maximum(self.cand_len - n + 1, 0).sum()
                   + np.maximum(self.ref_len - n + 1, 0).sum())

    def subset(self, count: int) -> "Workload":
        """The first `count` sentence groups (used for bounded CPU timing samples)."""
        c = min(count, self.B)
        return Workload(self.name + f"[:{c}]", self.vocab, self.cand[:c].copy(),
                        self.cand_len[:c].copy(), self.refs[:c].copy(), self.ref_len[:c].copy(),
                        self.max_n, self.weights, list(self.runs))


def _substitute(tokens: np.ndarray, p: float, sampler: TokenSampler, seed: int, sent: int,
                seq: int) -> np.ndarray:
    """Each position independently replaced, with probability p, by a fresh draw."""
    n = len(tokens)
    base = seq * _STREAMS_PER_SEQ
    mask = uniforms(seed, sent, base + _S_SUB_MASK, n) < p
    fresh = sampler.draw(uniforms(seed, sent, base + _S_SUB_DRAW, n))
    return np.where(mask, fresh, tokens).astype(np.int32)


def _pad_rows(rows: List[np.ndarray], stride: int) -> Tuple[np.ndarray, np.ndarray]:
    out = np.zeros((len(rows), stride), dtype=np.int32)
    lens = np.zeros(len(rows), dtype=np.int32)
    for i, r in enumerate(rows):
        assert len(r) <= stride
        out[i, :len(r)] = r
        lens[i] = len(r)
    return out, lens


def config1(B: int = 16, L: int = 256) -> Workload:
    """Small case: one same-length reference, Zipf(1.1), 0.3 substitution, vocab 32000."""
    seed, V = BASE_SEED + 1, 32000
    smp = TokenSampler(V, 1.1)
    cands, refs = [], []
    for i in range(B):
        ref = smp.draw(uniforms(seed, i, _S_BASE, L))
        refs.append(ref)
        cands.append(_substitute(ref, 0.3, smp, seed, i, 1))
    cand, cl = _pad_rows(cands, L)
    ref, rl = _pad_rows(refs, L)
    return Workload("cfg1_B16_L256", V, cand, cl, ref[:, None, :].copy(), rl[:, None].copy(),
                    runs=[Run("none"), Run("add-k", 1.0)])


def config2(B: int = 256, L: int = 1024) -> Workload:
    """One reference; candidate = 0.3 substitution + ~5% insert/delete, ragged, pad id 0."""
    seed, V = BASE_SEED + 2, 50257
    smp = TokenSampler(V, 1.1)
    lo, hi = int(round(L * 0.95)), int(round(L * 1.05))
    stride = ((hi + 63) // 64) * 64
    cands, refs = [], []
    for i in range(B):
        ref = smp.draw(uniforms(seed, i, _S_BASE, L))
        sub = _substitute(ref, 0.3, smp, seed, i, 1)
        delete = uniforms(seed, i, _STREAMS_PER_SEQ + _S_DEL, L) < 0.025
        insert = uniforms(seed, i, _STREAMS_PER_SEQ + _S_INS, L) < 0.025
        fresh = smp.draw(uniforms(seed, i, _STREAMS_PER_SEQ + _S_INS_DRAW, L))
        # left-to-right edit pass: before each source token maybe insert a fresh one, then
        # emit the token unless deleted
        pieces = np.stack([fresh, sub], axis=1).reshape(-1)
        keep = np.stack([insert, ~delete], axis=1).reshape(-1)
        c = pieces[keep]
        if len(c) > hi:
            c = c[:hi]
        elif len(c) < lo:
            extra = smp.draw(uniforms(seed, i, _STREAMS_PER_SEQ + _S_EXT, lo - len(c)))
            c = np.concatenate([c, extra])
        refs.append(ref)
        cands.append(c.astype(np.int32))
    cand, cl = _pad_rows(cands, stride)
    ref, rl = _pad_rows(refs, L)
    return Workload(f"cfg2_B{B}_L{L}_ragged", V, cand, cl, ref[:, None, :].copy(),
                    rl[:, None].copy(), runs=[Run("floor", 0.1)])


def config3(B: int = 512, L: int = 1024, R: int = 4) -> Workload:
    """Headline: four references of length U{0.75L..1.25L}, shared base sequence."""
    seed, V = BASE_SEED + 3, 50257
    smp = TokenSampler(V, 1.1)
    lo, hi = (3 * L) // 4, (5 * L) // 4
    cands, ref_rows, ref_lens = [], [], np.zeros((B, R), dtype=np.int32)
    for i in range(B):
        base = smp.draw(uniforms(seed, i, _S_BASE, hi))
        ul = uniforms(seed, i, _S_LEN, R)
        rows = []
        for j in range(R):
            lr = lo + int(np.floor(ul[j] * (hi - lo + 1)))
            lr = min(lr, hi)
            rows.append(_substitute(base[:lr], 0.3, smp, seed, i, 2 + j))
            ref_lens[i, j] = lr
        ref_rows.append(rows)
        cands.append(_substitute(base[:L], 0.4, smp, seed, i, 1))
    cand, cl = _pad_rows(cands, L)
    refs = np.zeros((B, R, hi), dtype=np.int32)
    for i in range(B):
        for j in range(R):
            refs[i, j, :ref_lens[i, j]] = ref_rows[i][j]
    return Workload(f"cfg3_B{B}_L{L}_R{R}", V, cand, cl, refs, ref_lens, runs=[Run("exp")])


def config4(B: int = 1024, L: int = 2048) -> Workload:
    """Large vocabulary (2^18): 4-gram keys need 72 bits."""
    seed, V = BASE_SEED + 4, 262144
    smp = TokenSampler(V, 1.05)
    cands, refs = [], []
    for i in range(B):
        ref = smp.draw(uniforms(seed, i, _S_BASE, L))
        refs.append(ref)
        cands.append(_substitute(ref, 0.25, smp, seed, i, 1))
    cand, cl = _pad_rows(cands, L)
    ref, rl = _pad_rows(refs, L)
    return Workload(f"cfg4_B{B}_L{L}_V262144", V, cand, cl, ref[:, None, :].copy(),
                    rl[:, None].copy(),
                    runs=[Run("add-k", 1.0), Run("add-k", 1.0, corpus=True)])


def config5(B: int = 4096) -> Workload:
    """Ragged, tiny vocabulary (64, uniform ids): heavy n-gram repetition."""
    seed, V = BASE_SEED + 5, 64
    smp = TokenSampler(V, None)
    cs, rs = 512, 640
    cand = np.zeros((B, cs), dtype=np.int32)
    refs = np.zeros((B, 2, rs), dtype=np.int32)
    cl = np.zeros(B, dtype=np.int32)
    rl = np.zeros((B, 2), dtype=np.int32)
    for i in range(B):
        ul = uniforms(seed, i, _S_LEN, 3)
        lc = 32 + min(int(np.floor(ul[0] * 481)), 480)
        l0 = int(round(lc * (0.8 + 0.4 * ul[1])))
        l1 = int(round(lc * (0.8 + 0.4 * ul[2])))
        r0 = smp.draw(uniforms(seed, i, _S_BASE, l0))
        r1 = smp.draw(uniforms(seed, i, _STREAMS_PER_SEQ * 3 + _S_BASE, l1))
        src = r0[:lc]
        if len(src) < lc:
            src = np.concatenate([src, smp.draw(uniforms(seed, i, _S_EXT, lc - len(src)))])
        c = _substitute(src, 0.5, smp, seed, i, 1)
        cand[i, :lc], cl[i] = c, lc
        refs[i, 0, :l0], rl[i, 0] = r0, l0
        refs[i, 1, :l1], rl[i, 1] = r1, l1
    return Workload(f"cfg5_B{B}_ragged_V64", V, cand, cl, refs, rl,
                    runs=[Run("none"), Run("floor", 0.1)])


CONFIGS = {1: config1, 2: config2, 3: config3, 4: config4, 5: config5}


def make(config: int, **kw) -> Workload:
    return CONFIGS[config](**kw)


def random_small(seed: int, B: int, R: int, vocab: int, max_len: int, min_len: int = 0,
                 cand_stride: int | None = None, ref_stride: int | None = None,
                 related: bool = True) -> Workload:
    """Small ragged batch with arbitrary lengths (including 0) for edge-case tests."""
    smp = TokenSampler(vocab, None)
    cs = cand_stride or max(max_len, 1)
    rs = ref_stride or max(max_len, 1)
    cand = np.zeros((B, cs), dtype=np.int32)
    refs = np.zeros((B, R, rs), dtype=np.int32)
    cl = np.zeros(B, dtype=np.int32)
    rl = np.zeros((B, R), dtype=np.int32)
    span = max_len - min_len + 1
    for i in range(B):
        ul = uniforms(seed, i, _S_LEN, R + 1)
        lc = min_len + min(int(ul[0] * span), span - 1)
        c = smp.draw(uniforms(seed, i, _S_BASE, lc))
        cand[i, :lc], cl[i] = c, lc
        for j in range(R):
            lr = min_len + min(int(ul[1 + j] * span), span - 1)
            r = smp.draw(uniforms(seed, i, (2 + j) * _STREAMS_PER_SEQ + _S_BASE, lr))
            if related and lr and lc:
                m = min(lr, lc)
                keep = uniforms(seed, i, (2 + j) * _STREAMS_PER_SEQ + _S_SUB_MASK, m) < 0.6
                r[:m] = np.where(keep, c[:m], r[:m])
            refs[i, j, :lr], rl[i, j] = r, lr
    return Workload(f"small_s{seed}_B{B}_R{R}_V{vocab}", vocab, cand, cl, refs, rl)


def long_form(B: int = 128, L: int = 8192, vocab: int = 50257) -> Workload:
    """Long generations (the paper's Section 6 names them as a direction): B candidates of about
    L tokens with one reference each, Zipf(1.1) tokens, the reference a 0.3-substitution of the
    candidate's base text with its own length in [0.9 L, L].  Groups of ~2 L tokens: beyond one
    LDS table for L > 6144."""
    seed = 0x7B1E0100 + L
    smp = TokenSampler(vocab, 1.1)
    cand = np.zeros((B, L), dtype=np.int32)
    refs = np.zeros((B, 1, L), dtype=np.int32)
    cl = np.zeros(B, dtype=np.int32)
    rl = np.zeros((B, 1), dtype=np.int32)
    lo = (9 * L) // 10
    for i in range(B):
        ul = uniforms(seed, i, _S_LEN, 2)
        lc = lo + min(int(ul[0] * (L - lo + 1)), L - lo)
        lr = lo + min(int(ul[1] * (L - lo + 1)), L - lo)
        base = smp.draw(uniforms(seed, i, _S_BASE, L))
        cand[i, :lc], cl[i] = _substitute(base[:lc], 0.3, smp, seed, i, 1), lc
        refs[i, 0, :lr], rl[i, 0] = _substitute(base[:lr], 0.3, smp, seed, i, 2), lr
    return Workload(f"long_B{B}_L{L}_R1_V{vocab}", vocab, cand, cl, refs, rl, runs=[Run("exp")])


def ref_counts(seed: int, B: int, R: int) -> np.ndarray:
    """Per-candidate number of references in use, uniform in 1..R (for ragged reference counts)."""
    u = uniforms(seed, 0, 15, B)
    return (np.minimum(np.floor(u * R), R - 1) + 1).astype(np.int32)


def pack_reference_lists(refs: np.ndarray, ref_len: np.ndarray, counts: np.ndarray):
    """Fixed-R references [B, R, Lr] with per-candidate counts -> reference lists in CSR form:
    rows [sum(counts), Lr], their lengths [rows], offsets [B + 1] (candidate i owns the rows
    offsets[i] .. offsets[i + 1] - 1, its first counts[i] references in order).  Layout only."""
    B = refs.shape[0]
    offsets = np.zeros(B + 1, np.int32)
    offsets[1:] = np.cumsum(counts)
    rows = np.zeros((int(offsets[-1]), refs.shape[2]), np.int32)
    lens = np.zeros(int(offsets[-1]), np.int32)
    for i in range(B):
        k = int(counts[i])
        rows[offsets[i]:offsets[i] + k] = refs[i, :k]
        lens[offsets[i]:offsets[i] + k] = ref_len[i, :k]
    return rows, lens, offsets
