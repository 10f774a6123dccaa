"""Pins for the CPU oracle: closed forms, hand-worked cases, brute force and invariants.

None of these re-type the oracle's own formula for a general input: each either evaluates a
closed form that holds for one constructed family of inputs, compares against a dictionary-free
brute-force enumerator, or checks a property that any correct implementation has.
"""
import itertools
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from oracle import paper_pipeline
import synth_inputs as syn

MODES = [("none", 0.0), ("floor", 0.1), ("add-k", 1.0), ("exp", 0.0)]
GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "hand_worked.txt")


def pad_batch(cands, refs_per_cand):
    """Lists of token lists -> padded arrays. refs_per_cand: list (per candidate) of lists."""
    B = len(cands)
    R = len(refs_per_cand[0])
    cs = max(1, max(len(c) for c in cands))
    rs = max(1, max(len(r) for rr in refs_per_cand for r in rr))
    cand = np.full((B, cs), 0, np.int32)
    refs = np.full((B, R, rs), 0, np.int32)
    cl = np.zeros(B, np.int32)
    rl = np.zeros((B, R), np.int32)
    for i, c in enumerate(cands):
        cand[i, :len(c)] = c
        cl[i] = len(c)
        assert len(refs_per_cand[i]) == R
        for j, r in enumerate(refs_per_cand[i]):
            refs[i, j, :len(r)] = r
            rl[i, j] = len(r)
    return cand, cl, refs, rl


def one(cand, refs, smoothing="none", param=0.0, weights=None, max_n=4):
    c, cl, r, rl = pad_batch([cand], [refs])
    res = oracle.bleu(c, cl, r, rl, max_n=max_n, weights=weights, smoothing=smoothing,
                      smooth_param=param)
    return res


# ----------------------------------------------------------------------------- closed forms

@pytest.mark.parametrize("mode,param", MODES)
@pytest.mark.parametrize("L", [4, 5, 17, 300])
def test_identical_candidate_and_reference_scores_one(mode, param, L):
    toks = list(syn.TokenSampler(1000, 1.1).draw(syn.uniforms(5, L, 0, L)))
    res = one(toks, [toks], mode, param)
    assert (res.clipped[0] == res.total[0]).all()
    assert list(res.total[0]) == [L, L - 1, L - 2, L - 3]
    assert res.bleu[0] == pytest.approx(1.0, abs=1e-12)


@pytest.mark.parametrize("mode,param", MODES)
def test_no_shared_unigram_scores_zero_in_every_mode(mode, param):
    res = one([1, 2, 3, 4, 5, 6], [[7, 8, 9, 10, 11, 12], [13, 14, 15, 16]], mode, param)
    assert list(res.clipped[0]) == [0, 0, 0, 0]
    assert res.bleu[0] == 0.0


@pytest.mark.parametrize("c,m", [(5, 2), (9, 1), (12, 7), (3, 3), (6, 0)])
def test_repeated_token_is_clipped_at_reference_count(c, m):
    ref = [9] * m + list(range(100, 100 + 10))       # token 9 exactly m times
    ref = ref[m // 2:] + ref[:m // 2]                 # not all at the front
    res = one([9] * c, [ref], max_n=1, weights=[1.0])
    assert res.clipped[0, 0] == min(c, m)
    assert res.total[0, 0] == c


def test_clip_uses_max_over_references_not_sum():
    filler0, filler1 = [50, 51, 52, 53], [60, 61, 62]
    res = one([7] * 5, [[7, 7] + filler0, filler1 + [7, 7, 7]])
    assert res.clipped[0, 0] == 3          # max(2, 3); a sum would give 5
    # bigram (7,7): candidate 4, references 1 and 2 -> 2; trigram: 0 and 1 -> 1; 4-gram 0
    assert list(res.clipped[0]) == [3, 2, 1, 0]


@pytest.mark.parametrize("c,r", [(4, 4), (4, 9), (10, 11), (33, 100), (50, 50)])
def test_prefix_candidate_gives_pure_brevity_penalty(c, r):
    ref = list(range(1, r + 1))
    res = one(ref[:c], [ref])
    assert (res.clipped[0] == res.total[0]).all()
    assert res.bleu[0] == pytest.approx(math.exp(1.0 - r / c), rel=1e-13)


@pytest.mark.parametrize("c,r", [(9, 5), (20, 4), (6, 6), (5, 8), (40, 39)])
def test_single_repeated_token_closed_form(c, r):
    res = one([3] * c, [[3] * r])
    if c > r:
        expect = 1.0
        for n in range(1, 5):
            expect *= ((r - n + 1) / (c - n + 1)) ** 0.25
        assert list(res.clipped[0]) == [r - n + 1 for n in range(1, 5)]
    else:
        expect = math.exp(1.0 - r / c)
        assert list(res.clipped[0]) == [c - n + 1 for n in range(1, 5)]
    assert res.bleu[0] == pytest.approx(expect, rel=1e-13)


@pytest.mark.parametrize("L,k", [(10, 0), (10, 4), (10, 9), (12, 1), (7, 5), (30, 28)])
def test_single_substitution_closed_form(L, k):
    ref = list(range(1, L + 1))
    cand = list(ref)
    cand[k] = 10_000
    res = one(cand, [ref])
    prod = 1.0
    for n in range(1, 5):
        windows = L - n + 1
        covering = min(k, L - n) - max(0, k - n + 1) + 1
        assert res.clipped[0, n - 1] == windows - covering
        assert res.total[0, n - 1] == windows
        prod *= ((windows - covering) / windows) ** 0.25
    assert res.bleu[0] == pytest.approx(prod, rel=1e-13)     # c == r -> BP = 1


def test_closest_reference_length_tie_goes_to_shorter():
    cand = list(range(1, 11))                                  # c = 10
    short, long_ = list(range(1, 9)), list(range(1, 13))       # 8 and 12: both 2 away
    for refs in ([short, long_], [long_, short]):
        res = one(cand, refs)
        assert res.closest_ref_len[0] == 8
        assert (res.clipped[0] == res.total[0]).all()
        assert res.bleu[0] == pytest.approx(1.0, abs=1e-12)    # c > r, not exp(-0.2)


def test_closest_reference_length_prefers_nearest():
    cand = list(range(1, 11))
    res = one(cand, [list(range(1, 30)), list(range(1, 12)), list(range(1, 5))])
    assert res.closest_ref_len[0] == 11
    assert res.bleu[0] == pytest.approx(math.exp(1 - 11 / 10), rel=1e-13)


def test_empty_candidate_and_empty_reference():
    res = one([], [[1, 2, 3]])
    assert list(res.clipped[0]) == [0, 0, 0, 0] and list(res.total[0]) == [0, 0, 0, 0]
    assert res.bleu[0] == 0.0
    res = one([1, 2, 3, 4], [[], [1, 2, 3, 4]])
    assert res.closest_ref_len[0] == 4 and res.bleu[0] == pytest.approx(1.0)
    res = one([1, 2, 3, 4], [[]])
    assert res.closest_ref_len[0] == 0 and res.bleu[0] == 0.0


def test_weights_used_as_given_and_zero_weight_drops_order():
    cand, ref = [1, 2, 3, 4, 5], [1, 2, 3, 9, 4, 5, 6]         # p = 1, 3/4, 1/3, 0
    bp = math.exp(1 - 7 / 5)
    res = one(cand, [ref], weights=[0.5, 0.5, 0.0, 0.0])
    assert res.bleu[0] == pytest.approx(bp * math.sqrt(0.75), rel=1e-13)
    res = one(cand, [ref], weights=[1.0, 1.0, 1.0, 0.0])        # not renormalised
    assert res.bleu[0] == pytest.approx(bp * 0.75 / 3, rel=1e-13)
    res = one(cand, [ref], max_n=2, weights=[0.5, 0.5])
    assert res.bleu[0] == pytest.approx(bp * math.sqrt(0.75), rel=1e-13)


# ------------------------------------------------------------------- hand-worked golden file

def _parse_golden():
    cases, cur = [], None
    for raw in open(GOLDEN):
        line = raw.strip()
        if not line or line.startswith("#"):
            continue
        key, _, val = line.partition(":")
        key, val = key.strip(), val.strip()
        if key == "case":
            cur = {"name": val, "refs": [], "modes": {}}
            cases.append(cur)
        elif key == "cand":
            cur["cand"] = [int(x) for x in val.split()]
        elif key == "ref":
            cur["refs"].append([int(x) for x in val.split()])
        elif key in ("clipped", "total"):
            cur[key] = [int(x) for x in val.split()]
        elif key == "closest_ref_len":
            cur[key] = int(val)
        elif key == "bp_exponent":
            cur[key] = float(val)
        else:
            parts = key.split()
            mode, param = parts[0], float(parts[1]) if len(parts) > 1 else 0.0
            cur["modes"][(mode, param)] = None if val == "zero" else val.split()
    return cases


def _frac(s):
    num, den = s.split("/")
    return float(Fraction(num)) / float(Fraction(den))


@pytest.mark.parametrize("case", _parse_golden(), ids=lambda c: c["name"])
def test_hand_worked_cases(case):
    assert len(case["modes"]) == 4
    for (mode, param), precisions in case["modes"].items():
        res = one(case["cand"], case["refs"], mode, param)
        assert list(res.clipped[0]) == case["clipped"]
        assert list(res.total[0]) == case["total"]
        assert res.closest_ref_len[0] == case["closest_ref_len"]
        if precisions is None:
            assert res.bleu[0] == 0.0
        else:
            expect = math.exp(case["bp_exponent"])
            for p in precisions:
                expect *= _frac(p) ** 0.25
            assert res.bleu[0] == pytest.approx(expect, rel=1e-12)


# ------------------------------------------------------------------------------- brute force

def brute_force_stats(cand, refs, max_n):
    """Dictionary-free counting: O(L^2) window comparisons, de-duplicated by first occurrence."""
    clipped, total = [], []
    for n in range(1, max_n + 1):
        cw = [tuple(cand[p:p + n]) for p in range(len(cand) - n + 1)]
        acc = 0
        for p, g in enumerate(cw):
            if any(cw[q] == g for q in range(p)):
                continue                                   # counted at its first occurrence
            in_cand = sum(1 for x in cw if x == g)
            best = 0
            for ref in refs:
                in_ref = sum(1 for q in range(len(ref) - n + 1) if tuple(ref[q:q + n]) == g)
                best = max(best, in_ref)
            acc += min(in_cand, best)
        clipped.append(acc)
        total.append(max(len(cand) - n + 1, 0))
    return clipped, total


def brute_force_distinct(cand, refs, max_n):
    """Sizes of the candidate's and of the whole group's n-gram dictionaries: set of windows."""
    group, own = [], []
    for n in range(1, max_n + 1):
        cw = {tuple(cand[p:p + n]) for p in range(len(cand) - n + 1)}
        allw = set(cw)
        for ref in refs:
            allw |= {tuple(ref[p:p + n]) for p in range(len(ref) - n + 1)}
        own.append(len(cw))
        group.append(len(allw))
    return group, own


def test_exhaustive_tiny_inputs_match_brute_force():
    # every candidate/reference pair over a 2-letter alphabet with lengths 0..5 (R = 1)
    seqs = [list(t) for L in range(0, 6) for t in itertools.product([0, 1], repeat=L)]
    cands, refs = [], []
    for c in seqs:
        for r in seqs:
            cands.append(c)
            refs.append([r])
    cand, cl, ref, rl = pad_batch(cands, refs)
    res = oracle.bleu(cand, cl, ref, rl)
    for i in range(len(cands)):
        bc, bt = brute_force_stats(cands[i], refs[i], 4)
        assert list(res.clipped[i]) == bc, (cands[i], refs[i])
        assert list(res.total[i]) == bt
        gd, cd = brute_force_distinct(cands[i], refs[i], 4)
        assert list(res.group_distinct[i]) == gd and list(res.cand_distinct[i]) == cd


def test_dictionary_sizes_closed_forms():
    # L distinct tokens: L - n + 1 distinct n-grams; one token repeated: one n-gram per order;
    # a reference sharing nothing doubles the group's dictionary, an identical one adds nothing
    L = 9
    a, b = list(range(10, 10 + L)), list(range(50, 50 + L))
    cand, cl, ref, rl = pad_batch([a, a, [7] * L], [[a], [b], [[7] * 4]])
    res = oracle.bleu(cand, cl, ref, rl)
    full = [L - n + 1 for n in range(1, 5)]
    assert res.cand_distinct[0].tolist() == full and res.group_distinct[0].tolist() == full
    assert res.group_distinct[1].tolist() == [2 * x for x in full]
    assert res.cand_distinct[2].tolist() == [1, 1, 1, 1] == res.group_distinct[2].tolist()
    cand, cl, ref, rl = pad_batch([a], [[a, b]])
    res = oracle.bleu(cand, cl, ref, rl)
    assert res.group_distinct[0].tolist() == [2 * x for x in full]
    assert res.cand_distinct[0].tolist() == full


def test_exhaustive_tiny_two_references_match_brute_force():
    seqs = [list(t) for L in range(0, 4) for t in itertools.product([0, 1, 2], repeat=L)]
    cand4 = [list(t) for t in itertools.product([0, 1], repeat=4)]
    cands, refs = [], []
    for c in cand4:
        for r0 in seqs:
            for r1 in seqs[::3]:
                cands.append(c)
                refs.append([r0, r1])
    cand, cl, ref, rl = pad_batch(cands, refs)
    res = oracle.bleu(cand, cl, ref, rl)
    for i in range(len(cands)):
        bc, bt = brute_force_stats(cands[i], refs[i], 4)
        assert list(res.clipped[i]) == bc, (cands[i], refs[i])
        gd, cd = brute_force_distinct(cands[i], refs[i], 4)
        assert list(res.group_distinct[i]) == gd and list(res.cand_distinct[i]) == cd


@pytest.mark.parametrize("seed,V,R", [(1, 3, 1), (2, 5, 3), (3, 64, 2), (4, 1000, 4)])
def test_random_small_match_brute_force(seed, V, R):
    w = syn.random_small(seed, B=24, R=R, vocab=V, max_len=40)
    res = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len)
    for i in range(w.B):
        c = list(w.cand[i, :w.cand_len[i]])
        rr = [list(w.refs[i, j, :w.ref_len[i, j]]) for j in range(R)]
        bc, bt = brute_force_stats(c, rr, 4)
        assert list(res.clipped[i]) == bc
        assert list(res.total[i]) == bt
        gd, cd = brute_force_distinct(c, rr, 4)
        assert list(res.group_distinct[i]) == gd and list(res.cand_distinct[i]) == cd


# ------------------------------------------------- the paper's batched formulation agrees

@pytest.mark.parametrize("seed,V,R,L", [(11, 4, 2, 30), (12, 50, 1, 64), (13, 2000, 3, 48)])
def test_paper_unique_bincount_pipeline_matches_definition(seed, V, R, L):
    w = syn.random_small(seed, B=12, R=R, vocab=V, max_len=L)
    res = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len)
    clipped, total, _ = paper_pipeline.clipped_counts(w.cand, w.cand_len, w.refs, w.ref_len)
    assert (clipped == res.clipped).all()
    assert (total == res.total).all()


def test_paper_pipeline_on_config1():
    w = syn.make(1)
    res = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len)
    clipped, total, num_unique = paper_pipeline.clipped_counts(w.cand, w.cand_len, w.refs,
                                                               w.ref_len)
    assert (clipped == res.clipped).all() and (total == res.total).all()
    # a batch-wide dictionary can never be larger than the sum of per-group dictionaries
    assert (num_unique <= res.group_distinct.sum(axis=0)).all()


# -------------------------------------------------------------------------------- invariants

@pytest.fixture(scope="module")
def small():
    return syn.random_small(77, B=40, R=3, vocab=12, max_len=60)


def _run(w, **kw):
    return oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, **kw)


@pytest.mark.parametrize("mode,param", MODES)
def test_ranges(small, mode, param):
    res = _run(small, smoothing=mode, smooth_param=param)
    assert (res.clipped >= 0).all() and (res.clipped <= res.total).all()
    assert (res.bleu >= 0).all() and (res.bleu <= 1 + 1e-12).all()
    assert (res.cand_distinct <= res.group_distinct).all()
    assert (res.cand_distinct <= np.maximum(res.total, 0)).all()


def test_single_reference_clipped_counts_decrease_with_order():
    w = syn.random_small(78, B=60, R=1, vocab=6, max_len=50)
    res = _run(w)
    assert (res.clipped[:, 1:] <= res.clipped[:, :-1]).all()


def test_reference_order_and_duplicates_do_not_matter(small):
    base = _run(small, smoothing="exp")
    perm = small.refs[:, ::-1, :].copy(), small.ref_len[:, ::-1].copy()
    res = oracle.bleu(small.cand, small.cand_len, perm[0], perm[1], smoothing="exp")
    assert (res.clipped == base.clipped).all() and np.array_equal(res.bleu, base.bleu)
    dup_refs = np.concatenate([small.refs, small.refs[:, :1]], axis=1)
    dup_len = np.concatenate([small.ref_len, small.ref_len[:, :1]], axis=1)
    res = oracle.bleu(small.cand, small.cand_len, dup_refs, dup_len, smoothing="exp")
    assert (res.clipped == base.clipped).all() and np.array_equal(res.bleu, base.bleu)


def test_batch_permutation_equivariance_and_independence(small):
    base = _run(small, smoothing="floor", smooth_param=0.1)
    perm = np.random.default_rng(0).permutation(small.B)
    res = oracle.bleu(small.cand[perm], small.cand_len[perm], small.refs[perm],
                      small.ref_len[perm], smoothing="floor", smooth_param=0.1)
    assert (res.clipped == base.clipped[perm]).all()
    assert np.array_equal(res.bleu, base.bleu[perm])
    # sentence 0 does not depend on the rest of the batch
    other = syn.random_small(79, B=small.B, R=3, vocab=12, max_len=60)
    cand, cl = other.cand.copy(), other.cand_len.copy()
    refs, rl = other.refs.copy(), other.ref_len.copy()
    cand[0], cl[0], refs[0], rl[0] = small.cand[0], small.cand_len[0], small.refs[0], \
        small.ref_len[0]
    res = oracle.bleu(cand, cl, refs, rl, smoothing="floor", smooth_param=0.1)
    assert (res.clipped[0] == base.clipped[0]).all() and res.bleu[0] == base.bleu[0]


def test_pad_cells_are_never_interpreted(small):
    base = _run(small)
    rng = np.random.default_rng(1)
    cand, refs = small.cand.copy(), small.refs.copy()
    cpad = np.arange(cand.shape[1])[None, :] >= small.cand_len[:, None]
    rpad = np.arange(refs.shape[2])[None, None, :] >= small.ref_len[:, :, None]
    cand[cpad] = rng.integers(0, 12, cpad.sum())            # hot in-vocabulary garbage
    refs[rpad] = rng.integers(0, 12, rpad.sum())
    res = oracle.bleu(cand, small.cand_len, refs, small.ref_len)
    assert (res.clipped == base.clipped).all() and np.array_equal(res.bleu, base.bleu)


def test_injective_relabelling_leaves_scores_unchanged(small):
    base = _run(small, smoothing="add-k", smooth_param=1.0)
    table = (np.arange(12, dtype=np.int64) * 178_956_970 + 65_537).astype(np.int32)  # > 2^16
    assert len(set(table.tolist())) == 12
    res = oracle.bleu(table[small.cand], small.cand_len, table[small.refs], small.ref_len,
                      smoothing="add-k", smooth_param=1.0)
    # pad cells changed too (table[0] != 0) -- they are outside the lengths
    assert (res.clipped == base.clipped).all() and np.array_equal(res.bleu, base.bleu)


def test_corpus_of_one_sentence_equals_sentence_score():
    w = syn.random_small(80, B=9, R=2, vocab=8, max_len=30, min_len=4)
    for mode, param in MODES:
        for i in range(w.B):
            res = oracle.bleu(w.cand[i:i + 1], w.cand_len[i:i + 1], w.refs[i:i + 1],
                              w.ref_len[i:i + 1], smoothing=mode, smooth_param=param)
            assert res.corpus_bleu == res.bleu[0]


def test_corpus_statistics_are_sums_and_score_closed_form():
    # two sentences: first matches fully (c=6, r=6), second is a 4-token prefix of a 10-token
    # reference.  corpus: clipped = total = (10, 8, 6, 4), c = 10, r = 16 -> exp(1 - 1.6)
    a = [1, 2, 3, 4, 5, 6]
    b_ref = list(range(11, 21))
    cand, cl, ref, rl = pad_batch([a, b_ref[:4]], [[a], [b_ref]])
    res = oracle.bleu(cand, cl, ref, rl)
    assert list(res.corpus_stats) == [10, 8, 6, 4, 10, 8, 6, 4, 10, 16]
    assert res.corpus_bleu == pytest.approx(math.exp(1 - 16 / 10), rel=1e-13)


def test_threads_give_identical_results():
    w = syn.make(1)
    a = _run(w, smoothing="exp", threads=1)
    b = _run(w, smoothing="exp", threads=5)
    assert (a.clipped == b.clipped).all() and np.array_equal(a.bleu, b.bleu)
    assert a.corpus_bleu == b.corpus_bleu


def test_group_counts_agree_with_sentence_statistics(small):
    base = _run(small)
    for i in range(0, small.B, 7):
        for n in range(1, 5):
            grams, cc, rm = oracle.group_counts(small.cand[i], small.cand_len[i], small.refs[i],
                                                small.ref_len[i], n)
            assert len(grams) == base.group_distinct[i, n - 1]
            assert np.minimum(cc, rm).sum() == base.clipped[i, n - 1]
            assert cc.sum() == base.total[i, n - 1]
            assert (cc > 0).sum() == base.cand_distinct[i, n - 1]


# ------------------------------------------------------------------------ workload generator

def test_generator_is_deterministic_and_shaped():
    a, b = syn.make(1), syn.make(1)
    assert np.array_equal(a.cand, b.cand) and np.array_equal(a.refs, b.refs)
    assert a.cand.shape == (16, 256) and a.refs.shape == (16, 1, 256) and a.vocab == 32000
    assert a.cand.max() < a.vocab and a.cand.min() >= 0
    # ~30 % of positions substituted (a substitution can redraw the same token)
    frac = (a.cand != a.refs[:, 0, :]).mean()
    assert 0.2 < frac < 0.32
    # Zipf: id 0 is the most frequent token
    counts = np.bincount(a.refs.reshape(-1), minlength=10)
    assert counts[0] == counts.max()


def test_ragged_generators_respect_lengths():
    w = syn.config2(B=8)
    assert w.cand.shape[1] >= w.cand_len.max() and (w.cand_len >= 973).all()
    assert (w.cand_len <= 1075).all() and len(set(w.cand_len.tolist())) > 1
    w = syn.config3(B=4)
    assert w.refs.shape == (4, 4, 1280) and (w.ref_len >= 768).all() and (w.ref_len <= 1280).all()
    w = syn.config5(B=64)
    assert (w.cand_len >= 32).all() and (w.cand_len <= 512).all() and w.cand.max() < 64
    assert (w.ref_len <= 640).all() and (w.ref_len >= 0.79 * w.cand_len[:, None] - 1).all()


# ---------------------------------------------------- per-candidate reference counts (ragged R)

def _ref_counts(seed, B, R):
    return syn.ref_counts(seed, B, R)


@pytest.mark.parametrize("mode,param", MODES)
def test_reference_count_equal_to_R_changes_nothing(small, mode, param):
    full = _run(small, smoothing=mode, smooth_param=param)
    same = _run(small, smoothing=mode, smooth_param=param,
                ref_count=np.full(small.B, small.R, np.int32))
    np.testing.assert_array_equal(same.clipped, full.clipped)
    np.testing.assert_array_equal(same.closest_ref_len, full.closest_ref_len)
    np.testing.assert_array_equal(same.bleu, full.bleu)
    assert same.corpus_bleu == full.corpus_bleu


@pytest.mark.parametrize("mode,param", MODES)
def test_reference_count_equals_scoring_against_the_sliced_references(small, mode, param):
    """Candidate i with ref_count[i] = k is, by definition, candidate i with references 0..k-1:
    compared sentence by sentence with a batch of one that holds only those rows; the rows
    beyond k are overwritten with tokens that would change every count if they were read."""
    rc = _ref_counts(5, small.B, small.R)
    assert rc.min() >= 1 and rc.max() <= small.R and len(set(rc.tolist())) > 1
    poisoned = small.refs.copy()
    poisoned_len = small.ref_len.copy()
    for i in range(small.B):
        poisoned[i, rc[i]:] = small.cand[i, :1].repeat(poisoned.shape[2])[None, :]
        poisoned_len[i, rc[i]:] = small.cand_len[i]          # would also win the closest length
    res = oracle.bleu(small.cand, small.cand_len, poisoned, poisoned_len, smoothing=mode,
                      smooth_param=param, ref_count=rc)
    for i in range(small.B):
        k = int(rc[i])
        one_ = oracle.bleu(small.cand[i:i + 1], small.cand_len[i:i + 1], small.refs[i:i + 1, :k],
                           small.ref_len[i:i + 1, :k], smoothing=mode, smooth_param=param)
        np.testing.assert_array_equal(res.clipped[i], one_.clipped[0])
        assert res.closest_ref_len[i] == one_.closest_ref_len[0]
        assert res.bleu[i] == one_.bleu[0]
    # corpus statistics are the sums of the per-sentence ones
    np.testing.assert_array_equal(res.corpus_stats[:4], res.clipped.sum(0))
    assert res.corpus_stats[9] == res.closest_ref_len.sum()


def test_reference_count_brute_force():
    w = syn.random_small(31, B=12, R=3, vocab=4, max_len=9, min_len=1)
    rc = _ref_counts(8, w.B, w.R)
    res = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, ref_count=rc)
    for i in range(w.B):
        refs = [w.refs[i, j, :w.ref_len[i, j]].tolist() for j in range(rc[i])]
        clipped, total = brute_force_stats(w.cand[i, :w.cand_len[i]].tolist(), refs, 4)
        assert res.clipped[i].tolist() == clipped and res.total[i].tolist() == total


def test_reference_count_out_of_range_is_rejected():
    w = syn.random_small(32, B=4, R=2, vocab=5, max_len=8)
    for bad in (0, 3):
        with pytest.raises(ValueError):
            oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len,
                        ref_count=np.array([1, 2, bad, 1], np.int32))


# ------------------------------------------------------------------- more than four orders

@pytest.mark.parametrize("N", [5, 6, 8])
def test_more_than_four_orders_closed_forms_and_brute_force(N):
    """Nothing in the definition is special about N = 4: identity, the prefix brevity penalty,
    the single-substitution window count and the brute-force enumerator at N up to 8."""
    L = 30
    ref = list(range(100, 100 + L))
    assert one(ref, [ref], max_n=N).bleu[0] == pytest.approx(1.0, abs=1e-15)
    assert one(ref[:20], [ref], max_n=N).bleu[0] == pytest.approx(np.exp(1 - L / 20), rel=1e-13)
    k = 11
    cand = list(ref)
    cand[k] = 7
    res = one(cand, [ref], max_n=N)
    expect = 1.0
    for n in range(1, N + 1):
        total = L - n + 1
        covering = min(k, L - n) - max(0, k - n + 1) + 1
        assert res.clipped[0, n - 1] == total - covering
        expect *= ((total - covering) / total) ** (1.0 / N)
    assert res.bleu[0] == pytest.approx(expect, rel=1e-12)
    w = syn.random_small(91, B=10, R=2, vocab=3, max_len=14, min_len=1)
    res = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, max_n=N)
    for i in range(w.B):
        refs = [w.refs[i, j, :w.ref_len[i, j]].tolist() for j in range(w.R)]
        clipped, total = brute_force_stats(w.cand[i, :w.cand_len[i]].tolist(), refs, N)
        assert res.clipped[i].tolist() == clipped and res.total[i].tolist() == total


# ------------------------------------------------------------------- reference lists (CSR)

def test_reference_lists_equal_each_candidate_scored_alone_with_its_own_references():
    """A batch with reference lists of different lengths is, by definition, every candidate
    scored against its own list: the CSR form must equal B separate single-candidate calls."""
    w = syn.random_small(91, B=14, R=5, vocab=9, max_len=26, min_len=3)
    counts = syn.ref_counts(91, w.B, w.R)
    rows, lens, offsets = syn.pack_reference_lists(w.refs, w.ref_len, counts)
    assert rows.shape[0] == counts.sum() and offsets[-1] == counts.sum()
    res = oracle.bleu(w.cand, w.cand_len, rows, lens, smoothing="add-k", smooth_param=1.0,
                      ref_offsets=offsets)
    for i in range(w.B):
        k = int(counts[i])
        alone = oracle.bleu(w.cand[i:i + 1], w.cand_len[i:i + 1], w.refs[i:i + 1, :k],
                            w.ref_len[i:i + 1, :k], smoothing="add-k", smooth_param=1.0)
        assert res.clipped[i].tolist() == alone.clipped[0].tolist()
        assert res.closest_ref_len[i] == alone.closest_ref_len[0]
        assert res.bleu[i] == alone.bleu[0]
        rouge = oracle.rouge_n(w.cand, w.cand_len, rows, lens, n=2, ref_offsets=offsets)
        rouge_alone = oracle.rouge_n(w.cand[i:i + 1], w.cand_len[i:i + 1], w.refs[i:i + 1, :k],
                                     w.ref_len[i:i + 1, :k], n=2)
        assert rouge.overlap[i, :k].tolist() == rouge_alone.overlap[0].tolist()
        assert rouge.best[i] == rouge_alone.best[0]


def test_a_candidate_without_references_matches_nothing():
    cand, cl, ref, rl = pad_batch([[1, 2, 3, 4, 5], [1, 2, 3, 4, 5]], [[[1, 2, 3, 4, 5]]] * 2)
    rows, lens = ref[:1, 0], rl[:1, 0]
    res = oracle.bleu(cand, cl, rows, lens, smoothing="floor", smooth_param=0.1,
                      ref_offsets=np.array([0, 1, 1]))
    assert res.bleu.tolist() == [1.0, 0.0]
    assert res.clipped[1].tolist() == [0, 0, 0, 0] and res.total[1].tolist() == [5, 4, 3, 2]
    assert res.closest_ref_len.tolist() == [5, 0]
