"""Pins for the ROUGE-N oracle (oracle_rouge_n): closed forms, hand-worked cases, brute force.

ROUGE-N (Lin 2004) for one candidate/reference pair and one order n:
overlap = sum over distinct n-grams of min(count in candidate, count in reference),
precision = overlap / candidate n-grams, recall = overlap / reference n-grams,
F = (1 + beta^2) P R / (R + beta^2 P).  The paper names ROUGE as the first metric its counting
method extends to (Section 6, "Future Work")."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

import oracle
import synth_inputs as syn
from test_oracle_pins import pad_batch


def one(cand, refs, n=2, beta=1.0):
    c, cl, r, rl = pad_batch([cand], [refs])
    return oracle.rouge_n(c, cl, r, rl, n=n, beta=beta)


@pytest.mark.parametrize("n", [1, 2, 3, 4, 6])
def test_identical_sequences_give_one(n):
    seq = list(range(5, 25))
    res = one(seq, [seq], n=n)
    assert res.overlap[0, 0] == len(seq) - n + 1
    assert res.prf[0].tolist() == [1.0, 1.0, 1.0]


def test_disjoint_sequences_give_zero():
    res = one([1, 2, 3, 4], [[5, 6, 7, 8, 9]], n=1)
    assert res.overlap[0, 0] == 0 and res.prf[0].tolist() == [0.0, 0.0, 0.0]


@pytest.mark.parametrize("c,r,n", [(4, 10, 1), (7, 9, 2), (10, 30, 4), (12, 12, 3)])
def test_prefix_candidate_has_full_precision_and_length_ratio_recall(c, r, n):
    ref = list(range(100, 100 + r))
    res = one(ref[:c], [ref], n=n)
    P, R, F = res.prf[0]
    assert P == 1.0
    assert R == pytest.approx((c - n + 1) / (r - n + 1), rel=1e-15)
    assert F == pytest.approx(2 * P * R / (P + R), rel=1e-15)


@pytest.mark.parametrize("c,r,n", [(9, 4, 1), (4, 9, 1), (9, 4, 3), (5, 5, 2)])
def test_repeated_token_overlap_is_the_smaller_window_count(c, r, n):
    res = one([7] * c, [[7] * r], n=n)
    assert res.overlap[0, 0] == min(c, r) - n + 1
    assert res.prf[0, 0] == pytest.approx((min(c, r) - n + 1) / (c - n + 1))
    assert res.prf[0, 1] == pytest.approx((min(c, r) - n + 1) / (r - n + 1))


def test_hand_worked_bigram_case_and_beta():
    # candidate a b c a b d, reference a b a b a b: bigrams of the candidate ab bc ca ab bd,
    # of the reference ab ba ab ba ab; min(ab) = min(2, 3) = 2, nothing else shared
    cand, ref = [1, 2, 3, 1, 2, 4], [1, 2, 1, 2, 1, 2]
    res = one(cand, [ref], n=2)
    assert res.overlap[0, 0] == 2
    P, R = Fraction(2, 5), Fraction(2, 5)
    assert res.prf[0].tolist() == pytest.approx([float(P), float(R), float(2 * P * R / (P + R))])
    # unigrams: a 2/3, b 2/3, c 1/0, d 1/0 -> overlap 4, P = 4/6, R = 4/6
    assert one(cand, [ref], n=1).overlap[0, 0] == 4
    # beta = 2 weighs recall four times as much: F = 5 P R / (R + 4 P)
    res = one([1, 2, 3, 4], [[1, 2, 3, 9, 9]], n=2, beta=2.0)        # P = 2/3, R = 1/2
    P, R = Fraction(2, 3), Fraction(1, 2)
    assert res.prf[0, 2] == pytest.approx(float(5 * P * R / (R + 4 * P)), rel=1e-15)


def test_best_reference_is_the_one_with_the_highest_f_lowest_index_on_ties():
    cand = [1, 2, 3, 4, 5]
    refs = [[9, 9, 9, 9, 9], [1, 2, 3, 8, 8], [1, 2, 3, 4, 5], [1, 2, 3, 4, 5]]
    res = one(cand, refs, n=2)
    assert res.overlap[0].tolist() == [0, 2, 4, 4]
    assert res.best[0] == 2 and res.prf[0].tolist() == [1.0, 1.0, 1.0]
    # all references disjoint: F = 0 everywhere, reference 0 is reported
    res = one(cand, [[7, 7], [8, 8]], n=1)
    assert res.best[0] == 0 and res.prf[0].tolist() == [0.0, 0.0, 0.0]


def test_exactly_equal_f_goes_to_the_lowest_index_whatever_the_rounding():
    # beta = 1: F = 2 ov / (ct + rt).  ct = 5; reference A: ov 2, rt 5 -> 4/10; reference B: ov 3,
    # rt 10 -> 6/15: the same rational although P, R and their float quotients differ
    cand = [1, 2, 3, 4, 5]
    a, b = [1, 2, 9, 9, 9], [1, 2, 3, 9, 9, 9, 9, 9, 9, 9]
    for refs in ([a, b], [b, a]):
        res = one(cand, refs, n=1)
        assert sorted(res.overlap[0].tolist()) == [2, 3]
        assert res.best[0] == 0 and res.prf[0, 2] == pytest.approx(0.4, rel=1e-15)
    # a strictly better later reference wins: ov 3 of rt 9 -> 6/14 > 4/10
    res = one(cand, [a, b[:9]], n=1)
    assert res.best[0] == 1 and res.prf[0].tolist() == pytest.approx([3 / 5, 3 / 9, 6 / 14])
    # beta = 2 (recall weighs four times): F = 5 ov / (ct + 4 rt); A: 10/25, B: 15/45 -> A
    res = one(cand, [b, a], n=1, beta=2.0)
    assert res.best[0] == 1 and res.prf[0, 2] == pytest.approx(0.4, rel=1e-15)
    # beta = 0.5 (precision weighs more): F = 1.25 ov / (ct + rt / 4); A: 2.5/6.25, B: 3.75/7.5 -> B
    res = one(cand, [a, b], n=1, beta=0.5)
    assert res.best[0] == 1 and res.prf[0, 2] == pytest.approx(0.5, rel=1e-15)


def test_choice_follows_a_permutation_of_the_references():
    w = syn.random_small(431, B=40, R=4, vocab=5, max_len=24)
    res = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=2)
    perm = [2, 0, 3, 1]
    res_p = oracle.rouge_n(w.cand, w.cand_len, w.refs[:, perm], w.ref_len[:, perm], n=2)
    np.testing.assert_array_equal(res_p.overlap, res.overlap[:, perm])
    np.testing.assert_array_equal(res_p.prf[:, 2], res.prf[:, 2])      # the best F is the same
    for i in range(w.B):
        f = res.prf_all[i, :, 2]
        assert f[res.best[i]] == f.max() and (f[:res.best[i]] < f.max()).all()


def test_sequences_shorter_than_the_order_have_no_ngrams():
    res = one([1, 2], [[1, 2, 3, 4]], n=3)
    assert res.overlap[0, 0] == 0 and res.prf[0].tolist() == [0.0, 0.0, 0.0]
    res = one([1, 2, 3, 4], [[1, 2]], n=3)
    assert res.overlap[0, 0] == 0 and res.prf[0].tolist() == [0.0, 0.0, 0.0]
    res = one([], [[1, 2]], n=1)
    assert res.prf[0].tolist() == [0.0, 0.0, 0.0]


def brute_overlap(cand, ref, n):
    """Dictionary-free: every candidate window is matched to an unused equal reference window."""
    cw = [tuple(cand[p:p + n]) for p in range(len(cand) - n + 1)]
    rw = [tuple(ref[p:p + n]) for p in range(len(ref) - n + 1)]
    used = [False] * len(rw)
    ov = 0
    for g in cw:
        for q, h in enumerate(rw):
            if not used[q] and g == h:
                used[q] = True
                ov += 1
                break
    return ov


def test_exhaustive_tiny_inputs_match_the_matching_definition():
    seqs = [list(s) for L in range(0, 5) for s in itertools.product([0, 1], repeat=L)]
    cands, refs = zip(*[(c, [r]) for c in seqs for r in seqs])
    c, cl, r, rl = pad_batch(list(cands), list(refs))
    for n in (1, 2, 3):
        res = oracle.rouge_n(c, cl, r, rl, n=n)
        for i, (cand, ref) in enumerate(zip(cands, refs)):
            assert res.overlap[i, 0] == brute_overlap(cand, ref[0], n)


@pytest.mark.parametrize("seed,V,R,n", [(1, 3, 2, 2), (2, 5, 3, 1), (3, 2, 4, 3), (4, 50, 2, 4)])
def test_random_small_match_brute_force_and_invariants(seed, V, R, n):
    w = syn.random_small(seed + 400, B=30, R=R, vocab=V, max_len=18)
    res = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=n)
    for i in range(w.B):
        cand = w.cand[i, :w.cand_len[i]].tolist()
        fs = []
        for j in range(R):
            ref = w.refs[i, j, :w.ref_len[i, j]].tolist()
            ov = brute_overlap(cand, ref, n)
            assert res.overlap[i, j] == ov
            ct, rt = max(len(cand) - n + 1, 0), max(len(ref) - n + 1, 0)
            assert ov <= min(ct, rt)
            P, Rc = (Fraction(ov, ct) if ct else Fraction(0)), (Fraction(ov, rt) if rt else Fraction(0))
            fs.append(2 * P * Rc / (P + Rc) if P + Rc > 0 else Fraction(0))
            assert res.prf_all[i, j].tolist() == [float(P), float(Rc), float(fs[-1])]
        assert res.best[i] == fs.index(max(fs))              # the first maximum, exactly
        assert res.prf[i].tolist() == res.prf_all[i, res.best[i]].tolist()
    # symmetric roles: swapping candidate and (single) reference swaps precision and recall
    w1 = syn.random_small(seed + 500, B=20, R=1, vocab=V, max_len=18)
    a = oracle.rouge_n(w1.cand, w1.cand_len, w1.refs, w1.ref_len, n=n)
    L = max(w1.cand.shape[1], w1.refs.shape[2])
    c2 = np.zeros((w1.B, L), np.int32); c2[:, :w1.refs.shape[2]] = w1.refs[:, 0]
    r2 = np.zeros((w1.B, 1, L), np.int32); r2[:, 0, :w1.cand.shape[1]] = w1.cand
    b = oracle.rouge_n(c2, w1.ref_len[:, 0], r2, w1.cand_len[:, None], n=n)
    np.testing.assert_array_equal(a.overlap, b.overlap)
    np.testing.assert_allclose(a.prf[:, 0], b.prf[:, 1], rtol=0, atol=0)
    np.testing.assert_allclose(a.prf[:, 1], b.prf[:, 0], rtol=0, atol=0)


def test_reference_counts_and_relation_to_bleu_clipping():
    w = syn.random_small(77, B=25, R=3, vocab=6, max_len=30)
    rc = syn.ref_counts(3, w.B, w.R)
    res = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=2, ref_count=rc)
    full = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=2)
    for i in range(w.B):
        k = int(rc[i])
        np.testing.assert_array_equal(res.overlap[i, :k], full.overlap[i, :k])
        assert (res.overlap[i, k:] == 0).all() and res.best[i] < k
    # with one reference the overlap is BLEU's clipped count of the same order
    w1 = syn.random_small(78, B=25, R=1, vocab=6, max_len=30)
    bleu = oracle.bleu(w1.cand, w1.cand_len, w1.refs, w1.ref_len)
    for n in (1, 2, 3, 4):
        r = oracle.rouge_n(w1.cand, w1.cand_len, w1.refs, w1.ref_len, n=n)
        np.testing.assert_array_equal(r.overlap[:, 0], bleu.clipped[:, n - 1])
    with pytest.raises(ValueError):
        oracle.rouge_n(w1.cand, w1.cand_len, w1.refs, w1.ref_len, n=0)
    with pytest.raises(ValueError):
        oracle.rouge_n(w1.cand, w1.cand_len, w1.refs, w1.ref_len, n=2, beta=0.0)
