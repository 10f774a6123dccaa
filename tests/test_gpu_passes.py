"""GPU parity of the GLOBAL path one pass at a time (pack, dictionary, count/clip, finalize).

Expected keys are formed here from the definition with Python integers; the dictionary's ids are
internal (any bijection is correct), so the test checks what is unique: ids are equal exactly
when the n-grams are equal, they are dense in the group's offset range, and the dictionary size
equals the oracle's count of distinct n-grams.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05485_amd as tb
import synth_inputs as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def stage_all(w, run=syn.Run("exp"), corpus=False):
    cfg = tb.make_config(max_n=w.max_n, weights=w.weights, smoothing=run.smoothing,
                         smooth_param=run.smooth_param, vocab_size=w.vocab, path="global")
    cs, rs = w.cand.shape[1], w.refs.shape[2]
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, cs, rs, cfg)
    ws = tb.allocate_workspace(w.B, w.R, cs, rs, cfg, DEV)
    ws.fill_(0xAB)                                   # the workspace needs no initialisation
    stats = tb.Stats.allocate(w.B, w.max_n, DEV)
    cand, cl, refs, rl = dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len)
    tb.tensorbleu_pack(cand, cl, refs, rl, cfg, ws, stats)
    tb.tensorbleu_dictionary(cl, rl, cs, rs, cfg, ws, stats)
    tb.tensorbleu_count_clip(cl, rl, cs, rs, cfg, ws, stats)
    out = torch.empty(1 if corpus else w.B, dtype=torch.float32, device=DEV)
    tb.tensorbleu_finalize(cl, rl, cs, rs, cfg, corpus, out, ws, stats)
    torch.cuda.synchronize()
    return lay, ws.cpu().numpy(), stats, out.cpu().numpy()


def read_keys(wsb, lay, n, count):
    kb = lay.key_bytes[n - 1]
    raw = wsb[lay.keys_off[n - 1]: lay.keys_off[n - 1] + count * kb].view(np.uint64)
    if kb == 8:
        return [int(x) for x in raw]
    return [int(lo) | (int(hi) << 64) for lo, hi in raw.reshape(-1, 2)]


def expected_key(tokens, bits):
    k = 0
    for t in tokens:
        k = (k << bits) | int(t)
    return k


@pytest.mark.parametrize("seed,B,R,V,L", [(201, 6, 2, 64, 50), (202, 4, 1, 50257, 1100),
                                          (203, 3, 1, 262144, 1300), (204, 2, 3, 2 ** 31 - 1, 80)])
def test_pack_dictionary_count_passes(seed, B, R, V, L):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L, min_len=L // 2)
    lay, wsb, stats, out = stage_all(w)
    cap = lay.group_cap
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
    assert lay.global_candidate_first == (0 if V > 2 ** 20 else 1)
    cand_distinct = wsb[lay.cand_distinct_off: lay.cand_distinct_off + B * 4 * 4].view(
        np.int32).reshape(B, 4)
    for n in range(1, 5):
        keys = read_keys(wsb, lay, n, B * cap)
        inv = wsb[lay.inv_off[n - 1]: lay.inv_off[n - 1] + B * cap * 4].view(np.uint32)
        for g in range(B):
            rows = [(w.cand[g], w.cand_len[g])] + [
                (w.refs[g, j], w.ref_len[g, j]) for j in range(R)]
            seen, slot = {}, g * cap          # group-compact: sequences stored back to back
            for row, ln in rows:
                for p in range(max(ln - n + 1, 0)):
                    gram = tuple(int(t) for t in row[p:p + n])
                    assert keys[slot] == expected_key(gram, lay.bits), (n, g, p)
                    local = int(inv[slot]) - g * cap
                    assert seen.setdefault(gram, local) == local      # equal n-gram -> equal id
                    slot += 1
            ids = sorted(seen.values())
            assert ids == list(range(len(ids)))                        # dense and injective
            assert len(ids) == ref.group_distinct[g, n - 1]
            if lay.global_candidate_first:
                # ids below cand_distinct[g][n] are exactly the n-grams the candidate contains
                cd = int(cand_distinct[g, n - 1])
                assert cd == ref.cand_distinct[g, n - 1]
                in_cand = {tuple(int(t) for t in w.cand[g, p:p + n])
                           for p in range(max(w.cand_len[g] - n + 1, 0))}
                assert all((gram in in_cand) == (local < cd) for gram, local in seen.items())
    np.testing.assert_array_equal(stats.group_distinct.cpu().numpy(), ref.group_distinct)
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), ref.clipped)
    np.testing.assert_array_equal(stats.total.cpu().numpy(), ref.total)
    assert np.abs(out - ref.bleu).max() <= 1e-5


def test_staged_calls_equal_the_single_call_on_config1():
    w = syn.make(1)
    _, _, stats, out = stage_all(w, syn.Run("add-k", 1.0))
    cfg = tb.make_config(smoothing="add-k", smooth_param=1.0, vocab_size=w.vocab, path="global")
    st2 = tb.Stats.allocate(w.B, 4, DEV)
    out2 = tb.tensorbleu_sentence(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len), cfg,
                                  stats=st2)
    torch.cuda.synchronize()
    np.testing.assert_array_equal(out, out2.cpu().numpy())
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), st2.clipped.cpu().numpy())
    _, _, cstats, cout = stage_all(w, syn.Run("add-k", 1.0), corpus=True)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="add-k", smooth_param=1.0)
    np.testing.assert_array_equal(cstats.corpus_stats.cpu().numpy(), ref.corpus_stats)
    assert abs(cout[0] - ref.corpus_bleu) <= 1e-5


@pytest.mark.parametrize("seed,B,R,L", [(231, 13, 2, 700), (232, 37, 1, 300), (233, 3, 4, 1500)])
def test_score_inside_the_count_kernel_with_a_group_spread_over_xcds(seed, B, R, L):
    # With a batch size that is no multiple of eight, the count workgroups of one group (one per
    # order, B workgroup indices apart) run on different XCDs, each with its own L2: the
    # statistics and the arrival counter then have to travel through device-scope operations.
    w = syn.random_small(seed, B=B, R=R, vocab=5000, max_len=L, min_len=L // 2)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
    cfg = tb.make_config(smoothing="exp", vocab_size=w.vocab, path="global")
    cand, cl, refs, rl = dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len)
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, cand.shape[1], refs.shape[2], cfg)
    assert lay.global_candidate_first == 1      # the hierarchical-key kernels
    st = tb.Stats.allocate(w.B, 4, DEV, corpus_stats=False)
    ws = tb.allocate_workspace(w.B, w.R, cand.shape[1], refs.shape[2], cfg, DEV)
    out = torch.empty(w.B, dtype=torch.float32, device=DEV)
    first = None
    for _ in range(300):
        out.fill_(-1.0)
        st.closest_ref_len.fill_(-1)
        st.clipped.fill_(12345)     # a scoring workgroup that read stale statistics would show
        st.total.fill_(1)
        tb.tensorbleu_sentence(cand, cl, refs, rl, cfg, out=out, stats=st, workspace=ws)
        if first is None:
            first = out.clone()
            np.testing.assert_array_equal(st.clipped.cpu().numpy(), ref.clipped)
            np.testing.assert_array_equal(st.closest_ref_len.cpu().numpy(), ref.closest_ref_len)
            assert np.abs(first.cpu().numpy().astype(np.float64) - ref.bleu).max() <= 1e-5
        assert torch.equal(out, first)
    assert st.device_status.item() == 0


@pytest.mark.parametrize("k", [2, 5])
def test_single_global_call_scores_inside_the_count_kernel(k):
    # A single per-sentence call on the hierarchical-key kernels launches no score kernel: of a
    # group's count workgroups, the one that finishes last scores the sentence.  Whichever
    # workgroup that is, the result has to be the staged passes' (which end with the score
    # kernel), bit for bit and on every repetition; without corpus statistics, so that the
    # single call takes that route.
    w = syn.make(k)
    run = [r for r in w.runs if not r.corpus][-1]
    _, _, stats, out = stage_all(w, run)
    cfg = tb.make_config(max_n=w.max_n, weights=w.weights, smoothing=run.smoothing,
                         smooth_param=run.smooth_param, vocab_size=w.vocab, path="global")
    cand, cl, refs, rl = dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len)
    st2 = tb.Stats.allocate(w.B, w.max_n, DEV, corpus_stats=False)
    ws = tb.allocate_workspace(w.B, w.R, cand.shape[1], refs.shape[2], cfg, DEV)
    out2 = torch.empty(w.B, dtype=torch.float32, device=DEV)
    expect, closest = torch.from_numpy(out).to(DEV), stats.closest_ref_len
    for _ in range(100):
        out2.fill_(-1.0)
        st2.closest_ref_len.fill_(-1)
        st2.clipped.fill_(12345)    # a scoring workgroup that read stale statistics would show
        st2.total.fill_(1)
        tb.tensorbleu_sentence(cand, cl, refs, rl, cfg, out=out2, stats=st2, workspace=ws)
        assert torch.equal(out2, expect)
        assert torch.equal(st2.closest_ref_len, closest)
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), st2.clipped.cpu().numpy())
    np.testing.assert_array_equal(stats.total.cpu().numpy(), st2.total.cpu().numpy())
    assert st2.device_status.item() == 0


@pytest.mark.parametrize("seed,B,R,L,P", [
    (205, 2, 2, 5000, 4),    # one scatter workgroup per (group, order)
    (206, 1, 1, 12000, 8),   # few long groups: the scatter is split over chunks of 16 384 slots
])
def test_partitioned_dictionary_ids_are_a_bijection_within_the_group(seed, B, R, L, P):
    """Groups of 12 289 .. 65 536 slots: the dictionary is split over P workgroups and ids are
    p * 6144 + a number dense within partition p.  What is unique: equal n-gram <=> equal id, ids
    below id_stride, and the distinct count."""
    w = syn.random_small(seed, B=B, R=R, vocab=300, max_len=L, min_len=L * 17 // 20)
    lay, wsb, stats, out = stage_all(w)
    assert lay.global_partitions == P and lay.id_stride == P * 6144
    assert lay.global_tables_in_hbm == 0
    cap, stride = lay.group_cap, lay.id_stride
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
    for n in range(1, 5):
        inv = wsb[lay.inv_off[n - 1]: lay.inv_off[n - 1] + w.B * cap * 4].view(np.uint32)
        for g in range(w.B):
            rows = [(w.cand[g], w.cand_len[g])] + [
                (w.refs[g, j], w.ref_len[g, j]) for j in range(w.R)]
            seen, slot = {}, g * cap
            for row, ln in rows:
                for p in range(max(ln - n + 1, 0)):
                    gram = tuple(int(t) for t in row[p:p + n])
                    local = int(inv[slot]) - g * stride
                    assert 0 <= local < stride
                    assert seen.setdefault(gram, local) == local
                    slot += 1
            assert len(set(seen.values())) == len(seen) == ref.group_distinct[g, n - 1]
    assert stats.device_status.item() == 0
    np.testing.assert_array_equal(stats.group_distinct.cpu().numpy(), ref.group_distinct)
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), ref.clipped)
    np.testing.assert_array_equal(stats.total.cpu().numpy(), ref.total)
    assert np.abs(out - ref.bleu).max() <= 1e-5


def test_partition_overflow_is_reported_not_hidden():
    """More distinct n-grams in one hash partition than it can hold (6144) is only possible with
    tokens chosen to collide; the kernels then finish normally, set TB_DEV_TABLE_OVERFLOW and
    give the group the score NaN."""
    M = 1 << 32
    part = lambda t: ((((t * 0x9E3779B1) % M) * 0x85EBCA6B + 0x27D4EB2F) % M) >> 30   # P = 4
    colliding = [t for t in range(40000) if part(t) == 0][:7000]
    assert len(colliding) == 7000
    L = 8000
    cand = np.zeros((1, L), np.int32)
    cand[0, :7000] = colliding
    refs = np.zeros((1, 1, L), np.int32)
    refs[0, 0, :7000] = colliding[::-1]
    cl, rl = np.array([7000], np.int32), np.array([[7000]], np.int32)
    cfg = tb.make_config(vocab_size=40000, path="global")
    lay = tb.tensorbleu_workspace_layout(1, 1, L, L, cfg)
    assert lay.global_partitions == 4
    st = tb.Stats.allocate(1, 4, DEV)
    out = tb.tensorbleu_sentence(dev(cand), dev(cl), dev(refs), dev(rl), cfg, stats=st)
    torch.cuda.synchronize()
    assert st.device_status.item() & tb.TB_DEV_TABLE_OVERFLOW
    assert np.isnan(out.cpu().numpy()).all()      # not a number: cannot pass for a reward
    cout = tb.tensorbleu_corpus(dev(cand), dev(cl), dev(refs), dev(rl), cfg)
    torch.cuda.synchronize()
    assert np.isnan(cout.cpu().numpy()).all()
    # the remedy the header names: the same call with the tables in the workspace, which have no
    # capacity to exceed -- right statistics and score, nothing flagged
    safe = tb.make_config(vocab_size=40000, path="global", workspace_tables=True)
    slay = tb.tensorbleu_workspace_layout(1, 1, L, L, safe)
    assert slay.global_partitions == 0 and slay.global_tables_in_hbm == 1
    exact = oracle.bleu(cand, cl, refs, rl)
    st = tb.Stats.allocate(1, 4, DEV)
    out = tb.tensorbleu_sentence(dev(cand), dev(cl), dev(refs), dev(rl), safe, stats=st)
    torch.cuda.synchronize()
    assert st.device_status.item() == 0
    np.testing.assert_array_equal(st.clipped.cpu().numpy(), exact.clipped)
    assert np.abs(out.cpu().numpy().astype(np.float64) - exact.bleu).max() <= 1e-5
    # the same shape with ordinary tokens is scored and not flagged
    w = syn.random_small(206, B=1, R=1, vocab=40000, max_len=L, min_len=7000)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len)
    st = tb.Stats.allocate(1, 4, DEV)
    tb.tensorbleu_sentence(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len), cfg, stats=st)
    torch.cuda.synchronize()
    assert st.device_status.item() == 0
    np.testing.assert_array_equal(st.clipped.cpu().numpy(), ref.clipped)
