"""GPU tests of int64 token ingestion and of the PyTorch-facing convenience layer."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05485_amd as tb
import synth_inputs as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"


def dev(a, dtype=None):
    t = torch.from_numpy(np.ascontiguousarray(a)).to(DEV)
    return t.to(dtype) if dtype is not None else t


@pytest.mark.parametrize("path", ["fused", "global"])
@pytest.mark.parametrize("config", [1, 4])
def test_int64_tokens_give_the_same_bits_as_int32(config, path):
    w = syn.make(config) if config == 1 else syn.config4(B=32)
    run = w.runs[0]
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing=run.smoothing,
                      smooth_param=run.smooth_param, threads=8)
    outs = []
    for dt in (torch.int32, torch.int64):
        cfg = tb.make_config(smoothing=run.smoothing, smooth_param=run.smooth_param,
                             vocab_size=w.vocab, path=path)
        st = tb.Stats.allocate(w.B, 4, DEV)
        out = tb.tensorbleu_sentence(dev(w.cand, dt), dev(w.cand_len), dev(w.refs, dt),
                                     dev(w.ref_len), cfg, stats=st)
        torch.cuda.synchronize()
        assert st.device_status.item() == 0
        np.testing.assert_array_equal(st.clipped.cpu().numpy(), ref.clipped)
        assert np.abs(out.cpu().numpy() - ref.bleu).max() <= 1e-5
        outs.append(out.cpu().numpy())
    np.testing.assert_array_equal(outs[0], outs[1])


@pytest.mark.parametrize("path", ["fused", "global"])
def test_int64_ids_beyond_int32_are_flagged(path):
    w = syn.random_small(301, B=4, R=1, vocab=100, max_len=30, min_len=10)
    cand = dev(w.cand, torch.int64)
    cand[1, 2] = 2 ** 40 + 5          # low 32 bits would be a valid id: must not be truncated
    cfg = tb.make_config(vocab_size=w.vocab, path=path)
    st = tb.Stats.allocate(w.B, 4, DEV)
    tb.tensorbleu_sentence(cand, dev(w.cand_len), dev(w.refs, torch.int64), dev(w.ref_len), cfg,
                           stats=st)
    torch.cuda.synchronize()
    assert st.device_status.item() & tb.binding.TB_DEV_TOKEN_RANGE


def test_mixed_token_dtypes_are_rejected():
    w = syn.random_small(302, B=2, R=1, vocab=50, max_len=12, min_len=6)
    cfg = tb.make_config(vocab_size=w.vocab)
    with pytest.raises(tb.TensorBLEUError):
        tb.tensorbleu_sentence(dev(w.cand, torch.int64), dev(w.cand_len), dev(w.refs),
                               dev(w.ref_len), cfg)


def test_scorer_reuses_its_buffers_and_matches_the_oracle():
    w = syn.config3(B=24)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp", threads=8)
    scorer = tb.BleuScorer(w.B, w.R, w.cand.shape[1], w.refs.shape[2], vocab_size=w.vocab,
                           smoothing="exp", device=DEV)
    cand, refs = dev(w.cand, torch.int64), dev(w.refs, torch.int64)
    cl, rl = dev(w.cand_len), dev(w.ref_len)
    first = scorer(cand, cl, refs, rl)
    ptr = first.data_ptr()
    for _ in range(3):
        again = scorer(cand, cl, list(refs.unbind(dim=1)), rl.to(torch.int64))
    torch.cuda.synchronize()
    assert again.data_ptr() == ptr
    assert np.abs(again.cpu().numpy() - ref.bleu).max() <= 1e-5
    c = scorer.corpus(cand, cl, refs, rl)
    assert abs(float(c.item()) - ref.corpus_bleu) <= 1e-5
    one_shot = tb.sentence_bleu(cand, cl, refs, rl, vocab_size=w.vocab, smoothing="exp")
    np.testing.assert_array_equal(one_shot.cpu().numpy(), again.cpu().numpy())
    assert abs(float(tb.corpus_bleu(cand, cl, refs, rl, vocab_size=w.vocab,
                                    smoothing="exp").item()) - ref.corpus_bleu) <= 1e-5
    with pytest.raises(tb.TensorBLEUError):
        scorer(cand[:, :100], cl, refs, rl)


@pytest.mark.parametrize("path", ["fused", "global"])
def test_hip_graph_capture_and_replay(path):
    """The call allocates nothing and never synchronises, so it can be captured in a HIP graph.
    Every replay (with the inputs rewritten in place between replays) must equal the oracle."""
    w1 = syn.random_small(401, B=48, R=2, vocab=300, max_len=120, min_len=20)
    w2 = syn.random_small(402, B=48, R=2, vocab=300, max_len=120, min_len=20)
    scorer = tb.BleuScorer(w1.B, w1.R, w1.cand.shape[1], w1.refs.shape[2], vocab_size=300,
                           smoothing="floor", smooth_param=0.1, path=path, device=DEV)
    cand, cl = dev(w1.cand), dev(w1.cand_len)
    refs, rl = dev(w1.refs), dev(w1.ref_len)
    scorer(cand, cl, refs, rl)                      # warm-up outside capture
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = scorer(cand, cl, refs, rl)
    for rep, w in enumerate([w1, w2, w1, w2]):
        cand.copy_(dev(w.cand)); cl.copy_(dev(w.cand_len))
        refs.copy_(dev(w.refs)); rl.copy_(dev(w.ref_len))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="floor",
                          smooth_param=0.1)
        assert np.abs(out.cpu().numpy() - ref.bleu).max() <= 1e-5, (path, rep)
        eager = tb.sentence_bleu(cand, cl, refs, rl, vocab_size=300, smoothing="floor",
                                 smooth_param=0.1, path=path)
        np.testing.assert_array_equal(out.cpu().numpy(), eager.cpu().numpy())


def test_hip_graph_replay_of_the_partitioned_kernels():
    """A long group (several launches: zero fill, partitioned dictionary per key kind, count/clip,
    finalize) captured and replayed with fresh inputs."""
    V = 200000                                        # 18 bits: the 4-grams take the derived keys
    ws = [syn.random_small(s, B=3, R=1, vocab=V, max_len=7000, min_len=6500) for s in (411, 412)]
    scorer = tb.BleuScorer(3, 1, ws[0].cand.shape[1], ws[0].refs.shape[2], vocab_size=V,
                           smoothing="exp", path="auto", device=DEV)
    lay = tb.tensorbleu_workspace_layout(3, 1, ws[0].cand.shape[1], ws[0].refs.shape[2], scorer.cfg)
    assert lay.global_partitions == 4
    cand, cl = dev(ws[0].cand), dev(ws[0].cand_len)
    refs, rl = dev(ws[0].refs), dev(ws[0].ref_len)
    scorer(cand, cl, refs, rl)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        out = scorer(cand, cl, refs, rl)
    for rep, w in enumerate([ws[0], ws[1], ws[0]]):
        cand.copy_(dev(w.cand)); cl.copy_(dev(w.cand_len))
        refs.copy_(dev(w.refs)); rl.copy_(dev(w.ref_len))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
        assert np.abs(out.cpu().numpy() - ref.bleu).max() <= 1e-5, rep


def test_scorer_accepts_reference_counts():
    w = syn.random_small(61, B=20, R=3, vocab=30, max_len=50)
    rc = syn.ref_counts(61, w.B, w.R)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp", ref_count=rc)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    scorer = tb.BleuScorer(w.B, w.R, w.cand.shape[1], w.refs.shape[2], vocab_size=w.vocab,
                           smoothing="exp")
    out = scorer(to(w.cand).long(), to(w.cand_len), to(w.refs).long(), to(w.ref_len),
                 ref_count=to(rc).long()).cpu().numpy()
    assert np.abs(out.astype(np.float64) - ref.bleu).max() <= 1e-5
    full = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
    out = scorer(to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len)).cpu().numpy()
    assert np.abs(out.astype(np.float64) - full.bleu).max() <= 1e-5   # count cleared again


def test_pad_references_with_ragged_reference_lists():
    rng = np.random.default_rng(5)
    B, V = 12, 40
    cands = [rng.integers(0, V, rng.integers(5, 30)).tolist() for _ in range(B)]
    refs = [[rng.integers(0, V, rng.integers(3, 35)).tolist() for _ in range(rng.integers(1, 5))]
            for _ in range(B)]
    drefs, dref_len, dcount = tb.pad_references(refs)
    L = max(len(c) for c in cands)
    cand = np.zeros((B, L), np.int32)
    for i, c in enumerate(cands):
        cand[i, :len(c)] = c
    cand_len = np.array([len(c) for c in cands], np.int32)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    scorer = tb.BleuScorer(B, drefs.shape[1], L, drefs.shape[2], vocab_size=V, smoothing="floor",
                           smooth_param=0.1)
    out = scorer(to(cand), to(cand_len), drefs, dref_len, ref_count=dcount).cpu().numpy()
    for i in range(B):       # each candidate against exactly its own references, one at a time
        k = len(refs[i])
        Lr = max(len(r) for r in refs[i])
        r = np.zeros((1, k, Lr), np.int32)
        for j, seq in enumerate(refs[i]):
            r[0, j, :len(seq)] = seq
        rl = np.array([[len(seq) for seq in refs[i]]], np.int32)
        ref = oracle.bleu(cand[i:i + 1], cand_len[i:i + 1], r, rl, smoothing="floor",
                          smooth_param=0.1)
        assert abs(float(out[i]) - ref.bleu[0]) <= 1e-5


def test_pack_reference_lists_and_scorer_status_check():
    rng = np.random.default_rng(6)
    B, V = 10, 30
    cands = [rng.integers(0, V, rng.integers(5, 30)).tolist() for _ in range(B)]
    refs = [[rng.integers(0, V, rng.integers(3, 35)).tolist() for _ in range(rng.integers(1, 7))]
            for _ in range(B)]
    rows, row_len, offsets, max_refs = tb.pack_reference_lists(refs)
    assert rows.shape[0] == sum(len(g) for g in refs) and max_refs == max(len(g) for g in refs)
    L = max(len(c) for c in cands)
    cand = np.zeros((B, L), np.int32)
    for i, c in enumerate(cands):
        cand[i, :len(c)] = c
    cand_len = np.array([len(c) for c in cands], np.int32)
    to = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to("cuda:0")
    cfg = tb.make_config(vocab_size=V, smoothing="exp", ref_offsets=offsets, max_refs=max_refs)
    out = tb.tensorbleu_sentence(to(cand), to(cand_len), rows, row_len, cfg).cpu().numpy()
    ref = oracle.bleu(cand, cand_len, rows.cpu().numpy(), row_len.cpu().numpy(), smoothing="exp",
                      ref_offsets=offsets.cpu().numpy())
    assert np.abs(out.astype(np.float64) - ref.bleu).max() <= 1e-5
    # the scorer's status word: clean after a good call, raised (and cleared) after a bad one
    w = syn.random_small(88, B=6, R=1, vocab=50, max_len=40, min_len=10)
    scorer = tb.BleuScorer(w.B, 1, w.cand.shape[1], w.refs.shape[2], vocab_size=50)
    scorer(to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len))
    scorer.check()
    narrow = tb.BleuScorer(w.B, 1, w.cand.shape[1], w.refs.shape[2], vocab_size=8)
    narrow(to(w.cand), to(w.cand_len), to(w.refs), to(w.ref_len))
    with pytest.raises(tb.TensorBLEUError, match="token id out of range"):
        narrow.check()
    narrow.check()                                     # cleared by the failed check


def test_plain_c_caller_of_the_abi():
    """The C ABI is usable without PyTorch: a C99 program (built beforehand by build.py) links the
    library, runs both paths on three closed-form cases and compares them itself."""
    import os
    import subprocess
    exe = os.path.join(os.path.dirname(tb.LIB_PATH), "c_caller")
    if not os.path.exists(exe):       # normally built beforehand; a host-only gcc step otherwise
        from paper_2510_05485_amd import build
        try:
            build.build_example(verbose=False)
        except (OSError, subprocess.CalledProcessError) as err:
            pytest.skip(f"example caller not built and cannot be built here: {err}")
    res = subprocess.run([exe], capture_output=True, text=True, timeout=60)
    assert res.returncode == 0, res.stdout + res.stderr
    rows = [tuple(map(float, line.split())) for line in res.stdout.split("\n") if line.strip()]
    assert len(rows) == 6
    for got, want in rows:
        assert abs(got - want) <= 1e-5
    assert rows[1][1] == pytest.approx(np.exp(-0.5), abs=1e-6)


def test_two_streams_with_their_own_workspaces_run_side_by_side():
    """The stream argument: calls on two streams (default priority), each with its own scorer
    (workspace, outputs), enqueued alternately without waiting, give what the same calls give one
    at a time.  One scorer runs the fused kernel, the other the GLOBAL passes."""
    wa = syn.random_small(421, B=64, R=2, vocab=5000, max_len=400, min_len=100)
    wb = syn.random_small(422, B=40, R=3, vocab=300, max_len=700, min_len=50)
    mk = lambda w, path: tb.BleuScorer(w.B, w.R, w.cand.shape[1], w.refs.shape[2],
                                       vocab_size=w.vocab, smoothing="exp", path=path, device=DEV)
    sa, sb = mk(wa, "fused"), mk(wb, "global")
    ins = lambda w: (dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    ia, ib = ins(wa), ins(wb)
    serial_a, serial_b = sa(*ia).clone(), sb(*ib).clone()
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(20):
        with torch.cuda.stream(s1):
            oa = sa(*ia)
        with torch.cuda.stream(s2):
            ob = sb(*ib)
        s1.synchronize(); s2.synchronize()
        outs.append((oa.clone(), ob.clone()))
    for oa, ob in outs:
        assert torch.equal(oa, serial_a) and torch.equal(ob, serial_b)
    sa.check(); sb.check()
    ref = oracle.bleu(wb.cand, wb.cand_len, wb.refs, wb.ref_len, smoothing="exp")
    assert np.abs(serial_b.cpu().numpy() - ref.bleu).max() <= 1e-5
