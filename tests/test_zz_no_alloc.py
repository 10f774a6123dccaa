"""The allocation-free entry point (tensorbleu_sentence_static, built-in scratch buffer) against
tensorbleu_sentence on the same inputs: two calls in a row, the second on a smaller batch, plus
the size limit.  Runs last (file name) so that a failure here hides no other test."""
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


def both(w, path, smoothing="exp"):
    """Scores and integer statistics of the static entry point and of the ordinary one."""
    cfg = tb.make_config(max_n=w.max_n, smoothing=smoothing, vocab_size=w.vocab, path=path)
    args = (dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    got, want = [], []
    for fn, res in ((tb.tensorbleu_sentence_static, got), (tb.tensorbleu_sentence, want)):
        st = tb.Stats.allocate(w.B, w.max_n, DEV, corpus_stats=False)
        out = torch.full((w.B,), -1.0, dtype=torch.float32, device=DEV)
        fn(*args, cfg, out=out, stats=st)
        torch.cuda.synchronize()
        assert st.device_status.item() == 0
        res.extend([out.cpu().numpy(), st.clipped.cpu().numpy(), st.total.cpu().numpy(),
                    st.closest_ref_len.cpu().numpy()])
    return got, want


@pytest.mark.parametrize("path", ["auto", "global"])
def test_static_entry_point_matches_the_ordinary_one_twice_in_a_row(path):
    big = syn.random_small(901, B=48, R=3, vocab=300, max_len=200, min_len=20)
    small = syn.random_small(902, B=5, R=1, vocab=40, max_len=33)
    for w in (big, small):          # the second call reuses the buffer the first one left dirty
        got, want = both(w, path)
        for g, x in zip(got[1:], want[1:]):
            np.testing.assert_array_equal(g, x)
        assert np.abs(got[0].astype(np.float64) - want[0]).max() <= 1e-5
        ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
        np.testing.assert_array_equal(got[1], ref.clipped)
        assert np.abs(got[0].astype(np.float64) - ref.bleu).max() <= 1e-5


def test_static_entry_point_without_statistics_and_its_size_limit():
    w = syn.random_small(903, B=20, R=2, vocab=64, max_len=90, min_len=10)
    cfg = tb.make_config(vocab_size=w.vocab, smoothing="floor", smooth_param=0.1)
    args = (dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    out = torch.empty(w.B, dtype=torch.float32, device=DEV)
    tb.tensorbleu_sentence_static(*args, cfg, out=out)       # statistics live in the scratch
    want = tb.tensorbleu_sentence(*args, cfg)
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    limit = tb.tensorbleu_static_scratch_bytes()
    assert limit == 4 << 20
    # the GLOBAL path on this shape needs far more than the built-in buffer: refused, nothing runs
    gcfg = tb.make_config(vocab_size=50257, path="global")
    wide = syn.random_small(904, B=64, R=2, vocab=50257, max_len=2000, min_len=100)
    assert tb.tensorbleu_workspace_bytes(wide.B, wide.R, wide.cand.shape[1], wide.refs.shape[2],
                                         gcfg) > limit
    sentinel = torch.full((wide.B,), -7.0, dtype=torch.float32, device=DEV)
    with pytest.raises(tb.TensorBLEUError, match="built-in static buffer"):
        tb.tensorbleu_sentence_static(dev(wide.cand), dev(wide.cand_len), dev(wide.refs),
                                      dev(wide.ref_len), gcfg, out=sentinel)
    torch.cuda.synchronize()
    assert (sentinel == -7.0).all()
