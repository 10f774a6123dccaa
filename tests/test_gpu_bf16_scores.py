"""GPU tests of bfloat16 score outputs (cfg.score_bytes = 2): the stored value is the fp32 score
rounded to nearest even.  Two checks: bit-exact against a library conversion of the fp32 output of
the same kernels, and against the oracle's score rounded by the oracle's own bfloat16 rule (at most
one bfloat16 step apart, since the two fp32 scores may differ by the fp32 tolerance)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05485_amd as tb
import synth_inputs as syn

pytestmark = pytest.mark.gpu
DEV = "cuda:0"
TOL = 1e-5


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def close_in_bf16(got, want64):
    """got: bfloat16 tensor; want64: oracle fp64 scores.  One bfloat16 step (2^-7 relative) plus
    the fp32 tolerance."""
    g = got.to(torch.float64).cpu().numpy()
    w = oracle.to_bfloat16(want64)
    return np.all(np.abs(g - w) <= np.abs(w) * 2.0 ** -7 + TOL), np.mean(g != w)


@pytest.mark.parametrize("path", ["fused", "global"])
@pytest.mark.parametrize("smoothing", ["none", "exp"])
def test_sentence_and_corpus_scores_in_bfloat16(path, smoothing):
    w = syn.config5(B=96) if path == "fused" else syn.make(1)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing=smoothing, threads=8)
    args = (dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    c32 = tb.make_config(smoothing=smoothing, vocab_size=w.vocab, path=path)
    c16 = tb.make_config(smoothing=smoothing, vocab_size=w.vocab, path=path,
                         score_dtype=torch.bfloat16)
    s32, s16 = tb.tensorbleu_sentence(*args, c32), tb.tensorbleu_sentence(*args, c16)
    k32, k16 = tb.tensorbleu_corpus(*args, c32), tb.tensorbleu_corpus(*args, c16)
    torch.cuda.synchronize()
    assert s16.dtype == torch.bfloat16 and k16.dtype == torch.bfloat16
    # exactly the rounding of the kernels' own fp32 scores (conversion done by the library on the CPU)
    assert torch.equal(s16.cpu(), s32.cpu().to(torch.bfloat16))
    assert torch.equal(k16.cpu(), k32.cpu().to(torch.bfloat16))
    ok, differing = close_in_bf16(s16, ref.bleu)
    assert ok and differing <= 0.05
    ok, _ = close_in_bf16(k16, np.array([ref.corpus_bleu]))
    assert ok
    assert float(s32.max()) > 0.0     # the case is not all zeros


def test_rouge_scores_in_bfloat16():
    w = syn.config5(B=64)
    ref = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=2)
    args = (dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    p32 = tb.tensorrouge_n(*args, n=2, vocab_size=w.vocab)
    p16, _, best = tb.tensorrouge_n(*args, n=2, vocab_size=w.vocab, score_dtype=torch.bfloat16,
                                    want_best=True)
    torch.cuda.synchronize()
    assert p16.dtype == torch.bfloat16 and tuple(p16.shape) == (w.B, 3)
    assert torch.equal(p16.cpu(), p32.cpu().to(torch.bfloat16))
    # the oracle's numbers for the reference the kernel chose (near-ties may go either way)
    chosen = ref.prf_all[np.arange(w.B), best.cpu().numpy()]
    assert (chosen[:, 2] >= ref.prf[:, 2] * (1.0 - 4.0 * 2.0 ** -24)).all()
    ok, _ = close_in_bf16(p16, chosen)
    assert ok


def test_scorer_with_bfloat16_rewards_and_wrong_out_dtype():
    w = syn.random_small(77, B=9, R=2, vocab=40, max_len=40, min_len=12)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="add-k", smooth_param=1.0)
    scorer = tb.BleuScorer(w.B, w.R, w.cand.shape[1], w.refs.shape[2], vocab_size=w.vocab,
                           smoothing="add-k", smooth_param=1.0, device=DEV,
                           score_dtype=torch.bfloat16)
    out = scorer(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len))
    torch.cuda.synchronize()
    ok, _ = close_in_bf16(out, ref.bleu)
    assert out.dtype == torch.bfloat16 and ok
    cfg = tb.make_config(vocab_size=w.vocab, score_dtype=torch.bfloat16)
    with pytest.raises(tb.TensorBLEUError):
        tb.tensorbleu_sentence(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len), cfg,
                               out=torch.empty(w.B, dtype=torch.float32, device=DEV))
    with pytest.raises(tb.TensorBLEUError):
        tb.make_config(vocab_size=w.vocab, score_dtype=torch.float16)
