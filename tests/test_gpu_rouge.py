"""GPU parity for ROUGE-N (tensorrouge_n through the C ABI) against the CPU oracle: overlap
counts bit-exactly, the chosen reference valid (its exact F within single-precision round-off of
the best exact F), precision / recall / F of that reference within 1e-5."""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05485_amd as tb
import synth_inputs as syn
from rouge_validity import check_rouge

pytestmark = pytest.mark.gpu
TOL = 1e-5
DEV = "cuda:0"


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


def check(w, n, beta=1.0, ref_count=None, int64=False, path="auto"):
    ref = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=n, beta=beta,
                         ref_count=ref_count)
    cand, refs = dev(w.cand), dev(w.refs)
    if int64:
        cand, refs = cand.long(), refs.long()
    stats = tb.Stats.allocate(w.B, n, DEV)
    out, overlap, best = tb.tensorrouge_n(
        cand, dev(w.cand_len), refs, dev(w.ref_len), n=n, beta=beta, vocab_size=w.vocab,
        ref_count=dev(ref_count) if ref_count is not None else None, want_overlap=True,
        want_best=True, stats=stats, path=path)
    torch.cuda.synchronize()
    assert stats.device_status.item() == 0
    check_rouge(ref, overlap.cpu().numpy(), best.cpu().numpy(), out.cpu().numpy(), TOL,
                ref_count=ref_count)
    return out


@pytest.mark.parametrize("n", [1, 2, 3, 4, 6])
@pytest.mark.parametrize("seed,B,R,V,L", [
    (501, 33, 1, 3, 14),          # tiny vocabulary
    (502, 17, 3, 7, 70),          # several references, empty rows included
    (503, 9, 2, 50257, 300),
    (504, 5, 1, 262144, 1500),    # 18-bit ids
    (505, 4, 40, 300, 100),       # forty references
])
def test_rouge_n_random_ragged_batches(n, seed, B, R, V, L):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L)
    check(w, n)


def test_rouge_n_beta_reference_counts_and_int64():
    w = syn.random_small(506, B=40, R=4, vocab=9, max_len=80)
    for beta in (0.5, 2.0):
        check(w, 2, beta=beta)
    check(w, 2, ref_count=syn.ref_counts(506, w.B, w.R))
    check(w, 3, int64=True)


@pytest.mark.parametrize("path", ["auto", "global"])
@pytest.mark.parametrize("k", [1, 2, 3, 4, 5])
def test_rouge_n_full_size_configs(k, path):
    w = syn.make(k)
    for n in (1, 2, 4):
        check(w, n, path=path)


@pytest.mark.parametrize("n", [1, 2, 3, 5])
@pytest.mark.parametrize("seed,B,R,V,L", [
    (511, 21, 3, 7, 70),          # several references, empty rows included
    (512, 9, 2, 50257, 300),
    (513, 5, 1, 262144, 1500),    # 18-bit ids: 16-byte packed keys from order 4 on
    (514, 4, 40, 300, 100),       # forty references
])
def test_rouge_n_global_path_random_ragged_batches(n, seed, B, R, V, L):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L)
    check(w, n, path="global")
    if R > 1:
        check(w, n, beta=2.0, ref_count=syn.ref_counts(seed, w.B, w.R), path="global")


@pytest.mark.parametrize("seed,B,R,V,L,parts", [
    (521, 3, 1, 50257, 5000, 0),      # beyond the fused plans, one LDS table per group
    (522, 2, 2, 300, 5467, 1),        # 16 401 slots per group: partitions per (group, order)
    (523, 2, 1, 50257, 40000, 1),     # long generation, partitioned
    (524, 2, 14, 300, 1500, 1),       # partitioned, references counted in passes
])
def test_rouge_n_beyond_the_fused_plans(seed, B, R, V, L, parts):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L, min_len=L * 9 // 10)
    cfg = tb.make_config(max_n=2, vocab_size=V)
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.fused_ok == 0 and (lay.global_partitions > 0) == bool(parts)
    for n in (1, 2, 4):
        check(w, n)
    check(w, 2, beta=0.5, ref_count=syn.ref_counts(seed, w.B, w.R) if R > 1 else None)


def test_rouge_n_closed_forms_and_unsupported_shapes():
    L = 64
    ref = np.arange(100, 100 + L, dtype=np.int32)
    cand = np.zeros((2, L), np.int32)
    cand[0] = ref
    cand[1, :40] = ref[:40]
    refs = np.stack([ref, ref])[:, None, :]
    out = tb.tensorrouge_n(dev(cand), dev(np.array([L, 40], np.int32)), dev(refs),
                           dev(np.array([[L], [L]], np.int32)), n=2, vocab_size=1000)
    out = out.cpu().numpy()
    assert out[0].tolist() == [1.0, 1.0, 1.0]
    assert out[1, 0] == 1.0 and out[1, 1] == pytest.approx(39 / 63, abs=1e-6)
    big = syn.random_small(507, B=2, R=2, vocab=50, max_len=9000)     # beyond the fused plans
    with pytest.raises(tb.TensorBLEUError):
        tb.tensorrouge_n(dev(big.cand), dev(big.cand_len), dev(big.refs), dev(big.ref_len), n=2,
                         vocab_size=big.vocab, path="fused")
    # 31-bit ids on the GLOBAL path: the packed-key LDS kernels score BLEU only, so the entry
    # point refuses the shape as planned by default ...
    wide = syn.random_small(508, B=2, R=1, vocab=2 ** 31 - 1, max_len=60)
    wcfg = tb.make_config(max_n=2, vocab_size=wide.vocab, path="global")
    wws = tb.allocate_workspace(wide.B, wide.R, wide.cand.shape[1], wide.refs.shape[2], wcfg, DEV)
    with pytest.raises(tb.TensorBLEUError):
        tb.tensorrouge_n(dev(wide.cand), dev(wide.cand_len), dev(wide.refs), dev(wide.ref_len),
                         n=2, vocab_size=wide.vocab, path="global", workspace=wws)
    # ... and serves it on the workspace-table kernels, which the wrapper selects by itself
    check(wide, 2, path="global")


@pytest.mark.parametrize("seed,B,R,V,L", [
    (531, 4, 70, 300, 120),          # more references than the LDS kernels' one lane each
    (532, 3, 2, 2 ** 31 - 1, 900),   # (id, token) keys beyond 32 bits
    (533, 2, 3, 50257, 2500),        # a shape the hierarchical-key kernels would take
])
def test_rouge_n_on_workspace_tables(seed, B, R, V, L):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L, min_len=L // 4)
    for n, beta in ((1, 1.0), (3, 2.0)):
        rr = oracle.rouge_n(w.cand, w.cand_len, w.refs, w.ref_len, n=n, beta=beta)
        o, ov, best = tb.tensorrouge_n(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len),
                                       n=n, beta=beta, vocab_size=V, want_overlap=True,
                                       want_best=True, path="global", workspace_tables=True)
        check_rouge(rr, ov.cpu().numpy(), best.cpu().numpy(), o.cpu().numpy(), 1e-5)
