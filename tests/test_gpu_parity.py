"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle.

Integer statistics (clipped, total, closest reference length, dictionary sizes) must match
bit-exactly; scores (fp32 on the GPU, fp64 in the oracle) within 1e-5 absolute.  The fp32 tail
evaluates at most four log terms and two exps with |log p| < 25, each correctly rounded to a
few ulp (~1e-7 relative), so 1e-5 leaves two orders of magnitude of slack.
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2510_05485_amd as tb
import synth_inputs as syn

pytestmark = pytest.mark.gpu
TOL = 1e-5
DEV = "cuda:0"
PATHS = ["global", "fused"]


def dev(a):
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class Device:
    def __init__(self, w: syn.Workload):
        self.w = w
        self.cand, self.cand_len = dev(w.cand), dev(w.cand_len)
        self.refs, self.ref_len = dev(w.refs), dev(w.ref_len)


_WORKLOADS = {}


def cached_small(*args, **kw):
    """random_small, memoised (both paths of a test reuse the batch)."""
    key = (args, tuple(sorted(kw.items())))
    if key not in _WORKLOADS:
        _WORKLOADS[key] = syn.random_small(*args, **kw)
    return _WORKLOADS[key]


def path_supported(w, path, max_n=4):
    cfg = tb.make_config(max_n=max_n, vocab_size=w.vocab, path="auto")
    lay = tb.binding.tb_layout_t()
    import ctypes
    rc = tb.load_library().tensorbleu_workspace_layout(
        w.B, w.R, w.cand.shape[1], w.refs.shape[2], ctypes.byref(cfg), ctypes.byref(lay))
    assert rc in (0, 3), rc       # ok, or the forced path does not support the shape
    return bool(lay.fused_ok if path == "fused" else lay.global_ok)


def run_gpu(d: Device, run: syn.Run, path, max_n=None, weights=None, corpus=None):
    w = d.w
    max_n = max_n or w.max_n
    cfg = tb.make_config(max_n=max_n, weights=weights if weights is not None else w.weights,
                         smoothing=run.smoothing, smooth_param=run.smooth_param,
                         vocab_size=w.vocab, path=path)
    stats = tb.Stats.allocate(w.B, max_n, DEV)
    corpus = run.corpus if corpus is None else corpus
    fn = tb.tensorbleu_corpus if corpus else tb.tensorbleu_sentence
    out = fn(d.cand, d.cand_len, d.refs, d.ref_len, cfg, stats=stats)
    torch.cuda.synchronize()
    return out.cpu().numpy(), stats


def run_oracle(w, run, max_n=None, weights=None, threads=8):
    max_n = max_n or w.max_n
    weights = weights if weights is not None else w.weights
    return oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, max_n=max_n, weights=weights,
                       smoothing=run.smoothing, smooth_param=run.smooth_param, threads=threads)


def check(w, run, path, max_n=None, weights=None, d=None):
    resolved = path
    if path == "auto":
        resolved = "fused" if path_supported(w, "fused", max_n or w.max_n) else "global"
    if not path_supported(w, resolved, max_n or w.max_n):
        pytest.skip(f"{path} path does not support this shape")
    d = d or Device(w)
    ref = run_oracle(w, run, max_n, weights)
    out, st = run_gpu(d, run, path, max_n, weights, corpus=False)
    assert st.device_status.item() == 0
    np.testing.assert_array_equal(st.clipped.cpu().numpy(), ref.clipped)
    np.testing.assert_array_equal(st.total.cpu().numpy(), ref.total)
    np.testing.assert_array_equal(st.closest_ref_len.cpu().numpy(), ref.closest_ref_len)
    expect_distinct = ref.group_distinct if resolved == "global" else ref.cand_distinct
    np.testing.assert_array_equal(st.group_distinct.cpu().numpy(), expect_distinct)
    assert np.isfinite(out).all()
    assert np.abs(out.astype(np.float64) - ref.bleu).max() <= TOL
    cout, cst = run_gpu(d, run, path, max_n, weights, corpus=True)
    np.testing.assert_array_equal(cst.corpus_stats.cpu().numpy(), ref.corpus_stats)
    assert abs(float(cout[0]) - ref.corpus_bleu) <= TOL
    return out, ref


ALL_MODES = [syn.Run("none"), syn.Run("floor", 0.1), syn.Run("add-k", 1.0), syn.Run("exp")]


# ------------------------------------------------------------------------ small and edge cases

@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("run", ALL_MODES, ids=lambda r: r.smoothing)
def test_config1_all_smoothing_modes(path, run):
    check(syn.make(1), run, path)


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("seed,B,R,V,L", [
    (101, 33, 1, 3, 12),        # tiny vocabulary: almost every n-gram repeats
    (102, 17, 3, 7, 70),        # several references, lengths 0..70 (empty rows included)
    (103, 9, 2, 50257, 300),    # 64-bit keys at exactly 64 bits for n = 4
    (104, 5, 1, 262144, 1500),  # 128-bit keys, more than one pack tile and a ragged tail
    (105, 64, 5, 2, 40),        # binary vocabulary, five references
    (106, 3, 1, 2 ** 31 - 1, 90),  # widest ids: 31 bits per token, 124-bit 4-grams
    (107, 40, 2, 1000, 3),      # candidates shorter than the highest order
    (108, 3, 40, 500, 200),     # forty references: counters no longer fit one field per sequence
])
def test_random_ragged_batches(path, seed, B, R, V, L):
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L)
    d = Device(w)
    for run in ALL_MODES:
        check(w, run, path, d=d)


@pytest.mark.parametrize("path", PATHS)
def test_lower_orders_and_custom_weights(path):
    w = syn.random_small(111, B=20, R=2, vocab=9, max_len=50)
    d = Device(w)
    check(w, syn.Run("none"), path, max_n=1, weights=[1.0], d=d)
    check(w, syn.Run("floor", 0.1), path, max_n=2, weights=[0.7, 0.3], d=d)
    check(w, syn.Run("exp"), path, max_n=3, weights=[0.2, 0.3, 0.5], d=d)
    check(w, syn.Run("add-k", 1.0), path, max_n=4, weights=[0.5, 0.5, 0.0, 0.0], d=d)
    check(w, syn.Run("add-k", 0.5), path, max_n=4, weights=[1.0, 1.0, 1.0, 1.0], d=d)


@pytest.mark.parametrize("path", PATHS)
def test_closed_forms_on_the_gpu(path):
    # identical -> 1; prefix -> exp(1 - r/c); disjoint -> 0; clipping by max over references
    L = 40
    ref = np.arange(1, L + 1, dtype=np.int32)
    cands = [ref.copy(), ref[:25].copy(), ref + 1000, np.full(L, 7, np.int32)]
    refs = [[ref, ref], [ref, ref], [ref, ref],
            [np.r_[np.full(2, 7), ref[7:37]].astype(np.int32),
             np.r_[ref[7:27], np.full(3, 7)].astype(np.int32)]]
    B, R = len(cands), 2
    cand = np.zeros((B, 64), np.int32)
    refa = np.zeros((B, R, 64), np.int32)
    cl = np.zeros(B, np.int32)
    rl = np.zeros((B, R), np.int32)
    for i in range(B):
        cand[i, :len(cands[i])] = cands[i]
        cl[i] = len(cands[i])
        for j in range(R):
            refa[i, j, :len(refs[i][j])] = refs[i][j]
            rl[i, j] = len(refs[i][j])
    w = syn.Workload("closed", 2048, cand, cl, refa, rl)
    if not path_supported(w, path):
        pytest.skip("unsupported")
    out, st = run_gpu(Device(w), syn.Run("none"), path)
    assert abs(out[0] - 1.0) <= TOL
    assert abs(out[1] - np.exp(1 - 40 / 25)) <= TOL
    assert out[2] == 0.0
    clipped = st.clipped.cpu().numpy()
    assert list(clipped[3]) == [3, 2, 1, 0]      # max(2, 3) sevens, then 7-7 bigrams etc.
    assert out[3] == 0.0


@pytest.mark.parametrize("path", PATHS)
def test_pad_cells_and_other_sentences_do_not_matter(path):
    w = syn.random_small(120, B=24, R=2, vocab=30, max_len=90)
    if not path_supported(w, path):
        pytest.skip("unsupported")
    run = syn.Run("exp")
    base, st0 = run_gpu(Device(w), run, path)
    rng = np.random.default_rng(5)
    cand, refs = w.cand.copy(), w.refs.copy()
    cpad = np.arange(cand.shape[1])[None, :] >= w.cand_len[:, None]
    rpad = np.arange(refs.shape[2])[None, None, :] >= w.ref_len[:, :, None]
    cand[cpad] = rng.integers(0, 30, cpad.sum())
    refs[rpad] = rng.integers(0, 30, rpad.sum())
    w2 = syn.Workload("poisoned", w.vocab, cand, w.cand_len, refs, w.ref_len)
    out, st = run_gpu(Device(w2), run, path)
    np.testing.assert_array_equal(out, base)
    np.testing.assert_array_equal(st.clipped.cpu().numpy(), st0.clipped.cpu().numpy())
    # sentence 3 alone gives the same bits as sentence 3 inside the batch
    w3 = syn.Workload("alone", w.vocab, w.cand[3:4].copy(), w.cand_len[3:4].copy(),
                      w.refs[3:4].copy(), w.ref_len[3:4].copy())
    out3, _ = run_gpu(Device(w3), run, path)
    assert out3[0] == base[3]


@pytest.mark.parametrize("path", PATHS)
def test_device_status_reports_bad_tokens_and_lengths(path):
    w = syn.random_small(130, B=6, R=1, vocab=50, max_len=40, min_len=10)
    if not path_supported(w, path):
        pytest.skip("unsupported")
    w.cand[2, 3] = 50                       # == vocab_size: out of range, inside the length
    _, st = run_gpu(Device(w), syn.Run("none"), path)
    assert st.device_status.item() & tb.binding.TB_DEV_TOKEN_RANGE
    w = syn.random_small(130, B=6, R=1, vocab=50, max_len=40, min_len=10)
    w.cand_len[4] = 41                      # beyond the stride: clamped, flagged, no fault
    w.ref_len[1, 0] = -3
    _, st = run_gpu(Device(w), syn.Run("none"), path)
    assert st.device_status.item() & tb.binding.TB_DEV_LENGTH_RANGE


@pytest.mark.parametrize("max_len,min_len", [(4000, 3400), (9000, 8500)])
def test_device_status_on_partitioned_groups(max_len, min_len):
    # groups beyond one LDS table: a whole call extracts the n-grams inside the partitioned
    # kernels (the pack kernel does not run), which then also have to report bad tokens; the two
    # sizes take the scatter kernel for groups of at most 16 384 slots and the general one
    w = syn.random_small(131, B=2, R=3, vocab=300, max_len=max_len, min_len=min_len)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.path == 2 and lay.global_partitions > 0
    _, st = run_gpu(Device(w), syn.Run("none"), "auto")
    assert st.device_status.item() == 0
    w.refs[1, 2, int(w.ref_len[1, 2]) - 1] = 300   # == vocab_size, the last token inside a length
    _, st = run_gpu(Device(w), syn.Run("none"), "auto")
    assert st.device_status.item() & tb.binding.TB_DEV_TOKEN_RANGE
    w.refs[1, 2, int(w.ref_len[1, 2]) - 1] = 299
    w.refs[1, 2, int(w.ref_len[1, 2]):] = 300       # beyond the length: never looked at
    _, st = run_gpu(Device(w), syn.Run("none"), "auto")
    assert st.device_status.item() == 0


@pytest.mark.parametrize("path", PATHS)
def test_32_bit_keys_that_use_the_top_bit(path):
    # 18-bit token ids and 12 000 n-gram slots per group: keys (id of the prefix, last token) reach
    # 12 000 * 2^18 > 2^31, so the hash tables hold keys with the top bit set (still below the
    # all-ones empty marker); the GLOBAL path keeps its 32-bit-key kernels for this shape (the
    # fused plan does not fit: 32-bit staged tokens).  Tokens are drawn from the top of the id
    # range so that such keys do occur.
    w = syn.random_small(141, B=3, R=2, vocab=262144, max_len=4000, min_len=3600)
    rng = np.random.default_rng(141)
    hi = rng.integers(262144 - 40, 262144, size=w.cand.shape, dtype=np.int64)
    w.cand[:, 1::2] = hi[:, 1::2].astype(w.cand.dtype)
    w.refs[:, :, 1::2] = w.cand[:, None, 1::2]      # (equal strides) shared with the references
    cfg = tb.make_config(vocab_size=w.vocab, path="global")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.group_cap == 12000 and lay.global_candidate_first == 1 and lay.global_partitions == 0
    check(w, syn.Run("exp"), path)


def test_fused_keys_that_use_the_top_bit():
    # the same on the fused kernel, whose keys are (candidate position that made the prefix's
    # entry, last token): 20-bit token ids and a candidate of up to 4000 tokens reach 4000 * 2^20
    w = syn.random_small(142, B=4, R=1, vocab=1 << 20, max_len=4000, min_len=3700)
    rng = np.random.default_rng(142)
    hi = rng.integers((1 << 20) - 40, 1 << 20, size=w.cand.shape, dtype=np.int64)
    w.cand[:, 1::2] = hi[:, 1::2].astype(w.cand.dtype)
    w.refs[:, :, 1::2] = w.cand[:, None, 1::2]
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.fused_ok == 1 and lay.path == 1
    check(w, syn.Run("exp"), "fused")
    check(w, syn.Run("exp"), "global")


@pytest.mark.parametrize("seed,B,R,V,L", [(143, 9, 2, 300, 200), (144, 3, 1, 262144, 3000)])
def test_workspace_tables_on_shapes_that_fit_lds(seed, B, R, V, L):
    # cfg->workspace_tables: the kernels with tables in the workspace on shapes that would
    # otherwise take an LDS plan give the same statistics and scores
    w = syn.random_small(seed, B=B, R=R, vocab=V, max_len=L, min_len=L // 3)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp")
    cfg = tb.make_config(smoothing="exp", vocab_size=V, path="global", workspace_tables=True)
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_tables_in_hbm == 1 and lay.global_candidate_first == 0
    d = Device(w)
    st = tb.Stats.allocate(w.B, 4, DEV)
    out = tb.tensorbleu_sentence(d.cand, d.cand_len, d.refs, d.ref_len, cfg, stats=st)
    torch.cuda.synchronize()
    assert st.device_status.item() == 0
    np.testing.assert_array_equal(st.clipped.cpu().numpy(), ref.clipped)
    np.testing.assert_array_equal(st.total.cpu().numpy(), ref.total)
    np.testing.assert_array_equal(st.group_distinct.cpu().numpy(), ref.group_distinct)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref.bleu).max() <= TOL


@pytest.mark.parametrize("path", PATHS)
def test_largest_supported_group(path):
    # cand_stride + R * ref_stride = 12288 n-gram slots: the limit of both LDS plans
    w = syn.random_small(140, B=3, R=2, vocab=5000, max_len=4096, min_len=3000)
    check(w, syn.Run("exp"), path)


@pytest.mark.parametrize("path", PATHS)
def test_many_tiny_sentences_and_a_single_one(path):
    w = cached_small(141, B=70000, R=1, vocab=11, max_len=9)         # grid beyond 65535 groups
    check(w, syn.Run("floor", 0.1), path)
    w = syn.random_small(142, B=1, R=1, vocab=100, max_len=33, min_len=33)
    check(w, syn.Run("add-k", 1.0), path)


@pytest.mark.parametrize("path", PATHS)
def test_sixty_three_references(path):
    w = syn.random_small(143, B=2, R=63, vocab=40, max_len=90)
    check(w, syn.Run("none"), path)


@pytest.mark.parametrize("vocab", [50, 50257, 262144])
def test_group_too_large_for_one_lds_table(vocab):
    # cand_stride + R * ref_stride = 16400 > 12288: neither single-table LDS plan applies.  With
    # The dictionary is split over eight workgroups per (group, order); the 72-bit 4-grams of the
    # largest vocabulary are keyed there by (id of the 3-gram prefix, last token).
    w = cached_small(144, B=3, R=3, vocab=vocab, max_len=4100, min_len=3500)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.fused_ok == 0 and lay.global_ok == 1 and lay.path == 2
    assert lay.global_tables_in_hbm == 0 and lay.global_partitions == 8
    assert lay.id_stride == 8 * 6144
    d = Device(w)
    for run in (syn.Run("exp"), syn.Run("add-k", 1.0)):
        check(w, run, "auto", d=d)


@pytest.mark.parametrize("vocab", [50, 262144])
def test_partitioned_group_of_at_most_16384_slots(vocab):
    # 12 288 < group_cap <= 16 384: four partitions, and the scatter kernel that keeps a group's
    # keys in registers (with the largest vocabulary also for the derived keys of the 4-grams)
    w = cached_small(155, B=3, R=3, vocab=vocab, max_len=4000, min_len=3400)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.path == 2 and lay.global_partitions == 4 and lay.group_cap <= 16384
    check(w, syn.Run("exp"), "auto")


def test_long_form_sequences_of_300k_tokens():
    # two groups of ~600 000 tokens each (a candidate and one reference of up to 300 000): 256
    # partitions, and with a 3-token vocabulary single n-gram counts far beyond 16 bits
    w = cached_small(145, B=2, R=1, vocab=3, max_len=300000, min_len=250000)
    assert np.bincount(w.cand[0, :w.cand_len[0]]).max() > 65535
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 256 and lay.global_tables_in_hbm == 0
    check(w, syn.Run("exp"), "auto")
    w = cached_small(146, B=2, R=1, vocab=50257, max_len=300000, min_len=250000)
    check(w, syn.Run("add-k", 1.0), "global")


def test_groups_beyond_the_partitioned_kernels_use_tables_in_the_workspace():
    # a candidate and a reference of ~1.1 million tokens: more than 2 097 152 slots per group
    w = cached_small(156, B=1, R=1, vocab=50257, max_len=1100000, min_len=1060000)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 0 and lay.global_tables_in_hbm == 1
    check(w, syn.Run("exp"), "auto")
    # just below: 512 partitions
    w = cached_small(157, B=1, R=1, vocab=1000, max_len=1040000, min_len=1000000)
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 512 and lay.global_tables_in_hbm == 0
    check(w, syn.Run("floor", 0.1), "auto")


def test_sixty_four_partitions():
    # groups of ~150 000 slots: 64 workgroups per (group, order); the second case has 72-bit
    # 4-grams, keyed by (id of the 3-gram prefix, last token)
    w = cached_small(147, B=2, R=3, vocab=3000, max_len=40000, min_len=35000)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 64 and lay.global_tables_in_hbm == 0
    check(w, syn.Run("exp"), "auto")
    w = cached_small(148, B=1, R=2, vocab=200000, max_len=50000, min_len=45000)
    check(w, syn.Run("add-k", 1.0), "auto")


def test_partitions_with_sequences_beyond_65535_tokens():
    # 32-bit counters in the partitioned count kernel: with three tokens in the vocabulary single
    # n-grams occur more than 65 535 times in a sequence of 100 000
    w = cached_small(149, B=2, R=1, vocab=3, max_len=100000, min_len=90000)
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 64 and lay.global_tables_in_hbm == 0
    assert np.bincount(w.cand[0, :w.cand_len[0]]).max() > 20000
    check(w, syn.Run("exp"), "auto")
    w = cached_small(150, B=1, R=2, vocab=50257, max_len=70000, min_len=66000)
    check(w, syn.Run("floor", 0.1), "auto")


def test_partitions_with_more_references_than_counter_fields():
    # more than 11 references (5 with 32-bit counters): the partitioned count kernel takes the
    # references in passes of 10 (4) and keeps a running maximum per dictionary entry
    for seed, B, R, V, L, P in [(151, 2, 16, 1000, 1024, 8), (152, 1, 30, 50, 600, 8),
                                (153, 1, 6, 5, 70000, 128)]:
        w = cached_small(seed, B=B, R=R, vocab=V, max_len=L, min_len=L * 4 // 5)
        cfg = tb.make_config(vocab_size=w.vocab, path="auto")
        lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
        assert lay.global_partitions == P and lay.global_tables_in_hbm == 0
        check(w, syn.Run("exp"), "auto")


def test_long_texts_with_skewed_token_frequencies():
    # Zipf-distributed tokens: the most frequent token makes up a seventh of a text, so its
    # unigram's partition holds several times the expected members (the crowded-partition code)
    w = syn.long_form(B=2, L=60000)
    group = np.concatenate([w.cand[0, :w.cand_len[0]], w.refs[0, 0, :w.ref_len[0, 0]]])
    assert np.bincount(group).max() > 2 * 4096
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.global_partitions == 32
    check(w, syn.Run("exp"), "auto")
    check(w, syn.Run("add-k", 1.0), "global")


def test_long_form_workload_at_full_size():
    """The long-generation workload bench.py --long-form times (128 groups of ~16 000 tokens, four
    partitions per group and order), every sentence against the oracle."""
    w = syn.long_form()
    cfg = tb.make_config(vocab_size=w.vocab, path="auto")
    lay = tb.tensorbleu_workspace_layout(w.B, w.R, w.cand.shape[1], w.refs.shape[2], cfg)
    assert lay.path == 2 and lay.global_partitions == 4
    check(w, syn.Run("exp"), "auto")


def test_determinism_of_integer_statistics():
    w = syn.make(1)
    d = Device(w)
    a, sa = run_gpu(d, syn.Run("exp"), "global")
    b, sb = run_gpu(d, syn.Run("exp"), "global")
    np.testing.assert_array_equal(a, b)
    np.testing.assert_array_equal(sa.clipped.cpu().numpy(), sb.clipped.cpu().numpy())


def test_paths_agree_bit_for_bit():
    w = syn.config3(B=32)
    if not (path_supported(w, "fused") and path_supported(w, "global")):
        pytest.skip("needs both paths")
    d = Device(w)
    a, sa = run_gpu(d, syn.Run("exp"), "global")
    b, sb = run_gpu(d, syn.Run("exp"), "fused")
    np.testing.assert_array_equal(sa.clipped.cpu().numpy(), sb.clipped.cpu().numpy())
    np.testing.assert_array_equal(sa.total.cpu().numpy(), sb.total.cpu().numpy())
    np.testing.assert_array_equal(a, b)


# ------------------------------------------------------------------- full-size configurations

@pytest.mark.parametrize("path", PATHS + ["auto"])
@pytest.mark.parametrize("config", [2, 3, 4, 5])
def test_full_size_configs(config, path):
    w = syn.make(config)
    d = Device(w)
    for run in w.runs:
        if run.corpus:
            continue                        # check() always covers the corpus variant too
        check(w, run, path, d=d)


# ------------------------------------------------- per-candidate reference counts (ragged R)

def _ragged_case(seed, B, R, V, L):
    """A batch whose candidates use 1..R references; the unused rows are filled with copies of
    the candidate (and its length), which would change every statistic if they were read."""
    w = cached_small(seed, B=B, R=R, vocab=V, max_len=L)
    rc = syn.ref_counts(seed, B, R)
    refs, ref_len = w.refs.copy(), w.ref_len.copy()
    for i in range(B):
        m = min(w.cand.shape[1], refs.shape[2])
        refs[i, rc[i]:, :m] = w.cand[i, :m]
        ref_len[i, rc[i]:] = min(int(w.cand_len[i]), m)
    return w, rc, refs, ref_len


@pytest.mark.parametrize("path", PATHS)
@pytest.mark.parametrize("seed,B,R,V,L", [
    (201, 37, 4, 11, 60),          # LDS kernels, one field per sequence
    (202, 6, 3, 262144, 700),      # 128-bit keys
    (203, 5, 40, 300, 120),        # many references (pair-phase count kernel on the global path)
    (204, 3, 2, 50, 9000),         # group beyond one LDS table: partitioned kernels
    (205, 3, 14, 300, 1000),       # the same with the references counted in two passes
])
def test_ragged_reference_counts(path, seed, B, R, V, L):
    w, rc, refs, ref_len = _ragged_case(seed, B, R, V, L)
    if not path_supported(w, path):
        pytest.skip(f"{path} path does not support this shape")
    cand, cand_len = dev(w.cand), dev(w.cand_len)
    drefs, dref_len, drc = dev(refs), dev(ref_len), dev(rc)
    for run in ALL_MODES:
        ref = oracle.bleu(w.cand, w.cand_len, refs, ref_len, smoothing=run.smoothing,
                          smooth_param=run.smooth_param, ref_count=rc, threads=8)
        cfg = tb.make_config(smoothing=run.smoothing, smooth_param=run.smooth_param,
                             vocab_size=w.vocab, path=path, ref_count=drc)
        for corpus in (False, True):
            stats = tb.Stats.allocate(w.B, 4, DEV)
            fn = tb.tensorbleu_corpus if corpus else tb.tensorbleu_sentence
            out = fn(cand, cand_len, drefs, dref_len, cfg, stats=stats).cpu().numpy()
            assert stats.device_status.item() == 0
            np.testing.assert_array_equal(stats.clipped.cpu().numpy(), ref.clipped)
            np.testing.assert_array_equal(stats.total.cpu().numpy(), ref.total)
            np.testing.assert_array_equal(stats.closest_ref_len.cpu().numpy(), ref.closest_ref_len)
            if corpus:
                np.testing.assert_array_equal(stats.corpus_stats.cpu().numpy(), ref.corpus_stats)
                assert abs(float(out[0]) - ref.corpus_bleu) <= TOL
            else:
                assert np.abs(out.astype(np.float64) - ref.bleu).max() <= TOL


@pytest.mark.parametrize("path", PATHS)
def test_reference_count_out_of_range_is_clamped_and_flagged(path):
    w = cached_small(205, B=8, R=3, vocab=20, max_len=30)
    rc = np.array([1, 2, 3, 0, 7, -4, 3, 1], np.int32)       # 0 and -4 -> 1, 7 -> 3
    clamped = np.clip(rc, 1, 3).astype(np.int32)
    cfg = tb.make_config(vocab_size=w.vocab, path=path, ref_count=dev(rc))
    stats = tb.Stats.allocate(w.B, 4, DEV)
    out = tb.tensorbleu_sentence(dev(w.cand), dev(w.cand_len), dev(w.refs), dev(w.ref_len), cfg,
                                 stats=stats).cpu().numpy()
    assert stats.device_status.item() & tb.TB_DEV_LENGTH_RANGE
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, ref_count=clamped)
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), ref.clipped)
    assert np.abs(out.astype(np.float64) - ref.bleu).max() <= TOL


# ------------------------------------------------------------------- more than four orders

@pytest.mark.parametrize("N", [5, 6, 8])
@pytest.mark.parametrize("seed,B,R,V,L", [
    (301, 24, 2, 5, 40),           # tiny vocabulary: long n-grams still repeat
    (302, 6, 3, 50257, 600),
    (303, 4, 1, 262144, 1200),     # packed 8-grams would need 144 bits; hierarchical keys do not
])
def test_more_than_four_orders(N, seed, B, R, V, L):
    w = cached_small(seed, B=B, R=R, vocab=V, max_len=L)
    d = Device(w)
    weights = [1.0 / N] * N
    for run in ALL_MODES:
        check(w, run, "auto", max_n=N, weights=weights, d=d)
    bits = max(1, (V - 1).bit_length())
    if N * bits <= 128:                # the GLOBAL path packs the whole n-gram into a key
        for run in ALL_MODES:
            check(w, run, "global", max_n=N, weights=weights, d=d)
    else:
        cfg = tb.make_config(max_n=N, vocab_size=w.vocab, path="global")
        with pytest.raises(tb.TensorBLEUError):
            tb.tensorbleu_sentence(d.cand, d.cand_len, d.refs, d.ref_len, cfg)


@pytest.mark.parametrize("N", [5, 7, 8])
def test_more_than_four_orders_on_the_global_path_large_and_tiny_groups(N):
    w = cached_small(304, B=3, R=2, vocab=65536, max_len=1500)        # 16-byte keys from n = 5
    check(w, syn.Run("exp"), "global", max_n=N, weights=[1.0 / N] * N)
    w = cached_small(305, B=2, R=1, vocab=4, max_len=9000)            # partitioned LDS tables
    check(w, syn.Run("floor", 0.1), "global", max_n=N, weights=[1.0 / N] * N)
    # partitioned tables where every order from 3 (93 bits) to 4 needs 16-byte packed keys and is
    # keyed by (id of its prefix, last token) instead, each on the ids of the order below
    w = cached_small(307, B=2, R=2, vocab=2 ** 31 - 1, max_len=5000, min_len=4000)
    check(w, syn.Run("exp"), "global", max_n=min(N, 4), weights=[1.0 / min(N, 4)] * min(N, 4))
    w = cached_small(308, B=2, R=1, vocab=60000, max_len=8000, min_len=7000)   # 16 bits: wide from 5
    check(w, syn.Run("exp"), "global", max_n=N, weights=[1.0 / N] * N)
    w = cached_small(306, B=600, R=1, vocab=200, max_len=40)          # many groups: paired orders
    check(w, syn.Run("none"), "global", max_n=N, weights=[1.0 / N] * N)


def test_more_than_63_references_use_the_loop_fallback_of_the_group_index():
    """With 64 or more sequences per group the wave-wide length scan no longer applies: the
    GLOBAL kernels fall back to loops over the lengths (FUSED does not take such shapes)."""
    w = cached_small(401, B=3, R=70, vocab=30, max_len=25)
    assert not path_supported(w, "fused")
    d = Device(w)
    for run in ALL_MODES:
        check(w, run, "global", d=d)
    check(w, syn.Run("exp"), "auto", d=d)
    rc = syn.ref_counts(401, w.B, w.R)
    ref = oracle.bleu(w.cand, w.cand_len, w.refs, w.ref_len, smoothing="exp", ref_count=rc)
    cfg = tb.make_config(smoothing="exp", vocab_size=w.vocab, path="global", ref_count=dev(rc))
    stats = tb.Stats.allocate(w.B, 4, DEV)
    out = tb.tensorbleu_sentence(d.cand, d.cand_len, d.refs, d.ref_len, cfg, stats=stats)
    np.testing.assert_array_equal(stats.clipped.cpu().numpy(), ref.clipped)
    np.testing.assert_array_equal(stats.closest_ref_len.cpu().numpy(), ref.closest_ref_len)
    assert np.abs(out.cpu().numpy().astype(np.float64) - ref.bleu).max() <= TOL
