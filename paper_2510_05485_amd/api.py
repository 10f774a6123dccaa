"""Convenience layer over the C-ABI binding for PyTorch callers (e.g. an RL reward function).

Nothing is computed here: the functions build the config struct, allocate (or reuse) output and
workspace tensors, and call `tensorbleu_sentence` / `tensorbleu_corpus`.  Token-ID tensors may be
int32 or int64 (the usual tokenizer dtype); lengths are int32.  Everything lives on the GPU and
runs on the current stream without synchronising.
"""
from __future__ import annotations

from typing import Optional, Sequence

import torch

from . import binding as _b


def _refs3d(references) -> torch.Tensor:
    if isinstance(references, (list, tuple)):
        return torch.stack(list(references), dim=1)     # R tensors [B, L] -> [B, R, L]
    return references if references.dim() == 3 else references.unsqueeze(1)


def _len32(t: torch.Tensor) -> torch.Tensor:
    return t if t.dtype == torch.int32 else t.to(torch.int32)


class BleuScorer:
    """Per-sentence / corpus token-ID BLEU for one batch shape, with buffers allocated once.

    scorer = BleuScorer(B, R, cand_stride, ref_stride, vocab_size=50257, smoothing="exp")
    reward = scorer(cand, cand_len, refs, ref_len)          # float32 [B], on the GPU

    score_dtype=torch.bfloat16 stores the scores as bfloat16 (the fp32 score rounded to nearest
    even) for consumers that keep rewards in that type.

    Conditions that only the kernels can see (a token id outside [0, vocab_size), a clamped
    length or reference count, an overflowing table partition) are OR-ed into
    `scorer.device_status` (int32 [1] on the GPU) by every call and make the scores of the rows
    concerned unspecified; `scorer.check()` synchronises, raises if any bit is set and clears
    them.  Poll it where a silent wrong reward would hurt (a mis-set vocab_size is enough).
    """

    def __init__(self, B: int, R: int, cand_stride: int, ref_stride: int, *, vocab_size: int,
                 max_n: int = 4, weights: Optional[Sequence[float]] = None,
                 smoothing: str = "none", smooth_param: float = 0.0, path: str = "auto",
                 device="cuda:0", want_stats: bool = False,
                 score_dtype: torch.dtype = torch.float32):
        self.shape = (int(B), int(R), int(cand_stride), int(ref_stride))
        self.cfg = _b.make_config(max_n=max_n, weights=weights, smoothing=smoothing,
                                  smooth_param=smooth_param, vocab_size=vocab_size, path=path,
                                  score_dtype=score_dtype)
        self.workspace = _b.allocate_workspace(B, R, cand_stride, ref_stride, self.cfg, device)
        self.out = torch.empty(B, dtype=score_dtype, device=device)
        self.corpus_out = torch.zeros(1, dtype=score_dtype, device=device)
        self.stats = (_b.Stats.allocate(B, max_n, device) if want_stats else
                      _b.Stats(device_status=torch.zeros(1, dtype=torch.int32, device=device)))
        self.device_status = self.stats.device_status

    def check(self) -> None:
        """Synchronise, raise TensorBLEUError if a kernel reported a condition since the last
        check, and clear the status word."""
        bits = int(self.device_status.item())
        if bits:
            self.device_status.zero_()
            names = [n for n, b in (("token id out of range", _b.TB_DEV_TOKEN_RANGE),
                                    ("length or reference count clamped", _b.TB_DEV_LENGTH_RANGE),
                                    ("table partition overflow", _b.TB_DEV_TABLE_OVERFLOW))
                     if bits & b]
            raise _b.TensorBLEUError("device status " + str(bits) + ": " + ", ".join(names))

    def _check(self, cand, refs):
        B, R, cs, rs = self.shape
        if tuple(cand.shape) != (B, cs) or tuple(refs.shape) != (B, R, rs):
            raise _b.TensorBLEUError(f"scorer was built for cand {(B, cs)} / refs {(B, R, rs)}, "
                                     f"got {tuple(cand.shape)} / {tuple(refs.shape)}")

    def _set_ref_count(self, ref_count):
        """ref_count: int32/int64 device tensor [B] (candidate i uses its first ref_count[i]
        references) or None (all R)."""
        if ref_count is None:
            self.cfg.ref_count = None
            self._ref_count = None
            return
        t = _len32(ref_count).contiguous()
        if tuple(t.shape) != (self.shape[0],) or not t.is_cuda:
            raise _b.TensorBLEUError("ref_count must be a device tensor of shape [B]")
        self._ref_count = t                    # keeps the memory alive for the call
        self.cfg.ref_count = t.data_ptr()

    def __call__(self, cand, cand_len, refs, ref_len, ref_count=None) -> torch.Tensor:
        refs = _refs3d(refs)
        self._check(cand, refs)
        self._set_ref_count(ref_count)
        return _b.tensorbleu_sentence(cand, _len32(cand_len), refs, _len32(ref_len), self.cfg,
                                      out=self.out, stats=self.stats, workspace=self.workspace)

    def corpus(self, cand, cand_len, refs, ref_len, ref_count=None) -> torch.Tensor:
        refs = _refs3d(refs)
        self._check(cand, refs)
        self._set_ref_count(ref_count)
        return _b.tensorbleu_corpus(cand, _len32(cand_len), refs, _len32(ref_len), self.cfg,
                                    out=self.corpus_out, stats=self.stats,
                                    workspace=self.workspace)


def sentence_bleu(cand, cand_len, refs, ref_len, *, vocab_size: int, **kw) -> torch.Tensor:
    """One-shot per-sentence BLEU (allocates its buffers; use BleuScorer inside a loop)."""
    refs = _refs3d(refs)
    s = BleuScorer(cand.shape[0], refs.shape[1], cand.shape[1], refs.shape[2],
                   vocab_size=vocab_size, device=cand.device, **kw)
    return s(cand, cand_len, refs, ref_len).clone()


def corpus_bleu(cand, cand_len, refs, ref_len, *, vocab_size: int, **kw) -> torch.Tensor:
    """One-shot corpus-level BLEU over the batch."""
    refs = _refs3d(refs)
    s = BleuScorer(cand.shape[0], refs.shape[1], cand.shape[1], refs.shape[2],
                   vocab_size=vocab_size, device=cand.device, **kw)
    return s.corpus(cand, cand_len, refs, ref_len).clone()


def rouge_n(cand, cand_len, refs, ref_len, *, n: int = 2, beta: float = 1.0, vocab_size: int,
            ref_count=None, score_dtype: torch.dtype = torch.float32) -> torch.Tensor:
    """ROUGE-N precision, recall and F (float32 or bfloat16 [B, 3]) of every candidate against the best of
    its references; runs `tensorrouge_n` on the current stream."""
    refs = _refs3d(refs)
    rc = None if ref_count is None else _len32(ref_count).contiguous()
    return _b.tensorrouge_n(cand, _len32(cand_len), refs, _len32(ref_len), n=n, beta=beta,
                            vocab_size=vocab_size, ref_count=rc, score_dtype=score_dtype)


def pack_reference_lists(references, device="cuda:0", dtype=torch.int32):
    """Lay out a ragged list of references in CSR form (tb_config_t.ref_offsets): no padding rows.

    `references[i]` is the list of reference token sequences of candidate i.  Returns (rows
    [total, L], row_len [total] int32, ref_offsets [B + 1] int32, max_refs) with the tensors on
    `device`; pass them as make_config(ref_offsets=..., max_refs=...) and as `refs` / `ref_len`.
    Host-side convenience: builds the arrays on the CPU and copies them once."""
    flat = [seq for group in references for seq in group]
    L = max(1, max((len(s) for s in flat), default=1))
    rows = torch.zeros(max(len(flat), 1), L, dtype=dtype)
    row_len = torch.zeros(max(len(flat), 1), dtype=torch.int32)
    for r, seq in enumerate(flat):
        t = torch.as_tensor(seq, dtype=dtype)
        rows[r, :t.numel()] = t
        row_len[r] = t.numel()
    offsets = torch.zeros(len(references) + 1, dtype=torch.int32)
    offsets[1:] = torch.cumsum(torch.tensor([len(g) for g in references], dtype=torch.int32), 0)
    return (rows[:len(flat)].to(device), row_len[:len(flat)].to(device), offsets.to(device),
            max((len(g) for g in references), default=1))


def lengths_from_padding(tokens: torch.Tensor, pad_id: int) -> torch.Tensor:
    """int32 lengths of right-padded rows: the number of cells before the trailing run of
    `pad_id` (a pad-valued token inside the sentence is kept).  Plain torch on the tensor's device;
    for callers that hold (batch, seq_len) tensors without a length array."""
    keep = tokens != pad_id
    L = tokens.shape[-1]
    pos = torch.arange(1, L + 1, device=tokens.device, dtype=torch.int32)
    return (keep.to(torch.int32) * pos).amax(dim=-1).to(torch.int32)


def pad_references(references, device="cuda:0", dtype=torch.int32):
    """Lay out a ragged list of references for the fixed-R interface.

    `references[i]` is the list of reference token sequences (lists or 1-D tensors) of candidate
    i; candidates may have different numbers of references (at least one each).  Returns
    (refs [B, R, L], ref_len [B, R] int32, ref_count [B] int32) on `device`, with R the largest
    number of references and L the longest one; pass ref_count on to the scorer.  Host-side
    convenience: builds the arrays on the CPU and copies them once."""
    B = len(references)
    if B == 0 or any(len(r) == 0 for r in references):
        raise _b.TensorBLEUError("every candidate needs at least one reference")
    R = max(len(r) for r in references)
    L = max(1, max(len(s) for r in references for s in r))
    refs = torch.zeros(B, R, L, dtype=dtype)
    ref_len = torch.zeros(B, R, dtype=torch.int32)
    ref_count = torch.empty(B, dtype=torch.int32)
    for i, group in enumerate(references):
        ref_count[i] = len(group)
        for j, seq in enumerate(group):
            t = torch.as_tensor(seq, dtype=dtype)
            refs[i, j, :t.numel()] = t
            ref_len[i, j] = t.numel()
    return refs.to(device), ref_len.to(device), ref_count.to(device)
