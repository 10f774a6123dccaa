"""ctypes binding of libtensorbleu.so: argument marshalling only.

Every function here has the name of the C entry point it calls (see include/tensorbleu.h).
PyTorch supplies device memory and the current HIP stream; every step of the computation runs
in the library's kernels.  There is no CPU fallback: if the library is missing or no GPU is
present the calls raise.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtensorbleu.so")

TB_OK = 0
SMOOTHING = {"none": 0, "floor": 1, "add-k": 2, "exp": 3}
PATHS = {"auto": 0, "fused": 1, "global": 2}
TB_DEV_TOKEN_RANGE, TB_DEV_LENGTH_RANGE, TB_DEV_TABLE_OVERFLOW = 1, 2, 4

EXPORTS = [
    "tensorbleu_workspace_bytes", "tensorbleu_workspace_layout", "tensorbleu_sentence",
    "tensorbleu_corpus", "tensorbleu_pack", "tensorbleu_dictionary", "tensorbleu_count_clip",
    "tensorbleu_finalize", "tensorbleu_status_string", "tensorrouge_n",
    "tensorbleu_sentence_static", "tensorbleu_static_scratch_bytes",
]


class tb_config_t(ctypes.Structure):
    _fields_ = [("max_n", ctypes.c_int32), ("weights", ctypes.c_float * 8),
                ("smoothing", ctypes.c_int32), ("smooth_param", ctypes.c_float),
                ("vocab_size", ctypes.c_int32), ("force_path", ctypes.c_int32),
                ("token_bytes", ctypes.c_int32), ("score_bytes", ctypes.c_int32),
                ("ref_count", ctypes.c_void_p), ("ref_offsets", ctypes.c_void_p),
                ("ref_rows", ctypes.c_int64), ("workspace_tables", ctypes.c_int32)]


class tb_stats_t(ctypes.Structure):
    _fields_ = [("clipped", ctypes.c_void_p), ("total", ctypes.c_void_p),
                ("closest_ref_len", ctypes.c_void_p), ("group_distinct", ctypes.c_void_p),
                ("corpus_stats", ctypes.c_void_p), ("device_status", ctypes.c_void_p)]


class tb_layout_t(ctypes.Structure):
    _fields_ = [("path", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("key_bytes", ctypes.c_int32 * 8), ("group_cap", ctypes.c_int64),
                ("keys_off", ctypes.c_size_t * 8), ("inv_off", ctypes.c_size_t * 8),
                ("clipped_off", ctypes.c_size_t), ("total_off", ctypes.c_size_t),
                ("closest_off", ctypes.c_size_t), ("distinct_off", ctypes.c_size_t),
                ("cand_distinct_off", ctypes.c_size_t),
                ("corpus_off", ctypes.c_size_t), ("overlap_off", ctypes.c_size_t),
                ("bytes", ctypes.c_size_t),
                ("fused_ok", ctypes.c_int32), ("global_ok", ctypes.c_int32),
                ("global_tables_in_hbm", ctypes.c_int32), ("tables_off", ctypes.c_size_t),
                ("id_stride", ctypes.c_int64), ("global_candidate_first", ctypes.c_int32),
                ("global_partitions", ctypes.c_int32)]


class TensorBLEUError(RuntimeError):
    pass


_lib = None


def load_library() -> ctypes.CDLL:
    """Load the in-tree shared library (raises if it has not been built)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise TensorBLEUError(
            f"{LIB_PATH} is missing: run `python -m paper_2510_05485_amd.build` first")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64, ctypes.c_size_t
    cfgp, stp = ctypes.POINTER(tb_config_t), ctypes.POINTER(tb_stats_t)
    lib.tensorbleu_workspace_bytes.restype = sz
    lib.tensorbleu_workspace_bytes.argtypes = [i32, i32, i64, i64, cfgp]
    lib.tensorbleu_workspace_layout.restype = ctypes.c_int
    lib.tensorbleu_workspace_layout.argtypes = [i32, i32, i64, i64, cfgp,
                                                ctypes.POINTER(tb_layout_t)]
    full = [vp, i64, vp, vp, i64, vp, i32, i32, cfgp, vp, stp, vp, sz, vp]
    lib.tensorbleu_sentence.restype = ctypes.c_int
    lib.tensorbleu_sentence.argtypes = full
    lib.tensorbleu_corpus.restype = ctypes.c_int
    lib.tensorbleu_corpus.argtypes = full
    lib.tensorbleu_sentence_static.restype = ctypes.c_int
    lib.tensorbleu_sentence_static.argtypes = [vp, i64, vp, vp, i64, vp, i32, i32, cfgp, vp, stp, vp]
    lib.tensorbleu_static_scratch_bytes.restype = sz
    lib.tensorbleu_static_scratch_bytes.argtypes = []
    lib.tensorrouge_n.restype = ctypes.c_int
    lib.tensorrouge_n.argtypes = [vp, i64, vp, vp, i64, vp, i32, i32, cfgp, vp, vp, vp, stp, vp, sz, vp]
    lib.tensorbleu_pack.restype = ctypes.c_int
    lib.tensorbleu_pack.argtypes = [vp, i64, vp, vp, i64, vp, i32, i32, cfgp, stp, vp, sz, vp]
    stage = [vp, vp, i64, i64, i32, i32, cfgp, stp, vp, sz, vp]
    lib.tensorbleu_dictionary.restype = ctypes.c_int
    lib.tensorbleu_dictionary.argtypes = stage
    lib.tensorbleu_count_clip.restype = ctypes.c_int
    lib.tensorbleu_count_clip.argtypes = stage
    lib.tensorbleu_finalize.restype = ctypes.c_int
    lib.tensorbleu_finalize.argtypes = [vp, vp, i32, i32, i64, i64, cfgp, i32, vp, stp, vp, sz, vp]
    lib.tensorbleu_status_string.restype = ctypes.c_char_p
    lib.tensorbleu_status_string.argtypes = [ctypes.c_int]
    _lib = lib
    return lib


def tensorbleu_status_string(status: int) -> str:
    return load_library().tensorbleu_status_string(int(status)).decode()


def _check(rc: int, what: str) -> None:
    if rc != TB_OK:
        raise TensorBLEUError(f"{what}: {tensorbleu_status_string(rc)} (status {rc})")


def make_config(max_n: int = 4, weights: Optional[Sequence[float]] = None,
                smoothing: str = "none", smooth_param: float = 0.0, vocab_size: int = 1 << 16,
                path: str = "auto", ref_count: Optional[torch.Tensor] = None,
                score_dtype: torch.dtype = torch.float32,
                ref_offsets: Optional[torch.Tensor] = None, max_refs: int = 0,
                workspace_tables: bool = False) -> tb_config_t:
    """ref_count: optional int32 device tensor [B]; candidate i is scored against its first
    ref_count[i] references only.  The config keeps the tensor alive.
    ref_offsets: optional int32 device tensor [B + 1]: reference lists in CSR form (`refs` is then
    [rows, Lr] and `ref_len` [rows]; candidate i owns rows ref_offsets[i] .. ref_offsets[i+1]-1);
    max_refs is the largest number of references of any candidate.
    score_dtype: torch.float32, or torch.bfloat16 for scores stored as bfloat16.
    workspace_tables: the GLOBAL path with its hash tables in the workspace whatever the shape
    (slower; no table can overflow: for re-issuing a call that reported TB_DEV_TABLE_OVERFLOW)."""
    if score_dtype not in (torch.float32, torch.bfloat16):
        raise TensorBLEUError(f"score_dtype must be float32 or bfloat16 (got {score_dtype})")
    cfg = tb_config_t()
    cfg.max_n = int(max_n)
    w = [0.0] * 8
    if weights is not None:
        for n, x in enumerate(list(weights)[:8]):
            w[n] = float(x)
    cfg.weights = (ctypes.c_float * 8)(*w)
    cfg.smoothing = SMOOTHING[smoothing] if isinstance(smoothing, str) else int(smoothing)
    cfg.smooth_param = float(smooth_param)
    cfg.vocab_size = int(vocab_size)
    cfg.force_path = PATHS[path] if isinstance(path, str) else int(path)
    cfg.token_bytes = 4
    cfg.score_bytes = 2 if score_dtype == torch.bfloat16 else 4
    cfg.workspace_tables = 1 if workspace_tables else 0
    cfg.ref_count = None
    if ref_count is not None:
        if ref_count.dtype != torch.int32 or not ref_count.is_contiguous() or ref_count.dim() != 1:
            raise TensorBLEUError("ref_count must be a contiguous int32 tensor of shape [B]")
        cfg.ref_count = ref_count.data_ptr()
        cfg._ref_count_tensor = ref_count      # keeps the device memory alive with the config
    cfg.ref_offsets = None
    cfg.ref_rows = 0
    cfg._max_refs = 0
    if ref_offsets is not None:
        if ref_offsets.dtype != torch.int32 or not ref_offsets.is_contiguous() or \
                ref_offsets.dim() != 1 or max_refs < 1 or ref_count is not None:
            raise TensorBLEUError("ref_offsets must be a contiguous int32 tensor of shape [B + 1], "
                                  "given with max_refs >= 1 and without ref_count")
        cfg.ref_offsets = ref_offsets.data_ptr()
        cfg._ref_offsets_tensor = ref_offsets
        cfg._max_refs = int(max_refs)
    return cfg


@dataclass
class Stats:
    """Device tensors behind a tb_stats_t (allocated by `Stats.allocate`); None = not wanted."""
    clipped: Optional[torch.Tensor] = None
    total: Optional[torch.Tensor] = None
    closest_ref_len: Optional[torch.Tensor] = None
    group_distinct: Optional[torch.Tensor] = None
    corpus_stats: Optional[torch.Tensor] = None
    device_status: Optional[torch.Tensor] = None

    @staticmethod
    def allocate(B: int, N: int, device, corpus_stats: bool = True) -> "Stats":
        z = lambda *s, dt=torch.int32: torch.zeros(*s, dtype=dt, device=device)
        return Stats(z(B, N), z(B, N), z(B), z(B, N),
                     z(2 * N + 2, dt=torch.int64) if corpus_stats else None, z(1))

    def as_struct(self) -> tb_stats_t:
        ptr = lambda t: t.data_ptr() if t is not None else None
        s = tb_stats_t()
        s.clipped = ptr(self.clipped)
        s.total = ptr(self.total)
        s.closest_ref_len = ptr(self.closest_ref_len)
        s.group_distinct = ptr(self.group_distinct)
        s.corpus_stats = ptr(self.corpus_stats)
        s.device_status = ptr(self.device_status)
        return s


@dataclass
class _Batch:
    cand: torch.Tensor
    cand_len: torch.Tensor
    refs: torch.Tensor
    ref_len: torch.Tensor
    B: int
    R: int
    cand_stride: int
    ref_stride: int


def _batch(cand, cand_len, refs, ref_len, cfg: Optional[tb_config_t] = None) -> _Batch:
    for t, name in ((cand, "cand"), (cand_len, "cand_len"), (refs, "refs"), (ref_len, "ref_len")):
        if not t.is_cuda:
            raise TensorBLEUError(f"{name} must live on the GPU (got {t.device})")
    for t, name in ((cand_len, "cand_len"), (ref_len, "ref_len")):
        if t.dtype != torch.int32:
            raise TensorBLEUError(f"{name} must be int32 (got {t.dtype})")
    if cand.dtype not in (torch.int32, torch.int64) or refs.dtype != cand.dtype:
        raise TensorBLEUError("cand and refs must both be int32 or both int64 "
                              f"(got {cand.dtype}, {refs.dtype})")
    if cfg is not None:
        cfg.token_bytes = 8 if cand.dtype == torch.int64 else 4
    if cfg is not None and cfg.ref_offsets:           # CSR reference lists
        if cand.dim() != 2 or refs.dim() != 2 or tuple(ref_len.shape) != (refs.shape[0],):
            raise TensorBLEUError("with ref_offsets: expected cand [B, Lc], refs [rows, Lr] and "
                                  "ref_len [rows]")
        B = int(cand.shape[0])
        if tuple(cand_len.shape) != (B,) or cfg._ref_offsets_tensor.numel() != B + 1:
            raise TensorBLEUError("expected cand_len [B] and ref_offsets [B + 1]")
        cfg.ref_rows = int(refs.shape[0])
        return _Batch(cand.contiguous(), cand_len.contiguous(), refs.contiguous(),
                      ref_len.contiguous(), B, cfg._max_refs, int(cand.shape[1]),
                      int(refs.shape[1]))
    if cand.dim() != 2 or refs.dim() != 3 or refs.shape[0] != cand.shape[0]:
        raise TensorBLEUError("expected cand [B, Lc] and refs [B, R, Lr]")
    B, R = int(cand.shape[0]), int(refs.shape[1])
    if tuple(cand_len.shape) != (B,) or tuple(ref_len.shape) != (B, R):
        raise TensorBLEUError("expected cand_len [B] and ref_len [B, R]")
    cand, refs = cand.contiguous(), refs.contiguous()
    return _Batch(cand, cand_len.contiguous(), refs, ref_len.contiguous(), B, R,
                  int(cand.shape[1]), int(refs.shape[2]))


def _stream_ptr(stream) -> int:
    s = stream if stream is not None else torch.cuda.current_stream()
    return int(s.cuda_stream)


def tensorbleu_workspace_layout(B: int, R: int, cand_stride: int, ref_stride: int,
                                cfg: tb_config_t) -> tb_layout_t:
    lay = tb_layout_t()
    rc = load_library().tensorbleu_workspace_layout(B, R, cand_stride, ref_stride,
                                                    ctypes.byref(cfg), ctypes.byref(lay))
    _check(rc, "tensorbleu_workspace_layout")
    return lay


def tensorbleu_workspace_bytes(B: int, R: int, cand_stride: int, ref_stride: int,
                               cfg: tb_config_t) -> int:
    return int(load_library().tensorbleu_workspace_bytes(B, R, cand_stride, ref_stride,
                                                         ctypes.byref(cfg)))


def allocate_workspace(B: int, R: int, cand_stride: int, ref_stride: int, cfg: tb_config_t,
                       device) -> torch.Tensor:
    n = tensorbleu_workspace_bytes(B, R, cand_stride, ref_stride, cfg)
    if n == 0:
        raise TensorBLEUError("tensorbleu_workspace_bytes: invalid or unsupported shape")
    return torch.empty(n, dtype=torch.uint8, device=device)


def _score_out(out: Optional[torch.Tensor], cfg: tb_config_t, shape, device) -> torch.Tensor:
    """The score tensor of the dtype the config asks for (checked when the caller brings one)."""
    dtype = torch.bfloat16 if cfg.score_bytes == 2 else torch.float32
    if out is None:
        return torch.zeros(shape, dtype=dtype, device=device)
    if out.dtype != dtype or tuple(out.shape) != tuple(shape) or not out.is_contiguous():
        raise TensorBLEUError(f"out must be a contiguous {dtype} tensor of shape {tuple(shape)}")
    return out


def _full(entry: str, cand, cand_len, refs, ref_len, cfg, out, stats, workspace, stream):
    b = _batch(cand, cand_len, refs, ref_len, cfg)
    if workspace is None:
        workspace = allocate_workspace(b.B, b.R, b.cand_stride, b.ref_stride, cfg, b.cand.device)
    st = stats.as_struct() if stats is not None else None
    rc = getattr(load_library(), entry)(
        b.cand.data_ptr(), b.cand_stride, b.cand_len.data_ptr(), b.refs.data_ptr(), b.ref_stride,
        b.ref_len.data_ptr(), b.B, b.R, ctypes.byref(cfg), out.data_ptr(),
        ctypes.byref(st) if st is not None else None, workspace.data_ptr(), workspace.numel(),
        _stream_ptr(stream))
    _check(rc, entry)
    return out


def tensorbleu_sentence(cand, cand_len, refs, ref_len, cfg: tb_config_t,
                        out: Optional[torch.Tensor] = None, stats: Optional[Stats] = None,
                        workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """float32 (or bfloat16, see make_config) [B]: one BLEU score per candidate."""
    out = _score_out(out, cfg, (cand.shape[0],), cand.device)
    return _full("tensorbleu_sentence", cand, cand_len, refs, ref_len, cfg, out, stats,
                 workspace, stream)


def tensorbleu_static_scratch_bytes() -> int:
    return int(load_library().tensorbleu_static_scratch_bytes())


def tensorbleu_sentence_static(cand, cand_len, refs, ref_len, cfg: tb_config_t,
                               out: torch.Tensor, stats: Optional[Stats] = None,
                               stream=None) -> torch.Tensor:
    """tensorbleu_sentence without a workspace: the library's built-in scratch buffer is used and
    nothing is allocated (`out` must be brought by the caller for the same reason)."""
    out = _score_out(out, cfg, (cand.shape[0],), cand.device)
    b = _batch(cand, cand_len, refs, ref_len, cfg)
    st = stats.as_struct() if stats is not None else None
    rc = load_library().tensorbleu_sentence_static(
        b.cand.data_ptr(), b.cand_stride, b.cand_len.data_ptr(), b.refs.data_ptr(), b.ref_stride,
        b.ref_len.data_ptr(), b.B, b.R, ctypes.byref(cfg), out.data_ptr(),
        ctypes.byref(st) if st is not None else None, _stream_ptr(stream))
    _check(rc, "tensorbleu_sentence_static")
    return out


def tensorbleu_corpus(cand, cand_len, refs, ref_len, cfg: tb_config_t,
                      out: Optional[torch.Tensor] = None, stats: Optional[Stats] = None,
                      workspace: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """float32 (or bfloat16) [1]: one BLEU score for the batch."""
    out = _score_out(out, cfg, (1,), cand.device)
    return _full("tensorbleu_corpus", cand, cand_len, refs, ref_len, cfg, out, stats, workspace,
                 stream)


def tensorrouge_n(cand, cand_len, refs, ref_len, n: int = 2, beta: float = 1.0, *,
                  vocab_size: int, ref_count: Optional[torch.Tensor] = None,
                  want_overlap: bool = False, want_best: bool = False,
                  workspace: Optional[torch.Tensor] = None, stats: Optional[Stats] = None,
                  stream=None, score_dtype: torch.dtype = torch.float32, path: str = "auto",
                  ref_offsets: Optional[torch.Tensor] = None, max_refs: int = 0,
                  workspace_tables: bool = False):
    """ROUGE-N of every candidate against its references: float32 (or bfloat16) [B, 3] (precision,
    recall, F of the best reference), plus overlap int32 [B, R] and best-reference index int32 [B]
    on request (returned as a tuple then).  Without a workspace argument, a shape that the GLOBAL
    path would serve with its BLEU-only packed-key kernels is run with workspace_tables set."""
    cfg = make_config(max_n=n, smooth_param=beta, vocab_size=vocab_size, path=path,
                      ref_count=ref_count, score_dtype=score_dtype, ref_offsets=ref_offsets,
                      max_refs=max_refs, workspace_tables=workspace_tables)
    b = _batch(cand, cand_len, refs, ref_len, cfg)
    if workspace is None:
        lay = tensorbleu_workspace_layout(b.B, b.R, b.cand_stride, b.ref_stride, cfg)
        if lay.path == PATHS["global"] and not (lay.global_candidate_first or
                                                lay.global_partitions or
                                                lay.global_tables_in_hbm):
            cfg.workspace_tables = 1
        workspace = allocate_workspace(b.B, b.R, b.cand_stride, b.ref_stride, cfg, b.cand.device)
    dev = b.cand.device
    out = _score_out(None, cfg, (b.B, 3), dev)
    overlap = torch.zeros(b.B, b.R, dtype=torch.int32, device=dev) if want_overlap else None
    best = torch.zeros(b.B, dtype=torch.int32, device=dev) if want_best else None
    st = stats.as_struct() if stats is not None else None
    rc = load_library().tensorrouge_n(
        b.cand.data_ptr(), b.cand_stride, b.cand_len.data_ptr(), b.refs.data_ptr(), b.ref_stride,
        b.ref_len.data_ptr(), b.B, b.R, ctypes.byref(cfg), out.data_ptr(),
        overlap.data_ptr() if overlap is not None else None,
        best.data_ptr() if best is not None else None,
        ctypes.byref(st) if st is not None else None, workspace.data_ptr(), workspace.numel(),
        _stream_ptr(stream))
    _check(rc, "tensorrouge_n")
    if want_overlap or want_best:
        return out, overlap, best
    return out


def tensorbleu_pack(cand, cand_len, refs, ref_len, cfg, workspace, stats=None, stream=None):
    b = _batch(cand, cand_len, refs, ref_len, cfg)
    st = stats.as_struct() if stats is not None else None
    rc = load_library().tensorbleu_pack(
        b.cand.data_ptr(), b.cand_stride, b.cand_len.data_ptr(), b.refs.data_ptr(), b.ref_stride,
        b.ref_len.data_ptr(), b.B, b.R, ctypes.byref(cfg),
        ctypes.byref(st) if st is not None else None, workspace.data_ptr(), workspace.numel(),
        _stream_ptr(stream))
    _check(rc, "tensorbleu_pack")


def _stage(entry, cand_len, ref_len, cand_stride, ref_stride, cfg, workspace, stats, stream):
    B = int(cand_len.shape[0])
    R = cfg._max_refs if cfg.ref_offsets else int(ref_len.shape[1])
    st = stats.as_struct() if stats is not None else None
    rc = getattr(load_library(), entry)(
        cand_len.data_ptr(), ref_len.data_ptr(), cand_stride, ref_stride, B, R, ctypes.byref(cfg),
        ctypes.byref(st) if st is not None else None, workspace.data_ptr(), workspace.numel(),
        _stream_ptr(stream))
    _check(rc, entry)


def tensorbleu_dictionary(cand_len, ref_len, cand_stride, ref_stride, cfg, workspace,
                          stats=None, stream=None):
    _stage("tensorbleu_dictionary", cand_len, ref_len, cand_stride, ref_stride, cfg, workspace,
           stats, stream)


def tensorbleu_count_clip(cand_len, ref_len, cand_stride, ref_stride, cfg, workspace,
                          stats=None, stream=None):
    _stage("tensorbleu_count_clip", cand_len, ref_len, cand_stride, ref_stride, cfg, workspace,
           stats, stream)


def tensorbleu_finalize(cand_len, ref_len, cand_stride, ref_stride, cfg, corpus, out, workspace,
                        stats=None, stream=None):
    B = int(cand_len.shape[0])
    R = cfg._max_refs if cfg.ref_offsets else int(ref_len.shape[1])
    st = stats.as_struct() if stats is not None else None
    rc = load_library().tensorbleu_finalize(
        cand_len.data_ptr(), ref_len.data_ptr(), B, R, cand_stride, ref_stride, ctypes.byref(cfg),
        1 if corpus else 0, out.data_ptr(), ctypes.byref(st) if st is not None else None,
        workspace.data_ptr(), workspace.numel(), _stream_ptr(stream))
    _check(rc, "tensorbleu_finalize")
    return out
