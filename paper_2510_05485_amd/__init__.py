"""MI355X-native batched token-ID BLEU (per-sentence and corpus) behind a C ABI.

The computation lives in `libtensorbleu.so` (hand-written HIP for gfx950, built from `csrc/` by
`python -m paper_2510_05485_amd.build`); `binding` marshals PyTorch device tensors into it.
"""
from .binding import (  # noqa: F401
    LIB_PATH, TB_DEV_LENGTH_RANGE, TB_DEV_TABLE_OVERFLOW, TB_DEV_TOKEN_RANGE, Stats, TensorBLEUError, allocate_workspace, load_library, make_config,
    tensorbleu_corpus, tensorbleu_count_clip, tensorbleu_dictionary, tensorbleu_finalize,
    tensorbleu_pack, tensorbleu_sentence, tensorbleu_status_string, tensorbleu_workspace_bytes,
    tensorbleu_workspace_layout, tensorrouge_n, tensorbleu_sentence_static,
    tensorbleu_static_scratch_bytes,
)
from .api import (  # noqa: F401
    BleuScorer, corpus_bleu, lengths_from_padding, pack_reference_lists, pad_references, rouge_n,
    sentence_bleu,
)
