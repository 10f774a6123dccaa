"""Host-only checks of the C-ABI library: it loads, exports every declared symbol, and its pure
host functions (layout, argument validation, status strings) behave as the header says.  No
kernel is launched here."""
import ctypes
import os
import re

import pytest

import paper_2510_05485_amd as tb
from paper_2510_05485_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "tensorbleu.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(tb.LIB_PATH):
        from paper_2510_05485_amd import build
        build.build(verbose=False)
    return tb.load_library()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tensor(?:bleu|rouge)_\w+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_functions()
    assert len(names) >= 10 and "tensorrouge_n" in names
    for name in names:
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == names


def test_status_strings(lib):
    assert tb.tensorbleu_status_string(0) == "ok"
    seen = {tb.tensorbleu_status_string(k) for k in range(5)}
    assert len(seen) == 5
    assert tb.tensorbleu_status_string(99) == "unknown status"


def test_layout_key_widths_follow_vocab(lib):
    cfg = tb.make_config(vocab_size=50257, path="global")
    lay = tb.tensorbleu_workspace_layout(512, 4, 1024, 1280, cfg)
    assert lay.bits == 16 and list(lay.key_bytes) == [8, 8, 8, 8, 16, 16, 16, 16]
    assert lay.group_cap == 1024 + 4 * 1280 and lay.path == 2 and lay.global_ok == 1
    cfg = tb.make_config(vocab_size=262144, path="global")
    lay = tb.tensorbleu_workspace_layout(1024, 1, 2048, 2048, cfg)
    assert lay.bits == 18 and list(lay.key_bytes)[:4] == [8, 8, 8, 16]
    slots = 1024 * 4096
    assert lay.keys_off[3] - lay.keys_off[2] >= slots * 8
    assert lay.inv_off[0] - lay.keys_off[3] >= slots * 16
    assert lay.bytes >= lay.inv_off[3] + slots * 4
    assert lay.bytes == tb.tensorbleu_workspace_bytes(1024, 1, 2048, 2048, cfg)
    for off in list(lay.keys_off) + list(lay.inv_off) + [lay.corpus_off]:
        assert off % 256 == 0
    cfg = tb.make_config(vocab_size=64, path="global")
    assert tb.tensorbleu_workspace_layout(4096, 2, 512, 640, cfg).bits == 6
    cfg = tb.make_config(vocab_size=1, path="global")
    assert tb.tensorbleu_workspace_layout(1, 1, 8, 8, cfg).bits == 1


def test_invalid_arguments_are_rejected_on_the_host(lib):
    good = tb.make_config(vocab_size=100, path="global")
    assert tb.tensorbleu_workspace_bytes(4, 1, 16, 16, good) > 0
    assert tb.tensorbleu_workspace_bytes(-1, 1, 16, 16, good) == 0
    assert tb.tensorbleu_workspace_bytes(4, 0, 16, 16, good) == 0
    assert tb.tensorbleu_workspace_bytes(4, 1, 0, 16, good) == 0
    for bad in (tb.make_config(max_n=0, vocab_size=100), tb.make_config(max_n=9, vocab_size=100),
                tb.make_config(vocab_size=0), tb.make_config(vocab_size=100, smoothing=7),
                tb.make_config(vocab_size=100, path=3)):
        assert tb.tensorbleu_workspace_bytes(4, 1, 16, 16, bad) == 0
    lay = binding.tb_layout_t()
    rc = lib.tensorbleu_workspace_layout(4, 1, 16, 16, None, ctypes.byref(lay))
    assert rc == 1
    # more than four orders: the GLOBAL path needs the packed n-gram to fit 128 bits
    eight = tb.make_config(max_n=8, vocab_size=65536, path="global")       # 8 * 16 bits
    assert lib.tensorbleu_workspace_layout(4, 1, 16, 16, ctypes.byref(eight), ctypes.byref(lay)) == 0
    assert lay.global_ok == 1 and lay.keys_off[7] > lay.keys_off[6] > 0
    five = tb.make_config(max_n=5, vocab_size=2 ** 26, path="global")      # 5 * 26 bits
    assert lib.tensorbleu_workspace_layout(4, 1, 16, 16, ctypes.byref(five), ctypes.byref(lay)) == 3
    five = tb.make_config(max_n=5, vocab_size=2 ** 26, path="auto")
    assert lib.tensorbleu_workspace_layout(4, 1, 16, 16, ctypes.byref(five), ctypes.byref(lay)) == 0
    assert lay.path == 1 and lay.global_ok == 0 and lay.fused_ok == 1
    # shapes whose slot count would not fit the 32-bit ids (or int64 at all) are refused, not wrapped
    huge = tb.make_config(vocab_size=100, path="global")
    assert lib.tensorbleu_workspace_layout(2 ** 31 - 1, 2 ** 20, 2 ** 30, 2 ** 30, ctypes.byref(huge),
                                           ctypes.byref(lay)) == 3
    assert tb.tensorbleu_workspace_bytes(2 ** 31 - 1, 2 ** 20, 2 ** 30, 2 ** 30, huge) == 0
    assert tb.tensorbleu_workspace_bytes(1 << 20, 1, 4096, 4096, huge) == 0     # 2^33 slots
    # NULL data pointers / workspace are caught before any launch
    args = [None, 16, None, None, 16, None, 4, 1, ctypes.byref(good), None, None, None, 0, None]
    assert lib.tensorbleu_sentence(*args) == 1
    # B == 0 is a successful no-op
    args[6] = 0
    assert lib.tensorbleu_sentence(*args) == 0


def test_group_too_large_for_lds_falls_back_to_tables_in_the_workspace(lib):
    cfg = tb.make_config(vocab_size=50257, path="global")
    lay = binding.tb_layout_t()
    # 64 sequences: beyond the single-table kernels (12 288 slots) and, with more than 62
    # references, not for the partitioned ones either
    rc = lib.tensorbleu_workspace_layout(2, 63, 8192, 8192, ctypes.byref(cfg), ctypes.byref(lay))
    assert rc == 0 and lay.global_ok == 1 and lay.global_tables_in_hbm == 1
    assert lay.global_partitions == 0 and lay.id_stride == lay.group_cap
    cap = 64 * 8192
    slots = 1 << (2 * cap - 1).bit_length()
    assert lay.bytes >= lay.tables_off + 2 * 4 * (slots + 8) * 8
    fused = tb.make_config(vocab_size=50257, path="fused")
    assert lib.tensorbleu_workspace_layout(2, 63, 8192, 8192, ctypes.byref(fused),
                                           ctypes.byref(lay)) == 3
    assert tb.tensorbleu_workspace_bytes(2, 63, 8192, 8192, fused) == 0
    # up to 62 references the partitioned kernels take such groups (the count kernel then takes
    # the references a few at a time)
    lay = tb.tensorbleu_workspace_layout(2, 16, 8192, 8192, cfg)
    assert lay.global_tables_in_hbm == 0 and lay.global_partitions == 64


def test_partitioned_layout_between_the_lds_kernels_and_the_workspace_tables(lib):
    cfg = tb.make_config(vocab_size=50257, path="global")
    lay = tb.tensorbleu_workspace_layout(2, 8, 8192, 8192, cfg)       # 73 728 slots
    assert lay.global_ok == 1 and lay.global_tables_in_hbm == 0
    assert lay.global_partitions == 32 and lay.id_stride == 32 * 6144
    assert lay.bytes >= lay.tables_off + 2 * 4 * 32 * 4               # int32 [B, N, P]
    small = tb.tensorbleu_workspace_layout(2, 1, 8192, 8192, cfg)     # 16 384 slots
    assert small.global_partitions == 4 and small.id_stride == 4 * 6144
    # more references than the partitioned count kernel has counter fields for at once: still
    # partitioned (it takes them in passes); from 63 references on: tables in the workspace
    many = tb.tensorbleu_workspace_layout(2, 12, 2048, 2048, cfg)
    assert many.global_partitions == 8 and many.global_tables_in_hbm == 0
    most = tb.tensorbleu_workspace_layout(2, 63, 512, 512, cfg)
    assert most.global_partitions == 0 and most.global_tables_in_hbm == 1
    # 512 partitions at most: 41 * 65 535 slots would need more
    far = tb.tensorbleu_workspace_layout(1, 40, 65535, 65535, cfg)
    assert far.global_partitions == 0 and far.global_tables_in_hbm == 1
    most = tb.tensorbleu_workspace_layout(1, 31, 65535, 65535, cfg)     # 2 097 120 slots
    assert most.global_partitions == 512 and most.global_tables_in_hbm == 0
    wide = tb.tensorbleu_workspace_layout(1, 7, 65535, 65535, cfg)     # 524 280 slots
    assert wide.global_partitions == 128
    # strides above 65 535 are fine there (32-bit counters)
    long_rows = tb.tensorbleu_workspace_layout(2, 1, 100000, 100000, cfg)
    assert long_rows.global_partitions == 64 and long_rows.global_tables_in_hbm == 0
    # ids must still fit 32 bits
    assert tb.tensorbleu_workspace_bytes(1 << 16, 8, 8192, 8192, cfg) == 0


def test_lengths_from_padding():
    import torch
    x = torch.tensor([[5, 0, 7, 0, 0], [0, 0, 0, 0, 0], [1, 2, 3, 4, 5], [0, 0, 3, 0, 0]])
    assert tb.lengths_from_padding(x, 0).tolist() == [3, 0, 5, 3]      # inner pad ids are kept
    assert tb.lengths_from_padding(x, 7).tolist() == [5, 5, 5, 5]
    refs = x.view(2, 2, 5).to(torch.int64)
    got = tb.lengths_from_padding(refs, 0)
    assert got.dtype == torch.int32 and got.tolist() == [[3, 0], [5, 3]]


def test_partition_hash_spreads_realistic_and_structured_keys():
    """The partitioned kernels give a hash partition room for 6144 distinct n-grams.  The hash
    (re-stated here from the kernels' definition: a multiplicative hash of the packed key, the
    partition = the top bits of a second product) must keep every partition below that on keys as
    the workloads produce them -- Zipf tokens, and the most regular keys there are: consecutive
    ids -- with the number of partitions the plan chooses for the shape."""
    import numpy as np
    import synth_inputs as syn
    M = np.uint64(0xFFFFFFFF)

    def partitions(keys, log2_parts):
        keys = keys.astype(np.uint64)
        lo, hi = keys & M, keys >> np.uint64(32)
        rot = ((hi << np.uint64(15)) | (hi >> np.uint64(17))) & M
        h = ((lo ^ rot) * np.uint64(0x9E3779B1)) & M
        return ((h * np.uint64(0x85EBCA6B) + np.uint64(0x27D4EB2F)) & M) >> np.uint64(32 - log2_parts)

    def worst_load(seqs, bits, parts):
        log2_parts = parts.bit_length() - 1
        worst = 0
        for n in (1, 2, 3):                     # orders whose packed keys fit 64 bits at 16-bit ids
            keys = []
            for s in seqs:
                s = s.astype(np.uint64)
                k = np.zeros(max(len(s) - n + 1, 0), np.uint64)
                for j in range(n):
                    k = (k << np.uint64(bits)) | s[j:len(s) - n + 1 + j]
                keys.append(k)
            distinct = np.unique(np.concatenate(keys))
            worst = max(worst, int(np.bincount(partitions(distinct, log2_parts).astype(np.int64),
                                               minlength=parts).max()))
        return worst

    cfg = tb.make_config(vocab_size=50257, path="global")
    for L, name in ((8192, "zipf"), (8192, "consecutive"), (40000, "zipf"), (40000, "consecutive")):
        lay = tb.tensorbleu_workspace_layout(1, 1, L, L, cfg)
        assert lay.global_partitions > 0
        if name == "zipf":
            w = syn.long_form(B=1, L=L)
            seqs = [w.cand[0, :w.cand_len[0]], w.refs[0, 0, :w.ref_len[0, 0]]]
        else:
            seqs = [np.arange(L) % 50257, (np.arange(L) + L) % 50257]
        assert worst_load(seqs, 16, lay.global_partitions) <= 6144, (L, name)
