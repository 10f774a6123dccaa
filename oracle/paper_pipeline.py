"""The paper's tensor-op pipeline, step by step, in numpy -- TEST INFRASTRUCTURE ONLY.

This walks Sections 3.1-3.3 in the paper's order and notation with library primitives standing
in for the PyTorch calls it names (sliding windows for `unfold`, `np.unique(axis=0,
return_inverse=True)` for `torch.unique(dim=0, return_inverse=True)`, `np.bincount` for
`torch.bincount`).  The dictionary here is batch-wide and the count tensor is the dense
(batch_size, num_unique_ngrams) one, exactly as described, so it is only usable on small batches.
It exists to show that the per-sentence dictionary definition in `bleu_oracle.cpp` and the
paper's batched formulation give the same integer statistics.
"""
from __future__ import annotations

import numpy as np


def _valid_windows(rows: np.ndarray, lens: np.ndarray, n: int):
    """All valid order-n windows of a padded [S, stride] matrix, flattened, with owner ids.

    Section 3.1 (unfold) + Section 3.2 step 1 ("valid n-grams"): a window is valid when it lies
    inside the sequence's true length.
    """
    S, stride = rows.shape
    if stride < n:
        return np.zeros((0, n), rows.dtype), np.zeros(0, np.int64)
    win = np.lib.stride_tricks.sliding_window_view(rows, n, axis=1)  # (S, stride-n+1, n)
    pos = np.arange(stride - n + 1)[None, :]
    valid = pos + n <= lens[:, None]
    owner = np.broadcast_to(np.arange(S)[:, None], valid.shape)
    return win[valid], owner[valid].astype(np.int64)


def clipped_counts(cand: np.ndarray, cand_len: np.ndarray, refs: np.ndarray,
                   ref_len: np.ndarray, max_n: int = 4):
    """Numerators and denominators per sentence and order via unique + offset bincount.

    Returns (clipped [B, N], total [B, N], num_unique [N]).
    """
    B, R = refs.shape[0], refs.shape[1]
    clipped = np.zeros((B, max_n), np.int64)
    total = np.zeros((B, max_n), np.int64)
    num_unique = np.zeros(max_n, np.int64)
    for n in range(1, max_n + 1):
        # Section 3.2 step 1: unified collection of candidate and all reference n-grams
        cg, c_owner = _valid_windows(cand, cand_len, n)
        parts, owners = [cg], [c_owner]
        for j in range(R):
            rg, r_owner = _valid_windows(refs[:, j, :], ref_len[:, j], n)
            parts.append(rg)
            owners.append(r_owner)
        all_ngrams = np.concatenate(parts, axis=0)
        total[:, n - 1] = np.bincount(c_owner, minlength=B)
        if all_ngrams.shape[0] == 0:
            continue
        # Section 3.2 step 2: compact batch-specific dictionary
        unique_ngrams, inverse_indices = np.unique(all_ngrams, axis=0, return_inverse=True)
        inverse_indices = inverse_indices.reshape(-1)
        U = unique_ngrams.shape[0]
        num_unique[n - 1] = U
        # Section 3.3 steps 1-2: offset ids, one bincount, reshape to (batch, num_unique)
        bounds = np.cumsum([0] + [len(p) for p in parts])

        def batched_bincount(k):
            ids = inverse_indices[bounds[k]:bounds[k + 1]] + owners[k] * U
            return np.bincount(ids, minlength=B * U).reshape(B, U)

        candidate_counts = batched_bincount(0)
        # Section 3.3 step 3: maximum over reference sets, then minimum with candidate counts
        reference_max_counts = np.zeros((B, U), np.int64)
        for j in range(R):
            reference_max_counts = np.maximum(reference_max_counts, batched_bincount(1 + j))
        clipped[:, n - 1] = np.minimum(candidate_counts, reference_max_counts).sum(axis=1)
    return clipped, total, num_unique
