"""Token permutation / dispatch packing for one rank (the local stand-in for the
all-to-all dispatch of Sec. "Overhead-Aware Pipeline Orchestration": tokens are
sent to the devices of their experts, then the MoE computation runs).

Canonical order (the paper does not fix one): the rank's assignments sorted by
(local expert ascending, flat assignment index a = t*k + j ascending) -- a
stable sort by expert.
"""
import numpy as np


def permute_indices(topk_ids: np.ndarray, rank: int, n_local: int):
    """Returns expert_offsets int32 [n_local+1] (exclusive prefix of the local
    expert counts), row_to_assign int32 [R], assign_to_row int32 [T*k] (-1 for
    assignments of other ranks)."""
    ids = np.asarray(topk_ids, dtype=np.int64)
    flat = ids.reshape(-1)
    lo = rank * n_local
    local = np.nonzero((flat >= lo) & (flat < lo + n_local))[0]
    order = np.argsort(flat[local], kind="stable")
    row_to_assign = local[order].astype(np.int32)
    counts = np.bincount(flat[local] - lo, minlength=n_local)
    expert_offsets = np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)
    assign_to_row = np.full(flat.size, -1, dtype=np.int32)
    assign_to_row[row_to_assign] = np.arange(row_to_assign.size, dtype=np.int32)
    return expert_offsets, row_to_assign, assign_to_row


def gather_rows(x_bits: np.ndarray, row_to_assign: np.ndarray, k: int) -> np.ndarray:
    """Xperm[r] = x[row_to_assign[r] // k]  (bf16 patterns, copied unchanged)."""
    return np.asarray(x_bits)[np.asarray(row_to_assign, dtype=np.int64) // k]
