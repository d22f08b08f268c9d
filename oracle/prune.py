"""Pruning propagation on one device (Sec. 3.3.2 "pruning propagation", Algorithm 1).

TEST INFRASTRUCTURE.  Once the last stage has verified a token tau_hat, every
device prunes its tree mask M_i, its in-flight embeddings E_i and the pending
layer with the column mask col(tau_hat), and its KV cache with
row(tau_hat) OR col(tau_hat), because the verified token and the path that
leads to it must stay in the cache.  Dropping a rejected branch (used by the
synthetic workloads) keeps the complement of a column instead.

Masks are over the oracle's tree indices, root included (see tree.py).
"""
from __future__ import annotations

from dataclasses import dataclass

import numpy as np

from .tree import SpecTree


@dataclass
class PruneResult:
    table_keep: np.ndarray   # bool[n]: mask for M_i, E_i and the pending layer
    kv_keep: np.ndarray      # bool[n]: mask for the tree part of KV_i (root's row first)
    n_commit: int            # speculative nodes that become committed context


def accept_masks(tree: SpecTree, r: int) -> PruneResult:
    """tau_hat = node r: tables keep col(r); KV keeps row(r) OR col(r)."""
    if not (0 <= r < tree.n):
        raise ValueError("accept: no such node")
    col = tree.col(r)
    row = tree.row(r)
    return PruneResult(col, np.logical_or(row, col), int(row.sum()) - 1)


def drop_masks(tree: SpecTree, x: int) -> PruneResult:
    """Reject node x: x and everything below it goes; nothing is committed."""
    if not (1 <= x < tree.n):
        raise ValueError("drop: no such speculative node")
    keep = np.logical_not(tree.col(x))
    return PruneResult(keep, keep.copy(), 0)


def compact_rows(rows: np.ndarray, keep: np.ndarray) -> np.ndarray:
    """Stable selection of the kept rows (any dtype: used on float caches and on raw bytes)."""
    keep = np.asarray(keep, dtype=bool)
    if rows.shape[0] != keep.shape[0]:
        raise ValueError("compact_rows: mask length differs from row count")
    return rows[keep]
