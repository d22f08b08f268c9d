"""The dynamic speculative tree as the paper stores it (Sec. 3.2).

TEST INFRASTRUCTURE.  Three arrays represent a tree of n tokens indexed from
the root down, parents before children:

  I[i]    token id of tau_i,
  P[i]    probability of tau_i given its parent,
  M[i,j]  1 iff j == i or tau_j is an ancestor of tau_i; 0 above the diagonal.

Index 0 is the root tau_1 = the last verified token.  (The HIP library keeps
that root in the committed prefix and numbers only the speculative nodes, so
its node k is index k+1 here and its parent -1 is index 0 here; `view()`
converts.)

Nothing else is stored: parent and depth are read off M.
"""
from __future__ import annotations

from typing import Sequence, Tuple

import numpy as np


class SpecTree:
    def __init__(self, root_token: int = 0, root_prob: float = 1.0):
        self.I = np.array([root_token], dtype=np.int64)
        self.P = np.array([root_prob], dtype=np.float32)
        self.M = np.ones((1, 1), dtype=np.uint8)

    # -- size ---------------------------------------------------------------
    @property
    def n(self) -> int:
        return int(self.I.shape[0])

    def copy(self) -> "SpecTree":
        t = SpecTree()
        t.I, t.P, t.M = self.I.copy(), self.P.copy(), self.M.copy()
        return t

    # -- layer appending (Sec. 3.2, "Layer appending") ------------------------
    def append_layer(self, parents: Sequence[int], tokens: Sequence[int], probs: Sequence[float]) -> None:
        """Append a group of tokens whose parents all exist already.  M grows to
        [[M, 0], [rows of the parents, identity]]."""
        parents = np.asarray(parents, dtype=np.int64).reshape(-1)
        k = parents.shape[0]
        if k == 0:
            return
        n = self.n
        if parents.min() < 0 or parents.max() >= n:
            raise ValueError("append_layer: parent outside the existing tree")
        top = np.concatenate([self.M, np.zeros((n, k), dtype=np.uint8)], axis=1)
        bottom = np.concatenate([self.M[parents, :], np.eye(k, dtype=np.uint8)], axis=1)
        self.M = np.concatenate([top, bottom], axis=0)
        self.I = np.concatenate([self.I, np.asarray(tokens, dtype=np.int64).reshape(-1)])
        self.P = np.concatenate([self.P, np.asarray(probs, dtype=np.float32).reshape(-1)])

    def append(self, parents: Sequence[int], tokens: Sequence[int], probs: Sequence[float]) -> None:
        """Append tokens whose parent may be an existing node or a token earlier
        in this same call: the call is cut into consecutive groups whose parents
        all exist, and each group is appended as a layer."""
        parents = [int(p) for p in parents]
        tokens = list(tokens)
        probs = list(probs)
        start = 0
        while start < len(parents):
            n = self.n
            end = start
            while end < len(parents) and parents[end] < n:
                end += 1
            if end == start:
                raise ValueError("append: parent index not smaller than the child's")
            self.append_layer(parents[start:end], tokens[start:end], probs[start:end])
            start = end

    # -- what M implies -----------------------------------------------------
    def depth(self) -> np.ndarray:
        """Number of proper ancestors of each node (root: 0)."""
        return self.M.sum(axis=1).astype(np.int64) - 1

    def parent(self) -> np.ndarray:
        """Parent index of each node, -1 for the root: the proper ancestor with
        the largest index (ancestors of a node form a chain with growing index)."""
        out = np.full(self.n, -1, dtype=np.int64)
        for i in range(self.n):
            anc = np.nonzero(self.M[i, :i])[0]
            if anc.size:
                out[i] = anc[-1]
        return out

    def col(self, i: int) -> np.ndarray:
        """Temporary mask m of to-subtree pruning: m[j] = tau_j lies in the subtree rooted at tau_i."""
        return self.M[:, i].astype(bool)

    def row(self, i: int) -> np.ndarray:
        """row[j] = tau_j is tau_i or one of its ancestors."""
        return self.M[i, :].astype(bool)

    # -- to-subtree pruning (Sec. 3.2, "To-subtree pruning") ------------------
    def select(self, m: np.ndarray) -> None:
        """Apply a keep-mask to I and P and to both the rows and the columns of M."""
        m = np.asarray(m, dtype=bool)
        self.I = self.I[m]
        self.P = self.P[m]
        self.M = self.M[m][:, m]

    def to_subtree(self, i: int) -> np.ndarray:
        """Reroot at tau_i; returns the mask that was applied."""
        if not (0 <= i < self.n):
            raise ValueError("to_subtree: no such node")
        m = self.col(i)
        self.select(m)
        return m

    # -- the library's numbering: speculative nodes only ---------------------
    def view(self) -> Tuple[np.ndarray, np.ndarray, np.ndarray, np.ndarray, np.ndarray]:
        """(parent, depth, token, prob, M) over the non-root nodes, in the HIP
        library's numbering: node k = index k+1 here, parent -1 = the root,
        depth counted from the root's children (0)."""
        par = self.parent()[1:] - 1
        dep = self.depth()[1:] - 1
        return (par.astype(np.int32), dep.astype(np.int32), self.I[1:].astype(np.int32),
                self.P[1:].astype(np.float32), self.M[1:, 1:].copy())
