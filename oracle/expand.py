"""Fixed-width layer expansion, CPU oracle (TEST INFRASTRUCTURE, not product).

Sec. 3.3.3 ("Fixed-width tree") and Sec. 4.1: for each token at the tree bottom the token source
proposes k candidates with their probabilities; a candidate's cumulative probability is its own
probability times the probabilities, stored in P, of the bottom token and of all its ancestors;
the w candidates with the highest cumulative probabilities are appended, sorted by the order
of their parents (Sec. 3.2, "Layer appending"), so a level never holds more than w nodes.

Precision: the selection is an integer decision taken on floats, so both sides take it in the
same arithmetic, float32: the running product starts at 1, takes the ancestors from the root
downwards (ascending node index), then the bottom token, then the candidate.  Equal cumulative
probabilities go to the candidate that comes first in (bottom token, candidate) order.

Pins (tests/test_oracle_expand.py): a hand-worked two-level example, brute-force enumeration of
all size-w subsets on tiny inputs, and properties that hold for any correct selection.
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

F32 = np.float32


def cumulative_prob(parent: Sequence[int], prob: Sequence[float], node: int) -> np.float32:
    """Product of P over `node` and its ancestors (library numbering: parent -1 = child of the
    root, whose own probability is 1), multiplied from the root downwards in float32."""
    chain = []
    j = int(node)
    while j >= 0:
        chain.append(j)
        j = int(parent[j])
    c = F32(1.0)
    for j in reversed(chain):
        c = F32(c * F32(prob[j]))
    return c


def expand_fixed_width(parent: Sequence[int], prob: Sequence[float], bottom: Sequence[int],
                       cand_tokens: np.ndarray, cand_probs: np.ndarray, w: int
                       ) -> Tuple[List[int], List[int], List[float]]:
    """bottom: node indices (ascending; -1 = the root itself, for an empty tree) whose children are
    proposed; cand_tokens / cand_probs: [len(bottom), k]; a negative token marks an absent candidate.
    Returns the new level as (parents, tokens, probs), at most w entries, in parent order."""
    cand_tokens = np.asarray(cand_tokens)
    cand_probs = np.asarray(cand_probs, dtype=F32)
    nb, k = cand_tokens.shape
    keys = []
    for b in range(nb):
        base = cumulative_prob(parent, prob, bottom[b]) if bottom[b] >= 0 else F32(1.0)
        for c in range(k):
            if cand_tokens[b, c] < 0:
                continue
            keys.append((F32(base * cand_probs[b, c]), b * k + c))
    # highest cumulative probability first; the earlier candidate wins a tie
    keys.sort(key=lambda t: (-float(t[0]), t[1]))
    chosen = sorted(idx for _, idx in keys[:max(w, 0)])
    parents = [int(bottom[i // k]) for i in chosen]
    tokens = [int(cand_tokens[i // k, i % k]) for i in chosen]
    probs = [float(cand_probs[i // k, i % k]) for i in chosen]
    return parents, tokens, probs
