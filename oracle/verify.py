"""Last-stage verification, CPU oracle (TEST INFRASTRUCTURE, not product).

Sec. 3.3.2, node-wise computation: the last device infers the next token from the output of
the large model; Algorithm 1, "verify new token tau_hat on device m"; Sec. 3.3.3: validation
is against the top-1 prediction of the large model, which keeps decoding lossless.

For a node tau whose hidden state h leaves the last decoder layer, the model's next token is
    pred(tau) = argmax_v  ( RMSNorm(h; g, eps) . W_vocab[v] )          (Llama output head)
with the lowest vocabulary index among equal maxima.  The verified token of a step is the
child of the root tau_1 whose token equals pred(tau_1); if no child carries it the step is
a miss (pipeline stall) and the true token pred(tau_1) itself becomes the next level.

Pins (tests/test_oracle_verify.py): the head against Hugging Face's LlamaRMSNorm + a
torch Linear in float64; argmax ties by hand-made rows; and the lossless property: a
tree-speculative run with distractor tokens and misses emits exactly the token sequence
of plain one-token-at-a-time greedy decoding.
"""
from __future__ import annotations

from typing import Optional, Sequence

import numpy as np

F64 = np.float64


def lm_head_logits(h: np.ndarray, gain: np.ndarray, w_vocab: np.ndarray, eps: float) -> np.ndarray:
    """logits[i, v] = RMSNorm(h[i]) . W_vocab[v]; h [n, d], W_vocab [V, d]."""
    h = np.asarray(h, F64)
    rms = np.sqrt(np.mean(h * h, axis=-1, keepdims=True) + eps)
    return ((h / rms) * np.asarray(gain, F64)) @ np.asarray(w_vocab, F64).T


def greedy_token(logits: np.ndarray) -> np.ndarray:
    """Top-1 token of each row; the lowest index among equal maxima."""
    logits = np.asarray(logits, F64)
    out = np.empty(logits.shape[0], dtype=np.int64)
    for i in range(logits.shape[0]):
        best = 0
        for v in range(1, logits.shape[1]):
            if logits[i, v] > logits[i, best]:
                best = v
        out[i] = best
    return out


def greedy_token_fast(logits: np.ndarray) -> np.ndarray:
    """Same result through numpy (argmax returns the first maximum); for large vocabularies."""
    return np.argmax(np.asarray(logits, F64), axis=1).astype(np.int64)


def match_root_child(parent: Sequence[int], token: Sequence[int], root_pred: int) -> int:
    """Index (library numbering: speculative nodes only, parent -1 = child of the root) of the
    first root child whose token is the model's token for the root's successor; -1 on a miss."""
    for k, (p, t) in enumerate(zip(parent, token)):
        if p == -1 and int(t) == int(root_pred):
            return k
    return -1
