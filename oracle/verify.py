"""Last-stage verification, CPU oracle (TEST INFRASTRUCTURE, not product).

Sec. 3.3.2, node-wise computation: the last device infers the next token from the output of
the large model; Algorithm 1, "verify new token tau_hat on device m"; Sec. 3.4: validation
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

Lossy verification (Sec. 3.4, "Lossless and Lossy Acceleration", options (1) and (2)):
  relaxed: among the candidate tokens (the root's children) take the one the large model
           gives the highest probability -- every step verifies some child, no stall;
  top-p:   a child is acceptable if its token lies in the large model's top-p set (tokens in
           descending probability, the shortest prefix whose probabilities sum to >= p);
           among the acceptable children the one with the highest draft probability wins.
Readings where the paper is silent: equal probabilities are ordered by ascending token id,
equal candidates by ascending node index; a step with no acceptable child is a miss exactly
as in the lossless case (the model's top-1 token becomes the next level).
Pins (tests/test_oracle_lossy.py): the top-p set against an exhaustive search over all subsets
of a tiny vocabulary and against Hugging Face's TopPLogitsWarper; p -> 0 reduces top-p
verification to the lossless match, p = 1 to "highest draft probability"; relaxed verification
equals the lossless match whenever the top-1 token is among the candidates and never misses.
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


def softmax_probs(logits: np.ndarray) -> np.ndarray:
    """Probabilities of one row of logits (float64, max subtracted)."""
    z = np.asarray(logits, F64)
    e = np.exp(z - np.max(z))
    return e / np.sum(e)


def top_p_set(probs: np.ndarray, p: float) -> list:
    """Token ids of the top-p set, most probable first: tokens in descending probability (equal
    probabilities by ascending id), cut after the first token at which the running sum reaches p."""
    probs = np.asarray(probs, F64)
    order = sorted(range(len(probs)), key=lambda v: (-probs[v], v))
    out, run = [], 0.0
    for v in order:
        out.append(v)
        run += probs[v]
        if run >= p:
            break
    return out


def relaxed_choice(logits: np.ndarray, parent: Sequence[int], token: Sequence[int]) -> int:
    """Option (1): the root child whose token has the highest large-model probability (first one
    among equals); -1 only if the root has no child.  Tokens outside the vocabulary never win."""
    logits = np.asarray(logits, F64)
    best, best_l = -1, -np.inf
    for k, (par, t) in enumerate(zip(parent, token)):
        if par != -1 or not (0 <= int(t) < len(logits)):
            continue
        if best == -1 or logits[int(t)] > best_l:
            best, best_l = k, logits[int(t)]
    return best


def top_p_choice(logits: np.ndarray, parent: Sequence[int], token: Sequence[int], draft_prob: Sequence[float],
                 p: float) -> int:
    """Option (2): among the root children whose token is in the large model's top-p set, the one
    with the highest draft probability (first one among equals); -1 if there is none."""
    logits = np.asarray(logits, F64)
    inside = set(top_p_set(softmax_probs(logits), p))
    best, best_q = -1, -np.inf
    for k, (par, t) in enumerate(zip(parent, token)):
        if par != -1 or int(t) not in inside:
            continue
        q = float(np.float32(draft_prob[k]))
        if best == -1 or q > best_q:
            best, best_q = k, q
    return best


# ----------------------------------------------------------------------------
# Stochastic decoding at the verifier (Sec. 4.3, "Stochastic Decoding")
# ----------------------------------------------------------------------------
# The large model's next token is drawn instead of taken as the arg-max: temperature T, and
# candidates are collected in descending probability until their probabilities sum to top_p or
# top_k of them have been taken, whichever comes first (the paper's setting: T = 0.6, 0.9, 80).
# The drawn token then plays the part of the top-1 token: the step verifies the root child that
# carries it, or stalls.  Readings where the paper is silent: probabilities are those of
# softmax(logits / T) over the whole vocabulary (the running sum is measured against the full
# distribution, not against the top_k tokens' share of it); equal probabilities are ordered by
# ascending token id; the draw is the inverse CDF of the candidates' renormalised probabilities
# at a uniform number u in [0, 1) that the caller supplies: candidate j is drawn iff
# C_(j-1) <= u * C_m < C_j, C the running sums in candidate order and C_m their total.
# Pins (tests/test_oracle_sampling.py): Hugging Face's temperature / top-k / top-p warpers for the
# candidate set in the cases where the two cuts do not interact; the measure of u that draws each
# candidate equals its renormalised probability; T -> 0, top_k = 1 and top_p -> 0 all reduce to
# the arg-max; the candidates are a prefix of the descending order, by exhaustive check.
def sampling_candidates(logits: np.ndarray, temperature: float, top_p: float, top_k: int):
    """(tokens, probabilities under softmax(logits / T), most probable first) the stochastic decoder may emit."""
    z = np.asarray(logits, F64) / F64(temperature)
    probs = softmax_probs(z)
    order = sorted(range(len(probs)), key=lambda v: (-probs[v], v))
    toks, ps, run = [], [], 0.0
    for v in order:
        toks.append(v)
        ps.append(probs[v])
        run += probs[v]
        if run >= top_p or len(toks) >= top_k:
            break
    return toks, np.asarray(ps, F64)


def sample_token(logits: np.ndarray, temperature: float, top_p: float, top_k: int, u: float) -> int:
    """The token drawn at uniform number u in [0, 1)."""
    toks, ps = sampling_candidates(logits, temperature, top_p, top_k)
    run = np.cumsum(ps)
    x = F64(u) * run[-1]
    for j, t in enumerate(toks):
        if x < run[j]:
            return int(t)
    return int(toks[-1])          # u * total rounded up to the total itself
