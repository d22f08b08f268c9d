"""Pins for the oracle's lossy verification (Sec. 3.4, options (1) relaxed and (2) top-p)
against things other than itself: an exhaustive subset search, Hugging Face's top-p warper,
and the limits in which both options reduce to rules already pinned elsewhere."""
import itertools

import numpy as np
import pytest
import torch

from oracle.verify import (softmax_probs, top_p_set, relaxed_choice, top_p_choice, match_root_child,
                           greedy_token)


def _brute_top_p(probs, p):
    """Smallest subset whose mass reaches p; among those of that size the one of largest mass."""
    n = len(probs)
    for size in range(1, n + 1):
        best, best_mass = None, -1.0
        for sub in itertools.combinations(range(n), size):
            mass = float(sum(probs[v] for v in sub))
            if mass >= p and mass > best_mass:
                best, best_mass = sub, mass
        if best is not None:
            return set(best)
    return set(range(n))


@pytest.mark.parametrize("seed", range(6))
@pytest.mark.parametrize("p", [0.05, 0.3, 0.6, 0.9, 0.999])
def test_top_p_set_is_the_smallest_heaviest_subset(seed, p):
    rng = np.random.default_rng(seed)
    probs = softmax_probs(rng.normal(0, 2.0, size=9))
    got = top_p_set(probs, p)
    assert set(got) == _brute_top_p(probs, p)
    # listed most probable first
    assert all(probs[a] >= probs[b] for a, b in zip(got, got[1:]))


def test_top_p_set_hand_worked():
    probs = np.array([0.1, 0.4, 0.2, 0.3])
    assert top_p_set(probs, 0.4) == [1]              # reached exactly by the first token
    assert top_p_set(probs, 0.41) == [1, 3]
    assert top_p_set(probs, 0.7) == [1, 3]
    assert top_p_set(probs, 0.75) == [1, 3, 2]
    assert top_p_set(probs, 1.0) == [1, 3, 2, 0]
    # equal probabilities: ascending token id
    assert top_p_set(np.array([0.25, 0.25, 0.25, 0.25]), 0.5) == [0, 1]


@pytest.mark.parametrize("seed", range(5))
@pytest.mark.parametrize("p", [0.2, 0.5, 0.8, 0.95])
def test_top_p_set_matches_huggingface_warper(seed, p):
    from transformers.generation.logits_process import TopPLogitsWarper
    rng = np.random.default_rng(100 + seed)
    logits = rng.normal(0, 3.0, size=257)
    warped = TopPLogitsWarper(top_p=float(p))(None, torch.tensor(logits, dtype=torch.float64)[None, :])[0]
    kept = set(np.nonzero(np.isfinite(warped.numpy()))[0].tolist())
    assert set(top_p_set(softmax_probs(logits), p)) == kept


def _children(rng, n_nodes, vocab, n_root):
    parent = [-1] * n_root + [int(rng.integers(0, n_root)) for _ in range(n_nodes - n_root)]
    token = rng.choice(vocab, size=n_nodes, replace=False).tolist()
    prob = rng.uniform(0.01, 1.0, size=n_nodes).astype(np.float32).tolist()
    return parent, token, prob


@pytest.mark.parametrize("seed", range(8))
def test_tiny_p_is_the_lossless_match(seed):
    rng = np.random.default_rng(200 + seed)
    V = 50
    logits = rng.normal(0, 2.0, size=V)
    parent, token, prob = _children(rng, 12, V, 5)
    top1 = int(greedy_token(logits[None, :])[0])
    if seed % 2 == 0:
        token[int(rng.integers(0, 5))] = top1         # make it a hit
    assert top_p_choice(logits, parent, token, prob, 1e-9) == match_root_child(parent, token, top1)


@pytest.mark.parametrize("seed", range(5))
def test_p_one_takes_the_highest_draft_probability(seed):
    rng = np.random.default_rng(300 + seed)
    V = 40
    logits = rng.normal(0, 2.0, size=V)
    parent, token, prob = _children(rng, 10, V, 6)
    want = max(range(6), key=lambda k: (np.float32(prob[k]), -k))
    assert top_p_choice(logits, parent, token, prob, 1.0) == want


@pytest.mark.parametrize("seed", range(8))
def test_relaxed_never_misses_and_agrees_with_a_lossless_hit(seed):
    rng = np.random.default_rng(400 + seed)
    V = 64
    logits = rng.normal(0, 2.0, size=V)
    parent, token, prob = _children(rng, 14, V, 6)
    k = relaxed_choice(logits, parent, token)
    assert k != -1 and parent[k] == -1
    # no root child has a more probable token
    assert all(logits[token[j]] <= logits[token[k]] for j in range(14) if parent[j] == -1)
    top1 = int(greedy_token(logits[None, :])[0])
    token[3] = top1
    assert relaxed_choice(logits, parent, token) == match_root_child(parent, token, top1) == 3


def test_relaxed_and_top_p_edge_cases():
    logits = np.array([0.0, 3.0, 1.0, 3.0, -1.0])
    # no children of the root
    assert relaxed_choice(logits, [], []) == -1
    assert top_p_choice(logits, [], [], [], 0.9) == -1
    # only deeper nodes carry likely tokens
    assert relaxed_choice(logits, [-1, 0], [4, 1]) == 0
    # equal large-model probability: first node
    assert relaxed_choice(logits, [-1, -1], [3, 1]) == 0
    # a token outside the vocabulary never wins
    assert relaxed_choice(logits, [-1, -1], [99, 4]) == 1
    assert top_p_choice(logits, [-1, -1], [99, 1], [0.9, 0.1], 0.5) == 1
    # equal draft probabilities among acceptable children: first node
    assert top_p_choice(logits, [-1, -1, -1], [2, 1, 3], [0.5, 0.5, 0.5], 0.95) == 0
    # top-p set {1} (ties by id: token 1 before token 3): a child with token 3 is outside at small p
    assert top_p_choice(logits, [-1], [3], [1.0], 0.3) == -1
    assert top_p_choice(logits, [-1], [1], [1.0], 0.3) == 0
