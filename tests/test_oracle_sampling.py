"""Pins for the oracle's stochastic verification (Sec. 4.3: temperature 0.6, candidates collected until
their probabilities reach 0.9 or 80 have been taken): Hugging Face's logits warpers where the two cuts
do not interact, the measure of the uniform numbers that draw a candidate, limits that reduce to the
arg-max, and an exhaustive check of the candidate set on tiny vocabularies."""
import itertools

import numpy as np
import pytest
import torch

from oracle.verify import sample_token, sampling_candidates, softmax_probs, greedy_token


def hf_kept(logits, temperature, top_p=None, top_k=None):
    """Tokens Hugging Face's warpers keep (finite logits after warping)."""
    from transformers.generation.logits_process import TemperatureLogitsWarper, TopKLogitsWarper, TopPLogitsWarper
    x = torch.tensor(np.asarray(logits, np.float64))[None, :]
    ids = torch.zeros((1, 1), dtype=torch.long)
    x = TemperatureLogitsWarper(float(temperature))(ids, x)
    if top_k is not None:
        x = TopKLogitsWarper(int(top_k))(ids, x)
    if top_p is not None:
        x = TopPLogitsWarper(float(top_p))(ids, x)
    return sorted(int(v) for v in torch.nonzero(torch.isfinite(x[0]))[:, 0])


@pytest.mark.parametrize("seed", range(4))
def test_candidates_against_hugging_face_warpers(seed):
    rs = np.random.RandomState(seed)
    V = 300
    logits = rs.randn(V) * 3.0
    # only the probability cut (top_k out of reach)
    for T, p in ((0.6, 0.9), (1.0, 0.5), (1.7, 0.99), (0.3, 0.2)):
        toks, _ = sampling_candidates(logits, T, p, V)
        assert sorted(toks) == hf_kept(logits, T, top_p=p)
    # only the count cut (top_p = 1 is never reached before the last token)
    for T, k in ((0.6, 80), (1.0, 1), (2.0, 17)):
        toks, _ = sampling_candidates(logits, T, 1.0 + 1e-9, k)
        assert sorted(toks) == hf_kept(logits, T, top_k=k)
        assert len(toks) == k


def test_both_cuts_whichever_comes_first():
    logits = np.log(np.array([0.4, 0.25, 0.15, 0.1, 0.06, 0.04]))
    assert sampling_candidates(logits, 1.0, 0.9, 80)[0] == [0, 1, 2, 3]          # 0.4+0.25+0.15+0.1 reaches 0.9
    assert sampling_candidates(logits, 1.0, 0.9, 3)[0] == [0, 1, 2]              # the count cuts first
    assert sampling_candidates(logits, 1.0, 0.5, 3)[0] == [0, 1]                 # the probability cuts first
    # equal probabilities: ascending token id
    assert sampling_candidates(np.zeros(5), 1.0, 0.5, 80)[0] == [0, 1, 2]
    # temperature sharpens: at T = 0.5 the probabilities are proportional to p^2
    toks, ps = sampling_candidates(logits, 0.5, 0.999999, 80)
    want = np.array([0.4, 0.25, 0.15, 0.1, 0.06, 0.04]) ** 2
    assert np.allclose(ps / ps.sum(), (want / want.sum())[:len(ps)])


def test_candidate_set_is_the_shortest_descending_prefix_exhaustively():
    """Over every ordering of a small multiset of logits: the candidates are a prefix of the descending
    order, their mass reaches top_p (unless top_k cut first), and dropping the last one would not."""
    base = [0.0, 0.0, 0.7, -1.3, 2.1, 0.7]
    for perm in set(itertools.permutations(base)):
        logits = np.array(perm)
        for T, p, k in ((0.6, 0.9, 80), (1.0, 0.6, 2), (1.0, 0.6, 80)):
            toks, ps = sampling_candidates(logits, T, p, k)
            probs = softmax_probs(logits / T)
            order = sorted(range(len(perm)), key=lambda v: (-probs[v], v))
            assert toks == order[:len(toks)]
            assert len(toks) <= k
            if len(toks) < k:
                assert ps.sum() >= p
            assert len(toks) == 1 or ps[:-1].sum() < p


def test_measure_of_u_that_draws_a_candidate_is_its_probability():
    rs = np.random.RandomState(5)
    logits = rs.randn(40) * 2.0
    T, p, k = 0.6, 0.9, 80
    toks, ps = sampling_candidates(logits, T, p, k)
    grid = (np.arange(200000) + 0.5) / 200000.0
    drawn = np.array([sample_token(logits, T, p, k, u) for u in grid[::40]])       # 5000 points
    for t, q in zip(toks, ps / ps.sum()):
        assert abs(np.mean(drawn == t) - q) <= 1.0 / 2500, (t, q)
    assert set(drawn.tolist()) <= set(toks)
    assert sample_token(logits, T, p, k, 0.0) == toks[0]
    assert sample_token(logits, T, p, k, np.nextafter(1.0, 0.0)) == toks[-1]


def test_limits_reduce_to_the_arg_max():
    rs = np.random.RandomState(6)
    logits = rs.randn(3, 64)
    top1 = greedy_token(logits)
    for i in range(3):
        for u in (0.0, 0.37, 0.999):
            assert sample_token(logits[i], 1e-3, 0.9, 80, u) == top1[i]      # temperature -> 0
            assert sample_token(logits[i], 0.6, 0.9, 1, u) == top1[i]        # one candidate
            assert sample_token(logits[i], 0.6, 1e-12, 80, u) == top1[i]     # probability cut at once
