"""Pins for oracle/expand.py (fixed-width layer expansion, Sec. 3.3.3): a hand-worked example,
brute force over all subsets on tiny inputs, and properties of any correct selection."""
import itertools

import numpy as np
import pytest

from oracle.expand import expand_fixed_width, cumulative_prob

F32 = np.float32


def test_hand_worked_two_levels():
    # level 1 under the root: a (P=.5) and b (P=.25); a has a child c (P=.5)
    parent = [-1, -1, 0]
    prob = [0.5, 0.25, 0.5]
    assert cumulative_prob(parent, prob, 2) == F32(0.25)
    assert cumulative_prob(parent, prob, 1) == F32(0.25)
    # bottom tokens: b (node 1) and c (node 2), two candidates each
    toks = np.array([[10, 11], [20, 21]])
    prs = np.array([[0.5, 0.125], [0.75, 0.25]], dtype=F32)
    # cumulative: b->10: .125, b->11: .03125, c->20: .1875, c->21: .0625
    par, tok, pr = expand_fixed_width(parent, prob, [1, 2], toks, prs, 2)
    assert (par, tok) == ([1, 2], [10, 20]) and pr == [0.5, 0.75]
    par, tok, pr = expand_fixed_width(parent, prob, [1, 2], toks, prs, 3)
    assert (par, tok) == ([1, 2, 2], [10, 20, 21])                  # parent order, not probability order
    par, tok, _ = expand_fixed_width(parent, prob, [1, 2], toks, prs, 9)
    assert tok == [10, 11, 20, 21]                                  # fewer candidates than the width
    assert expand_fixed_width(parent, prob, [1, 2], toks, prs, 0) == ([], [], [])


def test_ties_go_to_the_earlier_candidate_and_absent_ones_are_skipped():
    parent, prob = [-1, -1], [0.5, 0.5]
    toks = np.array([[7, -1, 8], [9, 7, 6]])
    prs = np.array([[0.25, 0.9, 0.25], [0.25, 0.25, 0.125]], dtype=F32)
    par, tok, _ = expand_fixed_width(parent, prob, [0, 1], toks, prs, 3)
    assert (par, tok) == ([0, 0, 1], [7, 8, 9])                     # four equal keys: the first three
    # an empty tree: the root itself is the bottom token
    par, tok, _ = expand_fixed_width([], [], [-1], np.array([[3, 4, 5]]), np.array([[.2, .5, .3]], dtype=F32), 2)
    assert (par, tok) == ([-1, -1], [4, 5])


@pytest.mark.parametrize("seed", range(6))
def test_against_all_subsets(seed):
    """The chosen set maximises the sum of cumulative probabilities over all subsets of its size
    (a top-w set does; with distinct keys it is the only one), and it comes out in parent order."""
    rs = np.random.RandomState(seed)
    n = 5
    parent = [-1] + [int(rs.randint(-1, i)) for i in range(1, n)]
    prob = rs.uniform(0.1, 1.0, n).astype(F32)
    bottom = sorted(rs.choice(n, 3, replace=False).tolist())
    k, w = 3, 4
    toks = rs.randint(0, 50, (3, k))
    prs = rs.uniform(0.01, 1.0, (3, k)).astype(F32)
    par, tok, pr = expand_fixed_width(parent, prob, bottom, toks, prs, w)
    assert len(par) == w and par == sorted(par)
    cum = {}
    for b in range(3):
        c = 1.0
        j = bottom[b]
        while j >= 0:                       # float64, leaf upwards: another order on purpose
            c *= float(prob[j])
            j = parent[j]
        for i in range(k):
            cum[(b, i)] = c * float(prs[b, i])
    best = max(itertools.combinations(cum, w), key=lambda s: sum(cum[e] for e in s))
    chosen = set()
    for p_, t_, q_ in zip(par, tok, pr):
        b = bottom.index(p_)
        i = [i for i in range(k) if toks[b, i] == t_ and abs(prs[b, i] - q_) < 1e-7 and (b, i) not in chosen][0]
        chosen.add((b, i))
    assert chosen == set(best)
    # everything chosen is at least as likely as everything left out
    assert min(cum[e] for e in chosen) >= max(cum[e] for e in cum if e not in chosen) - 1e-9


def test_level_never_wider_than_w_over_many_steps():
    rs = np.random.RandomState(11)
    parent, prob = [], []
    bottom = [-1]
    w, k = 8, 4
    for step in range(6):
        toks = rs.randint(0, 1000, (len(bottom), k))
        prs = np.sort(rs.dirichlet(np.ones(k), len(bottom)).astype(F32), axis=1)[:, ::-1]
        par, tok, pr = expand_fixed_width(parent, prob, bottom, toks, prs, w)
        assert len(par) <= w and par == sorted(par)
        first = len(parent)
        parent += par
        prob += pr
        bottom = list(range(first, len(parent)))
    assert len(parent) <= 6 * w
