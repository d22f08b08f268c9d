"""Pins for oracle/tree.py: the (I, P, M) tree of Sec. 3.2 against brute force,
against the block form of layer appending, against rebuilding from survivors, and
against a hand-worked example."""
import os

import numpy as np
import pytest

import workloads as wl
from oracle import SpecTree

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def load_matrix(name):
    return np.loadtxt(os.path.join(GOLD, name), dtype=np.int64, comments="#", ndmin=2)


def build(parents_lib, tokens=None, probs=None):
    """parents in the library numbering (-1 = root)."""
    t = SpecTree(root_token=7)
    n = len(parents_lib)
    tokens = list(range(100, 100 + n)) if tokens is None else tokens
    probs = [0.5 + 0.001 * i for i in range(n)] if probs is None else probs
    t.append([p + 1 for p in parents_lib], tokens, probs)
    return t


def ancestors_by_walk(parents_lib):
    """Brute force: walk the parent list from every node up to the root."""
    n = len(parents_lib) + 1
    M = np.zeros((n, n), dtype=np.uint8)
    full = [-1] + [p + 1 for p in parents_lib]
    for i in range(n):
        j = i
        while j >= 0:
            M[i, j] = 1
            j = full[j]
    return M


TREES = {
    "c1": wl.tree_uniform_parents(0, 16, 6),
    "c2": wl.tree_branching(1, 64, 4, 8),
    "c3": wl.tree_branching(2, 128, 4, 12),
    "chain": wl.tree_chain(9),
    "star": wl.tree_star(11),
    "specinfer": wl.tree_static_levels([1, 1, 3, 1, 1, 1, 1, 1]),
    "one": [-1],
    "big": wl.tree_uniform_parents(5, 255, 40),
}


@pytest.mark.parametrize("name", sorted(TREES))
def test_mask_equals_ancestor_walk(name):
    par = TREES[name]
    t = build(par)
    assert np.array_equal(t.M, ancestors_by_walk(par))
    assert np.array_equal(np.triu(t.M, 1), np.zeros_like(t.M))
    assert np.all(np.diag(t.M) == 1)


@pytest.mark.parametrize("name", sorted(TREES))
def test_parent_and_depth_read_off_M(name):
    par = TREES[name]
    t = build(par)
    p, d, tok, pr, M = t.view()
    assert p.tolist() == list(par)
    assert d.tolist() == wl.levels_of(par)
    assert tok.tolist() == list(range(100, 100 + len(par)))
    assert M.shape == (len(par), len(par))
    assert np.array_equal(M, ancestors_by_walk(par)[1:, 1:])


def test_layer_append_block_structure():
    """Old M top-left, zeros top-right, predecessor rows bottom-left, identity bottom-right."""
    par = wl.bfs_sorted(wl.tree_branching(3, 40, 3, 6))[0]
    lev = wl.levels_of(par)
    t = SpecTree()
    for l in range(max(lev) + 1):
        idx = [i for i in range(len(par)) if lev[i] == l]
        old = t.M.copy()
        n0 = t.n
        t.append_layer([par[i] + 1 for i in idx], [0] * len(idx), [0.0] * len(idx))
        k = len(idx)
        assert np.array_equal(t.M[:n0, :n0], old)
        assert not t.M[:n0, n0:].any()
        assert np.array_equal(t.M[n0:, n0:], np.eye(k, dtype=np.uint8))
        for r, i in enumerate(idx):
            assert np.array_equal(t.M[n0 + r, :n0], old[par[i] + 1])
    assert np.array_equal(t.M, ancestors_by_walk(par))


def test_append_with_parents_inside_the_call_equals_one_by_one():
    par = wl.tree_uniform_parents(9, 60, 30)
    a = build(par)
    b = SpecTree(root_token=7)
    for i, p in enumerate(par):
        b.append_layer([p + 1], [100 + i], [0.5 + 0.001 * i])
    assert np.array_equal(a.M, b.M) and np.array_equal(a.I, b.I) and np.array_equal(a.P, b.P)


def test_append_rejects_forward_parent():
    t = SpecTree()
    with pytest.raises(ValueError):
        t.append([1], [0], [0.0])      # parent index 1 does not exist yet
    with pytest.raises(ValueError):
        t.append_layer([-1], [0], [0.0])


def test_hand_worked_example():
    par_lib = [-1, -1, 0, 0, 1, 2]
    t = build(par_lib)
    assert np.array_equal(t.M, load_matrix("tree7_M.txt"))
    t.to_subtree(1)
    assert np.array_equal(t.M, load_matrix("tree7_subtree1_M.txt"))
    assert t.parent().tolist() == [-1, 0, 0, 1]
    assert t.I.tolist() == [100, 102, 103, 105]


@pytest.mark.parametrize("name", ["c1", "c2", "c3", "specinfer", "big"])
def test_to_subtree_equals_rebuild_from_survivors(name):
    par = TREES[name]
    n = len(par)
    rs = np.random.RandomState(len(par))
    for r in rs.choice(n, size=min(n, 12), replace=False):
        t = build(par)
        m = t.to_subtree(int(r) + 1)
        # survivors by brute force: r and every node whose parent chain passes through r
        surv = [i for i in range(n) if i == r or r in chain_of(par, i)]
        assert np.nonzero(m[1:])[0].tolist() == surv and not m[0]
        new_of = {old: k for k, old in enumerate(surv)}           # k = index in the new tree (root = r = 0)
        fresh = SpecTree(root_token=100 + surv[0], root_prob=np.float32(0.5 + 0.001 * surv[0]))
        fresh.append([new_of[par[i]] for i in surv[1:]], [100 + i for i in surv[1:]],
                     [0.5 + 0.001 * i for i in surv[1:]])
        assert np.array_equal(t.M, fresh.M)
        assert np.array_equal(t.I, fresh.I)
        assert np.array_equal(t.P, fresh.P)


def chain_of(par, i):
    out = []
    j = par[i]
    while j >= 0:
        out.append(j)
        j = par[j]
    return out


def test_bfs_sorted_keeps_the_tree():
    par = wl.tree_uniform_parents(11, 50, 8)
    new_par, order = wl.bfs_sorted(par)
    lev = wl.levels_of(new_par)
    assert lev == sorted(lev)
    # same tree: node order[new] has parent order[new_par[new]]
    for new, old in enumerate(order):
        assert (par[old] == -1 and new_par[new] == -1) or order[new_par[new]] == par[old]
    # within a level, parents are non-decreasing (the order layer appending assumes)
    for a in range(1, len(new_par)):
        if lev[a] == lev[a - 1]:
            assert new_par[a] >= new_par[a - 1]
