"""Pins for pruning propagation in the oracle (Sec. 3.2 to-subtree pruning, Sec. 3.3.2
device-level pruning, Algorithm 1 lines 5-7): brute-force survivor sets, the committed
path landing at the tail of the context in order, prune == rebuild from the survivors
(tables and cache), unchanged positions of the survivors, and prune-then-continue."""
import numpy as np
import pytest

import workloads as wl
from oracle import StageOracle, SpecTree, accept_masks, drop_masks, compact_rows

SMALL = wl.ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, d_head=16, d_ff=96,
                      rms_eps=1e-6, rope_theta=500000.0, dtype="f32")


def make(seed, P, capacity=None, shape=SMALL):
    ws = [wl.layer_weights(shape, seed, l) for l in range(shape.n_layers)]
    pk, pv = zip(*[wl.prefix_kv(shape, seed, l, P) for l in range(shape.n_layers)])
    st = StageOracle(shape, ws)
    st.request_init(0, pk, pv, capacity or P + 300)
    return st


def chain_of(par, i):
    out = []
    j = par[i]
    while j >= 0:
        out.append(j)
        j = par[j]
    return out[::-1]


def tree_of(par):
    t = SpecTree()
    t.append([p + 1 for p in par], list(range(len(par))), [0.0] * len(par))
    return t


PARS = [wl.tree_uniform_parents(0, 16, 6), wl.tree_branching(1, 64, 4, 8),
        wl.tree_uniform_parents(4, 200, 25), wl.tree_chain(5), wl.tree_star(6)]


@pytest.mark.parametrize("par", PARS, ids=["c1", "c2", "deep", "chain", "star"])
def test_masks_by_brute_force(par):
    n = len(par)
    t = tree_of(par)
    for r in range(n):
        path = chain_of(par, r) + [r]
        below = [i for i in range(n) if r in chain_of(par, i)]
        a = accept_masks(t, r + 1)
        assert np.nonzero(a.table_keep)[0].tolist() == [r + 1] + [i + 1 for i in below]
        assert np.nonzero(a.kv_keep)[0].tolist() == sorted([0] + [i + 1 for i in path + below])
        assert a.n_commit == len(path)
        d = drop_masks(t, r + 1)
        assert np.nonzero(d.table_keep)[0].tolist() == [0] + [i + 1 for i in range(n) if i != r and i not in below]
        assert np.array_equal(d.table_keep, d.kv_keep) and d.n_commit == 0
        # the two prunes of one node split the speculative nodes between them, but for the path
        assert not np.any(a.table_keep[1:] & d.table_keep[1:])


def test_compact_rows_is_a_stable_selection_for_any_dtype():
    rows = np.arange(40, dtype=np.uint16).reshape(10, 4)
    keep = np.array([1, 0, 0, 1, 1, 0, 1, 0, 0, 1], bool)
    assert compact_rows(rows, keep).tolist() == [rows[i].tolist() for i in (0, 3, 4, 6, 9)]
    with pytest.raises(ValueError):
        compact_rows(rows, keep[:5])


@pytest.mark.parametrize("mode", ["accept_root_child", "accept_deep", "drop"])
def test_prune_equals_rebuild_and_reforward(mode):
    """After a prune, tables and cache equal those of a stage that was only ever given the
    survivors: the committed path as ordinary context, the kept nodes as its tree."""
    P = 20
    par = wl.tree_branching(12, 28, 3, 6)
    n = len(par)
    x = wl.hidden_rows(SMALL, 12, ("p",), n)
    lev = wl.levels_of(par)
    if mode == "accept_root_child":
        r = [i for i in range(n) if par[i] < 0][0]
    elif mode == "accept_deep":
        r = [i for i in range(n) if lev[i] == 2 and i in par][0]
    else:
        r = [i for i in range(n) if lev[i] == 1 and i in par][0]

    a = make(12, P)
    a.tree_insert(0, par, tokens=list(range(n)), probs=[i / 100 for i in range(n)])
    a.stage_forward(0, 0, x)
    pos_before = (a.req[0].P - 1) + a.req[0].tree.depth()
    pr = a.accept(0, r) if mode != "drop" else a.drop(0, r)

    below = [i for i in range(n) if r in chain_of(par, i)]
    if mode == "drop":
        path, surv = [], [i for i in range(n) if i != r and i not in below]
    else:
        path, surv = chain_of(par, r) + [r], below
    assert a.req[0].P == P + len(path)
    # positions of the survivors did not change, so their rotated K rows stay valid
    pos_after = (a.req[0].P - 1) + a.req[0].tree.depth()
    assert pos_after[1:].tolist() == [pos_before[i + 1] for i in surv]

    b = make(12, P)
    if path:                                   # the committed path, decoded as a chain and accepted
        b.tree_insert(0, wl.tree_chain(len(path)))
        b.stage_forward(0, 0, x[path])
        b.accept(0, len(path) - 1)
    new_of = {old: k for k, old in enumerate(surv)}
    b.tree_insert(0, [new_of.get(par[i], -1) for i in surv], tokens=surv, probs=[i / 100 for i in surv])
    b.stage_forward(0, 0, x[surv])

    ta, tb = a.req[0].tree, b.req[0].tree
    assert np.array_equal(ta.M, tb.M)
    assert np.array_equal(ta.I[1:], tb.I[1:]) and np.array_equal(ta.P[1:], tb.P[1:])
    assert a.req[0].P == b.req[0].P
    hi = a.req[0].P + len(surv)
    for l in range(SMALL.n_layers):
        assert np.allclose(a.req[0].K[l][:hi], b.req[0].K[l][:hi], rtol=1e-12, atol=1e-12)
        assert np.allclose(a.req[0].V[l][:hi], b.req[0].V[l][:hi], rtol=1e-12, atol=1e-12)

    # prune, then keep going: new children under the survivors give the same outputs on both
    if surv:
        more = [len(surv) - 1, -1, len(surv)]
        xm = wl.hidden_rows(SMALL, 12, ("more",), len(more))
        fa = a.tree_insert(0, more)
        fb = b.tree_insert(0, more)
        assert fa == fb == len(surv)
        assert np.allclose(a.stage_forward(0, fa, xm), b.stage_forward(0, fb, xm), rtol=1e-12, atol=1e-12)


def test_committed_path_lands_at_the_tail_in_order():
    P = 10
    par = [-1, 0, 0, 1, 3, -1, 4, 2]
    a = make(3, P)
    a.tree_insert(0, par)
    a.stage_forward(0, 0, wl.hidden_rows(SMALL, 3, ("o",), len(par)))
    before = [a.req[0].K[l].copy() for l in range(SMALL.n_layers)]
    a.accept(0, 4)                                  # path 0 -> 1 -> 3 -> 4, survivor 6
    assert a.req[0].P == P + 4
    for l in range(SMALL.n_layers):
        K = a.req[0].K[l]
        assert np.array_equal(K[:P], before[l][:P])
        for k, node in enumerate([0, 1, 3, 4, 6]):
            assert np.array_equal(K[P + k], before[l][P + node])
    assert a.req[0].tree.view()[0].tolist() == [-1]


def test_hidden_rows_follow_the_table_mask():
    par = [-1, 0, 0, -1, 3]
    t = tree_of(par)
    rows = np.arange(5 * 3).reshape(5, 3)
    pr = accept_masks(t, 1)                          # accept node 0: keeps 0 (new root), 1, 2
    assert StageOracle.prune_hidden_rows(rows, [0, 1, 2, 3, 4], pr).tolist() == rows[[0, 1, 2]].tolist()
    pr = drop_masks(t, 4)                            # drop node 3 and its child
    assert StageOracle.prune_hidden_rows(rows[[1, 3, 4]], [1, 3, 4], pr).tolist() == rows[[1]].tolist()


def test_accept_everything_and_empty_tree():
    a = make(1, 8)
    a.tree_insert(0, [-1])
    a.stage_forward(0, 0, wl.hidden_rows(SMALL, 1, ("e",), 1))
    pr = a.accept(0, 0)
    assert pr.n_commit == 1 and a.req[0].tree.n == 1 and a.req[0].P == 9
    # the next level hangs off the new tail
    assert a.tree_insert(0, [-1, -1]) == 0
    assert a.req[0].tree.view()[1].tolist() == [0, 0]
