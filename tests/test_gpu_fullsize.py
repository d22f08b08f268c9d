"""The named configurations at their own size and depth: the 70B-shaped stage with all 10 layers and 128
nodes, the streaming schedule on the 4-layer 8B-shaped stage behind a 32768-token context (trees of more
than 64 live nodes included), and the 32-request batch with its cold step and steady steps.  Every output
row the oracle follows is compared element by element; tables, fresh K/V rows and compaction as in the
small cases.  These are the slow GPU tests (the float64 oracle gathers every visible key per node and KV
head): each prints its progress."""
import time

import numpy as np
import pytest
import torch

import workloads as wl
import paper_2504_04104_amd as sp
from gpu_harness import Pair, elementwise_figure, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu

TOL = 2e-2


def say(*a):
    print(*a, flush=True)


def test_c3_all_ten_layers():
    """Config 3: 10 decoder layers at d=8192, 64/8 heads, FFN 28672 (17 GB of bf16 weights), context 4096,
    the 128-node tree: bf16 parity through the whole depth.  The oracle takes the weights one layer at a
    time (6.8 GB in float64); the host keeps them as bf16 bit patterns in between."""
    w = wl.CONFIGS["C3"]
    shape = w.shape
    t0 = time.time()
    bits = {}

    def layer(l):
        if l not in bits:
            ww = wl.layer_weights(shape, w.seed, l)
            bits[l] = {k: wl.to_bf16_bits(v) for k, v in ww.items()}
            say("C3 layer", l, "weights drawn, %.0f s" % (time.time() - t0))
            return ww
        say("C3 layer", l, "to the oracle, %.0f s" % (time.time() - t0))
        return {k: wl.from_bf16_bits(v) for k, v in bits[l].items()}

    pair = Pair(shape, w.seed, {0: w.prefix_len}, max_batch_nodes=128, flags=sp.SP_FLAG_PACKED_WEIGHTS, weights=layer)
    par = wl.tree_branching(w.seed, w.n_nodes, w.max_children, w.max_levels)
    x = wl.hidden_rows(shape, w.seed, ("x",), w.n_nodes)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [w.n_nodes], x)
    e = rel_err(y, ref)
    say("C3 full depth: rel err %.3e over %d layers; increment: rel %.3e, element-wise figure %.2f (a = 1e-2 rms)"
        % (e, shape.n_layers, rel_err(y - x, ref - x), elementwise_figure(y - x, ref - x, TOL)))
    assert e <= TOL
    assert rel_err(y - x, ref - x) <= TOL
    pair.check_kv(0, TOL)
    pair.check_tables(0)
    roots = [i for i, p in enumerate(par) if p < 0]
    pair.prune(0, sp.SP_ACCEPT, roots[0], x_rows=y, row_nodes=list(range(w.n_nodes)))
    pair.close()


def f64_weights(shape, seed):
    """Layer weights converted to float64 once, so that the oracle does not convert them again on every call."""
    return [{k: v.astype(np.float64) for k, v in wl.layer_weights(shape, seed, l).items()} for l in range(shape.n_layers)]


def test_c4_four_layers_streaming_with_large_trees():
    """Config 4: the 4-layer stage behind a 32768-token context.  The first call forwards an 80-node tree
    (more rows than one 64-row block, a tree region longer than two attention tiles in the last of the 32
    chunks); the streaming steps that follow insert 1-8 nodes under a live tree of 60-85 nodes, then under
    small ones; prune + compaction of the cache and of the in-flight rows after every step."""
    w = wl.CONFIGS["C4"]
    shape = w.shape
    t0 = time.time()
    w64 = f64_weights(shape, w.seed)
    say("C4 weights drawn, %.0f s" % (time.time() - t0))
    pair = Pair(shape, w.seed, {0: w.prefix_len}, tree_room=320, max_batch_nodes=128, flags=sp.SP_FLAG_PACKED_WEIGHTS,
                weights=w64.__getitem__)
    init = wl.tree_deep(w.seed, 80, 12, window=6, name=("c4init", 2))
    host = wl._HostTree()
    host.parents = list(init)
    host.apply(wl.PruneOp(wl.ACCEPT, 0))
    steps = [wl.StreamStep(init, wl.PruneOp(wl.ACCEPT, 0))]
    steps += wl.streaming_schedule(w.seed, 8, max_new=8, cap=256, p_accept=0.7, name=("c4full", 2), initial=host.parents)
    worst, big = 0.0, 0
    for s_, st in enumerate(steps):
        n = len(st.parents)
        first = pair.insert(0, st.parents)
        live = first + n
        big += live > 64
        x = wl.hidden_rows(shape, w.seed, ("full", s_), n)
        y, ref = pair.forward([0], [first], [n], x)
        e = rel_err(y, ref)
        worst = max(worst, e)
        say("C4 step %d: %d new nodes under %d live, rel err %.3e, increment rel %.3e, %.0f s"
            % (s_, n, live, e, rel_err(y - x, ref - x), time.time() - t0))
        assert e <= TOL and rel_err(y - x, ref - x) <= TOL
        pair.check_kv(0, TOL)
        if st.prune is not None:
            pair.prune(0, st.prune.mode, st.prune.node, x_rows=y, row_nodes=list(range(first, first + n)))
    assert big >= 4                      # forward calls that ran on a tree of more than 64 live nodes
    assert len(steps) >= 9
    say("C4 worst rel err %.3e" % worst)
    pair.close()


def test_c5_four_layers_cold_and_steady_steps():
    """Config 5: 32 requests (contexts of 512-4096 tokens, trees of 8-32 nodes) on the 4-layer stage: the cold
    step forwards every tree in one call, two steady steps then prune every request (batched), compact
    (batched), insert (batched) and forward the new nodes.  The GPU runs all 32 requests; the oracle follows
    four of them (first, last, largest and smallest tree) through every step."""
    w = wl.CONFIGS["C5"]
    shape = w.shape
    t0 = time.time()
    reqs = wl.batch_requests(w.seed, n_req=32, p_lo=512, p_hi=4096, t_lo=8, t_hi=32, max_levels=6)
    sizes = [len(r.parents) for r in reqs]
    sample = sorted({0, 31, int(np.argmax(sizes)), int(np.argmin(sizes))})
    w64 = f64_weights(shape, w.seed)
    say("C5 weights drawn, %.0f s; oracle follows requests" % (time.time() - t0), sample)
    pair = Pair(shape, w.seed, {r.req: r.prefix_len for r in reqs}, tree_room=64, max_batch_nodes=sum(sizes),
                flags=sp.SP_FLAG_PACKED_WEIGHTS, oracle_reqs=sample, weights=w64.__getitem__)
    g = pair.gpu
    ids = [r.req for r in reqs]

    def forward_and_compare(tag, act, firsts, counts, x):
        y = to_np(g.stage_forward(act, firsts, counts, to_dev(x, g)))
        assert np.isfinite(y).all()
        row0 = np.concatenate([[0], np.cumsum(counts)])
        worst = 0.0
        for i, r in enumerate(act):
            if r in sample and counts[i]:
                xr = x[row0[i]:row0[i + 1]]
                ref = pair.ora.stage_forward(r, firsts[i], xr)
                e = rel_err(y[row0[i]:row0[i + 1]], ref)
                worst = max(worst, e)
                assert e <= TOL, (tag, r, e)
                assert rel_err(y[row0[i]:row0[i + 1]] - xr, ref - xr) <= TOL, (tag, r)
                pair.check_kv(r, TOL)
                pair.check_tables(r)
        say("C5 %s: %d rows, worst rel err over the followed requests %.3e, %.0f s" % (tag, sum(counts), worst, time.time() - t0))

    pair.insert_batch(ids, [r.parents for r in reqs])
    forward_and_compare("cold step", ids, [0] * 32, sizes, wl.hidden_rows(shape, w.seed, ("cold",), sum(sizes)))
    sched = wl.batch_schedule(w.seed, reqs, 2, max_new=8, max_levels=6)
    for s_, row in enumerate(sched):
        modes = [st.prune.mode if st.prune else -1 for st in row]
        nodes = [st.prune.node if st.prune else 0 for st in row]
        before = {}
        for r, st in zip(reqs, row):
            if st.prune and r.req in sample:
                o = pair.ora.req[r.req]
                before[r.req] = (o.P, pair.tree_region(r.req, o.P, o.tree.n - 1), pair.rows(r.req, 0, o.P))
        live, commit = g.tree_prune_batch(ids, modes, nodes)
        g.kv_compact_batch([i for i, m in zip(ids, modes) if m >= 0])
        for i, (r, st) in enumerate(zip(reqs, row)):
            if not (st.prune and r.req in sample):
                continue
            pr = pair.ora.accept(r.req, st.prune.node) if st.prune.mode == sp.SP_ACCEPT else pair.ora.drop(r.req, st.prune.node)
            assert commit[i] == pr.n_commit and live[i] == pair.ora.req[r.req].tree.n - 1
            P_old, reg, ctx = before[r.req]
            keep = pr.kv_keep[1:]
            sel = torch.from_numpy(np.nonzero(keep)[0]).to(reg.device)
            after = pair.tree_region(r.req, P_old, int(keep.sum()))
            assert torch.equal(after.view(torch.uint8), reg.index_select(3, sel).contiguous().view(torch.uint8))
            assert torch.equal(pair.rows(r.req, 0, P_old).view(torch.uint8), ctx.view(torch.uint8))
            pair.check_tables(r.req)
        act = [r.req for r, st in zip(reqs, row) if st.parents]
        new = [st.parents for st in row if st.parents]
        counts = [len(p) for p in new]
        firsts = pair.insert_batch(act, new)
        forward_and_compare("steady step %d" % s_, act, firsts, counts, wl.hidden_rows(shape, w.seed, ("steady", s_), sum(counts)))
    pair.close()
