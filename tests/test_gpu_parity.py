"""HIP path against the CPU oracle, through the C ABI, on seeded inputs.

Bars: bit-exact for tables (parent, depth, token, prob, mask) and for cache/hidden-row
compaction; hidden states and freshly written K/V rows within max|gpu - oracle| / max|oracle|
<= 2e-2 for bf16 storage (the oracle computes in float64 from the same bf16-rounded weights,
inputs and context) and <= 2e-4 for float32 storage (float32 accumulation over up to
14336 terms against float64)."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2504_04104_amd as sp
from gpu_harness import Pair, rel_err, to_dev, to_np

pytestmark = pytest.mark.gpu

TOL = {"bf16": 2e-2, "f32": 2e-4}

# small shapes that still span several tiles of every kernel and leave ragged tails
MINI_BF16 = wl.ModelShape(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=2, d_head=128, d_ff=768)
MINI_GQA4 = wl.ModelShape(n_layers=2, d_model=768, n_q_heads=8, n_kv_heads=2, d_head=128, d_ff=1280)
MINI_F32 = wl.ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, d_head=64, d_ff=688,
                         rms_eps=1e-6, dtype="f32")


def say(*a):
    print(*a, flush=True)


# ---------------------------------------------------------------------------------------
def test_c1_tiny_fp32_forward_drop_compact():
    """Config 1: 2 layers, d=256, 4 heads of 64, FFN 688, fp32, prefix 128, 16 nodes."""
    w = wl.CONFIGS["C1"]
    say("C1", w.shape)
    pair = Pair(w.shape, w.seed, {0: w.prefix_len})
    par = wl.tree_uniform_parents(w.seed, w.n_nodes, w.max_levels)
    x = wl.hidden_rows(w.shape, w.seed, ("c1",), w.n_nodes)
    pair.insert(0, par, tokens=list(range(100, 116)), probs=[0.5 + i / 64 for i in range(16)])
    pair.check_tables(0)
    y, ref = pair.forward([0], [0], [w.n_nodes], x)
    e = rel_err(y, ref)
    say("C1 rel err", e)
    assert e <= TOL["f32"]
    pair.check_kv(0, TOL["f32"])
    node = int(wl.rng(w.seed, "c1drop").integers(0, w.n_nodes))
    pair.prune(0, sp.SP_DROP, node, x_rows=y, row_nodes=list(range(w.n_nodes)))
    pair.close()


@pytest.mark.parametrize("flags", [sp.SP_FLAG_SIMPLE_KERNELS, 0, sp.SP_FLAG_PACKED_WEIGHTS],
                         ids=["simple", "mfma", "mfma_packed"])
@pytest.mark.parametrize("shape", [MINI_BF16, MINI_GQA4], ids=["g2", "g4"])
def test_mini_bf16_forward(shape, flags):
    """Several attention tiles with a ragged tail (prefix 300), 37 nodes (ragged M), both kernel sets."""
    say("mini bf16", shape, flags)
    pair = Pair(shape, 11, {0: 300}, flags=flags)
    par = wl.tree_branching(11, 37, 3, 7)
    x = wl.hidden_rows(shape, 11, ("m",), 37)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [37], x)
    e = rel_err(y, ref)
    say("rel err", e)
    assert e <= TOL["bf16"]
    pair.check_kv(0, TOL["bf16"])
    pair.close()


def test_mini_f32_gqa_forward_in_pieces():
    """fp32, grouped heads, nodes forwarded over several calls in ancestor order."""
    pair = Pair(MINI_F32, 12, {0: 77})
    par = wl.bfs_sorted(wl.tree_branching(12, 29, 3, 6))[0]
    x = wl.hidden_rows(MINI_F32, 12, ("p",), 29)
    cuts = [0, 2, 9, 10, 29]
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        pair.insert(0, par[lo:hi])
        y, ref = pair.forward([0], [lo], [hi - lo], x[lo:hi])
        assert rel_err(y, ref) <= TOL["f32"]
    pair.check_tables(0)
    pair.check_kv(0, TOL["f32"])
    pair.close()


@pytest.mark.parametrize("n", [1, 15, 16, 17, 33, 64, 65, 128, 130, 255, 256])
def test_row_counts_across_tile_edges(n):
    """M below, at and above the 16-row MFMA tile and the 64-row block."""
    shape = MINI_BF16
    pair = Pair(shape, 13, {0: 129}, max_batch_nodes=256, flags=sp.SP_FLAG_PACKED_WEIGHTS if n % 2 else 0)
    par = wl.tree_uniform_parents(13, n, 9, name=("t", n))
    x = wl.hidden_rows(shape, 13, ("r", n), n)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [n], x)
    e = rel_err(y, ref)
    say("n", n, "rel err", e)
    assert e <= TOL["bf16"]
    pair.close()


@pytest.mark.parametrize("d_ff,n,packed", [(2048, 17, True), (6144, 33, False), (10240, 48, True), (14336, 64, True),
                                           (14336, 50, False), (16384, 64, False), (14336, 16, True), (14336, 20, False),
                                           (14336, 40, True), (14336, 100, True), (16384, 128, False), (14336, 65, False)])
def test_ffn_widths_by_increment(d_ff, n, packed):
    """The FFN at several widths up to the 8B shape's, both weight layouts, ragged row counts from two row
    tiles to the 128-row block (d_ff = 14336 and 16384 give each of 256 CUs 56 and 64 gate/up columns: the
    one-workgroup-per-CU kernel with a short and with a full last column group).  Small inputs and the
    increment y - x element by element, so that a wrong strip of gate/up columns or a wrong split of the down
    projection cannot hide behind the residual."""
    from gpu_harness import elementwise_figure
    shape = wl.ModelShape(n_layers=1, d_model=512, n_q_heads=4, n_kv_heads=2, d_head=128, d_ff=d_ff)
    pair = Pair(shape, 61, {0: 40}, max_batch_nodes=128, flags=sp.SP_FLAG_PACKED_WEIGHTS if packed else 0)
    par = wl.tree_uniform_parents(61, n, 9, name=("gu", n))
    x = wl.hidden_rows(shape, 61, ("gu", n), n) * np.float32(2.0 ** -6)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [n], x)
    inc_gpu, inc_ref = y.astype(np.float64) - x, ref - x
    e = float(np.max(np.abs(inc_gpu - inc_ref)) / np.max(np.abs(inc_ref)))
    fig = elementwise_figure(inc_gpu, inc_ref, 2e-2, 5e-2)
    say("d_ff", d_ff, "rows", n, ": increment rel err %.3e, element-wise figure %.2f" % (e, fig))
    assert e <= TOL["bf16"] and fig <= 1.0
    pair.close()


def test_empty_and_degenerate_calls():
    """Calls that carry no work leave everything as it was and report success: an insert of no
    nodes, a forward / output head over no nodes (alone and as an empty request inside a batch), a
    compaction without hidden rows, an expansion of width 0; a one-node tree accepted (the tree
    becomes empty, the context grows by one) and a chain accepted at its leaf (the whole chain is
    committed)."""
    shape = MINI_BF16
    pair = Pair(shape, 19, {0: 30, 1: 17}, vocab=128)
    g = pair.gpu
    assert g.tree_insert(0, []) == 0
    x0 = torch.empty((0, shape.d_model), dtype=torch.bfloat16, device="cuda:0")
    assert g.stage_forward([0], [0], [0], x0).shape[0] == 0
    assert g.verify_head(pair.head, [0], [0], [0], x0).shape[0] == 0
    assert g.tree_expand(0, [-1], torch.tensor([[5, 6]], dtype=torch.int32).cuda(), torch.tensor([[.5, .5]]).cuda(), 0) == ([], [], [])
    pair.check_tables(0)
    # request 1 has no new nodes in a batched call
    pair.insert(0, [-1, 0, 1])
    x = wl.hidden_rows(shape, 19, ("e",), 3)
    y, ref = pair.forward([0, 1], [0, 0], [3, 0], x)
    assert rel_err(y, ref) <= TOL["bf16"]
    # a chain accepted at its leaf: three tokens committed, nothing left
    live, commit = g.tree_prune(0, sp.SP_ACCEPT, 2)
    pair.ora.accept(0, 2)
    assert (live, commit) == (0, 3)
    g.kv_compact(0)
    pair.check_tables(0)
    assert g.request_info(0)[:2] == (33, 0)
    # a one-node tree
    pair.insert(1, [-1])
    x1 = wl.hidden_rows(shape, 19, ("e1",), 1)
    y, ref = pair.forward([1], [0], [1], x1)
    assert rel_err(y, ref) <= TOL["bf16"]
    pair.prune(1, sp.SP_ACCEPT, 0)
    assert g.request_info(1)[:2] == (18, 0)
    # clearing an empty tree is allowed and changes nothing
    pair.prune(1, sp.SP_CLEAR, 0)
    assert g.request_info(1)[:2] == (18, 0)
    assert g.tree_match([0, 1]) == [-1, -1]
    pair.close()


def test_paged_cache_f32_and_page_accounting():
    """The plain (fp32) kernels on a paged cache, and the allocator's bookkeeping: pages follow the
    live slots, an insert that would need more pages than are free fails without changing anything,
    a release returns every page."""
    shape = MINI_F32
    PG = 32
    pair = Pair(shape, 25, {0: 70, 1: 45}, tree_room=64, page_slots=PG)
    g = pair.gpu
    total_pages = g.sizes.kv_bytes // (shape.n_layers * 2 * shape.n_kv_heads * shape.d_head * 4) // PG
    assert len(g.request_pages(0)) == 3 and len(g.request_pages(1)) == 2
    assert g.free_pages() == total_pages - 5
    assert sorted(g.request_pages(0) + g.request_pages(1)) != g.request_pages(0) + g.request_pages(1)   # out of order
    par = wl.tree_uniform_parents(25, 30, 6, name=("pg",))
    x = wl.hidden_rows(shape, 25, ("pg",), 30)
    pair.insert(0, par)
    assert len(g.request_pages(0)) == 4                                   # 70 + 30 slots
    y, ref = pair.forward([0], [0], [30], x)
    assert rel_err(y, ref) <= TOL["f32"]
    pair.check_kv(0, TOL["f32"])
    roots = [i for i, p in enumerate(par) if p < 0]
    pair.prune(0, sp.SP_DROP, roots[0], x_rows=y, row_nodes=list(range(30)))
    pair.check_kv(0, TOL["f32"])
    # another request takes all free pages but one; request 1 then asks for two more
    free = g.free_pages()
    g.request_init(2, 0, (free - 1) * PG, (free - 1) * PG)
    assert g.free_pages() == 1
    with pytest.raises(sp.SpError) as ei:
        g.tree_insert(1, [-1] * 64)                                       # 45 + 64 slots = 4 pages, 2 held
    assert ei.value.status == -2                                          # SP_E_CAPACITY
    assert g.free_pages() == 1 and g.request_info(1)[1] == 0 and len(g.request_pages(1)) == 2
    pair.insert(1, [-1] * 40)                                             # 85 slots = 3 pages: takes the last one
    assert g.free_pages() == 0
    x1 = wl.hidden_rows(shape, 25, ("pg1",), 40)
    y, ref = pair.forward([1], [0], [40], x1)
    assert rel_err(y, ref) <= TOL["f32"]
    g.request_release(2)
    g.request_release(0)
    g.request_release(1)
    assert g.free_pages() == total_pages
    pair.close()


def test_forward_replays_from_a_hip_graph():
    """sp_stage_forward only enqueues kernels on the caller's stream (no allocation, no host wait, no
    memset), so a caller may capture it into a HIP graph.  Replays are interleaved with eager calls and
    host synchronisation, and each replay is compared with the eager result for the same input rows."""
    shape = MINI_BF16
    pair = Pair(shape, 26, {0: 90}, flags=sp.SP_FLAG_PACKED_WEIGHTS, oracle=True)
    g = pair.gpu
    n = 21
    pair.insert(0, wl.tree_uniform_parents(26, n, 6, name=("g",)))
    xs = [to_dev(wl.hidden_rows(shape, 26, ("g", i), n), g) for i in range(4)]
    x = xs[0].clone()
    y = torch.empty_like(x)
    y_ref, ref = pair.forward([0], [0], [n], wl.hidden_rows(shape, 26, ("g", 0), n))     # eager, also warms up
    assert rel_err(y_ref, ref) <= TOL["bf16"]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            g.stage_forward([0], [0], [n], x, y)
    torch.cuda.current_stream().wait_stream(side)
    for i in (1, 2, 3, 0, 2):
        x.copy_(xs[i])
        graph.replay()
        torch.cuda.synchronize()
        got = y.clone()
        eager = g.stage_forward([0], [0], [n], xs[i])                     # eager call between replays
        torch.cuda.synchronize()
        assert torch.equal(got.view(torch.int16), eager.view(torch.int16)), i
    pair.close()


def test_forward_graph_of_its_own_matches_eager_calls():
    """On a stream that can be captured the forward call replays a graph of its own launches from the
    second time a shape is seen.  The same steps on a stage that may not (SP_FLAG_NO_GRAPHS) must give
    the same bits, call after call, with other shapes and a prune in between."""
    shape = MINI_GQA4
    a = Pair(shape, 27, {0: 70}, flags=sp.SP_FLAG_PACKED_WEIGHTS, oracle=False)
    b = Pair(shape, 27, {0: 70}, flags=sp.SP_FLAG_PACKED_WEIGHTS | sp.SP_FLAG_NO_GRAPHS, oracle=False)
    assert torch.cuda.current_stream() != torch.cuda.default_stream()
    par = wl.tree_uniform_parents(27, 19, 5, name=("r",))
    for rep in range(5):
        outs = []
        for pair in (a, b):
            g = pair.gpu
            g.request_init(0, pair.base[0], pair.cap[0], 70)
            g.tree_insert(0, par)
            x = to_dev(wl.hidden_rows(shape, 27, ("r", rep), 19), g)
            y = g.stage_forward([0], [0], [19], x)                      # shape seen again: replayed on `a`
            g.tree_insert(0, [3, 3, 7])
            y2 = g.stage_forward([0], [19], [3], to_dev(wl.hidden_rows(shape, 27, ("r2", rep), 3), g))
            g.tree_prune(0, sp.SP_DROP, 2)
            g.kv_compact(0)
            outs.append((y.clone(), y2.clone(), pair.rows(0, 0, 70 + 22)))
        torch.cuda.synchronize()
        for u, v in zip(outs[0], outs[1]):
            assert torch.equal(u.view(torch.int16), v.view(torch.int16)), rep
    a.close()
    b.close()


def test_tables_only_random_sequences():
    """Insert / accept / drop sequences up to the 256-node cap: tables bit-exact after every call."""
    pair = Pair(MINI_F32, 14, {0: 5}, tree_room=4096, max_batch_nodes=256)
    g = wl.rng(14, "seq")
    n_live = 0

    def forward_zeros(first, k):
        # an accept commits the K/V rows of the accepted path, so they must exist: the library refuses
        # to accept a node that was never forwarded
        if k:
            pair.gpu.stage_forward([0], [first], [k], torch.zeros(k, MINI_F32.d_model, device="cuda:0"))

    for step in range(60):
        room = 256 - n_live
        k = int(g.integers(0, min(room, 40) + 1))
        parents = [int(g.integers(-1, n_live + i)) for i in range(k)]
        toks = [int(g.integers(0, 1 << 20)) for _ in range(k)]
        prbs = [float(g.random()) for _ in range(k)]
        forward_zeros(pair.insert(0, parents, toks, prbs), k)
        n_live += k
        pair.check_tables(0)
        if n_live and g.random() < 0.8:
            node = int(g.integers(0, n_live))
            mode = sp.SP_ACCEPT if g.random() < 0.5 else sp.SP_DROP
            pair.prune(0, mode, node)
            n_live = pair.gpu.request_info(0)[1]
    # fill to the cap exactly, then prune at the last node
    forward_zeros(pair.insert(0, [-1] * (256 - n_live)), 256 - n_live)
    pair.check_tables(0)
    pair.prune(0, sp.SP_DROP, 255)
    pair.prune(0, sp.SP_ACCEPT, 0)
    pair.close()


@pytest.mark.parametrize("page_slots", [0, 32, 128], ids=["contiguous", "pages32", "pages128"])
def test_streaming_mini(page_slots):
    """Config 4 in miniature: per step insert 1-8 nodes, forward only those, prune, compact
    (cache and in-flight hidden rows); every step checked.  Also with the cache in pages that
    the request holds out of physical order and returns as the tree shrinks."""
    shape = MINI_BF16
    pair = Pair(shape, 15, {0: 200}, tree_room=700, flags=sp.SP_FLAG_PACKED_WEIGHTS, page_slots=page_slots)
    steps = wl.streaming_schedule(15, 40, max_new=8, cap=256, p_accept=0.7)
    worst = 0.0
    for s, st in enumerate(steps):
        n = len(st.parents)
        first = pair.insert(0, st.parents)
        y = None
        if n:
            x = wl.hidden_rows(shape, 15, ("s", s), n)
            y, ref = pair.forward([0], [first], [n], x)
            worst = max(worst, rel_err(y, ref))
        if st.prune is not None:
            if y is not None:
                pair.prune(0, st.prune.mode, st.prune.node, x_rows=y, row_nodes=list(range(first, first + n)))
            else:
                pair.prune(0, st.prune.mode, st.prune.node)
        pair.check_kv(0, TOL["bf16"])
    say("streaming worst rel err", worst)
    assert worst <= TOL["bf16"]
    pair.close()


@pytest.mark.parametrize("page_slots", [0, 64], ids=["contiguous", "pages64"])
def test_ragged_batch_mini(page_slots):
    """Config 5 in miniature: several requests with their own prefix and tree in one call;
    block-diagonal masks; batched prune + compaction.  Also with a paged cache shared by the
    requests (the storage of the multi-request version, Sec. 4 "Implementation")."""
    shape = MINI_GQA4
    reqs = wl.batch_requests(16, n_req=5, p_lo=40, p_hi=333, t_lo=3, t_hi=20, max_levels=5)
    pair = Pair(shape, 16, {r.req: r.prefix_len for r in reqs}, max_batch_nodes=128, page_slots=page_slots)
    for r in reqs:
        pair.insert(r.req, r.parents)
    counts = [len(r.parents) for r in reqs]
    x = wl.hidden_rows(shape, 16, ("b",), sum(counts))
    y, ref = pair.forward([r.req for r in reqs], [0] * len(reqs), counts, x)
    e = rel_err(y, ref)
    say("batch cold rel err", e)
    assert e <= TOL["bf16"]
    sched = wl.batch_schedule(16, reqs, 6, max_new=6, max_levels=5)
    for s, row in enumerate(sched):
        # batched prune + compaction
        ids = [r.req for r in reqs]
        modes = [st.prune.mode if st.prune else -1 for st in row]
        nodes = [st.prune.node if st.prune else 0 for st in row]
        before = {}
        for r, st in zip(reqs, row):
            if st.prune:
                o = pair.ora.req[r.req]
                before[r.req] = (o.P, o.tree.n - 1, pair.tree_region(r.req, o.P, o.tree.n - 1))
        live, commit = pair.gpu.tree_prune_batch(ids, modes, nodes)
        act = [i for i, m in zip(ids, modes) if m >= 0]
        pair.gpu.kv_compact_batch(act)
        for i, (r, st) in enumerate(zip(reqs, row)):
            if not st.prune:
                continue
            pr = pair.ora.accept(r.req, st.prune.node) if st.prune.mode == sp.SP_ACCEPT else pair.ora.drop(r.req, st.prune.node)
            assert commit[i] == pr.n_commit
            P_old, T_old, reg = before[r.req]
            keep = pr.kv_keep[1:]
            sel = torch.from_numpy(np.nonzero(keep)[0]).to(reg.device)
            after = pair.tree_region(r.req, P_old, int(keep.sum()))
            assert torch.equal(after.view(torch.uint8), reg.index_select(3, sel).contiguous().view(torch.uint8))
            pair.check_tables(r.req)
        # batched insert: one launch for all requests with new nodes (tokens and probabilities too)
        act_ids = [r.req for r, st in zip(reqs, row) if st.parents]
        new = [st.parents for st in row if st.parents]
        counts = [len(p) for p in new]
        toks = [[1000 * s + 10 * i + k for k in range(len(p))] for i, p in enumerate(new)]
        prbs = [[(k + 1) / 64.0 for k in range(len(p))] for p in new]
        firsts = pair.insert_batch(act_ids, new, toks, prbs) if act_ids else []
        for rid in act_ids:
            pair.check_tables(rid)
        if act_ids:
            x = wl.hidden_rows(shape, 16, ("b", s), sum(counts))
            y, ref = pair.forward(act_ids, firsts, counts, x)
            e = rel_err(y, ref)
            assert e <= TOL["bf16"], (s, e)
    pair.close()


@pytest.mark.parametrize("page_slots", [0, 32], ids=["contiguous", "pages32"])
def test_ragged_batch_of_64_requests(page_slots):
    """The largest batch one call takes (64 requests): contexts of 1-120 tokens, trees of 1-3 nodes, one forward
    call, a batched prune and compaction of every request, a batched insert and a second forward call; one
    request more than the maximum is refused before anything is launched."""
    shape = MINI_GQA4
    reqs = wl.batch_requests(23, n_req=64, p_lo=1, p_hi=120, t_lo=1, t_hi=3, max_levels=3, name=("batch64",))
    pair = Pair(shape, 23, {r.req: r.prefix_len for r in reqs}, max_batch_nodes=256, page_slots=page_slots)
    for r in reqs:
        pair.insert(r.req, r.parents)
    ids = [r.req for r in reqs]
    counts = [len(r.parents) for r in reqs]
    x = wl.hidden_rows(shape, 23, ("b64",), sum(counts))
    y, ref = pair.forward(ids, [0] * 64, counts, x)
    e = rel_err(y, ref)
    say("64 requests, first call rel err", e, "rows", sum(counts))
    assert e <= TOL["bf16"]
    one_more = torch.zeros(sum(counts) + 1, shape.d_model, dtype=pair.gpu.tdtype, device="cuda")
    with pytest.raises(sp.SpError):                 # the library's own check: 65 requests in one call
        pair.gpu.stage_forward(ids + [0], [0] * 65, counts + [1], one_more)
    # every request accepts a child of its root (node 0 is one: parents start with -1) or drops it
    modes = [sp.SP_ACCEPT if r.req % 3 else sp.SP_DROP for r in reqs]
    nodes = [0] * 64
    live, commit = pair.gpu.tree_prune_batch(ids, modes, nodes)
    pair.gpu.kv_compact_batch(ids)
    for i, r in enumerate(reqs):
        pr = pair.ora.accept(r.req, 0) if modes[i] == sp.SP_ACCEPT else pair.ora.drop(r.req, 0)
        assert commit[i] == pr.n_commit and live[i] == pair.ora.req[r.req].tree.n - 1
        pair.check_tables(r.req)
    new = [[-1, -1] if r.req % 2 else [-1] for r in reqs]
    firsts = pair.insert_batch(ids, new, [[7 * r.req + k for k in range(len(p))] for r, p in zip(reqs, new)],
                               [[0.5] * len(p) for p in new])
    counts = [len(p) for p in new]
    x = wl.hidden_rows(shape, 23, ("b64", 1), sum(counts))
    y, ref = pair.forward(ids, firsts, counts, x)
    e = rel_err(y, ref)
    say("64 requests, second call rel err", e)
    assert e <= TOL["bf16"]
    for r in reqs:
        pair.check_kv(r.req, TOL["bf16"])
    pair.close()


WIDE_BATCHES = {
    # rows 387: one block of 256 and a ragged block of 131
    "387": {0: (150, 333), 1: (97, 64), 2: (140, 200)},          # request: (nodes, prefix)
    # rows 574: two blocks of 256 and a short last block of 62
    "574": {0: (200, 100), 1: (180, 257), 2: (130, 31), 3: (64, 500)},
    # rows 200: blocks of 128, the last with 72 rows
    "200": {0: (120, 90), 1: (80, 300)},
    # rows 130: blocks of 128, the last with 2 rows
    "130": {0: (130, 77)},
}


@pytest.mark.parametrize("batch", list(WIDE_BATCHES))
@pytest.mark.parametrize("packed", [0, sp.SP_FLAG_PACKED_WEIGHTS], ids=["rowmajor", "packed"])
def test_wide_batch(packed, batch):
    """A cold batch of several hundred rows goes through the many-row projection kernels: full
    row blocks of 128 or 256 and a ragged last block that runs a body of its own height."""
    shape = MINI_GQA4
    sizes = WIDE_BATCHES[batch]
    total = sum(n for n, _ in sizes.values())
    pair = Pair(shape, 18, {r: p for r, (n, p) in sizes.items()}, max_batch_nodes=total, flags=packed)
    counts = []
    for r, (n, p) in sizes.items():
        pair.insert(r, wl.tree_uniform_parents(18, n, 12, name=("w", r)))
        counts.append(n)
    x = wl.hidden_rows(shape, 18, ("w",), sum(counts))
    y, ref = pair.forward(list(sizes), [0] * len(sizes), counts, x)
    e = rel_err(y, ref)
    say("wide batch", batch, "rel err", e)
    assert e <= TOL["bf16"]
    for r in sizes:
        pair.check_kv(r, TOL["bf16"])
    pair.close()


def test_c4_full_prefix_first_steps():
    """Config 4's launch shape: the 8B-shaped layer dimensions, a committed context of 32768 tokens
    (each KV head's range cut into 32 chunks over the chip, merged by the second kernel), 1-8 new
    nodes per step, prune + compaction after each.  One layer and the first steps of the schedule:
    the float64 oracle gathers 33 MB per (node, head) at this length."""
    w = wl.CONFIGS["C4"]
    shape = wl.scaled(w.shape, n_layers=1)
    say("C4 prefix, 1 layer")
    pair = Pair(shape, w.seed, {0: w.prefix_len}, tree_room=64, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    steps = wl.streaming_schedule(w.seed, 3, max_new=8, cap=256, p_accept=0.7)
    worst = 0.0
    for s_, st in enumerate(steps):
        n = len(st.parents)
        first = pair.insert(0, st.parents)
        x = wl.hidden_rows(shape, w.seed, ("s", s_), n)
        y, ref = pair.forward([0], [first], [n], x)
        worst = max(worst, rel_err(y, ref))
        say("C4 step", s_, "nodes", n, "rel err", rel_err(y, ref))
        if st.prune is not None:
            pair.prune(0, st.prune.mode, st.prune.node, x_rows=y, row_nodes=list(range(first, first + n)))
        pair.check_kv(0, TOL["bf16"])
    assert worst <= TOL["bf16"]
    pair.close()


def test_c5_full_batch_cold_step_sampled():
    """Config 5's cold step at full size: 32 requests with contexts of 512-4096 tokens and trees of
    8-32 nodes forwarded in one call (several hundred rows: the many-row projection kernels, ragged
    attention segments).  The GPU runs the whole batch; the oracle follows a sample of the requests
    (first, last, the largest and the smallest tree), whose rows are compared element by element.
    One layer: the batch shape, not the depth, is what this case adds."""
    w = wl.CONFIGS["C5"]
    shape = wl.scaled(w.shape, n_layers=1)
    reqs = wl.batch_requests(w.seed, n_req=32, p_lo=512, p_hi=4096, t_lo=8, t_hi=32, max_levels=6)
    sizes = [len(r.parents) for r in reqs]
    sample = sorted({0, 31, int(np.argmax(sizes)), int(np.argmin(sizes))})
    total = sum(sizes)
    say("C5 cold batch:", total, "rows; oracle follows requests", sample)
    pair = Pair(shape, w.seed, {r.req: r.prefix_len for r in reqs}, tree_room=64, max_batch_nodes=total,
                flags=sp.SP_FLAG_PACKED_WEIGHTS, oracle_reqs=sample)
    # 574 new nodes in one call: the library cuts it into launches of at most 256
    pair.insert_batch([r.req for r in reqs], [r.parents for r in reqs])
    x = wl.hidden_rows(shape, w.seed, ("cold",), total)
    y = to_np(pair.gpu.stage_forward([r.req for r in reqs], [0] * 32, sizes, to_dev(x, pair.gpu)))
    row0 = np.concatenate([[0], np.cumsum(sizes)])
    for r in sample:
        ref = pair.ora.stage_forward(r, 0, x[row0[r]:row0[r + 1]])
        e = rel_err(y[row0[r]:row0[r + 1]], ref)
        say("C5 request", r, "nodes", sizes[r], "prefix", reqs[r].prefix_len, "rel err", e)
        assert e <= TOL["bf16"]
        pair.check_kv(r, TOL["bf16"])
        pair.check_tables(r)
    assert np.isfinite(y).all()
    pair.close()


# ---------------------------------------------------------------------------------------
# verification on the last stage
@pytest.mark.parametrize("flags", [0, sp.SP_FLAG_PACKED_WEIGHTS, sp.SP_FLAG_SIMPLE_KERNELS],
                         ids=["mfma", "mfma_packed", "simple"])
def test_verify_head_bf16(flags):
    """Output head + top-1 token on tree nodes of two requests, bf16; vocabulary of 1088 = 17 tiles."""
    shape = MINI_BF16
    pair = Pair(shape, 21, {0: 40, 1: 75}, flags=flags, vocab=1088)
    counts = [37, 21]
    for r, n in enumerate(counts):
        pair.insert(r, wl.tree_uniform_parents(21, n, 8, name=("v", r)), tokens=list(range(100 * r, 100 * r + n)))
    x = wl.hidden_rows(shape, 21, ("v",), sum(counts))
    y = pair.gpu.stage_forward([0, 1], [0, 0], counts, to_dev(x, pair.gpu))
    for r, n, row0 in ((0, counts[0], 0), (1, counts[1], counts[0])):       # oracle state: forward as well
        pair.ora.stage_forward(r, 0, x[row0:row0 + n])
    pred, differ = pair.verify_head([0, 1], [0, 0], counts, y, TOL["bf16"])
    say("verify head rows decided differently:", differ, "of", sum(counts))
    assert differ <= 1
    assert len(set(pred.tolist())) > 5                                     # not a constant
    for r in (0, 1):
        pair.check_tables(r)
    # a partial range of one request: rows are its nodes 5..14
    y1 = y[5:15].contiguous()
    pred2, _ = pair.verify_head([0], [5], [10], y1, TOL["bf16"])
    assert np.array_equal(pred2, pred[5:15])
    pair.close()


def test_verify_head_f32_odd_vocab():
    """fp32 config, vocabulary that is no multiple of anything: the plain kernels and full logits."""
    pair = Pair(MINI_F32, 22, {0: 33}, vocab=97)
    n = 29
    pair.insert(0, wl.tree_uniform_parents(22, n, 6, name=("v",)), tokens=list(range(n)))
    x = wl.hidden_rows(MINI_F32, 22, ("v",), n)
    y = pair.gpu.stage_forward([0], [0], [n], to_dev(x, pair.gpu))
    pair.ora.stage_forward(0, 0, x)
    pred, differ = pair.verify_head([0], [0], [n], y, TOL["f32"])
    assert differ == 0
    pair.check_tables(0)
    pair.close()


def test_verify_head_many_rows_and_order_error():
    """More than 64 rows (two passes of the row tiles) and the error for a node that was not forwarded."""
    shape = MINI_GQA4
    pair = Pair(shape, 23, {0: 50}, max_batch_nodes=128, vocab=640)
    n = 100
    pair.insert(0, wl.tree_uniform_parents(23, n, 10, name=("v",)), tokens=list(range(n)))
    x = wl.hidden_rows(shape, 23, ("v",), n)
    with pytest.raises(sp.SpError) as ei:
        pair.gpu.verify_head(pair.head, [0], [0], [n], to_dev(x, pair.gpu))
    assert ei.value.status == -6                                           # SP_E_ORDER
    y = pair.gpu.stage_forward([0], [0], [n], to_dev(x, pair.gpu))
    pair.ora.stage_forward(0, 0, x)
    pred, differ = pair.verify_head([0], [0], [n], y, TOL["bf16"])
    assert differ <= 1
    pair.check_tables(0)
    pair.close()


@pytest.mark.parametrize("handover", ["host", "device"])
@pytest.mark.parametrize("shape,flags,tol", [(MINI_F32, 0, "f32"), (MINI_BF16, sp.SP_FLAG_PACKED_WEIGHTS, "bf16")],
                         ids=["f32", "bf16_packed"])
def test_verified_decoding_loop(shape, flags, tol, handover):
    """Insert a level, forward, predict, match the root's successor, accept or stall -- the loop of
    Algorithm 1 with the stage as the whole model -- on the GPU and on the oracle side by side.  The
    guesses hold the right token about two times in three, so hits, misses (SP_CLEAR + the true token
    as a level of its own) and the hand-over of the accepted node's prediction to the root all occur.
    handover "device": the verified node never visits the host before the prune: sp_tree_prune_verified reads
    it from the match kernel's output (accept, or clear on a miss) and compacts the cache in the same call;
    the host's view of the request catches up afterwards."""
    V = 128
    pair = Pair(shape, 24, {0: 12}, tree_room=300, vocab=V, page_slots=32 if handover == "device" and tol == "bf16" else 0)
    emb = wl.embedding_table(shape, 24, V)
    rs = np.random.RandomState(24)
    pair.gpu.set_root_pred(0, 17)
    pair.ora.set_root_pred(0, 17)
    hits = misses = 0
    emitted = []
    for step in range(12):
        v = pair.gpu.tree_read(0)
        par, tok, n = v["parent"], v["token"], v["n_live"]
        leaves = [k for k in range(n) if k not in set(par.tolist())] if n else [-1]
        parents, tokens = [], []
        for leaf in leaves:
            known = int(v["pred"][leaf]) if leaf >= 0 else int(v["root_pred"])
            guesses = [known] if rs.rand() < 0.67 else []
            while len(guesses) < 3:
                g = int(rs.randint(V))
                if g != known and g not in guesses:
                    guesses.append(g)
            rs.shuffle(guesses)
            parents += [leaf] * 3
            tokens += guesses
        if n + len(parents) > 200:
            break
        first = pair.insert(0, parents, tokens)
        x = emb[tokens]
        y = pair.gpu.stage_forward([0], [first], [len(tokens)], to_dev(x, pair.gpu))
        ref = pair.ora.stage_forward(0, first, x)
        assert rel_err(to_np(y), ref) <= TOL[tol], step                       # a 12..24-token context: the mask shows
        assert rel_err(to_np(y) - x, ref - x) <= 4 * TOL[tol], step            # the layers' own contribution (y is rounded to the storage type)
        pair.verify_head([0], [first], [len(tokens)], y, TOL[tol])
        pair.check_tables(0)
        want = int(pair.ora.req[0].pred[0])
        emitted.append(want)
        if handover == "device":
            node = pair.ora.match(0)
            nodes_dev = pair.gpu.tree_match_dev([0])
            pair.prune_verified([0], nodes_dev, [node])              # no host read between match and prune
            assert int(nodes_dev[0]) == node
        else:
            node = pair.gpu.tree_match([0])[0]
            assert node == pair.ora.match(0)
            if node >= 0:
                pair.prune(0, sp.SP_ACCEPT, node)
            else:
                pair.prune(0, sp.SP_CLEAR, 0)
        if node >= 0:
            hits += 1
        else:
            misses += 1
            k = pair.insert(0, [-1], [want])
            y1 = pair.gpu.stage_forward([0], [k], [1], to_dev(emb[[want]], pair.gpu))
            assert rel_err(to_np(y1), pair.ora.stage_forward(0, k, emb[[want]])) <= TOL[tol], step
            pair.verify_head([0], [k], [1], y1, TOL[tol])
            pair.prune(0, sp.SP_ACCEPT, k)
        assert pair.gpu.tree_read(0)["root_pred"] == pair.ora.req[0].pred[0]
    say("verified decoding: hits", hits, "misses", misses, "tokens", emitted, "near-ties decided by the GPU:", pair.pred_overrides)
    assert pair.pred_overrides <= 2
    assert hits >= 3 and misses >= 1
    assert pair.gpu.request_info(0)[0] == 12 + len(emitted)
    pair.close()


# error of a single logit relative to the largest |logit|: fp32 accumulation order; bf16 rounding of the
# normalised row (2^-9 per element, adding up like a random walk over d_model terms)
TOL_LOGIT = {"f32": 1e-5, "bf16": 2e-3}


@pytest.mark.parametrize("shape,flags,tol,V", [(MINI_F32, 0, "f32", 97), (MINI_BF16, 0, "bf16", 1088),
                                               (MINI_BF16, sp.SP_FLAG_PACKED_WEIGHTS, "bf16", 4160),
                                               (MINI_BF16, sp.SP_FLAG_SIMPLE_KERNELS, "bf16", 2113)],
                         ids=["f32_v97", "bf16_v1088", "bf16_packed_v4160", "bf16_simple_v2113"])
def test_lossy_verification(shape, flags, tol, V):
    """Relaxed and top-p verification (Sec. 3.4) of the roots' children for three requests at once:
    vocabularies of one slice, of several slices with a short last one, and of odd size; children with
    duplicate tokens, a token outside the vocabulary, deeper nodes that must not count, a request
    whose root has no child."""
    pair = Pair(shape, 31, {0: 20, 1: 33, 2: 9}, vocab=V, head_gain=8.0)
    rs = np.random.RandomState(31)
    x_np = wl.hidden_rows(shape, 31, ("root",), 3)
    x_root = to_dev(x_np, pair.gpu)
    # the model's distribution after each root, to plant candidates at chosen places of the cumulative mass
    from oracle.verify import lm_head_logits, softmax_probs
    logits = lm_head_logits(x_np.astype(np.float64), pair.head_np["norm"], pair.head_np["wvocab"], shape.rms_eps)
    order = np.argsort(-logits, axis=1, kind="stable")
    for r, n_root in ((0, 9), (1, 14)):
        before = np.concatenate(([0.0], np.cumsum(softmax_probs(logits[r])[order[r]])[:-1]))   # by rank
        likely = [int(t) for t in order[r, 1:4]] + [int(order[r, 2])]             # near the top, one of them twice
        middle = [int(order[r, int(np.argmin(np.abs(before - m)))]) for m in (0.75, 0.85)]
        tail = [int(t) for t in order[r, V - (n_root - 7):]]                       # the least likely tokens
        tokens = likely + middle + tail + [V + 5]                                 # and one outside the vocabulary
        assert len(tokens) == n_root
        rs.shuffle(tokens)
        parents = [-1] * n_root
        deeper = [int(order[r, 0])] * 3                                           # the top-1 token, but not under the root
        pair.insert(r, parents + [0, 1, n_root], tokens + deeper,
                    probs=[float(q) for q in rs.uniform(0.05, 0.95, n_root + 3).astype(np.float32)])
    results = {}
    n_marginal = 0
    for mode, p in (("relaxed", 1.0), ("top_p", 0.55), ("top_p", 0.93), ("top_p", 0.999), ("top_p", 1e-6)):
        got, marginal = pair.verify_lossy([0, 1, 2], x_root, mode, p, TOL_LOGIT[tol])
        n_marginal += marginal
        say("lossy", mode, p, got, "marginal", marginal)
        results[(mode, p)] = got
        assert got[2][0] == -1                                                    # no children
        for r in (0, 1, 2):
            assert pair.gpu.tree_read(r)["root_pred"] == got[r][1] == int(order[r, 0])
    assert n_marginal <= 2                                                       # of 15 decisions; the others are compared exactly
    assert all(results[("relaxed", 1.0)][r][0] >= 0 for r in (0, 1))             # relaxed never misses
    assert all(results[("top_p", 1e-6)][r][0] == -1 for r in (0, 1))             # only the top-1 token passes
    assert any(results[("top_p", 0.999)][r][0] != results[("relaxed", 1.0)][r][0] for r in (0, 1))
    # a single request out of the three, in another order of arguments
    one, _ = pair.verify_lossy([1], x_root[1:2].contiguous(), "top_p", 0.93, TOL_LOGIT[tol])
    assert one[0] == results[("top_p", 0.93)][1]
    # device-side hand-over: the (node, top-1) pairs stay on the device and the prune reads them with stride 2;
    # request 1 accepts its relaxed choice, request 2 (no children) clears an empty tree
    n1 = pair.gpu.request_info(1)[1]
    pair.forward([1], [0], [n1], wl.hidden_rows(shape, 31, ("fw1",), n1))          # the accepted path's K/V rows exist
    res_dev = pair.gpu.verify_lossy_dev(pair.head, [1, 2], x_root[1:3].contiguous(), sp.SP_VERIFY_RELAXED, 1.0)
    want1 = results[("relaxed", 1.0)][1][0]
    pair.prune_verified([1, 2], res_dev, [want1, -1], stride=2)
    assert res_dev.tolist() == [want1, int(order[1, 0]), -1, int(order[2, 0])]
    with pytest.raises(sp.SpError):
        pair.gpu.verify_lossy(pair.head, [0], x_root[:1].contiguous(), sp.SP_VERIFY_TOP_P, 0.0)
    with pytest.raises(sp.SpError):
        pair.gpu.verify_lossy(pair.head, [0, 0], x_root[:2].contiguous(), sp.SP_VERIFY_RELAXED, 1.0)
    with pytest.raises(sp.SpError):
        pair.gpu.verify_lossy(pair.head, [0], x_root[:1].contiguous(), 3, 0.5)
    with pytest.raises(sp.SpError) as ei:
        pair.gpu.verify_lossy(pair.head, [7], x_root[:1].contiguous(), sp.SP_VERIFY_RELAXED, 1.0)
    assert ei.value.status == -4                                                 # SP_E_BAD_REQ
    assert pair.gpu.verify_lossy(pair.head, [], x_root[:1].contiguous(), sp.SP_VERIFY_RELAXED, 1.0) == []
    # while a compaction is pending the tables are between two states: refused
    pair.gpu.tree_prune(0, sp.SP_DROP, 0)
    with pytest.raises(sp.SpError) as ei:
        pair.gpu.verify_lossy(pair.head, [0], x_root[:1].contiguous(), sp.SP_VERIFY_RELAXED, 1.0)
    assert ei.value.status == -7                                                 # SP_E_PENDING
    pair.gpu.kv_compact(0)
    pair.close()


@pytest.mark.parametrize("shape,flags,tol,V,distinct",
                         [(MINI_F32, 0, "f32", 97, 0), (MINI_F32, 0, "f32", 5003, 0), (MINI_F32, 0, "f32", 5003, 7),
                          (MINI_F32, 0, "f32", 5003, 1), (MINI_F32, 0, "f32", 40007, 0),
                          (MINI_BF16, sp.SP_FLAG_PACKED_WEIGHTS, "bf16", 4160, 0)],
                         ids=["f32_v97", "f32_v5003", "f32_v5003_ties_of_7", "f32_v5003_all_equal", "f32_v40007",
                              "bf16_packed_v4160"])
def test_stochastic_verification(shape, flags, tol, V, distinct):
    """Stochastic decoding at the verifier (Sec. 4.3): the token after the root is drawn at temperature T among
    the candidates collected until their probabilities reach top_p or top_k have been taken; the uniform
    numbers are inputs.  The GPU forms probabilities in float32 from its own logits, the oracle in float64,
    so a draw is compared exactly unless the uniform number lies within a margin of an interval boundary
    (or the cut itself is within the margin of top_p), where the neighbouring outcome is accepted too.
    Vocabulary rows that repeat make logits tie exactly (equal probabilities go by ascending token id): with
    seven distinct rows every candidate comes out of a run of ties, with one the whole row is a tie, which is
    also the case the kernel's bound on the k-th largest logit cannot narrow down."""
    from oracle.verify import lm_head_logits, sampling_candidates, sample_token, match_root_child
    pair = Pair(shape, 35, {0: 20, 1: 33, 2: 9}, vocab=V, head_gain=8.0, head_distinct=distinct)
    rs = np.random.RandomState(35)
    x_np = wl.hidden_rows(shape, 35, ("root",), 3)
    x_root = to_dev(x_np, pair.gpu)
    logits = lm_head_logits(x_np.astype(np.float64), pair.head_np["norm"], pair.head_np["wvocab"], shape.rms_eps)
    order = np.argsort(-logits, axis=1, kind="stable")
    # root children: the most likely tokens (one twice), a token outside the vocabulary; deeper nodes must not count
    for r, n_root in ((0, 6), (1, 9)):
        toks = [int(t) for t in order[r, :n_root - 2]] + [int(order[r, 1]), V + 3]
        rs.shuffle(toks)
        pair.insert(r, [-1] * n_root + [0, 1], toks + [int(order[r, 0])] * 2)
    eps_logit = TOL_LOGIT[tol] * float(np.max(np.abs(logits)))
    n_checked = n_marginal = 0
    for T, p, k in ((0.6, 0.9, 80), (1.0, 0.5, 8), (0.3, 0.99, 128), (1.5, 1.0, 5), (0.6, 0.9, 1)):
        slack = 6.0 * eps_logit / T + 2e-6
        cands = [sampling_candidates(logits[r], T, p, k) for r in range(3)]
        us = []
        # centres of the three widest intervals, then uniform numbers anywhere
        for which in range(3):
            row = []
            for r in range(3):
                toks, ps = cands[r]
                c = np.concatenate(([0.0], np.cumsum(ps))) / ps.sum()
                j = int(np.argsort(-ps, kind="stable")[min(which, len(ps) - 1)])
                row.append(0.5 * (c[j] + c[j + 1]))
            us.append(row)
        us += [[float(v) for v in rs.uniform(0.0, 1.0, 3)] for _ in range(12)] + [[0.0, 0.0, 0.0]]
        for u in us:
            u32 = [float(np.float32(min(v, 0.9999999))) for v in u]
            got = pair.gpu.verify_sample(pair.head, [0, 1, 2], x_root, T, p, k, u32)
            for r in range(3):
                node, tok = got[r]
                toks, ps = cands[r]
                want = sample_token(logits[r], T, p, k, u32[r])
                # outcomes the margin allows: cut one candidate earlier / later where the running sum is within
                # the margin of top_p, boundaries moved by the margin
                allowed = set()
                full_t, full_p = sampling_candidates(logits[r], T, 1.0 + 1e-9, min(k, len(toks) + 1))
                run = np.cumsum(full_p)
                for m in range(max(1, len(toks) - 1), min(len(full_t), len(toks) + 1) + 1):
                    cut_ok = (m == len(toks)) or (m < len(toks) and run[m - 1] >= p - slack) or \
                             (m > len(toks) and run[len(toks) - 1] < p + slack and m <= k)
                    if not cut_ok:
                        continue
                    c = np.concatenate(([0.0], run[:m])) / run[m - 1]
                    for j in range(m):
                        if c[j] - slack <= u32[r] < c[j + 1] + slack:
                            allowed.add(int(full_t[j]))
                assert tok in allowed, (T, p, k, r, u32[r], tok, want, sorted(allowed))
                n_checked += 1
                n_marginal += len(allowed) > 1
                if len(allowed) == 1:
                    assert tok == want
                par, _, tk, _, _ = pair.ora.req[r].tree.view()
                assert node == match_root_child(par, tk, tok), (r, node, tok)
                assert pair.gpu.tree_read(r)["root_pred"] == tok
                pair.ora.set_root_pred(r, tok)
    say("stochastic verification:", n_checked, "draws,", n_marginal, "inside a margin")
    # float32 logits: the selection, the order, the running sums and the draw are compared exactly (a handful of
    # uniform numbers may sit on a boundary); bf16 logits move every probability by several per cent at these
    # temperatures, so there the margin rule above is the whole check
    if tol == "f32":
        # tied rows and the larger vocabulary (more candidates before top_p is reached) have more boundaries
        assert n_marginal <= n_checked // (8 if distinct or V > 5003 else 20)
    for bad in (dict(temperature=0.0), dict(top_p=0.0), dict(top_k=0), dict(top_k=129), dict(u=[1.0])):
        kw = dict(temperature=0.6, top_p=0.9, top_k=80, u=[0.5])
        kw.update(bad)
        with pytest.raises(sp.SpError) as ei:
            pair.gpu.verify_sample(pair.head, [0], x_root[:1].contiguous(), kw["temperature"], kw["top_p"], kw["top_k"], kw["u"])
        assert ei.value.status == -1
    pair.close()


# ---------------------------------------------------------------------------------------
# fixed-width expansion
def test_fixed_width_expansion_matches_oracle():
    """Grow a tree level by level with sp_tree_expand (k candidates per bottom token, the w most
    likely by cumulative probability kept, parent order) and compare every level with the oracle's
    selection, exactly: parents, tokens and probability bits.  Includes ties (probabilities drawn
    from a small set), absent candidates, w larger than the candidate count and the 4096 limit."""
    from oracle.expand import expand_fixed_width
    pair = Pair(MINI_F32, 31, {0: 6}, tree_room=300, oracle=True)
    g = pair.gpu
    rs = np.random.RandomState(31)
    bottom = [-1]
    for step, (k, w) in enumerate([(5, 9), (8, 3), (16, 40), (4, 64), (32, 64), (7, 30)]):
        nb = len(bottom)
        toks = rs.randint(0, 5000, (nb, k)).astype(np.int32)
        toks[rs.rand(nb, k) < 0.1] = -1                                    # absent candidates
        prs = (rs.randint(1, 9, (nb, k)) / 8.0).astype(np.float32)         # few distinct values: many ties
        if step % 2 == 0:
            prs = rs.uniform(0.01, 1.0, (nb, k)).astype(np.float32)
        par, _, _, prob, _ = pair.ora.req[0].tree.view()
        want = expand_fixed_width(par, prob, bottom, toks, prs, w)
        got = g.tree_expand(0, bottom, torch.from_numpy(toks).cuda(), torch.from_numpy(prs).cuda(), w)
        assert got[0] == want[0] and got[1] == want[1], (step, got[:2], want[:2])
        assert np.array_equal(np.asarray(got[2], np.float32).view(np.uint32), np.asarray(want[2], np.float32).view(np.uint32))
        assert len(got[0]) <= w and got[0] == sorted(got[0])
        if not got[0]:
            break
        first = pair.insert(0, got[0], got[1], got[2])
        pair.check_tables(0)
        bottom = list(range(first, first + len(got[0])))
    # the documented limits
    T = pair.gpu.request_info(0)[1]
    with pytest.raises(sp.SpError) as ei:
        g.tree_expand(0, list(range(min(T, 129))), torch.zeros((min(T, 129), 32), dtype=torch.int32).cuda(),
                      torch.ones((min(T, 129), 32)).cuda(), 8)
    assert ei.value.status == -2                                           # SP_E_CAPACITY: 129 * 32 > 4096
    with pytest.raises(sp.SpError) as ei:
        g.tree_expand(0, [3, 2], torch.zeros((2, 4), dtype=torch.int32).cuda(), torch.ones((2, 4)).cuda(), 2)
    assert ei.value.status == -1                                           # not ascending
    pair.close()


def test_error_codes():
    pair = Pair(MINI_F32, 17, {0: 10}, tree_room=30, oracle=False)
    g = pair.gpu

    def status(fn, *a, **k):
        try:
            fn(*a, **k)
        except sp.SpError as e:
            return e.status
        return 0

    assert status(g.tree_insert, 3, [-1]) == -4                     # request never initialised
    assert status(g.tree_insert, 0, [0]) == -3                      # parent does not exist
    assert status(g.tree_insert, 0, [-1, 2]) == -3                  # parent not before child
    assert status(g.tree_insert, 0, [-1] * 31) == -2                # slot range full
    assert g.request_info(0) == (10, 0, 0)                          # nothing changed
    g.tree_insert(0, [-1, 0, 1])
    x = torch.zeros(1, MINI_F32.d_model, device=g.device)
    assert status(g.stage_forward, [0], [2], [1], x) == -6          # parent 1 not forwarded
    assert status(g.stage_forward, [0], [2], [5], torch.zeros(5, 256, device=g.device)) == -5
    assert status(g.tree_prune, 0, sp.SP_ACCEPT, 3) == -5
    assert status(g.tree_prune, 0, sp.SP_ACCEPT, 1) == -6           # its K/V rows do not exist yet
    assert status(g.kv_compact, 0) == -7                            # nothing pending
    g.tree_prune(0, sp.SP_DROP, 2)
    assert status(g.tree_insert, 0, [-1]) == -7                     # compaction pending
    assert status(g.tree_prune, 0, sp.SP_DROP, 0) == -7
    g.kv_compact(0)
    assert g.request_info(0) == (10, 2, 0)
    # a flushed tree: accept the only chain down to nothing, then hang a new level off the tail
    g.stage_forward([0], [0], [2], torch.zeros(2, 256, device=g.device))
    assert g.tree_prune(0, sp.SP_ACCEPT, 1) == (0, 2)
    g.kv_compact(0)
    assert g.request_info(0) == (12, 0, 0)
    assert g.tree_insert(0, [-1, -1]) == 0
    torch.cuda.synchronize()
    pair.close()


def test_c2_full_size_in_bench_configuration():
    """Config 2 at full size, launched exactly as bench.py does (one request, prefix 2048, the
    64-node tree, accept + compact): every output element against the oracle."""
    w = wl.CONFIGS["C2"]
    say("C2 full size")
    pair = Pair(w.shape, w.seed, {0: w.prefix_len}, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    par = wl.tree_branching(w.seed, w.n_nodes, w.max_children, w.max_levels)
    x = wl.hidden_rows(w.shape, w.seed, ("x",), w.n_nodes)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [w.n_nodes], x)
    e = rel_err(y, ref)
    say("C2 rel err", e)
    assert e <= TOL["bf16"]
    pair.check_kv(0, TOL["bf16"])
    roots = [i for i, p in enumerate(par) if p < 0]
    pair.prune(0, sp.SP_ACCEPT, roots[0], x_rows=y, row_nodes=list(range(w.n_nodes)))
    pair.close()


@pytest.mark.parametrize("n_nodes,flags", [(128, sp.SP_FLAG_PACKED_WEIGHTS), (60, 0), (100, 0),
                                           (8, sp.SP_FLAG_PACKED_WEIGHTS), (40, sp.SP_FLAG_PACKED_WEIGHTS), (12, 0)],
                         ids=["128_packed", "60_rowmajor", "100_rowmajor", "8_packed", "40_packed", "12_rowmajor"])
def test_c3_dimensions_one_layer(n_nodes, flags):
    """One layer at the 70B shape (d=8192, 64/8 heads, FFN 28672) with config 3's 128-node tree and
    prefix 4096: a 128-row block per projection (two strips of 16 weight rows per wave, 64 + 64 gate/up
    columns per workgroup), 8 query heads per KV head; and with 60 nodes, where the gate/up projection
    takes the same wide workgroups with four row tiles, the last one ragged; both weight layouts.
    With 8, 12 and 40 nodes the QKV and O products (K = 8192) run as one or three row tiles whose
    workgroups walk their k slices from staggered starting chunks (slices of 10-11 and 16 chunks).
    (All ten layers: the full-depth test.)"""
    w = wl.CONFIGS["C3"]
    shape = wl.scaled(w.shape, n_layers=1)
    say("C3 dims, 1 layer,", n_nodes, "nodes")
    pair = Pair(shape, w.seed, {0: w.prefix_len}, max_batch_nodes=128, flags=flags)
    par = wl.tree_branching(w.seed, n_nodes, w.max_children, w.max_levels)
    x = wl.hidden_rows(shape, w.seed, ("x",), n_nodes)
    pair.insert(0, par)
    y, ref = pair.forward([0], [0], [n_nodes], x)
    e = rel_err(y, ref)
    say("C3-dims rel err", e)
    assert e <= TOL["bf16"]
    pair.check_kv(0, TOL["bf16"])
    pair.close()
