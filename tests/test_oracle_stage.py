"""Pins for oracle/stage.py.

The tree-masked stage must give, for every node, exactly what ordinary
sequential decoding gives along that node's root-to-leaf path (lossless
speculation: Sec. 3.3.2 "node-wise computation", Sec. 3.4 "Lossless and Lossy
Acceleration").  Sequential decoding is done by Hugging Face's Llama layer, which
the paper's implementation reuses (Sec. 4), so nothing of the oracle is on the
right-hand side.  The pieces are pinned separately against torch routines and
against identities that hold for any correct implementation."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import (StageOracle, SpecTree, rmsnorm, rope_rotate, silu, tree_attention)
from hf_reference import HFStage

SMALL = wl.ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, d_head=16, d_ff=96,
                      rms_eps=1e-6, rope_theta=500000.0, dtype="f32")
SMALL_MHA = wl.scaled(SMALL, n_kv_heads=4, rope_theta=10000.0, rms_eps=1e-5)


def make(shape, seed, P, capacity=None):
    ws = [wl.layer_weights(shape, seed, l) for l in range(shape.n_layers)]
    pk, pv = zip(*[wl.prefix_kv(shape, seed, l, P) for l in range(shape.n_layers)])
    st = StageOracle(shape, ws)
    st.request_init(0, pk, pv, capacity or P + 300)
    return st, ws, pk, pv


def path_to(par, i):
    out = [i]
    while par[out[-1]] >= 0:
        out.append(par[out[-1]])
    return out[::-1]


# ---------------------------------------------------------------- pieces
def test_rmsnorm_matches_torch():
    rs = np.random.RandomState(0)
    x = rs.randn(5, 48)
    g = 1 + 0.1 * rs.randn(48)
    ref = torch.nn.functional.rms_norm(torch.from_numpy(x), (48,), torch.from_numpy(g), 1e-6).numpy()
    assert np.allclose(rmsnorm(x, g, 1e-6), ref, rtol=1e-13, atol=1e-13)


def test_silu_matches_torch():
    z = np.linspace(-30, 30, 601)
    assert np.allclose(silu(z), torch.nn.functional.silu(torch.from_numpy(z)).numpy(), rtol=1e-13, atol=1e-15)


def test_rope_identities():
    rs = np.random.RandomState(1)
    q = rs.randn(1, 3, 32)
    k = rs.randn(1, 3, 32)
    # position 0 is the identity; rotation keeps the norm of every pair
    assert np.allclose(rope_rotate(q, [0], 500000.0), q)
    r = rope_rotate(q, [1234], 500000.0)
    assert np.allclose((r[..., :16] ** 2 + r[..., 16:] ** 2), (q[..., :16] ** 2 + q[..., 16:] ** 2))
    # the score depends on the position difference only
    a = (rope_rotate(q, [17], 1e4) * rope_rotate(k, [5], 1e4)).sum(-1)
    b = (rope_rotate(q, [112], 1e4) * rope_rotate(k, [100], 1e4)).sum(-1)
    assert np.allclose(a, b, rtol=1e-11)
    # complex form: (x_t + i x_{t+d/2}) * exp(i pos theta^(-2t/d))
    z = q[..., :16] + 1j * q[..., 16:]
    w = z * np.exp(1j * 37 * (1e4 ** (-np.arange(16) / 16.0)))
    rr = rope_rotate(q, [37], 1e4)
    assert np.allclose(rr[..., :16], w.real) and np.allclose(rr[..., 16:], w.imag)


def test_rope_matches_library():
    from transformers.models.llama.modeling_llama import apply_rotary_pos_emb
    hf = HFStage(SMALL, [wl.layer_weights(SMALL, 0, l) for l in range(SMALL.n_layers)])
    rs = np.random.RandomState(2)
    x = rs.randn(6, 4, 16)
    pos = [0, 1, 2, 50, 51, 129]
    cos, sin = hf.rot(torch.zeros(1, 6, 64, dtype=torch.float64), torch.tensor([pos]))
    xt = torch.from_numpy(x).permute(1, 0, 2)[None]                # [1, H, n, d]
    ref, _ = apply_rotary_pos_emb(xt, xt, cos, sin)
    assert np.allclose(rope_rotate(x, pos, SMALL.rope_theta), ref[0].permute(1, 0, 2).numpy(), atol=2e-5)


def test_tree_attention_matches_sdpa_with_explicit_mask():
    rs = np.random.RandomState(3)
    n, hq, hkv, dh, S = 7, 6, 2, 16, 40
    q = rs.randn(n, hq, dh)
    K = rs.randn(S, hkv, dh)
    V = rs.randn(S, hkv, dh)
    mask = rs.rand(n, S) < 0.6
    mask[:, 0] = True
    vis = [np.nonzero(mask[i])[0] for i in range(n)]
    out = tree_attention(q, K, V, vis)
    qt = torch.from_numpy(q).permute(1, 0, 2)[None]
    kt = torch.from_numpy(K).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    vt = torch.from_numpy(V).permute(1, 0, 2).repeat_interleave(hq // hkv, 0)[None]
    ref = torch.nn.functional.scaled_dot_product_attention(qt, kt, vt, attn_mask=torch.from_numpy(mask)[None, None])
    assert np.allclose(out, ref[0].permute(1, 0, 2).numpy(), rtol=1e-10, atol=1e-12)


# ---------------------------------------------------------------- whole stage
TREES = {
    "c1": wl.tree_uniform_parents(0, 16, 6),
    "branch": wl.tree_branching(7, 24, 3, 6),
    "chain": wl.tree_chain(6),
    "star": wl.tree_star(5),
    "one": [-1],
}


@pytest.mark.parametrize("shape", [SMALL, SMALL_MHA], ids=["gqa", "mha"])
@pytest.mark.parametrize("name", sorted(TREES))
def test_tree_forward_equals_sequential_decoding_along_every_path(shape, name):
    par = TREES[name]
    n, P = len(par), 21
    st, ws, pk, pv = make(shape, 5, P)
    x = wl.hidden_rows(shape, 5, ("t", name), n)
    st.tree_insert(0, par)
    y = st.stage_forward(0, 0, x)

    hf = HFStage(shape, ws)
    leaves = [i for i in range(n) if i not in par]
    seen = set()
    for leaf in leaves:
        path = path_to(par, leaf)
        cache = hf.fresh_cache(pk, pv)
        for k, node in enumerate(path):
            out = hf.run(x[node:node + 1], [P + k], cache)          # one ordinary decode step
            assert np.allclose(y[node], out[0], rtol=1e-5, atol=2e-5), (name, node)
            seen.add(node)
        # the cache rows this path produced are the rows the tree forward stored for its nodes
        for l in range(shape.n_layers):
            Kh, Vh = hf.cache_rows(cache, l)
            Ko, Vo = st.tree_kv(0, l)
            assert np.allclose(Kh[P:], Ko[path], atol=2e-5)
            assert np.allclose(Vh[P:], Vo[path], atol=2e-5)
    assert seen == set(range(n))


def test_tree_forward_equals_library_call_under_the_tree_mask():
    """One library call over all nodes with M as an explicit additive mask (Sec. 2.2, tree mask)."""
    shape, par, P = SMALL, TREES["branch"], 33
    n = len(par)
    st, ws, pk, pv = make(shape, 6, P)
    x = wl.hidden_rows(shape, 6, ("m",), n)
    st.tree_insert(0, par)
    y = st.stage_forward(0, 0, x)
    hf = HFStage(shape, ws)
    M = st.req[0].tree.view()[4].astype(bool)
    mask = np.concatenate([np.ones((n, P), bool), M], axis=1)
    pos = [P + d for d in wl.levels_of(par)]
    out = hf.run(x, pos, hf.fresh_cache(pk, pv), mask)
    assert np.allclose(y, out, rtol=1e-5, atol=2e-5)


def test_chain_is_causal_decoding():
    """A chain-shaped tree is one token per position: the tree mask is the causal mask (Sec. 2.2)."""
    shape, P, n = SMALL, 17, 8
    st, ws, pk, pv = make(shape, 8, P)
    x = wl.hidden_rows(shape, 8, ("c",), n)
    st.tree_insert(0, wl.tree_chain(n))
    y = st.stage_forward(0, 0, x)
    hf = HFStage(shape, ws)
    causal = np.concatenate([np.ones((n, P), bool), np.tril(np.ones((n, n), bool))], axis=1)
    out = hf.run(x, list(range(P, P + n)), hf.fresh_cache(pk, pv), causal)
    assert np.allclose(y, out, rtol=1e-5, atol=2e-5)


def test_forward_in_several_calls_equals_one_call():
    shape, P = SMALL, 19
    par = wl.bfs_sorted(wl.tree_branching(9, 30, 3, 6))[0]
    n = len(par)
    x = wl.hidden_rows(shape, 9, ("i",), n)
    a, *_ = make(shape, 9, P)
    a.tree_insert(0, par)
    ya = a.stage_forward(0, 0, x)
    b, *_ = make(shape, 9, P)
    cuts = [0, 3, 4, 11, 20, n]
    yb = []
    for lo, hi in zip(cuts[:-1], cuts[1:]):
        b.tree_insert(0, par[lo:hi])
        yb.append(b.stage_forward(0, lo, x[lo:hi]))
    yb = np.concatenate(yb)
    assert np.allclose(ya, yb, rtol=1e-12, atol=1e-12)
    for l in range(shape.n_layers):
        assert np.allclose(a.tree_kv(0, l)[0], b.tree_kv(0, l)[0], rtol=1e-12, atol=1e-12)


def test_star_is_independent_decode_steps():
    shape, P, n = SMALL, 23, 4
    x = wl.hidden_rows(shape, 10, ("s",), n)
    st, ws, pk, pv = make(shape, 10, P)
    st.tree_insert(0, wl.tree_star(n))
    y = st.stage_forward(0, 0, x)
    for i in range(n):
        one, *_ = make(shape, 10, P)
        one.tree_insert(0, [-1])
        assert np.allclose(one.stage_forward(0, 0, x[i:i + 1])[0], y[i], rtol=1e-12, atol=1e-13)


def test_a_planted_mistake_is_caught():
    """The sequential pin must notice a wrong position rule: shift one node's level by one."""
    shape, par, P = SMALL, TREES["branch"], 21
    n = len(par)
    st, ws, pk, pv = make(shape, 5, P)
    x = wl.hidden_rows(shape, 5, ("t", "branch"), n)
    st.tree_insert(0, par)
    good = st.stage_forward(0, 0, x)
    bad, *_ = make(shape, 5, P)
    bad.tree_insert(0, par)
    bad.req[0].P += 1          # every position off by one, cache slots too
    worse = bad.stage_forward(0, 0, x)
    assert not np.allclose(good, worse, rtol=1e-4, atol=1e-4)
