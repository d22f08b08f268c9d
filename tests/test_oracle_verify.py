"""Pins for oracle/verify.py and the verification state of oracle/stage.py.

The output head is checked against Hugging Face's LlamaRMSNorm and a torch Linear; the
greedy token against hand-made rows; the whole verify / accept / miss loop against the
property that makes the method lossless (Sec. 3.3.2: the selection strictly follows the
output of the large model; Sec. 3.4: top-1 validation): decoding through a speculative
tree full of wrong guesses must emit exactly the tokens of plain one-token-at-a-time greedy
decoding, which is the T=1 case already pinned against the Hugging Face layer."""
import numpy as np
import pytest
import torch

import workloads as wl
from oracle import (StageOracle, lm_head_logits, greedy_token, greedy_token_fast, match_root_child)

SMALL = wl.ModelShape(n_layers=2, d_model=64, n_q_heads=4, n_kv_heads=2, d_head=16, d_ff=96,
                      rms_eps=1e-6, rope_theta=500000.0, dtype="f32")
VOCAB = 53


def test_head_matches_hf_norm_and_torch_linear():
    from transformers.models.llama.modeling_llama import LlamaRMSNorm
    rs = np.random.RandomState(3)
    h = rs.randn(7, 64)
    g = 1 + 0.1 * rs.randn(64)
    W = 0.05 * rs.randn(VOCAB, 64)
    norm = LlamaRMSNorm(64, eps=1e-5).double()
    lin = torch.nn.Linear(64, VOCAB, bias=False).double()
    with torch.no_grad():
        norm.weight.copy_(torch.from_numpy(g))
        lin.weight.copy_(torch.from_numpy(W))
        ref = lin(norm(torch.from_numpy(h))).numpy()
    got = lm_head_logits(h, g, W, 1e-5)
    assert got.shape == (7, VOCAB)
    # the Hugging Face norm squares and averages in float32 whatever the module's dtype
    assert np.allclose(got, ref, rtol=1e-6, atol=1e-7)
    # torch's own rms_norm stays in float64
    ref64 = torch.nn.functional.linear(
        torch.nn.functional.rms_norm(torch.from_numpy(h), (64,), torch.from_numpy(g), 1e-5), torch.from_numpy(W)).numpy()
    assert np.allclose(got, ref64, rtol=1e-12, atol=1e-13)
    # a transposed projection or a dropped gain would not survive this
    assert not np.allclose(lm_head_logits(h, np.ones(64), W, 1e-5), ref, rtol=1e-6, atol=1e-6)


def test_greedy_token_takes_the_first_maximum():
    rows = np.array([[0.0, 2.0, 2.0, -1.0],       # tie: lowest index wins
                     [5.0, 1.0, 5.0, 5.0],
                     [-3.0, -2.0, -1.0, -0.5],
                     [-np.inf, -np.inf, 0.0, -np.inf]])
    assert greedy_token(rows).tolist() == [1, 0, 3, 2]
    rs = np.random.RandomState(4)
    big = np.round(rs.randn(40, 300), 1)           # many exact ties
    assert np.array_equal(greedy_token(big), greedy_token_fast(big))
    assert np.array_equal(greedy_token(big), [int(np.flatnonzero(r == r.max())[0]) for r in big])


def test_match_root_child():
    #          node: 0   1   2   3   4
    parent = [-1, -1, 0, -1, 1]
    token = [7, 9, 4, 9, 9]
    assert match_root_child(parent, token, 9) == 1          # first of two root children carrying 9
    assert match_root_child(parent, token, 7) == 0
    assert match_root_child(parent, token, 4) == -1         # 4 sits below a root child, not at level 1
    assert match_root_child([], [], 3) == -1


def _model(seed, P):
    ws = [wl.layer_weights(SMALL, seed, l) for l in range(SMALL.n_layers)]
    pk, pv = zip(*[wl.prefix_kv(SMALL, seed, l, P) for l in range(SMALL.n_layers)])
    head = wl.head_weights(SMALL, seed, VOCAB)
    emb = wl.embedding_table(SMALL, seed, VOCAB)
    st = StageOracle(SMALL, ws)
    st.request_init(0, pk, pv, P + 400)
    return st, head, emb


def _plain_greedy(seed, P, first_token, n_tokens):
    """One node per step under the root, forwarded alone, accepted at once."""
    st, head, emb = _model(seed, P)
    out, tok = [], first_token
    for _ in range(n_tokens):
        out.append(tok)
        k = st.tree_insert(0, [-1], [tok])
        h = st.stage_forward(0, k, emb[[tok]])
        pred, _ = st.verify_head(0, k, h, head["norm"], head["wvocab"])
        st.accept(0, k)
        tok = int(pred[0])
    return out


@pytest.mark.parametrize("seed,p_hit,width", [(5, 0.7, 3), (6, 1.0, 2), (7, 0.0, 2), (8, 0.5, 4)])
def test_speculative_decoding_is_lossless(seed, p_hit, width):
    P, n_tokens = 9, 14
    first = 11
    truth = _plain_greedy(seed, P, first, n_tokens + 4)
    # the model's token after y_i is y_{i+1}: what a perfect draft would guess
    nxt = {}
    for a, b in zip(truth, truth[1:]):
        nxt.setdefault(a, b)
    st, head, emb = _model(seed, P)
    st.set_root_pred(0, first)
    rs = np.random.RandomState(seed)
    emitted, misses, hits = [], 0, 0
    committed_path = []                       # tokens accepted so far
    while len(emitted) < n_tokens:
        # layer appending under every leaf: `width` guesses, the right one with probability p_hit
        par, dep, tok, _, _ = st.req[0].tree.view()
        n = len(par)
        leaves = [k for k in range(n) if k not in set(par.tolist())] if n else [-1]
        parents, tokens = [], []
        for leaf in leaves:
            # the true continuation of this leaf, if the leaf lies on the true path
            path = []
            k = leaf
            while k >= 0:
                path.append(int(tok[k]))
                k = int(par[k])
            path = path[::-1]
            i0 = len(committed_path)
            on_truth = truth[i0:i0 + len(path)] == path
            right = truth[i0 + len(path)] if on_truth and i0 + len(path) < len(truth) else None
            guesses = []
            if right is not None and rs.rand() < p_hit:
                guesses.append(right)
            while len(guesses) < width:
                g = int(rs.randint(VOCAB))
                if g != right and g not in guesses:
                    guesses.append(g)
            rs.shuffle(guesses)
            parents += [leaf] * width
            tokens += guesses
        if st.req[0].tree.n - 1 + len(parents) > 200:
            pytest.fail("tree grew without bound")
        k0 = st.tree_insert(0, parents, tokens)
        h = st.stage_forward(0, k0, emb[tokens])
        st.verify_head(0, k0, h, head["norm"], head["wvocab"])
        # verify the root's successor
        want = int(st.req[0].pred[0])
        node = st.match(0)
        if node >= 0:
            hits += 1
            par, _, tok, _, _ = st.req[0].tree.view()
            assert par[node] == -1 and tok[node] == want
            st.accept(0, node)
        else:
            misses += 1                       # pipeline stall: the true token becomes the next level
            st.clear(0)
            k = st.tree_insert(0, [-1], [want])
            hk = st.stage_forward(0, k, emb[[want]])
            st.verify_head(0, k, hk, head["norm"], head["wvocab"])
            st.accept(0, k)
        emitted.append(want)
        committed_path.append(want)
    assert emitted == truth[:n_tokens]
    if p_hit == 1.0:
        assert misses == 0
    if p_hit == 0.0:
        assert hits == 0
    # the committed context grew by one token per emitted token
    assert st.req[0].P == P + n_tokens
