"""Node-wise computation of one pipeline stage (Sec. 3.3.2; Algorithm 1, "Node-wise computation").

TEST INFRASTRUCTURE.  `for each layer in device i: E_i <- layer(E_i, M_i, KV_i)`
with the Llama-family decoder layer the paper builds on (Sec. 2.1, Sec. 4
"Implementation"/"Testbed"): pre-norm RMSNorm, grouped-query attention with
rotary positions, SwiGLU feed-forward, no biases.  Attention is
softmax(Q K^T / sqrt(d_h)) V (Sec. 2.1) restricted by the tree mask M
(Sec. 2.2, Sec. 3.3.2): a node sees the whole committed context and, among the
speculative tokens, itself and its ancestors only.  A node at tree level k
stands for the k-th future position (Sec. 3.2).

Everything is float64 numpy, one node and one head at a time where that is the
plain way to say it.  numpy's matmul is the only library step.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Callable, Dict, List, Optional, Sequence

import numpy as np

from .tree import SpecTree
from .prune import PruneResult, accept_masks, drop_masks, compact_rows

F64 = np.float64


# ----------------------------------------------------------------------------
# layer pieces
# ----------------------------------------------------------------------------
def rmsnorm(x: np.ndarray, gain: np.ndarray, eps: float) -> np.ndarray:
    x = np.asarray(x, F64)
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * np.asarray(gain, F64)


def silu(z: np.ndarray) -> np.ndarray:
    z = np.asarray(z, F64)
    return z / (1.0 + np.exp(-z))


def rope_rotate(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary position embedding, half-split pairing: coordinate t is paired with
    t + d_h/2 and the pair is rotated by the angle pos * theta^(-2t/d_h).
    x: [n, heads, d_h]; pos: [n]."""
    x = np.asarray(x, F64)
    dh = x.shape[-1]
    half = dh // 2
    inv_freq = F64(theta) ** (-(np.arange(half, dtype=F64) * 2.0) / dh)
    ang = np.asarray(pos, F64)[:, None] * inv_freq[None, :]          # [n, half]
    c = np.cos(ang)[:, None, :]
    s = np.sin(ang)[:, None, :]
    a, b = x[..., :half], x[..., half:]
    return np.concatenate([a * c - b * s, b * c + a * s], axis=-1)


def tree_attention(q: np.ndarray, K: np.ndarray, V: np.ndarray,
                   visible: Sequence[np.ndarray]) -> np.ndarray:
    """q: [n, H_q, d_h]; K, V: [slots, H_kv, d_h]; visible[i]: the cache slots
    node i may attend to, ascending.  Query head h reads KV head h // (H_q/H_kv).
    Masked keys are left out of the softmax altogether."""
    n, hq, dh = q.shape
    hkv = K.shape[1]
    g = hq // hkv
    out = np.zeros((n, hq, dh), dtype=F64)
    scale = 1.0 / np.sqrt(F64(dh))
    for i in range(n):
        vis = np.asarray(visible[i], dtype=np.int64)
        for kv in range(hkv):
            kh = K[vis, kv, :]                           # [len, d_h]: the keys node i may see, this KV head
            vh = V[vis, kv, :]
            for h in range(kv * g, (kv + 1) * g):        # the query heads that read this KV head
                s = (kh @ q[i, h, :]) * scale
                s = s - s.max()
                p = np.exp(s)
                p = p / p.sum()
                out[i, h, :] = p @ vh
    return out


def decoder_layer(x: np.ndarray, w: Dict[str, np.ndarray], *, n_q_heads: int, n_kv_heads: int,
                  d_head: int, eps: float, theta: float, pos: np.ndarray,
                  K: np.ndarray, V: np.ndarray, slots: np.ndarray,
                  visible: Sequence[np.ndarray]) -> np.ndarray:
    """One decoder layer on n tree nodes.  Writes the nodes' K (rotated) and V
    into cache rows `slots` first, then attends; returns the new hidden rows."""
    x = np.asarray(x, F64)
    n = x.shape[0]
    W = {k: np.asarray(v, F64) for k, v in w.items()}
    n1 = rmsnorm(x, W["norm1"], eps)
    q = (n1 @ W["wq"].T).reshape(n, n_q_heads, d_head)
    k = (n1 @ W["wk"].T).reshape(n, n_kv_heads, d_head)
    v = (n1 @ W["wv"].T).reshape(n, n_kv_heads, d_head)
    q = rope_rotate(q, pos, theta)
    k = rope_rotate(k, pos, theta)
    K[slots] = k
    V[slots] = v
    a = tree_attention(q, K, V, visible).reshape(n, n_q_heads * d_head)
    h = x + a @ W["wo"].T
    n2 = rmsnorm(h, W["norm2"], eps)
    y = h + (silu(n2 @ W["wg"].T) * (n2 @ W["wu"].T)) @ W["wd"].T
    return y


# ----------------------------------------------------------------------------
# device state {E_i, M_i, KV_i} of one request, and the stage
# ----------------------------------------------------------------------------
@dataclass
class RequestState:
    """P counts the committed tokens, root tau_1 (the last verified token)
    included; tree index j (root = 0) lives in cache slot P-1+j."""
    P: int
    tree: SpecTree
    K: List[np.ndarray]           # per layer [capacity, H_kv, d_h] float64
    V: List[np.ndarray]
    # pred[j]: the model's next token after tree node j (root = 0), -1 while unknown
    # (set once the node has left the last stage: Algorithm 1, "verify new token")
    pred: np.ndarray = None


class StageOracle:
    """One pipeline stage: L decoder layers and, per request, a tree and a KV cache."""

    def __init__(self, shape, weights: Callable[[int], Dict[str, np.ndarray]] | Sequence[Dict[str, np.ndarray]]):
        self.shape = shape
        self._weights = weights
        self.req: Dict[int, RequestState] = {}

    def layer_weights(self, l: int) -> Dict[str, np.ndarray]:
        return self._weights(l) if callable(self._weights) else self._weights[l]

    # -- request set-up: a committed context whose K/V are given (post-RoPE) --
    def request_init(self, req: int, prefix_k: Sequence[np.ndarray], prefix_v: Sequence[np.ndarray],
                     capacity: int) -> None:
        sh = self.shape
        P = int(prefix_k[0].shape[0])
        if P < 1:
            raise ValueError("the committed context holds at least the root token")
        Ks, Vs = [], []
        for l in range(sh.n_layers):
            K = np.zeros((capacity, sh.n_kv_heads, sh.d_head), dtype=F64)
            V = np.zeros_like(K)
            K[:P] = prefix_k[l]
            V[:P] = prefix_v[l]
            Ks.append(K)
            Vs.append(V)
        self.req[req] = RequestState(P, SpecTree(), Ks, Vs, np.full(1, -1, dtype=np.int64))

    # -- layer appending; parents in the library's numbering (-1 = root) -------
    def tree_insert(self, req: int, parents: Sequence[int], tokens: Optional[Sequence[int]] = None,
                    probs: Optional[Sequence[float]] = None) -> int:
        st = self.req[req]
        first = st.tree.n - 1
        k = len(parents)
        tokens = [0] * k if tokens is None else tokens
        probs = [0.0] * k if probs is None else probs
        st.tree.append([p + 1 for p in parents], tokens, probs)
        st.pred = np.concatenate([st.pred, np.full(k, -1, dtype=np.int64)])
        return first

    # -- node-wise computation on nodes [first, first+n) (library numbering) ---
    def stage_forward(self, req: int, first: int, x: np.ndarray, mask: Optional[np.ndarray] = None) -> np.ndarray:
        """mask: attend under this matrix instead of the tree's own M (same indexing, root = 0).
        Positions still come from the true tree.  Tests use it to plant a wrong mask in the oracle
        and measure how far the outputs move."""
        sh = self.shape
        st = self.req[req]
        x = np.asarray(x, F64)
        n = x.shape[0]
        idx = np.arange(first + 1, first + 1 + n)                    # oracle tree indices
        if n and idx[-1] >= st.tree.n:
            raise ValueError("stage_forward: node not inserted")
        depth = st.tree.depth()
        pos = (st.P - 1) + depth[idx]
        slots = (st.P - 1) + idx
        committed = np.arange(st.P - 1)                              # everything before the root
        M = st.tree.M if mask is None else np.asarray(mask)
        visible = [np.concatenate([committed, (st.P - 1) + np.nonzero(M[i])[0]]) for i in idx]
        for l in range(sh.n_layers):
            x = decoder_layer(x, self.layer_weights(l), n_q_heads=sh.n_q_heads,
                              n_kv_heads=sh.n_kv_heads, d_head=sh.d_head, eps=sh.rms_eps,
                              theta=sh.rope_theta, pos=pos, K=st.K[l], V=st.V[l],
                              slots=slots, visible=visible)
        return x

    # -- pruning propagation ---------------------------------------------------
    def _apply(self, st: RequestState, pr: PruneResult, new_root: Optional[int]) -> None:
        n = st.tree.n
        lo = st.P - 1
        n_keep = int(pr.kv_keep.sum())
        for l in range(self.shape.n_layers):
            for C in (st.K[l], st.V[l]):
                C[lo:lo + n_keep] = compact_rows(C[lo:lo + n], pr.kv_keep)
        if new_root is not None:
            st.tree.to_subtree(new_root)          # tau_hat is the first kept node: it becomes the root
        else:
            st.tree.select(pr.table_keep)
        st.pred = st.pred[pr.table_keep]          # the new root's prediction is the accepted node's
        st.P += pr.n_commit

    def accept(self, req: int, node: int) -> PruneResult:
        """The verified token is speculative node `node` (library numbering)."""
        st = self.req[req]
        pr = accept_masks(st.tree, node + 1)
        self._apply(st, pr, node + 1)
        return pr

    def drop(self, req: int, node: int) -> PruneResult:
        st = self.req[req]
        pr = drop_masks(st.tree, node + 1)
        self._apply(st, pr, None)
        return pr

    def clear(self, req: int) -> PruneResult:
        """Pipeline stall: every speculative node goes, the root stays; nothing is committed."""
        st = self.req[req]
        keep = np.zeros(st.tree.n, dtype=bool)
        keep[0] = True
        pr = PruneResult(keep, keep.copy(), 0)
        self._apply(st, pr, None)
        return pr

    # -- verification on the last stage (Algorithm 1, "verify new token") ---------
    def set_root_pred(self, req: int, token: int) -> None:
        self.req[req].pred[0] = int(token)

    def verify_head(self, req: int, first: int, h: np.ndarray, gain: np.ndarray, w_vocab: np.ndarray):
        """Next-token predictions of nodes [first, first+n) from their last-layer outputs h.
        Returns (pred, logits)."""
        from .verify import lm_head_logits, greedy_token_fast
        st = self.req[req]
        logits = lm_head_logits(h, gain, w_vocab, self.shape.rms_eps)
        pred = greedy_token_fast(logits)
        st.pred[first + 1:first + 1 + len(pred)] = pred
        return pred, logits

    def match(self, req: int) -> int:
        """The root child that carries the model's token for the root's successor, or -1."""
        from .verify import match_root_child
        st = self.req[req]
        par, _, tok, _, _ = st.tree.view()
        return match_root_child(par, tok, int(st.pred[0]))

    def verify_lossy(self, req: int, h_root: np.ndarray, gain: np.ndarray, w_vocab: np.ndarray, mode: str,
                     top_p: float = 1.0):
        """Lossy verification of the root's children from the root's last-layer output h_root [d]
        (Sec. 3.4): mode "relaxed" or "top_p".  Returns (node or -1, top-1 token, logits) and
        records the top-1 token as the root's prediction."""
        from .verify import lm_head_logits, greedy_token_fast, relaxed_choice, top_p_choice
        st = self.req[req]
        logits = lm_head_logits(np.asarray(h_root)[None, :], gain, w_vocab, self.shape.rms_eps)[0]
        top1 = int(greedy_token_fast(logits[None, :])[0])
        par, _, tok, prob, _ = st.tree.view()
        if mode == "relaxed":
            node = relaxed_choice(logits, par, tok)
        elif mode == "top_p":
            node = top_p_choice(logits, par, tok, prob, top_p)
        else:
            raise ValueError(mode)
        st.pred[0] = top1
        return node, top1, logits

    @staticmethod
    def prune_hidden_rows(rows: np.ndarray, row_nodes: Sequence[int], pr: PruneResult) -> np.ndarray:
        """E_i pruned by the table mask: a row stays iff its node (library numbering) stays."""
        keep = np.array([bool(pr.table_keep[k + 1]) for k in row_nodes], dtype=bool)
        return compact_rows(rows, keep)

    # -- views for comparison ----------------------------------------------------
    def tree_kv(self, req: int, layer: int):
        """(K, V) rows of the speculative nodes, in node order."""
        st = self.req[req]
        lo, n = st.P, st.tree.n - 1
        return st.K[layer][lo:lo + n], st.V[layer][lo:lo + n]
