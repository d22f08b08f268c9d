"""Seeded synthetic inputs for the SpecPipe stage hot path.

This module is the only code shared by the CPU oracle and the HIP path.  It
holds no arithmetic of the method itself: it draws random numbers, rounds them
to the storage type, and draws tree shapes and prune schedules.  Everything is
a pure function of (seed, tensor name), so a tensor can be regenerated in any
process without shipping files around.

Shapes follow the paper's workloads: Llama-family decoder layers (Sec. 4,
"Testbed" and "GPU Memory Analysis"), a tree of at most w nodes per level
(Sec. 3.3.3, "Fixed-width tree"), a context of a few thousand to tens of
thousands of tokens (Fig. "scalinginference", Sec. 3.3.1), and up to 32
concurrent requests (Sec. 4.4).
"""
from __future__ import annotations

import hashlib
from dataclasses import dataclass, field, replace
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

__all__ = [
    "ModelShape", "Workload", "CONFIGS", "round_bf16", "to_bf16_bits", "from_bf16_bits",
    "rng", "normal", "layer_weights", "prefix_kv", "tree_uniform_parents",
    "tree_branching", "tree_deep", "tree_chain", "tree_star", "tree_static_levels", "bfs_sorted", "scaled", "hidden_rows",
    "levels_of", "PruneOp", "StreamStep", "streaming_schedule", "BatchRequest",
    "batch_requests", "batch_schedule",
]


# ----------------------------------------------------------------------------
# storage-type rounding (inputs only)
# ----------------------------------------------------------------------------
def round_bf16(a: np.ndarray) -> np.ndarray:
    """Round a float32 array to the nearest bfloat16 (ties to even) and return
    it as float32 again, so both sides read bit-identical values."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    u = a.view(np.uint32)
    bias = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    r = (u + bias) & np.uint32(0xFFFF0000)
    return r.view(np.float32)


def to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 values that are already bf16-representable -> uint16 bit patterns."""
    a = np.ascontiguousarray(a, dtype=np.float32)
    return (a.view(np.uint32) >> np.uint32(16)).astype(np.uint16)


def from_bf16_bits(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> float32."""
    b = np.ascontiguousarray(b, dtype=np.uint16)
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ----------------------------------------------------------------------------
# counter-based random streams
# ----------------------------------------------------------------------------
def rng(seed: int, *name) -> np.random.Generator:
    """Philox stream keyed by (seed, name): independent per tensor, reproducible
    in any process and any generation order."""
    h = hashlib.sha256(("%d|" % seed + "|".join(str(x) for x in name)).encode()).digest()
    key = int.from_bytes(h[:16], "little")
    return np.random.Generator(np.random.Philox(key=key))


def normal(seed: int, name: Sequence, shape, std: float = 1.0, mean: float = 0.0,
           dtype: str = "f32") -> np.ndarray:
    """N(mean, std) float32 tensor; rounded to bf16 when dtype == 'bf16'."""
    g = rng(seed, *name)
    a = g.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    if mean != 0.0:
        a += np.float32(mean)
    if dtype == "bf16":
        a = round_bf16(a)
    return a


# ----------------------------------------------------------------------------
# model shapes and the named configurations
# ----------------------------------------------------------------------------
@dataclass(frozen=True)
class ModelShape:
    n_layers: int
    d_model: int
    n_q_heads: int
    n_kv_heads: int
    d_head: int
    d_ff: int
    rms_eps: float = 1e-5
    rope_theta: float = 500000.0
    dtype: str = "bf16"          # storage type of weights / activations / KV: 'f32' or 'bf16'

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def d_q(self) -> int:
        return self.n_q_heads * self.d_head

    @property
    def d_kv(self) -> int:
        return self.n_kv_heads * self.d_head

    @property
    def params_per_layer(self) -> int:
        d, f = self.d_model, self.d_ff
        return d * (self.d_q + 2 * self.d_kv) + self.d_q * d + 3 * d * f

    @property
    def elt_bytes(self) -> int:
        return 2 if self.dtype == "bf16" else 4

    @property
    def kv_bytes_per_token_per_layer(self) -> int:
        return 2 * self.d_kv * self.elt_bytes


@dataclass(frozen=True)
class Workload:
    name: str
    seed: int
    shape: ModelShape
    prefix_len: int = 0
    n_nodes: int = 0
    max_levels: int = 0
    max_children: int = 0
    note: str = ""


TINY = ModelShape(2, 256, 4, 4, 64, 688, rms_eps=1e-6, dtype="f32")
LLAMA_8B_STAGE = ModelShape(4, 4096, 32, 8, 128, 14336)
LLAMA_70B_STAGE = ModelShape(10, 8192, 64, 8, 128, 28672)

CONFIGS: Dict[str, Workload] = {
    "C1": Workload("C1", 0, TINY, prefix_len=128, n_nodes=16, max_levels=6,
                   note="tiny fp32 stage; uniform random parents; forward, drop a subtree, compact"),
    "C2": Workload("C2", 1, LLAMA_8B_STAGE, prefix_len=2048, n_nodes=64, max_levels=8,
                   max_children=4, note="8B-shaped 4-layer stage, one tree of 64 nodes"),
    "C3": Workload("C3", 2, LLAMA_70B_STAGE, prefix_len=4096, n_nodes=128, max_levels=12,
                   max_children=4, note="70B-shaped 10-layer stage, one tree of 128 nodes"),
    "C4": Workload("C4", 3, LLAMA_8B_STAGE, prefix_len=32768, n_nodes=256,
                   note="streaming: 512 steps of insert 1-8 / forward / prune, <=256 live nodes"),
    "C5": Workload("C5", 4, LLAMA_8B_STAGE, prefix_len=4096, n_nodes=32, max_levels=6,
                   note="32 requests, ragged batch, 64 steps"),
}


def scaled(shape: ModelShape, **kw) -> ModelShape:
    """A shape with some fields replaced (used for small parity cases)."""
    return replace(shape, **kw)


# ----------------------------------------------------------------------------
# tensors
# ----------------------------------------------------------------------------
WEIGHT_STD = 0.02


def layer_weights(shape: ModelShape, seed: int, layer: int) -> Dict[str, np.ndarray]:
    """Weights of one decoder layer, every matrix stored [out_features, in_features]
    row-major (y = x W^T).  Projections are N(0, 0.02); the two RMSNorm gains are
    1 + N(0, 0.02) so that a dropped or misplaced gain shows up in parity."""
    d, f = shape.d_model, shape.d_ff
    dt = shape.dtype
    w = {
        "wq": normal(seed, ("wq", layer), (shape.d_q, d), WEIGHT_STD, dtype=dt),
        "wk": normal(seed, ("wk", layer), (shape.d_kv, d), WEIGHT_STD, dtype=dt),
        "wv": normal(seed, ("wv", layer), (shape.d_kv, d), WEIGHT_STD, dtype=dt),
        "wo": normal(seed, ("wo", layer), (d, shape.d_q), WEIGHT_STD, dtype=dt),
        "wg": normal(seed, ("wg", layer), (f, d), WEIGHT_STD, dtype=dt),
        "wu": normal(seed, ("wu", layer), (f, d), WEIGHT_STD, dtype=dt),
        "wd": normal(seed, ("wd", layer), (d, f), WEIGHT_STD, dtype=dt),
        "norm1": normal(seed, ("norm1", layer), (d,), WEIGHT_STD, mean=1.0, dtype=dt),
        "norm2": normal(seed, ("norm2", layer), (d,), WEIGHT_STD, mean=1.0, dtype=dt),
    }
    return w


def prefix_kv(shape: ModelShape, seed: int, layer: int, prefix_len: int, req: int = 0
              ) -> Tuple[np.ndarray, np.ndarray]:
    """Synthetic committed-context cache of one layer: K and V, each
    [prefix_len, n_kv_heads, d_head], N(0,1), taken to be post-RoPE."""
    k = normal(seed, ("pk", layer, req), (prefix_len, shape.n_kv_heads, shape.d_head), dtype=shape.dtype)
    v = normal(seed, ("pv", layer, req), (prefix_len, shape.n_kv_heads, shape.d_head), dtype=shape.dtype)
    return k, v


def head_weights(shape: ModelShape, seed: int, vocab: int) -> Dict[str, np.ndarray]:
    """Output head of the last stage: final RMSNorm gain 1 + N(0, 0.02) and the vocabulary
    projection [vocab, d_model], N(0, 0.02) (y = x W^T)."""
    return {
        "norm": normal(seed, ("head_norm",), (shape.d_model,), WEIGHT_STD, mean=1.0, dtype=shape.dtype),
        "wvocab": normal(seed, ("head_vocab",), (vocab, shape.d_model), WEIGHT_STD, dtype=shape.dtype),
    }


def embedding_table(shape: ModelShape, seed: int, vocab: int) -> np.ndarray:
    """Input embeddings [vocab, d_model], N(0, 1): the hidden row that enters the first layer
    for a token."""
    return normal(seed, ("embed",), (vocab, shape.d_model), dtype=shape.dtype)


def hidden_rows(shape: ModelShape, seed: int, name: Sequence, n: int) -> np.ndarray:
    """Input hidden states of n tree nodes, N(0,1), [n, d_model]."""
    return normal(seed, ("x",) + tuple(name), (n, shape.d_model), dtype=shape.dtype)


# ----------------------------------------------------------------------------
# tree shapes.  A tree is a parent list: parents[i] in {-1} U [0, i); -1 means
# "child of the last committed token".  levels_of() counts levels starting at 0.
# ----------------------------------------------------------------------------
def levels_of(parents: Sequence[int]) -> List[int]:
    lev: List[int] = []
    for i, p in enumerate(parents):
        assert -1 <= p < i
        lev.append(0 if p < 0 else lev[p] + 1)
    return lev


def tree_uniform_parents(seed: int, n: int, max_levels: int, name: Sequence = ("tree",)) -> List[int]:
    """Node i's parent is uniform in [-1, i-1]; a draw that would create level
    max_levels is repeated."""
    g = rng(seed, *name)
    parents: List[int] = []
    lev: List[int] = []
    for i in range(n):
        while True:
            p = int(g.integers(-1, i))  # high exclusive: -1 .. i-1
            l = 0 if p < 0 else lev[p] + 1
            if l < max_levels:
                break
        parents.append(p)
        lev.append(l)
    return parents


def tree_branching(seed: int, n: int, max_children: int, max_levels: int,
                   name: Sequence = ("tree",)) -> List[int]:
    """Sequential attachment with a cap on children per node (the committed
    tail included) and on the number of levels: every internal node ends up
    with 1..max_children children."""
    g = rng(seed, *name)
    parents: List[int] = []
    lev: List[int] = []
    nchild = {-1: 0}
    for i in range(n):
        elig = [j for j in range(-1, i)
                if nchild[j] < max_children and (j < 0 or lev[j] + 1 < max_levels)]
        if not elig:
            raise ValueError("tree_branching: no eligible parent (n too large for the caps)")
        p = elig[int(g.integers(0, len(elig)))]
        parents.append(p)
        lev.append(0 if p < 0 else lev[p] + 1)
        nchild[p] += 1
        nchild[i] = 0
    return parents


def tree_deep(seed: int, n: int, max_levels: int, window: int = 6, name: Sequence = ("deep",)) -> List[int]:
    """A deep, narrow tree: node i's parent is uniform among the `window` nodes before it (the
    committed tail while i < window), so levels grow with the index and a late node's ancestors are
    spread over the whole index range; a draw that would create level max_levels is repeated over all
    earlier nodes."""
    g = rng(seed, *name)
    parents: List[int] = []
    lev: List[int] = []
    for i in range(n):
        lo = max(-1, i - window)
        p = int(g.integers(lo, i))
        l = 0 if p < 0 else lev[p] + 1
        while l >= max_levels:
            p = int(g.integers(-1, i))
            l = 0 if p < 0 else lev[p] + 1
        parents.append(p)
        lev.append(l)
    return parents


def tree_chain(n: int) -> List[int]:
    return [i - 1 for i in range(n)]


def tree_star(n: int) -> List[int]:
    return [-1] * n


def tree_static_levels(widths: Sequence[int]) -> List[int]:
    """A static tree given by per-level branching: level l has prod(widths[:l+1])
    nodes, each node of level l-1 getting widths[l] children; BFS order."""
    parents: List[int] = []
    prev = [-1]
    for w in widths:
        cur = []
        for p in prev:
            for _ in range(w):
                cur.append(len(parents))
                parents.append(p)
        prev = cur
    return parents


def bfs_sorted(parents: Sequence[int]) -> Tuple[List[int], List[int]]:
    """Re-index a tree level by level, each level ordered by its parents' new
    order (the order the paper's layer appending assumes).  Returns (parents in
    the new indexing, order) where order[new] = old."""
    n = len(parents)
    lev = levels_of(parents)
    new_of = {-1: -1}
    order: List[int] = []
    for l in range((max(lev) + 1) if n else 0):
        nodes = [i for i in range(n) if lev[i] == l]
        nodes.sort(key=lambda i: (new_of[parents[i]], i))
        for i in nodes:
            new_of[i] = len(order)
            order.append(i)
    return [new_of[parents[old]] for old in order], order


# ----------------------------------------------------------------------------
# streaming and batch schedules
# ----------------------------------------------------------------------------
ACCEPT = 0
DROP = 1


@dataclass
class PruneOp:
    mode: int      # ACCEPT or DROP
    node: int


@dataclass
class StreamStep:
    parents: List[int]            # parents of the nodes inserted in this step (indices at insert time)
    prune: Optional[PruneOp]      # prune applied after the forward


class _HostTree:
    """Bookkeeping for schedule generation only: the live tree as a parent list."""

    def __init__(self):
        self.parents: List[int] = []

    def levels(self):
        return levels_of(self.parents)

    def descendants(self, x: int) -> List[bool]:
        n = len(self.parents)
        inside = [False] * n
        inside[x] = True
        for i in range(x + 1, n):
            p = self.parents[i]
            if p >= 0 and inside[p]:
                inside[i] = True
        return inside

    def apply(self, op: PruneOp):
        n = len(self.parents)
        inside = self.descendants(op.node)
        if op.mode == ACCEPT:
            keep = [inside[i] and i != op.node for i in range(n)]
        else:
            keep = [not inside[i] for i in range(n)]
        new_idx = {}
        out: List[int] = []
        for i in range(n):
            if keep[i]:
                new_idx[i] = len(out)
                p = self.parents[i]
                out.append(new_idx[p] if (p >= 0 and keep[p]) else -1)
        self.parents = out


def streaming_schedule(seed: int, n_steps: int, max_new: int = 8, cap: int = 256,
                       p_accept: float = 0.7, max_levels: int = 0,
                       name: Sequence = ("stream",), initial: Sequence[int] = ()) -> List[StreamStep]:
    """Per step: insert 1..max_new nodes under uniformly random live nodes or the
    committed tail (clamped so the tree never exceeds `cap` live nodes), then
    with probability p_accept accept a random child of the committed tail (the
    root advances, its siblings' subtrees go), else drop a random subtree."""
    g = rng(seed, *name)
    t = _HostTree()
    t.parents = list(initial)          # the live tree the schedule starts from (empty by default)
    steps: List[StreamStep] = []
    for _ in range(n_steps):
        n_new = int(g.integers(1, max_new + 1))
        n_new = min(n_new, cap - len(t.parents))
        new_par: List[int] = []
        for _k in range(n_new):
            cur = len(t.parents)
            while True:
                p = int(g.integers(-1, cur))
                if max_levels <= 0 or p < 0 or levels_of(t.parents)[p] + 1 < max_levels:
                    break
            t.parents.append(p)
            new_par.append(p)
        op: Optional[PruneOp] = None
        if t.parents:
            roots = [i for i, p in enumerate(t.parents) if p < 0]
            if float(g.random()) < p_accept:
                op = PruneOp(ACCEPT, roots[int(g.integers(0, len(roots)))])
            else:
                op = PruneOp(DROP, int(g.integers(0, len(t.parents))))
            t.apply(op)
        steps.append(StreamStep(new_par, op))
    return steps


@dataclass
class BatchRequest:
    req: int
    prefix_len: int
    target_nodes: int
    parents: List[int] = field(default_factory=list)


def batch_requests(seed: int, n_req: int = 32, p_lo: int = 512, p_hi: int = 4096,
                   t_lo: int = 8, t_hi: int = 32, max_levels: int = 6,
                   name: Sequence = ("batch",)) -> List[BatchRequest]:
    """Requests of the dynamic batch: own prefix length, own initial tree."""
    g = rng(seed, *name)
    out: List[BatchRequest] = []
    for r in range(n_req):
        p = int(g.integers(p_lo, p_hi + 1))
        t = int(g.integers(t_lo, t_hi + 1))
        parents = tree_uniform_parents(seed, t, max_levels, name=tuple(name) + ("tree", r))
        out.append(BatchRequest(r, p, t, parents))
    return out


def batch_schedule(seed: int, reqs: Sequence[BatchRequest], n_steps: int, max_new: int = 8,
                   max_levels: int = 6, p_accept: float = 0.7,
                   name: Sequence = ("batchsched",)) -> List[List[StreamStep]]:
    """Steady-state steps of the dynamic batch.  Step s holds one StreamStep per
    request: prune first (accept a child of the tail w.p. p_accept, else drop a
    random subtree), then insert 1..max_new nodes clamped to the request's drawn
    tree size and level cap.  Here the prune of a step precedes its insert, so
    StreamStep.prune is applied BEFORE StreamStep.parents."""
    g = rng(seed, *name)
    trees = []
    for r in reqs:
        t = _HostTree()
        t.parents = list(r.parents)
        trees.append(t)
    steps: List[List[StreamStep]] = []
    for _ in range(n_steps):
        row: List[StreamStep] = []
        for r, t in zip(reqs, trees):
            op: Optional[PruneOp] = None
            if t.parents:
                roots = [i for i, p in enumerate(t.parents) if p < 0]
                if float(g.random()) < p_accept:
                    op = PruneOp(ACCEPT, roots[int(g.integers(0, len(roots)))])
                else:
                    op = PruneOp(DROP, int(g.integers(0, len(t.parents))))
                t.apply(op)
            n_new = int(g.integers(1, max_new + 1))
            n_new = max(0, min(n_new, r.target_nodes - len(t.parents)))
            new_par: List[int] = []
            for _k in range(n_new):
                cur = len(t.parents)
                lev = levels_of(t.parents)
                while True:
                    p = int(g.integers(-1, cur))
                    if p < 0 or lev[p] + 1 < max_levels:
                        break
                t.parents.append(p)
                new_par.append(p)
            row.append(StreamStep(new_par, op))
        steps.append(row)
    return steps
