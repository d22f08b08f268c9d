"""Runs the HIP stage and the CPU oracle side by side on the same seeded inputs."""
from __future__ import annotations

from typing import Dict, List, Optional, Sequence

import numpy as np
import torch

import workloads as wl
import paper_2504_04104_amd as sp
from oracle import StageOracle


_OWN_STREAM = None


def use_own_stream():
    """The GPU tests run on a stream of their own, as bench.py does: the forward call captures and replays
    HIP graphs of its launches only on a stream that can be captured, and the parity tests should see that
    path whenever a shape comes back (streaming steps, repeated forwards)."""
    global _OWN_STREAM
    if _OWN_STREAM is None and torch.cuda.is_available():
        _OWN_STREAM = torch.cuda.Stream(device="cuda:0")
        torch.cuda.set_stream(_OWN_STREAM)


def elementwise_figure(gpu: np.ndarray, ref: np.ndarray, rtol: float, atol_rms: float = 1e-2) -> float:
    """The element-by-element figure next to the max-norm one: the largest |gpu - ref| measured in units of
    the allowance rtol * |ref| + atol_rms * rms(ref) of that element (<= 1 means every element is inside)."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    rms = float(np.sqrt(np.mean(ref * ref)))
    return float(np.max(np.abs(gpu - ref) / (rtol * np.abs(ref) + atol_rms * rms + 1e-300)))


def rel_err(gpu: np.ndarray, ref: np.ndarray) -> float:
    """max |gpu - ref| / max |ref| over a tensor."""
    ref = np.asarray(ref, np.float64)
    gpu = np.asarray(gpu, np.float64)
    return float(np.max(np.abs(gpu - ref)) / max(np.max(np.abs(ref)), 1e-30))


def to_np(t: torch.Tensor) -> np.ndarray:
    return t.detach().float().cpu().numpy()


def to_dev(a: np.ndarray, stage: sp.Stage) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(stage.device, stage.tdtype).contiguous()


class Pair:
    """A GPU stage and an oracle stage with identical weights and committed contexts."""

    def __init__(self, shape: wl.ModelShape, seed: int, prefixes: Dict[int, int], *, tree_room: int = 256 + 64,
                 flags: int = 0, max_batch_nodes: int = 64, oracle: bool = True, vocab: int = 0,
                 oracle_reqs: Optional[Sequence[int]] = None, page_slots: int = 0, head_gain: float = 1.0, head_distinct: int = 0,
                 norm1_gain: float = 1.0, prefix_k_scale: float = 1.0, weights=None):
        """norm1_gain (a power of two: exact in bf16) multiplies the gain of every attention RMSNorm, which
        scales the nodes' queries, keys and values; prefix_k_scale (same) the keys of the committed
        context.  Together they move the softmax mass between context and tree (mask tests)."""
        use_own_stream()
        self.shape, self.seed = shape, seed
        self.vocab = vocab
        self.pred_overrides = 0          # rows whose prediction the oracle took from the GPU (near-ties)
        # the float64 oracle may follow a sample of the requests only (large batches)
        self.oracle_reqs = None if oracle_reqs is None else set(oracle_reqs)
        if weights is None:
            self.weights = [wl.layer_weights(shape, seed, l) for l in range(shape.n_layers)]
            if norm1_gain != 1.0:
                for w in self.weights:
                    w["norm1"] = w["norm1"] * np.asarray(norm1_gain, w["norm1"].dtype)
            provider = self.weights.__getitem__
        else:
            # a callable layer -> weights: large models keep one layer at a time in host memory as float32
            self.weights = provider = weights
        layers = []
        for l in range(shape.n_layers):
            one = [sp.pack_layer_weights(provider(l), shape.dtype)]
            if flags & sp.SP_FLAG_PACKED_WEIGHTS:
                one = sp.pack_weights(shape, one)
            layers += one
        n_req = max(prefixes) + 1
        self.base: Dict[int, int] = {}
        self.cap: Dict[int, int] = {}
        self.page_slots = page_slots
        off = 0
        for r in sorted(prefixes):
            self.base[r] = 0 if page_slots else off
            self.cap[r] = prefixes[r] + tree_room
            off += self.cap[r] if not page_slots else -(-self.cap[r] // page_slots) * page_slots
        if page_slots:
            # paged cache: two extra requests are set up and released first, so that the free list
            # hands the real requests their pages out of physical order
            flags |= sp.SP_FLAG_PAGED_KV
            self.gpu = sp.Stage(shape, layers, kv_slots=off, max_requests=n_req + 2, max_batch_nodes=max_batch_nodes,
                                flags=flags, page_slots=page_slots)
            n_pages = off // page_slots
            a = max(1, n_pages // 3)
            self.gpu.request_init(n_req, 0, a * page_slots, a * page_slots)
            self.gpu.request_init(n_req + 1, 0, a * page_slots, a * page_slots)
            self.gpu.request_release(n_req)
            self.gpu.request_release(n_req + 1)
            assert self.gpu.free_pages() == n_pages
        else:
            self.gpu = sp.Stage(shape, layers, kv_slots=off, max_requests=n_req, max_batch_nodes=max_batch_nodes,
                                flags=flags)
        self.ora = StageOracle(shape, self.weights) if oracle else None
        if vocab:
            # output head of the last stage, same numbers on both sides
            self.head_np = wl.head_weights(shape, seed, vocab)
            if head_distinct:
                # vocabulary rows repeat with this period: logits tie exactly, on both sides
                self.head_np["wvocab"] = np.ascontiguousarray(self.head_np["wvocab"][np.arange(vocab) % head_distinct])
            # a power of two keeps the gains exact in bf16; larger gains make the distribution peakier
            self.head_np["norm"] = self.head_np["norm"] * np.asarray(head_gain, self.head_np["norm"].dtype)
            td = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
            wv = torch.from_numpy(self.head_np["wvocab"]).to("cuda:0", td).contiguous()
            if flags & sp.SP_FLAG_PACKED_WEIGHTS:
                wv = sp.pack_matrix(wv)
            self.head = {"norm": torch.from_numpy(self.head_np["norm"]).to("cuda:0", td).contiguous(), "wvocab": wv}
        for r, P in prefixes.items():
            pk, pv = zip(*[wl.prefix_kv(shape, seed, l, P, req=r) for l in range(shape.n_layers)])
            if prefix_k_scale != 1.0:
                pk = tuple(k * np.asarray(prefix_k_scale, k.dtype) for k in pk)
            if page_slots:
                self.gpu.request_init(r, 0, self.cap[r], P)          # takes the pages of the context
                idx = self.gpu.logical_slots(r, 0, P)
                kv = self.gpu.kv_view()
                for l in range(shape.n_layers):
                    kv[l, 0].index_copy_(1, idx, to_dev(pk[l], self.gpu).permute(1, 0, 2).contiguous())
                    kv[l, 1].index_copy_(1, idx, to_dev(pv[l], self.gpu).permute(1, 0, 2).contiguous())
            else:
                for l in range(shape.n_layers):
                    sp.write_prefix(self.gpu, l, self.base[r], pk[l], pv[l])
                self.gpu.request_init(r, self.base[r], self.cap[r], P)
            if self.ora is not None and (self.oracle_reqs is None or r in self.oracle_reqs):
                self.ora.request_init(r, pk, pv, self.cap[r])

    # -- the same call on both sides ------------------------------------------------
    def insert(self, req: int, parents: Sequence[int], tokens=None, probs=None) -> int:
        first = self.gpu.tree_insert(req, parents, tokens, probs)
        if self.ora is not None and (self.oracle_reqs is None or req in self.oracle_reqs):
            assert self.ora.tree_insert(req, parents, tokens, probs) == first
        return first

    def insert_batch(self, reqs: Sequence[int], parents_per_req, tokens_per_req=None, probs_per_req=None):
        """One launch for several requests on the GPU; one by one on the oracle."""
        firsts = self.gpu.tree_insert_batch(reqs, parents_per_req, tokens_per_req, probs_per_req)
        if self.ora is not None:
            for i, r in enumerate(reqs):
                if self.oracle_reqs is None or r in self.oracle_reqs:
                    f = self.ora.tree_insert(r, parents_per_req[i],
                                             None if tokens_per_req is None else tokens_per_req[i],
                                             None if probs_per_req is None else probs_per_req[i])
                    assert f == firsts[i]
        return firsts

    def forward(self, reqs: Sequence[int], firsts: Sequence[int], counts: Sequence[int], x: np.ndarray):
        """x: [sum counts, d] float32 (already rounded to the storage type).  Returns (gpu, oracle)."""
        y = to_np(self.gpu.stage_forward(reqs, firsts, counts, to_dev(x, self.gpu)))
        ref = None
        if self.ora is not None:
            outs, row = [], 0
            for r, f, n in zip(reqs, firsts, counts):
                if n:
                    outs.append(self.ora.stage_forward(r, f, x[row:row + n]))
                row += n
            ref = np.concatenate(outs) if outs else np.zeros_like(x, dtype=np.float64)
        return y, ref

    def verify_head(self, reqs: Sequence[int], firsts: Sequence[int], counts: Sequence[int], y_dev: torch.Tensor,
                    tol: float, max_differ: Optional[int] = None):
        """Output head + top-1 on both sides, the oracle fed with the GPU's own rows so that only the
        head is compared.  A row passes if the GPU's token is the oracle's, or if the oracle's logit of
        the GPU's token is within `tol` (relative to the largest |logit|) of the oracle's maximum: the
        GPU decides in bf16/fp32 arithmetic, the oracle in float64, and near-ties may fall either way.
        The oracle's state then takes the GPU's decision, as a real last stage would.
        Returns (gpu predictions, number of rows decided differently)."""
        pred, mx = self.gpu.verify_head(self.head, reqs, firsts, counts, y_dev, want_max=True)
        pred = pred.cpu().numpy().astype(np.int64)
        mx = mx.cpu().numpy().astype(np.float64)
        rows = to_np(y_dev).astype(np.float64)
        row, differ = 0, 0
        for r, f, n in zip(reqs, firsts, counts):
            if not n:
                continue
            want, logits = self.ora.verify_head(r, f, rows[row:row + n], self.head_np["norm"], self.head_np["wvocab"])
            scale = np.max(np.abs(logits))
            for i in range(n):
                g = int(pred[row + i])
                assert 0 <= g < self.vocab
                top = logits[i].max()
                assert logits[i, g] >= top - tol * scale, ("token far from the maximum", r, f + i, g, int(want[i]))
                assert abs(mx[row + i] - logits[i, g]) <= tol * scale, ("winning logit", r, f + i)
                if g != int(want[i]):
                    differ += 1
                    # both are maxima up to the tolerance; the lower index must win an exact tie
                    assert not (logits[i, g] == top and g > int(want[i]))
                    self.ora.req[r].pred[f + 1 + i] = g
            row += n
        # near-ties are rare: more than one row in 32 decided differently is a defect, not rounding
        total = int(sum(counts))
        assert differ <= (max(1, total // 32) if max_differ is None else max_differ), (differ, total)
        self.pred_overrides += differ
        return pred, differ

    def verify_lossy(self, reqs: Sequence[int], x_root: torch.Tensor, mode: str, top_p: float, tol: float):
        """Relaxed / top-p verification of the roots' children on both sides, the oracle fed with the
        GPU's own root rows.  The GPU forms logits in bf16/fp32 arithmetic and probabilities in
        float32, the oracle everything in float64, so the comparison leaves a margin around each
        decision: `tol` (relative to the largest |logit|) on logits, and the probability mass that
        such a logit error can move around top_p.  Outside the margins the decisions must be
        equal.  Returns the GPU's [(node, top1)] and how many requests had a decision inside a margin."""
        from oracle.verify import softmax_probs
        got = self.gpu.verify_lossy(self.head, reqs, x_root, sp.SP_VERIFY_RELAXED if mode == "relaxed" else sp.SP_VERIFY_TOP_P,
                                    top_p)
        rows = to_np(x_root).astype(np.float64)
        marginal = 0
        for i, r in enumerate(reqs):
            node, top1 = got[i]
            want, want_top1, logits = self.ora.verify_lossy(r, rows[i], self.head_np["norm"], self.head_np["wvocab"],
                                                             mode, top_p)
            scale = np.max(np.abs(logits))
            eps = tol * scale
            assert 0 <= top1 < self.vocab and logits[top1] >= logits.max() - eps, ("top-1 far from the maximum", r)
            assert not (logits[top1] == logits.max() and top1 > want_top1)
            self.ora.req[r].pred[0] = top1                       # the oracle follows the GPU's decision
            par, _, tok, prob, _ = self.ora.req[r].tree.view()
            cand = [k for k in range(len(par)) if par[k] == -1 and 0 <= tok[k] < self.vocab]
            if mode == "relaxed":
                if not cand:
                    assert node == -1 == want
                    continue
                assert node in cand, (r, node)
                best = max(logits[tok[k]] for k in cand)
                assert logits[tok[node]] >= best - eps, ("candidate far from the best", r, node, want)
                close = [k for k in cand if logits[tok[k]] >= best - 2 * eps]
                if len(close) == 1:
                    assert node == want, (r, node, want)
                else:
                    marginal += 1
                    assert not (logits[tok[node]] == best and node > want)
                continue
            # The mass in front of a candidate's token, bracketed.  A logit error of eps moves a probability by
            # a factor within exp(+-2 eps) (numerator and normaliser); as the masses in front of and behind the
            # token add up to one, the smaller of the two bounds the shift.  Tokens whose logit is within 2 eps
            # of the candidate's may also be counted on either side.
            probs = softmax_probs(logits)
            rank = sorted(range(self.vocab), key=lambda v: (-probs[v], v))
            before = np.zeros(self.vocab)
            before[rank] = np.concatenate(([0.0], np.cumsum(probs[rank])[:-1]))
            sure_in, maybe = [], []
            for k in cand:
                t = tok[k]
                near = float(np.sum(probs[np.abs(logits - logits[t]) <= 2 * eps])) - float(probs[t])
                slack = 4 * eps * min(before[t], 1.0 - before[t]) + near + 1e-6
                if before[t] + slack < top_p:
                    sure_in.append(k)
                elif before[t] - slack < top_p:
                    maybe.append(k)
            if not maybe:
                assert node == want, (r, node, want)
                continue
            marginal += 1
            if node == -1:
                assert not sure_in, (r, want)
            else:
                assert node in sure_in or node in maybe, (r, node)
                assert all(np.float32(prob[node]) >= np.float32(prob[k]) for k in sure_in), (r, node, want)
        return got, marginal

    def tree_region(self, req: int, P: int, n: int) -> torch.Tensor:
        """Raw slab rows of tree slots [P, P+n): [layer, K|V, head, n, d_head] (a copy)."""
        return self.rows(req, P, P + n)

    def rows(self, req: int, lo: int, hi: int) -> torch.Tensor:
        """The request's logical cache slots [lo, hi) of every plane (a copy), whatever the storage."""
        if self.page_slots:
            if hi <= lo:
                return self.gpu.kv_view()[:, :, :, 0:0, :].clone()
            return self.gpu.kv_view().index_select(3, self.gpu.logical_slots(req, lo, hi))
        b = self.base[req]
        return self.gpu.kv_view()[:, :, :, b + lo:b + hi, :].clone()

    def check_tables(self, req: int):
        v = self.gpu.tree_read(req)
        st = self.ora.req[req]
        par, dep, tok, prob, M = st.tree.view()
        assert v["prefix_len"] == st.P, (v["prefix_len"], st.P)
        assert v["n_live"] == len(par)
        assert np.array_equal(v["parent"], par)
        assert np.array_equal(v["depth"], dep)
        assert np.array_equal(v["token"], tok)
        assert np.array_equal(v["prob"].view(np.uint32), prob.view(np.uint32))
        assert np.array_equal(v["M"], M)
        assert np.array_equal(v["pred"], st.pred[1:]), (v["pred"], st.pred[1:])
        assert v["root_pred"] == st.pred[0]
        assert self.gpu.request_info(req)[:2] == (st.P, len(par))

    def check_kv(self, req: int, tol: float):
        """Tree-region K/V rows of every layer against the oracle's."""
        st = self.ora.req[req]
        n = st.tree.n - 1
        if n == 0:
            return
        g = self.tree_region(req, st.P, n).float().cpu().numpy()
        for l in range(self.shape.n_layers):
            K, V = self.ora.tree_kv(req, l)                  # [n, H, d]
            assert rel_err(g[l, 0].transpose(1, 0, 2), K) <= tol, ("K", l)
            assert rel_err(g[l, 1].transpose(1, 0, 2), V) <= tol, ("V", l)

    def prune(self, req: int, mode: int, node: int, x_rows: Optional[np.ndarray] = None,
              row_nodes: Optional[Sequence[int]] = None):
        """Prune + compact on both sides.  Checks that the cache compaction is the oracle's
        stable selection applied to the GPU's own bytes, bit for bit, that rows in front of
        the first dropped slot did not change, and the tables.  Returns surviving hidden rows
        (gpu, oracle) if x_rows was given."""
        st = self.ora.req[req]
        P_old, T_old = st.P, st.tree.n - 1
        before = self.tree_region(req, P_old, T_old)
        untouched = self.rows(req, 0, P_old)
        live, commit = self.gpu.tree_prune(req, mode, node)
        pr = (self.ora.accept(req, node) if mode == sp.SP_ACCEPT else
              self.ora.drop(req, node) if mode == sp.SP_DROP else self.ora.clear(req))
        assert commit == pr.n_commit and live == st.tree.n - 1
        xg = None
        if x_rows is not None:
            xg = to_dev(x_rows, self.gpu)
            n_out, new_nodes = self.gpu.kv_compact(req, xg, row_nodes)
        else:
            self.gpu.kv_compact(req)
        keep = pr.kv_keep[1:]
        n_keep = int(keep.sum())
        after = self.tree_region(req, P_old, n_keep)
        sel = torch.from_numpy(np.nonzero(keep)[0]).to(before.device)
        expect = before.index_select(3, sel)                # oracle: rows[keep], stable
        assert expect.shape[3] == n_keep
        assert torch.equal(after.view(torch.uint8), expect.contiguous().view(torch.uint8))
        now = self.rows(req, 0, P_old)
        assert torch.equal(now.contiguous().view(torch.uint8), untouched.contiguous().view(torch.uint8))
        if self.page_slots:
            # exactly the pages of the live slots stay with the request
            live_slots = self.ora.req[req].P + self.ora.req[req].tree.n - 1
            assert len(self.gpu.request_pages(req)) == -(-live_slots // self.page_slots)
        self.check_tables(req)
        if x_rows is not None:
            ref = self.ora.prune_hidden_rows(x_rows, row_nodes, pr)
            assert n_out == ref.shape[0]
            tab_new = np.cumsum(pr.table_keep) - 1           # new oracle index (root = 0)
            want = [int(tab_new[k + 1]) - 1 if mode == sp.SP_ACCEPT else int(tab_new[k + 1]) - 1
                    for k in row_nodes if pr.table_keep[k + 1]]
            assert new_nodes == want, (new_nodes, want)
            got = to_np(xg[:n_out])
            assert np.array_equal(got, ref.astype(np.float32))
            return got, ref
        return None

    def prune_verified(self, reqs: Sequence[int], nodes_dev: torch.Tensor, want_nodes: Sequence[int], stride: int = 1):
        """sp_tree_prune_verified (prune + compaction decided on the device from nodes_dev) against the
        oracle's accept / clear of want_nodes: same checks as prune(), the cache compared bit for bit."""
        before = {}
        for r in reqs:
            st = self.ora.req[r]
            before[r] = (st.P, self.tree_region(r, st.P, st.tree.n - 1), self.rows(r, 0, st.P))
        self.gpu.tree_prune_verified(reqs, nodes_dev, stride)
        for r, node in zip(reqs, want_nodes):
            st = self.ora.req[r]
            pr = self.ora.accept(r, node) if node >= 0 else self.ora.clear(r)
            P_old, reg, ctx = before[r]
            keep = pr.kv_keep[1:]
            sel = torch.from_numpy(np.nonzero(keep)[0]).to(reg.device)
            after = self.tree_region(r, P_old, int(keep.sum()))
            assert torch.equal(after.view(torch.uint8), reg.index_select(3, sel).contiguous().view(torch.uint8))
            assert torch.equal(self.rows(r, 0, P_old).contiguous().view(torch.uint8), ctx.contiguous().view(torch.uint8))
            self.check_tables(r)                         # also the host mirror: prefix_len and n_live
            if self.page_slots:
                live_slots = st.P + st.tree.n - 1
                assert len(self.gpu.request_pages(r)) == -(-live_slots // self.page_slots)

    def close(self):
        self.gpu.close()
