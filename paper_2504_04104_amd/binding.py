"""ctypes binding of libspecpipe.so: argument marshalling only.

Every step of the stage path runs inside the library's HIP kernels; this module
turns Python/torch arguments into the pointers and sizes of include/specpipe.h and
raises on a non-zero status.  torch is used for device memory and streams only.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libspecpipe.so")

SP_MAX_TREE_NODES = 256
SP_MAX_BATCH_REQ = 64
SP_F32, SP_BF16 = 0, 1
SP_ACCEPT, SP_DROP, SP_CLEAR = 0, 1, 2
SP_VERIFY_RELAXED, SP_VERIFY_TOP_P = 1, 2
SP_FLAG_SIMPLE_KERNELS = 1
SP_FLAG_PACKED_WEIGHTS = 2
SP_FLAG_PAGED_KV = 4
SP_FLAG_NO_GRAPHS = 8

# sp_kernel_kind
K_GEMM_QKV, K_GEMM_O, K_GEMM_GATEUP, K_GEMM_DOWN = 1, 2, 3, 4
K_ATTENTION, K_ATTENTION_MERGE, K_KV_COMPACT, K_TREE_PRUNE, K_TREE_INSERT, K_NORM, K_ROPE_KV = 5, 6, 7, 8, 9, 10, 11
K_VERIFY_HEAD = 12

STATUS = {0: "SP_OK", -1: "SP_E_INVALID", -2: "SP_E_CAPACITY", -3: "SP_E_BAD_PARENT", -4: "SP_E_BAD_REQ",
          -5: "SP_E_BAD_NODE", -6: "SP_E_ORDER", -7: "SP_E_PENDING", -8: "SP_E_HIP", -9: "SP_E_UNSUPPORTED"}


class SpError(RuntimeError):
    def __init__(self, status: int, what: str):
        self.status = status
        super().__init__("%s failed: %s (%d)" % (what, STATUS.get(status, "?"), status))


class sp_config(C.Structure):
    _fields_ = [("n_layers", C.c_int32), ("d_model", C.c_int32), ("n_q_heads", C.c_int32),
                ("n_kv_heads", C.c_int32), ("d_head", C.c_int32), ("d_ff", C.c_int32),
                ("rms_eps", C.c_float), ("rope_theta", C.c_float), ("dtype", C.c_int32),
                ("max_requests", C.c_int32), ("max_tree_nodes", C.c_int32), ("max_batch_nodes", C.c_int32),
                ("kv_slots", C.c_int64), ("flags", C.c_uint32), ("page_slots", C.c_int32)]


class sp_layer_weights(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("wqkv", "wo", "wgu", "wd", "norm1", "norm2")]


class sp_sizes(C.Structure):
    _fields_ = [(n, C.c_size_t) for n in ("kv_bytes", "tables_bytes", "workspace_bytes", "kv_plane_bytes",
                                          "kv_row_bytes")]


class sp_buffers(C.Structure):
    _fields_ = [("kv", C.c_void_p), ("kv_bytes", C.c_size_t), ("tables", C.c_void_p), ("tables_bytes", C.c_size_t),
                ("workspace", C.c_void_p), ("workspace_bytes", C.c_size_t)]


class sp_tree_view(C.Structure):
    _fields_ = [("prefix_len", C.c_int32), ("n_live", C.c_int32),
                ("parent", C.c_int32 * SP_MAX_TREE_NODES), ("depth", C.c_int32 * SP_MAX_TREE_NODES),
                ("token", C.c_int32 * SP_MAX_TREE_NODES), ("prob", C.c_float * SP_MAX_TREE_NODES),
                ("anc", (C.c_uint64 * 4) * SP_MAX_TREE_NODES),
                ("pred", C.c_int32 * SP_MAX_TREE_NODES), ("root_pred", C.c_int32)]


class sp_head_weights(C.Structure):
    _fields_ = [("norm", C.c_void_p), ("wvocab", C.c_void_p), ("vocab", C.c_int32), ("reserved", C.c_int32)]


_lib = None


def load_library(path: Optional[str] = None) -> C.CDLL:
    """Loads the built library; builds it first only if no build exists."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    p = path or LIB_PATH
    if not os.path.exists(p):
        from . import build as _build
        _build.build(verbose=False)
    if not os.path.exists(p):
        raise RuntimeError("libspecpipe.so is missing and could not be built: the HIP path is required")
    lib = C.CDLL(p)
    i32p, f32p, vp = C.POINTER(C.c_int32), C.POINTER(C.c_float), C.c_void_p
    sig = {
        "sp_stage_query_sizes": [C.POINTER(sp_config), C.POINTER(sp_sizes)],
        "sp_stage_create": [C.POINTER(sp_config), C.POINTER(sp_layer_weights), C.POINTER(sp_buffers), vp,
                            C.POINTER(vp)],
        "sp_pack_weights": [C.POINTER(sp_config), C.POINTER(sp_layer_weights), C.POINTER(sp_layer_weights), vp],
        "sp_pack_matrix": [vp, vp, C.c_int32, C.c_int32, vp],
        "sp_request_init": [vp, C.c_int32, C.c_int64, C.c_int32, C.c_int32, vp],
        "sp_stage_verify_head": [vp, C.POINTER(sp_head_weights), C.c_int32, i32p, i32p, i32p, vp, vp, vp, vp],
        "sp_stage_verify_head_noalloc": [vp, C.POINTER(sp_head_weights), C.c_int32, i32p, i32p, i32p, vp, vp, vp, vp],
        "sp_stage_verify_lossy": [vp, C.POINTER(sp_head_weights), C.c_int32, i32p, vp, C.c_int32, C.c_float, vp,
                                  i32p, vp],
        "sp_stage_verify_sample": [vp, C.POINTER(sp_head_weights), C.c_int32, i32p, vp, C.c_float, C.c_float, C.c_int32,
                                   f32p, vp, i32p, vp],
        "sp_request_set_root_pred": [vp, C.c_int32, C.c_int32, vp],
        "sp_tree_match": [vp, C.c_int32, i32p, vp, i32p, vp],
        "sp_tree_expand": [vp, C.c_int32, C.c_int32, i32p, C.c_int32, vp, vp, C.c_int32, vp, vp, vp, vp, vp],
        "sp_tree_insert": [vp, C.c_int32, C.c_int32, i32p, i32p, f32p, i32p, vp],
        "sp_request_pages": [vp, C.c_int32, i32p, C.c_int32, i32p],
        "sp_request_release": [vp, C.c_int32, vp],
        "sp_stage_free_pages": [vp],
        "sp_tree_insert_batch": [vp, C.c_int32, i32p, i32p, i32p, i32p, f32p, i32p, vp],
        "sp_stage_forward": [vp, C.c_int32, i32p, i32p, i32p, vp, vp, vp],
        "sp_tree_prune": [vp, C.c_int32, C.c_int32, C.c_int32, i32p, i32p, vp],
        "sp_kv_compact": [vp, C.c_int32, vp, C.c_int32, i32p, i32p, i32p, vp],
        "sp_tree_prune_verified": [vp, C.c_int32, i32p, vp, C.c_int32, vp],
        "sp_tree_prune_batch": [vp, C.c_int32, i32p, i32p, i32p, i32p, i32p, vp],
        "sp_kv_compact_batch": [vp, C.c_int32, i32p, vp],
        "sp_tree_read": [vp, C.c_int32, C.POINTER(sp_tree_view), vp],
        "sp_request_info": [vp, C.c_int32, i32p, i32p, i32p],
        "sp_profile_begin": [vp, C.c_int32, C.c_int32],
        "sp_profile_sample_every": [vp, C.c_int32],
        "sp_profile_end": [vp, i32p, f32p],
        "sp_last_hip_error": [vp],
        "sp_version": [],
    }
    for name, args in sig.items():
        fn = getattr(lib, name)
        fn.argtypes = args
        fn.restype = C.c_int
    lib.sp_stage_destroy.argtypes = [vp]
    lib.sp_stage_destroy.restype = None
    lib.sp_strerror.argtypes = [C.c_int]
    lib.sp_strerror.restype = C.c_char_p
    if path is None:
        _lib = lib
    return lib


def _i32(a: Optional[Sequence[int]]):
    if a is None:
        return None, None
    arr = np.ascontiguousarray(np.asarray(a, dtype=np.int32))
    return arr, arr.ctypes.data_as(C.POINTER(C.c_int32))


def _check(rc: int, what: str):
    if rc != 0:
        raise SpError(rc, what)


class Stage:
    """One pipeline stage on one GPU.  Owns (through torch) the KV slab, the table
    arena and the workspace, and forwards every call to the C ABI."""

    def __init__(self, shape, layers: List[Dict[str, "object"]], *, kv_slots: int, max_requests: int = 1,
                 max_batch_nodes: int = 64, max_tree_nodes: int = SP_MAX_TREE_NODES, flags: int = 0,
                 device: str = "cuda:0", page_slots: int = 0):
        import torch
        self.torch = torch
        self.lib = load_library()
        self.shape = shape
        self.device = torch.device(device)
        self.dtype = SP_BF16 if shape.dtype == "bf16" else SP_F32
        self.tdtype = torch.bfloat16 if shape.dtype == "bf16" else torch.float32
        self.cfg = sp_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.d_head,
                             shape.d_ff, shape.rms_eps, shape.rope_theta, self.dtype, max_requests,
                             max_tree_nodes, max_batch_nodes, kv_slots, flags, page_slots)
        self.page_slots = page_slots
        sz = sp_sizes()
        _check(self.lib.sp_stage_query_sizes(C.byref(self.cfg), C.byref(sz)), "sp_stage_query_sizes")
        self.sizes = sz
        with torch.cuda.device(self.device):
            self.kv = torch.zeros(sz.kv_bytes, dtype=torch.uint8, device=self.device)
            self.tables = torch.zeros(sz.tables_bytes, dtype=torch.uint8, device=self.device)
            self.workspace = torch.zeros(sz.workspace_bytes, dtype=torch.uint8, device=self.device)
        self.layers = layers                      # keeps the weight tensors alive
        arr = (sp_layer_weights * shape.n_layers)()
        for l, w in enumerate(layers):
            for name in ("wqkv", "wo", "wgu", "wd", "norm1", "norm2"):
                t = w[name]
                assert t.is_cuda and t.is_contiguous() and t.dtype == self.tdtype, name
                setattr(arr[l], name, t.data_ptr())
        bufs = sp_buffers(self.kv.data_ptr(), sz.kv_bytes, self.tables.data_ptr(), sz.tables_bytes,
                          self.workspace.data_ptr(), sz.workspace_bytes)
        h = C.c_void_p()
        _check(self.lib.sp_stage_create(C.byref(self.cfg), arr, C.byref(bufs), self._stream(), C.byref(h)),
               "sp_stage_create")
        self.handle = h

    # -- plumbing -----------------------------------------------------------------
    def _stream(self):
        return C.c_void_p(self.torch.cuda.current_stream(self.device).cuda_stream)

    def close(self):
        if getattr(self, "handle", None):
            self.torch.cuda.synchronize(self.device)
            self.lib.sp_stage_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def kv_view(self):
        """The slab as a tensor [layer, K|V, kv_head, slot, d_head] (no copy)."""
        s = self.shape
        return self.kv.view(self.tdtype).view(s.n_layers, 2, s.n_kv_heads, self.cfg.kv_slots, s.d_head)

    # -- the C ABI, one method per entry point --------------------------------------
    def request_pages(self, req: int) -> List[int]:
        """Paged cache: physical page of every logical page the request holds."""
        n = C.c_int32()
        _check(self.lib.sp_request_pages(self.handle, req, None, 0, C.byref(n)), "sp_request_pages")
        out = np.zeros(max(n.value, 1), dtype=np.int32)
        _check(self.lib.sp_request_pages(self.handle, req, out.ctypes.data_as(C.POINTER(C.c_int32)), n.value, None),
               "sp_request_pages")
        return [int(v) for v in out[:n.value]]

    def request_release(self, req: int):
        _check(self.lib.sp_request_release(self.handle, req, self._stream()), "sp_request_release")

    def free_pages(self) -> int:
        return int(self.lib.sp_stage_free_pages(self.handle))

    def logical_slots(self, req: int, lo: int, hi: int):
        """Physical slot index (tensor, on the device) of the request's logical slots [lo, hi) in paged mode."""
        pages = self.request_pages(req)
        pg = self.page_slots
        idx = [pages[s // pg] * pg + s % pg for s in range(lo, hi)]
        return self.torch.tensor(idx, dtype=self.torch.long, device=self.device)

    def request_init(self, req: int, slot_base: int, capacity: int, prefix_len: int):
        _check(self.lib.sp_request_init(self.handle, req, slot_base, capacity, prefix_len, self._stream()),
               "sp_request_init")

    def tree_insert(self, req: int, parents: Sequence[int], tokens: Optional[Sequence[int]] = None,
                    probs: Optional[Sequence[float]] = None) -> int:
        pa, pp = _i32(parents)
        ta, tp = _i32(tokens)
        fa = fp = None
        if probs is not None:
            fa = np.ascontiguousarray(np.asarray(probs, dtype=np.float32))
            fp = fa.ctypes.data_as(C.POINTER(C.c_float))
        first = C.c_int32(-1)
        _check(self.lib.sp_tree_insert(self.handle, req, len(pa), pp, tp, fp, C.byref(first), self._stream()),
               "sp_tree_insert")
        return first.value

    def tree_insert_batch(self, req_ids: Sequence[int], parents_per_req: Sequence[Sequence[int]],
                          tokens_per_req: Optional[Sequence[Sequence[int]]] = None,
                          probs_per_req: Optional[Sequence[Sequence[float]]] = None) -> List[int]:
        """One launch for the new nodes of several requests; returns each request's first new index."""
        ra, rp = _i32(req_ids)
        na, npn = _i32([len(p) for p in parents_per_req])
        pa, pp = _i32([x for p in parents_per_req for x in p])
        ta, tp = _i32([x for t in tokens_per_req for x in t]) if tokens_per_req is not None else (None, None)
        qa = fp = None
        if probs_per_req is not None:
            qa = np.ascontiguousarray(np.asarray([x for q in probs_per_req for x in q], dtype=np.float32))
            fp = qa.ctypes.data_as(C.POINTER(C.c_float))
        first = np.zeros(max(len(ra), 1), dtype=np.int32)
        _check(self.lib.sp_tree_insert_batch(self.handle, len(ra), rp, npn, pp, tp, fp,
                                             first.ctypes.data_as(C.POINTER(C.c_int32)), self._stream()),
               "sp_tree_insert_batch")
        return [int(v) for v in first[:len(ra)]]

    def stage_forward(self, req_ids: Sequence[int], first_node: Sequence[int], n_nodes: Sequence[int], x_in, x_out=None):
        ra, rp = _i32(req_ids)
        fa, fp = _i32(first_node)
        na, np_ = _i32(n_nodes)
        if x_out is None:
            x_out = self.torch.empty_like(x_in)
        assert x_in.is_cuda and x_in.is_contiguous() and x_in.dtype == self.tdtype
        assert x_out.is_cuda and x_out.is_contiguous() and x_out.dtype == self.tdtype and x_out.shape == x_in.shape
        assert x_in.shape[0] == int(na.sum()) and x_in.shape[1] == self.shape.d_model
        _check(self.lib.sp_stage_forward(self.handle, len(ra), rp, fp, np_, C.c_void_p(x_in.data_ptr()),
                                         C.c_void_p(x_out.data_ptr()), self._stream()), "sp_stage_forward")
        return x_out

    def tree_prune(self, req: int, mode: int, node: int):
        live, commit = C.c_int32(-1), C.c_int32(-1)
        _check(self.lib.sp_tree_prune(self.handle, req, mode, node, C.byref(live), C.byref(commit), self._stream()),
               "sp_tree_prune")
        return live.value, commit.value

    def kv_compact(self, req: int, x_rows=None, row_nodes: Optional[Sequence[int]] = None):
        """Returns (n_rows_out, new node index per surviving row)."""
        n_out = C.c_int32(0)
        if x_rows is None:
            _check(self.lib.sp_kv_compact(self.handle, req, None, 0, None, C.byref(n_out), None, self._stream()),
                   "sp_kv_compact")
            return 0, []
        ra, rp = _i32(row_nodes)
        out = np.full(max(len(ra), 1), -2, dtype=np.int32)
        assert x_rows.is_cuda and x_rows.is_contiguous() and x_rows.dtype == self.tdtype
        _check(self.lib.sp_kv_compact(self.handle, req, C.c_void_p(x_rows.data_ptr()), len(ra), rp, C.byref(n_out),
                                      out.ctypes.data_as(C.POINTER(C.c_int32)), self._stream()), "sp_kv_compact")
        return n_out.value, out[:n_out.value].tolist()

    def tree_prune_verified(self, req_ids: Sequence[int], nodes_dev, stride: int = 1):
        """Prune + cache compaction by the verified nodes a device tensor holds (int32; the result of
        tree_match_dev or of verify_lossy's device output)."""
        ra, rp = _i32(req_ids)
        _check(self.lib.sp_tree_prune_verified(self.handle, len(ra), rp, nodes_dev.data_ptr(), stride, self._stream()),
               "sp_tree_prune_verified")

    def tree_prune_batch(self, req_ids, modes, nodes):
        ra, rp = _i32(req_ids)
        ma, mp = _i32(modes)
        na, np_ = _i32(nodes)
        live = np.zeros(len(ra), np.int32)
        commit = np.zeros(len(ra), np.int32)
        _check(self.lib.sp_tree_prune_batch(self.handle, len(ra), rp, mp, np_,
                                            live.ctypes.data_as(C.POINTER(C.c_int32)),
                                            commit.ctypes.data_as(C.POINTER(C.c_int32)), self._stream()),
               "sp_tree_prune_batch")
        return live.tolist(), commit.tolist()

    def kv_compact_batch(self, req_ids):
        ra, rp = _i32(req_ids)
        _check(self.lib.sp_kv_compact_batch(self.handle, len(ra), rp, self._stream()), "sp_kv_compact_batch")

    def tree_read(self, req: int) -> Dict[str, np.ndarray]:
        v = sp_tree_view()
        _check(self.lib.sp_tree_read(self.handle, req, C.byref(v), self._stream()), "sp_tree_read")
        n = v.n_live
        anc = np.ctypeslib.as_array(v.anc).reshape(SP_MAX_TREE_NODES, 4)[:n].copy()
        M = np.zeros((n, n), dtype=np.uint8)
        for i in range(n):
            for j in range(n):
                M[i, j] = (int(anc[i, j >> 6]) >> (j & 63)) & 1
        return {"prefix_len": v.prefix_len, "n_live": n,
                "parent": np.ctypeslib.as_array(v.parent)[:n].copy(), "depth": np.ctypeslib.as_array(v.depth)[:n].copy(),
                "token": np.ctypeslib.as_array(v.token)[:n].copy(), "prob": np.ctypeslib.as_array(v.prob)[:n].copy(),
                "anc": anc, "M": M, "pred": np.ctypeslib.as_array(v.pred)[:n].copy(), "root_pred": v.root_pred}

    # -- verification on the last stage ------------------------------------------------------
    def verify_head(self, head: Dict[str, "object"], req_ids: Sequence[int], first_node: Sequence[int],
                    n_nodes: Sequence[int], x, want_max: bool = False, noalloc: bool = False, out=None):
        """head: {"norm": tensor [d], "wvocab": tensor [V, d] (re-laid if the stage uses packed weights)}.
        Returns the device tensor of predictions (int32 per row) and, if asked, the winning logits.
        noalloc: call sp_stage_verify_head_noalloc (scratch inside the library) with the caller's
        output tensors out = (pred int32 [rows], max float32 [rows] or None)."""
        import torch
        if noalloc:
            ra, rp = _i32(req_ids)
            fa, fp = _i32(first_node)
            na, npn = _i32(n_nodes)
            pred, mx = out
            h = sp_head_weights(head["norm"].data_ptr(), head["wvocab"].data_ptr(), int(head["wvocab"].shape[0]), 0)
            _check(self.lib.sp_stage_verify_head_noalloc(self.handle, C.byref(h), len(ra), rp, fp, npn, x.data_ptr(),
                                                         pred.data_ptr(), mx.data_ptr() if mx is not None else None,
                                                         self._stream()), "sp_stage_verify_head_noalloc")
            return pred, mx
        ra, rp = _i32(req_ids)
        fa, fp = _i32(first_node)
        na, npn = _i32(n_nodes)
        rows = int(sum(n_nodes))
        assert x.is_contiguous() and x.dtype == self.tdtype
        pred = torch.empty(max(rows, 1), dtype=torch.int32, device=self.device)
        mx = torch.empty(max(rows, 1), dtype=torch.float32, device=self.device) if want_max else None
        h = sp_head_weights(head["norm"].data_ptr(), head["wvocab"].data_ptr(), int(head["wvocab"].shape[0]), 0)
        _check(self.lib.sp_stage_verify_head(self.handle, C.byref(h), len(ra), rp, fp, npn, x.data_ptr(),
                                             pred.data_ptr(), mx.data_ptr() if want_max else None, self._stream()),
               "sp_stage_verify_head")
        return (pred[:rows], mx[:rows]) if want_max else pred[:rows]

    def tree_expand(self, req: int, bottom_nodes: Sequence[int], cand_tokens, cand_probs, w: int):
        """cand_tokens (int32) / cand_probs (float32): device tensors [len(bottom_nodes), k].  Returns the
        selected level as host lists (parents, tokens, probs), ready for tree_insert; waits for the stream."""
        import torch
        ba, bp = _i32(bottom_nodes)
        assert cand_tokens.is_contiguous() and cand_tokens.dtype == torch.int32
        assert cand_probs.is_contiguous() and cand_probs.dtype == torch.float32
        k = int(cand_tokens.shape[1])
        room = max(w, 1)
        # one buffer for parents | tokens | probabilities (float bits) | count: one copy back to the host
        out = torch.empty(3 * room + 1, dtype=torch.int32, device=self.device)
        base = out.data_ptr()
        _check(self.lib.sp_tree_expand(self.handle, req, len(ba), bp, k, cand_tokens.data_ptr(), cand_probs.data_ptr(),
                                       w, base, base + 4 * room, base + 8 * room, base + 12 * room, self._stream()),
               "sp_tree_expand")
        host = out.cpu().numpy()
        n = int(host[3 * room])
        return (host[:n].tolist(), host[room:room + n].tolist(),
                host[2 * room:2 * room + n].view(np.float32).tolist())

    def set_root_pred(self, req: int, token: int):
        _check(self.lib.sp_request_set_root_pred(self.handle, req, token, self._stream()), "sp_request_set_root_pred")

    def verify_lossy(self, head: Dict[str, "object"], req_ids: Sequence[int], x_root, mode: int,
                     top_p: float = 1.0) -> List[tuple]:
        """x_root: device tensor [len(req_ids), d_model], the roots' last-layer outputs.  Returns
        [(verified node or -1, top-1 token)] per request; waits for the stream."""
        import torch
        ra, rp = _i32(req_ids)
        n = len(ra)
        assert x_root.is_contiguous() and x_root.dtype == self.tdtype
        dev = torch.empty(max(2 * n, 2), dtype=torch.int32, device=self.device)
        host = torch.empty(max(2 * n, 2), dtype=torch.int32, pin_memory=True)
        h = sp_head_weights(head["norm"].data_ptr(), head["wvocab"].data_ptr(), int(head["wvocab"].shape[0]), 0)
        _check(self.lib.sp_stage_verify_lossy(self.handle, C.byref(h), n, rp, x_root.data_ptr(), int(mode),
                                              float(top_p), dev.data_ptr(),
                                              C.cast(host.data_ptr(), C.POINTER(C.c_int32)), self._stream()),
               "sp_stage_verify_lossy")
        torch.cuda.current_stream(self.device).synchronize()
        return [(int(host[2 * i]), int(host[2 * i + 1])) for i in range(n)]

    def verify_sample(self, head: Dict[str, "object"], req_ids: Sequence[int], x_root, temperature: float, top_p: float,
                      top_k: int, u: Sequence[float]) -> List[tuple]:
        """sp_stage_verify_sample: [(verified node or -1, drawn token)] per request; waits for the stream."""
        import torch
        ra, rp = _i32(req_ids)
        n = len(ra)
        ua = np.ascontiguousarray(np.asarray(u, dtype=np.float32))
        dev = torch.empty(max(2 * n, 2), dtype=torch.int32, device=self.device)
        host = torch.empty(max(2 * n, 2), dtype=torch.int32, pin_memory=True)
        h = sp_head_weights(head["norm"].data_ptr(), head["wvocab"].data_ptr(), int(head["wvocab"].shape[0]), 0)
        _check(self.lib.sp_stage_verify_sample(self.handle, C.byref(h), n, rp, x_root.data_ptr(), float(temperature),
                                               float(top_p), int(top_k), ua.ctypes.data_as(C.POINTER(C.c_float)),
                                               dev.data_ptr(), C.cast(host.data_ptr(), C.POINTER(C.c_int32)),
                                               self._stream()), "sp_stage_verify_sample")
        torch.cuda.current_stream(self.device).synchronize()
        return [(int(host[2 * i]), int(host[2 * i + 1])) for i in range(n)]

    def tree_match_dev(self, req_ids: Sequence[int]):
        """sp_tree_match without the host copy: the device tensor of verified nodes (int32 per request),
        valid in stream order; nothing waits."""
        import torch
        ra, rp = _i32(req_ids)
        dev = torch.empty(max(len(ra), 1), dtype=torch.int32, device=self.device)
        _check(self.lib.sp_tree_match(self.handle, len(ra), rp, dev.data_ptr(), None, self._stream()), "sp_tree_match")
        return dev

    def verify_lossy_dev(self, head: Dict[str, "object"], req_ids: Sequence[int], x_root, mode: int, top_p: float = 1.0):
        """sp_stage_verify_lossy without the host copy: device tensor [2 * len(req_ids)] of (node, top-1 token)."""
        import torch
        ra, rp = _i32(req_ids)
        n = len(ra)
        dev = torch.empty(max(2 * n, 2), dtype=torch.int32, device=self.device)
        h = sp_head_weights(head["norm"].data_ptr(), head["wvocab"].data_ptr(), int(head["wvocab"].shape[0]), 0)
        _check(self.lib.sp_stage_verify_lossy(self.handle, C.byref(h), n, rp, x_root.data_ptr(), int(mode),
                                              float(top_p), dev.data_ptr(), None, self._stream()), "sp_stage_verify_lossy")
        return dev

    def tree_match(self, req_ids: Sequence[int]) -> List[int]:
        """Verified root child per request (-1 = miss); waits for the stream."""
        import torch
        ra, rp = _i32(req_ids)
        dev = torch.empty(max(len(ra), 1), dtype=torch.int32, device=self.device)
        host = torch.empty(max(len(ra), 1), dtype=torch.int32, pin_memory=True)
        _check(self.lib.sp_tree_match(self.handle, len(ra), rp, dev.data_ptr(),
                                      C.cast(host.data_ptr(), C.POINTER(C.c_int32)), self._stream()), "sp_tree_match")
        torch.cuda.current_stream(self.device).synchronize()
        return [int(v) for v in host[:len(ra)]]

    def request_info(self, req: int):
        p, t, f = C.c_int32(), C.c_int32(), C.c_int32()
        _check(self.lib.sp_request_info(self.handle, req, C.byref(p), C.byref(t), C.byref(f)), "sp_request_info")
        return p.value, t.value, f.value

    def profile_begin(self, kind: int, max_launches: int, every: int = 1):
        _check(self.lib.sp_profile_begin(self.handle, kind, max_launches), "sp_profile_begin")
        if every > 1:
            _check(self.lib.sp_profile_sample_every(self.handle, every), "sp_profile_sample_every")

    def profile_end(self):
        n, ms = C.c_int32(), C.c_float()
        _check(self.lib.sp_profile_end(self.handle, C.byref(n), C.byref(ms)), "sp_profile_end")
        return n.value, ms.value


def pack_weights(shape, layers: List[Dict[str, "object"]], device: str = "cuda:0"):
    """sp_pack_weights on every layer: returns new layer dicts whose four projection matrices are in
    MFMA fragment order (create the Stage with SP_FLAG_PACKED_WEIGHTS).  The inputs can be dropped."""
    import torch
    lib = load_library()
    cfg = sp_config(shape.n_layers, shape.d_model, shape.n_q_heads, shape.n_kv_heads, shape.d_head, shape.d_ff,
                    shape.rms_eps, shape.rope_theta, SP_BF16, 1, SP_MAX_TREE_NODES, 1, 1, 0)
    stream = C.c_void_p(torch.cuda.current_stream(torch.device(device)).cuda_stream)
    out = []
    for w in layers:
        o = dict(w)
        a, b = sp_layer_weights(), sp_layer_weights()
        for name in ("wqkv", "wo", "wgu", "wd"):
            o[name] = torch.empty_like(w[name])
            setattr(a, name, w[name].data_ptr())
            setattr(b, name, o[name].data_ptr())
        for name in ("norm1", "norm2"):
            setattr(a, name, w[name].data_ptr())
            setattr(b, name, w[name].data_ptr())
        _check(lib.sp_pack_weights(C.byref(cfg), C.byref(a), C.byref(b), stream), "sp_pack_weights")
        out.append(o)
    torch.cuda.synchronize()
    return out


def pack_matrix(w, device: str = "cuda:0"):
    """sp_pack_matrix: a [rows, cols] bf16 device tensor re-laid into MFMA fragment order (new tensor)."""
    import torch
    lib = load_library()
    out = torch.empty_like(w)
    stream = C.c_void_p(torch.cuda.current_stream(torch.device(device)).cuda_stream)
    _check(lib.sp_pack_matrix(w.data_ptr(), out.data_ptr(), w.shape[0], w.shape[1], stream), "sp_pack_matrix")
    torch.cuda.synchronize()
    return out


# ---- data preparation helpers (layout only) ---------------------------------------------
def pack_layer_weights(w: Dict[str, np.ndarray], dtype: str, device: str = "cuda:0"):
    """numpy weights of one layer (separate q/k/v and gate/up, [out, in]) -> the stacked
    device tensors the ABI takes."""
    import torch
    td = torch.bfloat16 if dtype == "bf16" else torch.float32

    def dev(a):
        return torch.from_numpy(np.ascontiguousarray(a)).to(device=device, dtype=td).contiguous()

    return {
        "wqkv": dev(np.concatenate([w["wq"], w["wk"], w["wv"]], axis=0)),
        "wo": dev(w["wo"]),
        "wgu": dev(np.concatenate([w["wg"], w["wu"]], axis=0)),
        "wd": dev(w["wd"]),
        "norm1": dev(w["norm1"]),
        "norm2": dev(w["norm2"]),
    }


def write_prefix(stage: Stage, layer: int, slot_base: int, k: np.ndarray, v: np.ndarray):
    """Copies a committed context's K and V ([P, H_kv, d_head], already rotated) into the slab."""
    import torch
    kv = stage.kv_view()
    P = k.shape[0]
    kt = torch.from_numpy(np.ascontiguousarray(k)).to(stage.device, stage.tdtype).permute(1, 0, 2)
    vt = torch.from_numpy(np.ascontiguousarray(v)).to(stage.device, stage.tdtype).permute(1, 0, 2)
    kv[layer, 0, :, slot_base:slot_base + P, :] = kt
    kv[layer, 1, :, slot_base:slot_base + P, :] = vt
