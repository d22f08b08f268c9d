#!/usr/bin/env python3
"""Timing runs of the other workloads of the stage library (bench.py covers the headline one).

    python -m paper_2504_04104_amd.measure --run sweep        # n = 1..256 nodes on the 8B-shaped stage
    python -m paper_2504_04104_amd.measure --run c3           # 70B-shaped 10-layer stage, 128 nodes
    python -m paper_2504_04104_amd.measure --run c4           # streaming, prefix 32768, 1-8 nodes per step
    python -m paper_2504_04104_amd.measure --run c5           # 32 requests, ragged batch
    python -m paper_2504_04104_amd.measure --run compact      # batched prune + KV compaction, scaled
    python -m paper_2504_04104_amd.measure --run verify       # last stage: output head (vocab 128256) + match
    python -m paper_2504_04104_amd.measure --run wide         # many-row projections at 512 / 574 / 1024 rows
    python -m paper_2504_04104_amd.measure --run wide_context # the vendor library's GEMM on the same shapes (yardstick)

Each run prints one JSON line.  These runs only time the HIP path (parity is the tests' job), so
weights are drawn on the GPU (seeded N(0, 0.02)) instead of through the host generators; trees,
schedules and context lengths come from `workloads` with the configs' seeds.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

import numpy as np
import torch

import workloads as wl
import paper_2504_04104_amd as sp
from paper_2504_04104_amd import binding as B

DEV = "cuda:0"
HBM_PEAK = 8000.0
MFMA_PEAK = 2500.0


def gpu_layers(sh: wl.ModelShape, seed: int, share: bool = False):
    """Layer weights drawn on the device.  share=True reuses one layer's matrices for all layers
    (only to save set-up time where the footprint does not matter)."""
    g = torch.Generator(device=DEV).manual_seed(seed)

    def mat(n, k):
        return (torch.randn(n, k, generator=g, device=DEV, dtype=torch.float32) * 0.02).to(torch.bfloat16)

    def layer():
        return {"wqkv": mat(sh.d_q + 2 * sh.d_kv, sh.d_model), "wo": mat(sh.d_model, sh.d_q),
                "wgu": mat(2 * sh.d_ff, sh.d_model), "wd": mat(sh.d_model, sh.d_ff),
                "norm1": torch.ones(sh.d_model, device=DEV, dtype=torch.bfloat16),
                "norm2": torch.ones(sh.d_model, device=DEV, dtype=torch.bfloat16)}

    first = layer()
    layers = [first if share else layer() for _ in range(sh.n_layers)]
    layers[0] = first
    return sp.pack_weights(sh, layers, DEV)


def fill_kv(stage: sp.Stage, seed: int):
    g = torch.Generator(device=DEV).manual_seed(seed)
    kv = stage.kv_view()
    for l in range(kv.shape[0]):
        kv[l].copy_(torch.randn(kv[l].shape, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16))


def timed(fn, reps: int, warm: int = 3, rounds: int = 3):
    """Best of a few rounds (a stray host stall otherwise lands in one data point)."""
    for _ in range(warm):
        fn()
    best = None
    for _ in range(rounds):
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(reps):
            fn()
        torch.cuda.synchronize()
        t = (time.perf_counter() - t0) / reps
        best = t if best is None else min(best, t)
    return best


def kernel_us(stage: sp.Stage, fn, kind: int, reps: int = 10):
    stage.profile_begin(kind, 4096)
    for _ in range(reps):
        fn()
    n, ms = stage.profile_end()
    return ms * 1e3 / reps, n // reps


# ---------------------------------------------------------------------------------------------
def run_sweep(args):
    """Stage-step forward latency against the number of tree nodes (the shape of the paper's
    layer-latency figure: flat within a tile of rows, stepping at tile edges)."""
    w = wl.CONFIGS["C2"]
    sh, P = w.shape, w.prefix_len
    layers = gpu_layers(sh, w.seed)
    cap = P + 320
    stage = sp.Stage(sh, layers, kv_slots=cap, max_batch_nodes=256, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    fill_kv(stage, w.seed)
    out = {}
    for n in [1, 2, 4, 8, 16, 17, 31, 32, 33, 48, 63, 64, 65, 80, 96, 112, 128, 129, 192, 256]:
        par = wl.tree_uniform_parents(w.seed, n, 8, name=("sweep", n))
        x = torch.randn(n, sh.d_model, device=DEV).to(torch.bfloat16)
        y = torch.empty_like(x)

        def step():
            stage.request_init(0, 0, cap, P)
            stage.tree_insert(0, par)
            stage.stage_forward([0], [0], [n], x, y)
        out[n] = round(timed(step, 15) * 1e6, 1)
    print(json.dumps({"run": "sweep", "workload": "8B-shaped 4-layer stage, prefix 2048", "us_per_step_by_nodes": out}))
    stage.close()


def run_c3(args):
    w = wl.CONFIGS["C3"]
    sh, P, n = w.shape, w.prefix_len, w.n_nodes
    layers = gpu_layers(sh, w.seed)
    cap = P + 320
    stage = sp.Stage(sh, layers, kv_slots=cap, max_batch_nodes=128, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    fill_kv(stage, w.seed)
    par = wl.tree_branching(w.seed, n, w.max_children, w.max_levels)
    roots = [i for i, p in enumerate(par) if p < 0]
    x = torch.randn(n, sh.d_model, device=DEV).to(torch.bfloat16)
    y = torch.empty_like(x)
    rn = list(range(n))

    def step():
        stage.request_init(0, 0, cap, P)
        stage.tree_insert(0, par)
        stage.stage_forward([0], [0], [n], x, y)
        stage.tree_prune(0, sp.SP_ACCEPT, roots[0])
        stage.kv_compact(0, y, rn)
    t = timed(step, 10)
    gu_us, cnt = kernel_us(stage, step, B.K_GEMM_GATEUP)
    wbytes = sh.params_per_layer * 2 * sh.n_layers
    res = {"run": "c3", "workload": "70B-shaped 10-layer stage, prefix 4096, 128 nodes", "ms_per_step": round(t * 1e3, 3),
           "tree_tokens_per_s": round(n / t, 1), "weights_GB": round(wbytes / 1e9, 2),
           "step_hbm_frac": round(wbytes / t / 1e9 / HBM_PEAK, 4),
           "gateup_us_per_launch": round(gu_us / cnt, 1),
           "gateup_hbm_frac": round(2 * sh.d_ff * sh.d_model * 2 / (gu_us / cnt * 1e-6) / 1e9 / HBM_PEAK, 4)}
    print(json.dumps(res))
    stage.close()


def run_c4(args):
    """Streaming: per step insert 1-8 nodes, forward them, prune, compact; prefix 32768."""
    w = wl.CONFIGS["C4"]
    sh, P = w.shape, args.prefix or w.prefix_len
    layers = gpu_layers(sh, w.seed)
    steps = wl.streaming_schedule(w.seed, args.steps or 512, max_new=8, cap=256, p_accept=0.7)
    cap = P + 256 + sum(1 for s in steps if s.prune and s.prune.mode == wl.ACCEPT) * 9 + 64
    stage = sp.Stage(sh, layers, kv_slots=cap, max_batch_nodes=64, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    fill_kv(stage, w.seed)
    xs = torch.randn(8, sh.d_model, device=DEV).to(torch.bfloat16)
    ys = torch.empty_like(xs)

    def run(profile_kind=None):
        stage.request_init(0, 0, cap, P)
        tokens = 0
        for st in steps:
            n = len(st.parents)
            first = stage.tree_insert(0, st.parents)
            if n:
                stage.stage_forward([0], [first], [n], xs[:n], ys[:n])
                tokens += n
            if st.prune is not None:
                stage.tree_prune(0, st.prune.mode, st.prune.node)
                if n:
                    stage.kv_compact(0, ys[:n], list(range(first, first + n)))
                else:
                    stage.kv_compact(0)
        return tokens

    run()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    tokens = run()
    torch.cuda.synchronize()
    t = time.perf_counter() - t0
    stage.profile_begin(B.K_ATTENTION, 4096)
    run()
    cnt, ms = stage.profile_end()
    P_end = stage.request_info(0)[0]
    kv_bytes = ((P + P_end) / 2 + 128) * sh.kv_bytes_per_token_per_layer     # per launch, average context
    att_us = ms * 1e3 / cnt
    res = {"run": "c4", "workload": "streaming, 8B-shaped 4-layer stage, prefix %d, %d steps" % (P, len(steps)),
           "ms_per_step": round(t / len(steps) * 1e3, 4), "tree_tokens_per_s": round(tokens / t, 1),
           "tokens": tokens, "attention_us_per_launch": round(att_us, 1),
           "attention_GBps": round(kv_bytes / (att_us * 1e-6) / 1e9, 1),
           "attention_hbm_frac": round(kv_bytes / (att_us * 1e-6) / 1e9 / HBM_PEAK, 4),
           "final_prefix": P_end}
    print(json.dumps(res))
    stage.close()


def run_c5(args):
    """Dynamic batch: 32 requests, own prefix and tree; cold step then steady steps."""
    w = wl.CONFIGS["C5"]
    sh = w.shape
    layers = gpu_layers(sh, w.seed)
    reqs = wl.batch_requests(w.seed)
    n_steps = args.steps or 64
    sched = wl.batch_schedule(w.seed, reqs, n_steps - 1)
    room = 32 + 9 * n_steps + 64
    base, off = {}, 0
    for r in reqs:
        base[r.req] = off
        off += r.prefix_len + room
    total_nodes = sum(len(r.parents) for r in reqs)
    pg = args.page_slots
    if pg:          # paged cache: requests share a pool of pages instead of owning a range each
        off = -(-off // pg) * pg
        for r in reqs:
            base[r.req] = 0
    stage = sp.Stage(sh, layers, kv_slots=off, max_requests=len(reqs), max_batch_nodes=max(64, total_nodes),
                     flags=sp.SP_FLAG_PACKED_WEIGHTS | (sp.SP_FLAG_PAGED_KV if pg else 0), page_slots=pg)
    fill_kv(stage, w.seed)
    x = torch.randn(total_nodes, sh.d_model, device=DEV).to(torch.bfloat16)
    y = torch.empty_like(x)
    ids = [r.req for r in reqs]

    def cold():
        for r in reqs:
            stage.request_init(r.req, base[r.req], r.prefix_len + room, r.prefix_len)
        stage.tree_insert_batch(ids, [r.parents for r in reqs])
        stage.stage_forward(ids, [0] * len(reqs), [len(r.parents) for r in reqs], x, y)

    def steady():
        toks = 0
        for row in sched:
            modes = [st.prune.mode if st.prune else -1 for st in row]
            nodes = [st.prune.node if st.prune else 0 for st in row]
            stage.tree_prune_batch(ids, modes, nodes)
            stage.kv_compact_batch([i for i, m in zip(ids, modes) if m >= 0])
            act = [r.req for r, st in zip(reqs, row) if st.parents]
            new = [st.parents for st in row if st.parents]
            counts = [len(p) for p in new]
            firsts = stage.tree_insert_batch(act, new) if act else []
            if act:
                n = sum(counts)
                stage.stage_forward(act, firsts, counts, x[:n], y[:n])
                toks += n
        return toks

    cold(); steady()
    torch.cuda.synchronize()
    t0 = time.perf_counter(); cold(); torch.cuda.synchronize(); t_cold = time.perf_counter() - t0
    t0 = time.perf_counter(); toks = steady(); torch.cuda.synchronize(); t_steady = time.perf_counter() - t0
    stage.profile_begin(B.K_ATTENTION, 4096)
    cold(); steady()
    n_att, att_ms = stage.profile_end()
    flops_cold = 2.0 * total_nodes * sh.params_per_layer * sh.n_layers
    res = {"run": "c5", "page_slots": pg, "attention_us_per_launch_cold_and_steady": round(att_ms * 1e3 / max(n_att, 1), 1), "workload": "32 requests, 8B-shaped 4-layer stage", "cold_nodes": total_nodes,
           "cold_ms": round(t_cold * 1e3, 3), "cold_tree_tokens_per_s": round(total_nodes / t_cold, 1),
           "cold_gemm_TFLOPs": round(flops_cold / t_cold / 1e12, 1),
           "cold_mfma_frac": round(flops_cold / t_cold / 1e12 / MFMA_PEAK, 4),
           "steady_steps": len(sched), "steady_ms_per_step": round(t_steady / max(len(sched), 1) * 1e3, 3),
           "steady_tokens": toks, "steady_tree_tokens_per_s": round(toks / t_steady, 1)}
    print(json.dumps(res))
    stage.close()


def run_compact(args):
    """Batched prune + KV compaction at scale: 32 requests x 256 live nodes, 10 layers of the
    70B KV shape, drop a node near the front so that almost every row moves."""
    sh = wl.scaled(wl.LLAMA_70B_STAGE, d_model=256, d_ff=256, n_q_heads=8)     # KV shape is what matters here
    R, T, P = 32, 256, 64
    layers = gpu_layers(sh, 5, share=True)
    cap = P + T + 8
    stage = sp.Stage(sh, layers, kv_slots=R * cap, max_requests=R, max_batch_nodes=64,
                     flags=sp.SP_FLAG_PACKED_WEIGHTS)
    fill_kv(stage, 5)
    ids = list(range(R))
    par = [-1, -1] + [1] * (T - 2)                  # two root children; 254 nodes under the second

    def setup():
        for r in ids:
            stage.request_init(r, r * cap, cap, P)
            stage.tree_insert(r, par)

    def prune():
        stage.tree_prune_batch(ids, [sp.SP_DROP] * R, [0] * R)      # drop node 0: the other 255 rows all move by one
        stage.kv_compact_batch(ids)

    moved = R * (T - 1) * sh.kv_bytes_per_token_per_layer * sh.n_layers
    setup(); prune()
    torch.cuda.synchronize()
    reps = 20
    tk = 0.0
    for _ in range(reps):
        setup()
        stage.profile_begin(B.K_KV_COMPACT, 4)
        prune()
        n, ms = stage.profile_end()
        tk += ms
    res = {"run": "compact", "workload": "32 requests x 256 nodes x 10 layers of 8x128 bf16 KV, 255 rows move per request",
           "bytes_read": moved, "bytes_written": moved, "kv_compact_us": round(tk / reps * 1e3, 1),
           "GBps_read_plus_write": round(2 * moved / (tk / reps * 1e-3) / 1e9, 1),
           "hbm_frac": round(2 * moved / (tk / reps * 1e-3) / 1e9 / HBM_PEAK, 4)}
    print(json.dumps(res))
    stage.close()


def run_wide(args):
    """The many-row projection kernels on the 8B-shaped layer: forward calls of 512, 574 (the ragged cold
    batch of config 5) and 1024 rows spread over requests with short contexts, each projection kind
    bracketed by HIP events.  One layer; FLOP/s per projection against the dense bf16 matrix-core peak."""
    w = wl.CONFIGS["C5"]
    sh = wl.scaled(w.shape, n_layers=1)
    layers = gpu_layers(sh, w.seed)
    out = {}
    for M in (512, 574, 1024):
        if M == 574:
            sizes = [len(r.parents) for r in wl.batch_requests(w.seed)]
        else:
            sizes = [256] * (M // 256)
        assert sum(sizes) == M
        R, P, cap = len(sizes), 64, 64 + 256 + 8
        stage = sp.Stage(sh, layers, kv_slots=R * cap, max_requests=R, max_batch_nodes=M, flags=sp.SP_FLAG_PACKED_WEIGHTS)
        fill_kv(stage, w.seed)
        x = torch.randn(M, sh.d_model, device=DEV).to(torch.bfloat16)
        y = torch.empty_like(x)
        ids = list(range(R))
        pars = [wl.tree_uniform_parents(w.seed, n, 12, name=("wide", r)) for r, n in enumerate(sizes)]

        def step():
            for r in ids:
                stage.request_init(r, r * cap, cap, P)
            stage.tree_insert_batch(ids, pars)
            stage.stage_forward(ids, [0] * R, sizes, x, y)
        step()
        row = {}
        for kind, name, N, K in ((B.K_GEMM_QKV, "qkv", sh.d_q + 2 * sh.d_kv, sh.d_model), (B.K_GEMM_O, "o", sh.d_model, sh.d_q),
                                 (B.K_GEMM_GATEUP, "gateup", 2 * sh.d_ff, sh.d_model), (B.K_GEMM_DOWN, "down", sh.d_model, sh.d_ff)):
            us, cnt = kernel_us(stage, step, kind)
            us /= cnt
            row[name] = {"us": round(us, 1), "TFLOPs": round(2.0 * M * N * K / us / 1e6, 1),
                         "mfma_frac": round(2.0 * M * N * K / us / 1e6 / MFMA_PEAK, 4)}
        out[M] = row
        stage.close()
    print(json.dumps({"run": "wide", "workload": "8B-shaped layer, many-row projections (k_gemm_wide)", "by_rows": out}))


def run_wide_context(args):
    """A yardstick for `--run wide`, not a part of the path: the vendor library's bf16 GEMM (torch.matmul) on the
    same four shapes and row counts, random operands, timed with events.  It says what this chip sustains on
    these shapes with somebody else's kernel; the gate/up figure is for the two products alone (no SiLU)."""
    sh = wl.CONFIGS["C5"].shape
    g = torch.Generator(device=DEV).manual_seed(7)
    out = {}
    for M in (512, 574, 1024):
        row = {}
        for name, N, K in (("qkv", sh.d_q + 2 * sh.d_kv, sh.d_model), ("o", sh.d_model, sh.d_q),
                           ("gateup", 2 * sh.d_ff, sh.d_model), ("down", sh.d_model, sh.d_ff)):
            x = torch.randn(M, K, generator=g, device=DEV, dtype=torch.float32).to(torch.bfloat16)
            wt = (torch.randn(N, K, generator=g, device=DEV, dtype=torch.float32) * 0.02).to(torch.bfloat16)
            for _ in range(5):
                torch.matmul(x, wt.t())
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            torch.cuda.synchronize()
            e0.record()
            for _ in range(40):
                torch.matmul(x, wt.t())
            e1.record()
            torch.cuda.synchronize()
            us = e0.elapsed_time(e1) * 1e3 / 40
            row[name] = {"us": round(us, 1), "TFLOPs": round(2.0 * M * N * K / us / 1e6, 1),
                         "mfma_frac": round(2.0 * M * N * K / us / 1e6 / MFMA_PEAK, 4)}
            del x, wt
        out[M] = row
    print(json.dumps({"run": "wide_context", "workload": "vendor library bf16 GEMM (torch.matmul) on the shapes of --run wide",
                      "by_rows": out}))


def run_verify(args):
    """Last-stage step on the 8B-shaped stage: forward of 64 nodes, output head over a vocabulary of
    128256 with the top-1 token per node, match of the root's successor, accept, compaction."""
    w = wl.CONFIGS["C2"]
    sh, P, n = w.shape, w.prefix_len, w.n_nodes
    V = 128256
    layers = gpu_layers(sh, w.seed)
    g = torch.Generator(device=DEV).manual_seed(w.seed + 1)
    wv = (torch.randn(V, sh.d_model, generator=g, device=DEV, dtype=torch.float32) * 0.02).to(torch.bfloat16)
    head = {"norm": torch.ones(sh.d_model, device=DEV, dtype=torch.bfloat16), "wvocab": sp.pack_matrix(wv)}
    del wv
    cap = P + 320
    stage = sp.Stage(sh, layers, kv_slots=cap, max_batch_nodes=64, flags=sp.SP_FLAG_PACKED_WEIGHTS)
    fill_kv(stage, w.seed)
    par = wl.tree_branching(w.seed, n, w.max_children, w.max_levels)
    roots = [i for i, p in enumerate(par) if p < 0]
    tokens = list(range(1000, 1000 + n))
    x = torch.randn(n, sh.d_model, device=DEV).to(torch.bfloat16)
    y = torch.empty_like(x)
    rn = list(range(n))

    def head_only():
        stage.verify_head(head, [0], [0], [n], y)

    def step():
        stage.request_init(0, 0, cap, P)
        stage.set_root_pred(0, tokens[roots[0]])
        stage.tree_insert(0, par, tokens)
        stage.stage_forward([0], [0], [n], x, y)
        stage.verify_head(head, [0], [0], [n], y)
        node = stage.tree_match([0])[0]                      # waits for the stream: the host decides
        stage.tree_prune(0, sp.SP_ACCEPT, node)
        stage.kv_compact(0, y, rn)
    t = timed(step, 20)

    def step_device_handover():
        stage.request_init(0, 0, cap, P)
        stage.set_root_pred(0, tokens[roots[0]])
        stage.tree_insert(0, par, tokens)
        stage.stage_forward([0], [0], [n], x, y)
        stage.verify_head(head, [0], [0], [n], y)
        stage.tree_prune_verified([0], stage.tree_match_dev([0]))     # prune + compaction read the node on the device
    t_dev = timed(step_device_handover, 20)
    stage.request_init(0, 0, cap, P)
    stage.tree_insert(0, par, tokens)
    stage.stage_forward([0], [0], [n], x, y)
    t_head = timed(head_only, 30)
    hd_us, cnt = kernel_us(stage, head_only, B.K_VERIFY_HEAD)
    # fixed-width expansion of a full level: 64 bottom tokens x 16 candidates, width 64 (Sec. 4.1's setting)
    stage.request_init(0, 0, cap, P)
    stage.tree_insert(0, [-1] * 64, list(range(64)), [0.5] * 64)
    ct = torch.randint(0, V, (64, 16), device=DEV, dtype=torch.int32)
    cp = torch.rand(64, 16, device=DEV, dtype=torch.float32)
    t_expand = timed(lambda: stage.tree_expand(0, list(range(64)), ct, cp, 64), 30)
    # lossy verification of a full level of 64 root children from the root's row (one row of logits)
    stage.request_init(0, 0, cap, P)
    stage.tree_insert(0, [-1] * 64, [int(v) for v in torch.randint(0, V, (64,)).tolist()], [0.5] * 64)
    xr = y[:1].contiguous()
    t_relaxed = timed(lambda: stage.verify_lossy(head, [0], xr, sp.SP_VERIFY_RELAXED, 1.0), 30)
    t_top_p = timed(lambda: stage.verify_lossy(head, [0], xr, sp.SP_VERIFY_TOP_P, 0.9), 30)
    t_sample = timed(lambda: stage.verify_sample(head, [0], xr, 0.6, 0.9, 80, [0.37]), 30)
    hbytes = V * sh.d_model * 2
    res = {"run": "verify", "workload": "last stage of the 8B shape: 4 layers + output head, vocab 128256, 64 nodes",
           "ms_per_step": round(t * 1e3, 3), "tree_tokens_per_s": round(n / t, 1),
           "ms_per_step_device_handover": round(t_dev * 1e3, 3),
           "expand_call_us_with_host_copy": round(t_expand * 1e6, 1),
           "lossy_relaxed_call_us_with_host_wait": round(t_relaxed * 1e6, 1),
           "lossy_top_p_call_us_with_host_wait": round(t_top_p * 1e6, 1),
           "stochastic_T0.6_p0.9_k80_call_us_with_host_wait": round(t_sample * 1e6, 1),
           "head_call_us": round(t_head * 1e6, 1), "head_kernels_us": round(hd_us / cnt, 1),
           "head_weights_MB": round(hbytes / 1e6, 1),
           "head_GBps": round(hbytes / (hd_us / cnt * 1e-6) / 1e9, 1),
           "head_hbm_frac": round(hbytes / (hd_us / cnt * 1e-6) / 1e9 / HBM_PEAK, 4)}
    print(json.dumps(res))
    stage.close()


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--page-slots", type=int, default=0, help="c5: keep the cache in pages of this many slots")
    ap.add_argument("--run", required=True, choices=["sweep", "c3", "c4", "c5", "compact", "verify", "wide", "wide_context"])
    ap.add_argument("--steps", type=int, default=0)
    ap.add_argument("--prefix", type=int, default=0, help="c4: committed context length (default: the workload's 32768)")
    args = ap.parse_args()
    # a stream of our own: the forward call replays HIP graphs of its launches only on a stream that can be captured
    torch.cuda.set_stream(torch.cuda.Stream(device=DEV))
    {"sweep": run_sweep, "c3": run_c3, "c4": run_c4, "c5": run_c5, "compact": run_compact, "verify": run_verify, "wide": run_wide, "wide_context": run_wide_context}[args.run](args)


if __name__ == "__main__":
    main()
