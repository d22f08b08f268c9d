#!/usr/bin/env python3
"""Stage-step benchmark of the SpecPipe stage library on one MI355X.

A step is one pass of the whole hot path on the 8B-shaped 4-layer stage (BASELINE
config 2): reset the request to its 2048-token committed context, insert the 64-node
tree (sp_tree_insert), run the four decoder layers on those nodes under the tree mask
(sp_stage_forward), accept one child of the root (sp_tree_prune) and compact the KV
cache and the in-flight hidden rows (sp_kv_compact).  Inputs are seeded, synthetic and
already in HBM when the timed region starts.

Prints ONE JSON line with the stage-step rate in tree tokens per second, the roofline
figures of the dominant kernel (the gate/up projection, a weight stream from HBM) measured
with HIP events inside the timed region, and the CPU oracle timed on the host cores.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time
from concurrent.futures import ThreadPoolExecutor

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def profiled_traffic():
    """Bytes per gate/up launch as the rocprofv3 counter runs measured them: the line
    `bench.roofline.traffic_bytes = <number>` of profiles/pmc_hbm_traffic_stage_step_c2.txt, else None."""
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", "pmc_hbm_traffic_stage_step_c2.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("bench.roofline.traffic_bytes"):
                    return float(line.split("=", 1)[1])
    except (OSError, ValueError):
        pass
    return None


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", default="C2", choices=["C2", "C3"])
    ap.add_argument("--nodes", type=int, default=0, help="tree nodes per step (default: the workload's)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--kernels", action="store_true", help="also time every kernel kind (extra passes)")
    ap.add_argument("--unpacked", action="store_true",
                    help="keep the weights row-major instead of the load-time MFMA-fragment re-layout")
    ap.add_argument("--no-graphs", action="store_true",
                    help="keep sp_stage_forward from replaying HIP graphs of its launches (SP_FLAG_NO_GRAPHS)")
    ap.add_argument("--graph", action="store_true",
                    help="capture one step into a HIP graph and time replays (the step's device work is the "
                         "same every step; the host-side argument checks then run once, at capture)")
    ap.add_argument("--roofline-sample", type=int, default=20,
                    help="bracket the gate/up launches of one forward call in this many with HIP events (default 20); "
                         "a bracketed call is launched kernel by kernel instead of replaying its graph")
    ap.add_argument("--calib-copy", action="store_true",
                    help="first run three plain 1 GiB device copies (a known-size kernel that scales rocprofv3's "
                         "FETCH_SIZE / WRITE_SIZE counters)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one pipeline stage on ONE GPU; --gpus %d is not supported "
              "(no collectives or inter-stage transport are part of it)" % args.gpus, file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as wl
    import paper_2504_04104_amd as sp
    from paper_2504_04104_amd import binding as B

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    w = wl.CONFIGS[args.workload]
    sh = w.shape
    n = args.nodes or w.n_nodes
    P = w.prefix_len
    dev = "cuda:0"
    # A stream of the caller's own, as a serving loop would use: sp_stage_forward can only capture and
    # replay the graph of its launches on a stream that may be captured, which the default stream is not.
    torch.cuda.set_stream(torch.cuda.Stream(device=dev))
    t0 = time.time()
    with ThreadPoolExecutor(4) as ex:
        weights = list(ex.map(lambda l: wl.layer_weights(sh, w.seed, l), range(sh.n_layers)))
    layers = [sp.pack_layer_weights(x, sh.dtype, dev) for x in weights]
    flags = 0
    if not args.unpacked:
        layers = sp.pack_weights(sh, layers, dev)      # load-time re-layout, outside the timed region
        flags |= sp.SP_FLAG_PACKED_WEIGHTS
    if args.no_graphs:
        flags |= sp.SP_FLAG_NO_GRAPHS
    cap = P + 256 + 64
    stage = sp.Stage(sh, layers, kv_slots=cap, max_requests=1, max_batch_nodes=max(64, n), flags=flags)
    prefix = [wl.prefix_kv(sh, w.seed, l, P) for l in range(sh.n_layers)]
    for l, (k, v) in enumerate(prefix):
        sp.write_prefix(stage, l, 0, k, v)
    parents = wl.tree_branching(w.seed, n, w.max_children, w.max_levels)
    roots = [i for i, p in enumerate(parents) if p < 0]
    accept = roots[int(wl.rng(w.seed, "accept").integers(0, len(roots)))]
    x_np = wl.hidden_rows(sh, w.seed, ("x",), n)
    x = torch.from_numpy(x_np).to(dev, torch.bfloat16)
    y = torch.empty_like(x)
    row_nodes = list(range(n))
    setup_s = time.time() - t0

    def step():
        stage.request_init(0, 0, cap, P)
        stage.tree_insert(0, parents)
        stage.stage_forward([0], [0], [n], x, y)
        stage.tree_prune(0, sp.SP_ACCEPT, accept)
        stage.kv_compact(0, y, row_nodes)

    if args.calib_copy:
        src = torch.empty(1 << 30, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    if args.graph:
        graph = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(graph, stream=side):
                step()
        torch.cuda.current_stream().wait_stream(side)
        eager_step = step
        step = graph.replay
        for _ in range(3):
            step()
        torch.cuda.synchronize()

    # ---- timed region: K steps, with the dominant kernel bracketed by HIP events ----
    L = sh.n_layers
    # one gate/up launch in `sample` is bracketed by HIP events: the events open a gap of several
    # microseconds around the launch they bracket, so bracketing every launch would slow the step it times
    sample = max(1, args.roofline_sample)
    stage.profile_begin(B.K_GEMM_GATEUP, args.steps * L, every=sample)
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    if args.graph:
        # replays carry no events: every `sample`-th step is launched eagerly instead (same device work),
        # and one of its gate/up launches is bracketed
        for i in range(args.steps):
            if i % sample == 0:
                eager_step()
            else:
                step()
    else:
        for _ in range(args.steps):
            step()
    t_enq = time.perf_counter()
    torch.cuda.synchronize()
    t2 = time.perf_counter()
    n_launch, gu_ms = stage.profile_end()
    ms_per_step = (t2 - t1) * 1e3 / args.steps
    tok_per_s = n / (ms_per_step * 1e-3)

    # dominant kernel: gate/up projection.  Algorithmic bytes per launch: its weights once
    # (2 * d_ff * d_model bf16), the M x d input rows and the M x d_ff output rows.
    gu_bytes = 2 * sh.d_ff * sh.d_model * 2 + n * sh.d_model * 2 + n * sh.d_ff * 2
    gu_us = gu_ms * 1e3 / max(n_launch, 1)
    achieved = gu_bytes / (gu_us * 1e-6) / 1e9
    # HBM bytes per launch from rocprofv3 PMC runs of this same command (FETCH_SIZE x 2.00 + WRITE_SIZE x 1.00,
    # factors from a 1 GiB copy), read from the committed summary of those runs; it holds the profiled shape
    # only (C2 at 64 rows), and without the file or its line the field stays null.
    traffic = profiled_traffic() if (args.workload == "C2" and n == 64) else None
    roofline = {"bound": "hbm", "kernel": "gemm_gateup (k_gemm_bf16 GATEUP)", "achieved": round(achieved, 1),
                "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(achieved / HBM_PEAK_GBS, 4),
                "traffic": traffic, "avg_launch_us": round(gu_us, 2), "launches": n_launch,
                "bytes_per_launch": gu_bytes}

    # whole-step view against the HBM floor: all stage weights once + the KV the attention reads
    step_bytes = sh.params_per_layer * 2 * L + L * (P + n) * sh.kv_bytes_per_token_per_layer
    step_frac = step_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBS

    # informational: the same step replayed from a HIP graph captured by the caller (no host work per step)
    replay_ms = None
    if not args.graph:
        eager = eager_step if args.graph else step
        gr = torch.cuda.CUDAGraph()
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            with torch.cuda.graph(gr, stream=side):
                eager()
        torch.cuda.current_stream().wait_stream(side)
        for _ in range(5):
            gr.replay()
        torch.cuda.synchronize()
        tg = time.perf_counter()
        for _ in range(100):
            gr.replay()
        torch.cuda.synchronize()
        replay_ms = round((time.perf_counter() - tg) * 10.0, 4)
        del gr

    kernels = None
    if args.kernels:
        kernels = {}
        names = {B.K_GEMM_QKV: "gemm_qkv", B.K_GEMM_O: "gemm_o", B.K_GEMM_GATEUP: "gemm_gateup",
                 B.K_GEMM_DOWN: "gemm_down", B.K_ATTENTION: "attention", B.K_NORM: "norm",
                 B.K_ROPE_KV: "rope_kv", B.K_KV_COMPACT: "kv_compact", B.K_TREE_PRUNE: "tree_prune",
                 B.K_TREE_INSERT: "tree_insert"}
        reps = 20
        for kind, name in names.items():
            stage.profile_begin(kind, reps * 2 * L)
            for _ in range(reps):
                step()
            cnt, ms = stage.profile_end()
            kernels[name] = {"us_per_step": round(ms * 1e3 / reps, 2), "launches_per_step": cnt // reps}

    cpu = None
    if not args.no_cpu_baseline:
        # The oracle as it stands, one full step of the same workload on the host cores.
        from oracle import StageOracle
        import threadpoolctl
        ora = StageOracle(sh, weights)
        ora.request_init(0, [k for k, _ in prefix], [v for _, v in prefix], cap)
        c0 = time.perf_counter()
        ora.tree_insert(0, parents)
        ref = ora.stage_forward(0, 0, x_np)
        pr = ora.accept(0, accept)
        ora.prune_hidden_rows(ref, row_nodes, pr)
        c1 = time.perf_counter()
        threads = max([p.get("num_threads", 1) for p in threadpoolctl.threadpool_info()] or [1])
        got = y.float().cpu().numpy()          # rows after compaction; compare the survivors
        keep = [k for k in row_nodes if pr.table_keep[k + 1]]
        rel = float(np.max(np.abs(got[:len(keep)] - ref[keep])) / np.max(np.abs(ref)))
        cpu = {"value": round(n / (c1 - c0), 2), "unit": "tree tokens/s", "cores": int(threads), "kind": "oracle",
               "sample": "one full stage step of the same workload (%d nodes, %d layers, prefix %d)" % (n, L, P),
               "seconds": round(c1 - c0, 2), "gpu_vs_oracle_rel_err": rel}

    out = {
        "metric": ("8B-shape 4-layer" if args.workload == "C2" else "70B-shape 10-layer") +
                  " stage step: tree tokens/s (step latency in ms_per_step)",
        "value": round(tok_per_s, 1), "unit": "tree tokens/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "%s: %d-layer stage d=%d heads=%d/%d d_head=%d ffn=%d, prefix %d, tree of %d nodes, "
                               "step = insert + forward + accept + compact" %
                               (args.workload, L, sh.d_model, sh.n_q_heads, sh.n_kv_heads, sh.d_head, sh.d_ff, P, n),
                   "seed": w.seed, "tree_nodes": n, "prefix_len": P, "layers": L,
                   "weights_layout": "row-major" if args.unpacked else "mfma-fragment (sp_pack_weights)"},
        "step_latency_us": round(ms_per_step * 1e3, 1),
        "whole_step_graph_replay_ms": replay_ms,
        "host_enqueue_us_per_step": round((t_enq - t1) * 1e6 / args.steps, 1),
        "step_hbm_floor_frac": round(step_frac, 4),
        "roofline": roofline,
        "cpu_baseline": cpu,
        "setup_s": round(setup_s, 1),
    }
    if kernels is not None:
        out["kernels"] = kernels
    print(json.dumps(out), flush=True)
    stage.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
