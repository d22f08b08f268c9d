"""Closed forms the paper prints that fix the storage layout (Sec. 4.5 Table 1, Sec. 4.2)."""
import os

import workloads as wl

GOLD = os.path.join(os.path.dirname(__file__), "golden", "memory_table.txt")


def golden():
    out = {}
    for line in open(GOLD):
        if line.strip() and not line.startswith("#"):
            k, v = line.split()
            out[k] = float(v)
    return out


def test_memory_table_fixes_the_kv_row_size():
    g = golden()
    s = wl.LLAMA_70B_STAGE
    GiB = float(1 << 30)
    d, f, V = s.d_model, s.d_ff, 128256
    n_layer = 4 * d * d + 3 * d * f                       # the paper's count
    weights = 10 * n_layer * 2 / GiB
    kv = 81920 * 10 * s.kv_bytes_per_token_per_layer / GiB
    runtime = 0.25
    assert s.kv_bytes_per_token_per_layer == 4096         # K and V, 8 heads x 128, bf16
    assert round(weights + kv + runtime, 1) == g["gpu_middle"]
    emb = V * d * 2 / GiB
    assert round(weights + kv + runtime + emb, 1) == g["gpu_first"] == g["gpu_last"]


def test_hidden_row_size():
    g = golden()
    s = wl.LLAMA_70B_STAGE
    assert s.d_model * s.elt_bytes == g["hidden_one_token_KiB"] * 1024
    assert 64 * s.d_model * s.elt_bytes == g["hidden_64_tokens_MiB"] * (1 << 20)


def test_config_shapes():
    c2, c3 = wl.CONFIGS["C2"].shape, wl.CONFIGS["C3"].shape
    assert c2.params_per_layer == 218103808 and c3.params_per_layer == 855638016
    assert c2.group == 4 and c3.group == 8


def test_bench_traffic_comes_from_the_profile_summary():
    """bench.py's roofline.traffic is the figure of the committed counter summary, not a constant in the
    script: the summary's machine-readable line parses, and it is a plausible byte count for one gate/up
    launch of the 8B shape at 64 rows (at least the algorithmic bytes, at most a few per cent more)."""
    import bench
    import workloads as wl
    sh = wl.CONFIGS["C2"].shape
    algorithmic = 2 * sh.d_ff * sh.d_model * 2 + 64 * sh.d_model * 2 + 64 * sh.d_ff * 2
    t = bench.profiled_traffic()
    assert t is not None
    assert algorithmic <= t <= 1.1 * algorithmic
