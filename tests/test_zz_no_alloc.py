"""The allocation-free output-head entry point (sp_stage_verify_head_noalloc: scratch in a fixed array
inside the library) against sp_stage_verify_head (scratch in the stage's workspace), through the C ABI:
same predictions, same winning logits, on two calls in a row of which the second is smaller, and the
documented capacity error.  Runs last: it must pass alone in a fresh process and after every other test."""
import numpy as np
import pytest
import torch

import workloads as wl
import paper_2504_04104_amd as sp
from gpu_harness import Pair, to_dev

pytestmark = pytest.mark.gpu

MINI_BF16 = wl.ModelShape(n_layers=2, d_model=512, n_q_heads=4, n_kv_heads=2, d_head=128, d_ff=768)
MINI_F32 = wl.ModelShape(n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, d_head=64, d_ff=688,
                         rms_eps=1e-6, dtype="f32")


@pytest.mark.parametrize("shape,flags,V", [(MINI_BF16, sp.SP_FLAG_PACKED_WEIGHTS, 1088), (MINI_BF16, 0, 4160),
                                           (MINI_F32, 0, 97)], ids=["bf16_packed", "bf16", "f32_plain_kernels"])
def test_noalloc_head_matches_workspace_head(shape, flags, V):
    pair = Pair(shape, 41, {0: 40, 1: 75}, flags=flags, vocab=V, max_batch_nodes=128, oracle=False)
    g = pair.gpu
    counts = [37, 21]
    for r, n in enumerate(counts):
        g.tree_insert(r, wl.tree_uniform_parents(41, n, 8, name=("na", r)), list(range(100 * r, 100 * r + n)))
    x = to_dev(wl.hidden_rows(shape, 41, ("na",), sum(counts)), g)
    y = g.stage_forward([0, 1], [0, 0], counts, x)
    # first call: both requests (58 rows); second call: a smaller one (10 rows of request 0)
    for reqs, firsts, ns, rows in (([0, 1], [0, 0], counts, y), ([0], [5], [10], y[5:15].contiguous())):
        n = sum(ns)
        print("no-alloc head:", n, "rows, vocab", V, flush=True)
        want_pred, want_max = g.verify_head(pair.head, reqs, firsts, ns, rows, want_max=True)
        want_pred, want_max = want_pred.clone(), want_max.clone()
        stored = [g.tree_read(r)["pred"].copy() for r in reqs]
        pred = torch.full((n,), -7, dtype=torch.int32, device=g.device)
        mx = torch.full((n,), float("nan"), dtype=torch.float32, device=g.device)
        g.verify_head(pair.head, reqs, firsts, ns, rows, noalloc=True, out=(pred, mx))
        torch.cuda.synchronize()
        assert torch.equal(pred, want_pred)
        assert torch.equal(mx.view(torch.int32), want_max.view(torch.int32))
        assert len(set(pred.tolist())) > 3
        for r, s_ in zip(reqs, stored):
            assert np.array_equal(g.tree_read(r)["pred"], s_)
    # more rows than the fixed array is carved for: a clear error, nothing written
    g.tree_insert(0, [-1] * 40)
    x2 = to_dev(wl.hidden_rows(shape, 41, ("na2",), 40), g)
    y2 = g.stage_forward([0], [37], [40], x2)
    big = torch.cat([y[:37], y2]).contiguous()
    pred = torch.full((77,), -7, dtype=torch.int32, device=g.device)
    with pytest.raises(sp.SpError) as ei:
        g.verify_head(pair.head, [0], [0], [77], big, noalloc=True, out=(pred, None))
    assert ei.value.status == -2                                               # SP_E_CAPACITY
    torch.cuda.synchronize()
    assert int((pred != -7).sum()) == 0
    # the workspace entry point still takes them
    assert g.verify_head(pair.head, [0], [0], [77], big).shape[0] == 77
    pair.close()
