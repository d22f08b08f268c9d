"""CPU oracle for the SpecPipe stage hot path (TEST INFRASTRUCTURE, not product).

A plain, slow, float64 numpy statement of what one pipeline stage computes
over the dynamic speculative token tree and of how pruning propagation
compacts the tree tables and the KV cache.  It follows the paper's notation:
the tree is the triple (I, P, M) of Sec. 3.2 with the last verified token as
root tau_1, a device holds {E_i, M_i, KV_i} (Algorithm 1), and pruning uses
the column / row-OR-column masks of Sec. 3.3.2.

Only tests/, __graft_entry__.smoke() and bench.py's cpu_baseline leg may
import this package.  It shares no code with the HIP library and never falls
back to it or serves as a fallback for it.

Parity pins (tests/test_oracle_*.py): ancestor walk by brute force, the block
form of layer appending, prune == rebuild from survivors, Hugging Face's Llama
decoder layer run sequentially along every root-to-leaf path, torch SDPA with
an explicit mask, RoPE's relative-position identity, the closed forms of
the paper's memory table, and for verification Hugging Face's RMSNorm + a
torch Linear and the lossless property (tree-speculative decoding emits the
sequence of plain greedy decoding); for stochastic verification Hugging Face's temperature /
top-k / top-p warpers, the measure of the uniform numbers that draw each candidate, and the limits
that reduce the draw to the arg-max.  No function here is "parity unpinned".
"""
from .tree import SpecTree
from .stage import (StageOracle, RequestState, rmsnorm, rope_rotate, silu, tree_attention,
                    decoder_layer)
from .prune import (accept_masks, drop_masks, compact_rows, PruneResult)
from .verify import (lm_head_logits, greedy_token, greedy_token_fast, match_root_child, softmax_probs, top_p_set,
                     relaxed_choice, top_p_choice, sampling_candidates, sample_token)

__all__ = [
    "SpecTree", "StageOracle", "RequestState", "rmsnorm", "rope_rotate", "silu",
    "tree_attention", "decoder_layer", "accept_masks", "drop_masks", "compact_rows",
    "PruneResult", "lm_head_logits", "greedy_token", "greedy_token_fast", "match_root_child",
    "softmax_probs", "top_p_set", "relaxed_choice", "top_p_choice", "sampling_candidates", "sample_token",
]
