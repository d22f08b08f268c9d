"""Ordinary token-by-token decoding with Hugging Face's Llama decoder layer.

The paper builds on Hugging Face Transformers' Llama (Sec. 4, "Implementation"),
so that library is the independent statement of "what the large model would
have produced sequentially".  This helper feeds it the synthetic weights and a
cache that already holds the committed context, then decodes one token at a
time (plain causal decoding, no tree anywhere), or runs one call under an
explicit additive mask.  Float64 throughout; the library computes its rotary
tables in float32, which bounds the agreement at about 1e-6.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np
import torch
from transformers import DynamicCache, LlamaConfig
from transformers.models.llama.modeling_llama import LlamaDecoderLayer, LlamaRotaryEmbedding


class HFStage:
    def __init__(self, shape, weights: Sequence[Dict[str, np.ndarray]]):
        self.shape = shape
        cfg = LlamaConfig(hidden_size=shape.d_model, intermediate_size=shape.d_ff,
                          num_attention_heads=shape.n_q_heads, num_key_value_heads=shape.n_kv_heads,
                          head_dim=shape.d_head, rms_norm_eps=shape.rms_eps,
                          rope_theta=shape.rope_theta, num_hidden_layers=shape.n_layers,
                          attention_bias=False, mlp_bias=False, vocab_size=8,
                          max_position_embeddings=1 << 17)
        cfg._attn_implementation = "eager"
        self.cfg = cfg
        self.rot = LlamaRotaryEmbedding(cfg)
        self.layers: List[LlamaDecoderLayer] = []
        names = {"wq": "self_attn.q_proj", "wk": "self_attn.k_proj", "wv": "self_attn.v_proj",
                 "wo": "self_attn.o_proj", "wg": "mlp.gate_proj", "wu": "mlp.up_proj",
                 "wd": "mlp.down_proj", "norm1": "input_layernorm", "norm2": "post_attention_layernorm"}
        for l in range(shape.n_layers):
            layer = LlamaDecoderLayer(cfg, l).double().eval()
            sd = {names[k] + ".weight": torch.from_numpy(np.asarray(v, np.float64)) for k, v in weights[l].items()}
            missing = layer.load_state_dict(sd, strict=True)
            assert not missing.missing_keys and not missing.unexpected_keys
            self.layers.append(layer)

    def fresh_cache(self, prefix_k: Sequence[np.ndarray], prefix_v: Sequence[np.ndarray]) -> DynamicCache:
        """prefix_k[l], prefix_v[l]: [P, H_kv, d_h] (already rotated)."""
        cache = DynamicCache(config=self.cfg)
        for l in range(self.shape.n_layers):
            k = torch.from_numpy(np.asarray(prefix_k[l], np.float64)).permute(1, 0, 2)[None].contiguous()
            v = torch.from_numpy(np.asarray(prefix_v[l], np.float64)).permute(1, 0, 2)[None].contiguous()
            cache.update(k, v, l)
        return cache

    @torch.no_grad()
    def run(self, x: np.ndarray, positions: Sequence[int], cache: DynamicCache,
            mask: np.ndarray | None = None) -> np.ndarray:
        """x: [n, d]; positions: [n]; mask: None (every cached key and every key of
        this call visible: only valid for n == 1) or bool [n, cached + n]."""
        h = torch.from_numpy(np.asarray(x, np.float64))[None]
        pos = torch.tensor([list(positions)], dtype=torch.long)
        cos, sin = self.rot(h, pos)
        add = None
        if mask is not None:
            m = torch.from_numpy(np.asarray(mask, bool))
            add = torch.zeros(m.shape, dtype=torch.float64).masked_fill(~m, float("-inf"))[None, None]
        else:
            assert h.shape[1] == 1
        for layer in self.layers:
            h = layer(h, attention_mask=add, position_ids=pos, past_key_values=cache,
                      position_embeddings=(cos, sin))
        return h[0].numpy()

    def cache_rows(self, cache: DynamicCache, layer: int):
        """(K, V) as [slots, H_kv, d_h] numpy."""
        lay = cache.layers[layer]
        return (lay.keys[0].permute(1, 0, 2).numpy(), lay.values[0].permute(1, 0, 2).numpy())
