"""SpecPipe stage hot path for AMD MI355X: HIP kernels behind a C ABI (include/specpipe.h)
and a thin ctypes binding."""
from .binding import (Stage, SpError, load_library, pack_layer_weights, pack_weights, write_prefix, LIB_PATH,
                      SP_FLAG_PACKED_WEIGHTS, SP_FLAG_PAGED_KV, SP_FLAG_NO_GRAPHS,
                      SP_ACCEPT, SP_DROP, SP_CLEAR, SP_VERIFY_RELAXED, SP_VERIFY_TOP_P, pack_matrix, SP_F32, SP_BF16, SP_FLAG_SIMPLE_KERNELS, SP_MAX_TREE_NODES,
                      SP_MAX_BATCH_REQ)

__all__ = ["Stage", "SpError", "load_library", "pack_layer_weights", "pack_weights", "SP_FLAG_PACKED_WEIGHTS", "SP_FLAG_PAGED_KV", "SP_FLAG_NO_GRAPHS", "write_prefix", "LIB_PATH", "SP_ACCEPT",
           "SP_DROP", "SP_CLEAR", "SP_VERIFY_RELAXED", "SP_VERIFY_TOP_P", "pack_matrix", "SP_F32", "SP_BF16", "SP_FLAG_SIMPLE_KERNELS", "SP_MAX_TREE_NODES", "SP_MAX_BATCH_REQ"]
