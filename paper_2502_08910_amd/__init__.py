"""MI355X (gfx950) implementation of InfiniteHiP's pruning + block-sparse
attention hot path: HIP kernels behind a C ABI (include/ihip.h), with a thin
ctypes binding.  No CPU or PyTorch fallback exists."""
from .binding import (IhipError, Layer, Rope, PagedKV, ROPE_NONE, ROPE_RELATIVE, ROPE_CHUNK_INDEXED, ROPE_STREAMING, POOL_KV_HEAD, POOL_ALL_HEADS, HostKVCache, decode_layer_cached, prune_stage_cached, sparse_attn_decode_cached, first_stage_due, refresh_due, lib, LIB_PATH, mfma_rate, profile_enable, profile_read, OP_ATTN_DECODE, OP_ATTN_PREFILL,  # noqa: F401
                      OP_PRUNE_ALL, OP_DECODE_LAYER, OP_PREFILL_LAYER)
