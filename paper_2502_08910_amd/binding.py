"""ctypes binding of libihip.so: argument marshalling only.

Every step of the path runs in the library's HIP kernels; PyTorch supplies
device memory and the stream.  There is no fallback: if the library is
missing or a call fails this module raises.
"""
from __future__ import annotations

import ctypes
import math
import os
from typing import Optional, Sequence

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libihip.so")

OP_ATTN_DECODE, OP_ATTN_PREFILL, OP_PRUNE_ALL, OP_DECODE_LAYER, OP_PREFILL_LAYER = 1, 2, 3, 4, 5

c_i32, c_i64, c_f, vp, c_sz = (ctypes.c_int32, ctypes.c_int64, ctypes.c_float, ctypes.c_void_p,
                               ctypes.c_size_t)


class IhipError(RuntimeError):
    pass


class Tensor(ctypes.Structure):
    _fields_ = [("ptr", vp), ("stride_b", c_i64), ("stride_h", c_i64), ("stride_t", c_i64)]


class Shape(ctypes.Structure):
    _fields_ = [("B", c_i32), ("Hq", c_i32), ("Hkv", c_i32), ("d", c_i32), ("Tq", c_i32),
                ("b_q", c_i32), ("seq_lens", vp), ("max_seq_len", c_i32), ("n_sink", c_i32),
                ("n_stream", c_i32), ("b_q_range", c_i32)]


EXPORTS = {
    "ihip_prune_stage": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, vp, c_i32, c_i32, c_i32, c_i32,
                                 vp, vp, vp]),
    "ihip_prune_stage_rope": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, vp, c_i32, c_i32, c_i32, c_i32,
                                      vp, vp, vp, vp]),
    "ihip_sparse_attn_decode_rope": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                             c_f, vp, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer_rope": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f, vp,
                                       vp, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer_ex": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f, vp,
                                     vp, vp, vp, vp, c_sz, vp]),
    "ihip_sparse_attn_prefill_paged": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, vp, c_i32, c_i32,
                                               c_f, vp, vp, vp, vp, c_sz, vp]),
    "ihip_subdivide_blocks": (c_i32, [ctypes.POINTER(Shape), vp, c_i32, c_i32, vp, vp]),
    "ihip_sparse_attn_prefill_fp8kv": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                               c_f, c_f, c_f, vp, vp, vp, vp, c_sz, vp]),
    "ihip_prefill_layer_ex": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f, vp,
                                      vp, vp, vp, vp, c_sz, vp]),
    "ihip_sparse_attn_prefill_rope": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                              c_f, vp, vp, vp, vp, c_sz, vp]),
    "ihip_prefill_layer_rope": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f, vp,
                                        vp, vp, vp, vp, c_sz, vp]),
    "ihip_prune_stage_fp8kv": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, vp, c_i32, c_i32, c_i32, c_i32,
                                       c_f, vp, vp, vp]),
    "ihip_sparse_attn_decode_fp8kv": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                              c_f, c_f, c_f, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer_fp8kv": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f, c_f, c_f,
                                        vp, vp, vp, vp, c_sz, vp]),
    "ihip_prune_stage_paged": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, vp, vp, c_i32, c_i32, c_i32, c_i32,
                                       vp, vp, vp]),
    "ihip_sparse_attn_decode_paged": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, vp, c_i32, c_i32,
                                              c_f, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer_paged": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, vp, vp, c_f,
                                        vp, vp, vp, vp, c_sz, vp]),
    "ihip_stage1_slots": (c_i32, [ctypes.POINTER(Shape), c_i32]),
    "ihip_select_blocks": (c_i32, [ctypes.POINTER(Shape), vp, c_i32, vp, c_i32, c_i32, c_i32, c_i32,
                                   vp, vp]),
    "ihip_select_blocks_pooled": (c_i32, [ctypes.POINTER(Shape), vp, c_i32, vp, c_i32, c_i32, c_i32, c_i32, c_i32,
                                          vp, vp]),
    "ihip_decode_layer_pooled": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_i32, c_f,
                                         vp, vp, vp, vp, c_sz, vp]),
    "ihip_prefill_layer_pooled": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_i32, c_f,
                                          vp, vp, vp, vp, c_sz, vp]),
    "ihip_sparse_attn_decode": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                        c_f, vp, vp, vp, c_sz, vp]),
    "ihip_sparse_attn_prefill": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, vp, c_i32, c_i32,
                                         c_f, vp, vp, vp, c_sz, vp]),
    "ihip_prune_all": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, c_i32, vp, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f,
                                  vp, vp, vp, vp, c_sz, vp]),
    "ihip_decode_layer_static": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f,
                                         vp, vp, vp, vp]),
    "ihip_mask_state_elems": (c_sz, [ctypes.POINTER(Shape), c_i32, vp]),
    "ihip_decode_layer_masked": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_i32, vp,
                                         c_f, vp, vp, vp, c_sz, vp]),
    "ihip_prefill_layer": (c_i32, [ctypes.POINTER(Shape), Tensor, Tensor, Tensor, c_i32, vp, vp, c_f,
                                   vp, vp, vp, vp, c_sz, vp]),
    "ihip_cache_device_bytes": (c_sz, [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32]),
    "ihip_cache_device_bytes_fp8": (c_sz, [c_i32, c_i32, c_i64, c_i32, c_i32, c_i32]),
    "ihip_cache_create_fp8": (c_i32, [ctypes.POINTER(vp), vp, c_sz, Tensor, Tensor, c_i32, c_i32, c_i64, c_i32,
                                      c_i32, c_i32, vp]),
    "ihip_cache_create": (c_i32, [ctypes.POINTER(vp), vp, c_sz, Tensor, Tensor, c_i32, c_i32, c_i64, c_i32,
                                  c_i32, c_i32, vp]),
    "ihip_cache_destroy": (None, [vp]),
    "ihip_cache_create_paged": (c_i32, [ctypes.POINTER(vp), vp, c_sz, Tensor, Tensor, vp, c_i32, c_i32, c_i32, c_i64,
                                        c_i32, c_i32, c_i32, vp]),
    "ihip_cache_reset": (c_i32, [vp, vp]),
    "ihip_decode_layer_cached": (c_i32, [ctypes.POINTER(Shape), Tensor, vp, c_i32, vp, vp, c_f, vp, vp, vp,
                                         vp, c_sz, vp]),
    "ihip_prune_stage_cached": (c_i32, [ctypes.POINTER(Shape), Tensor, vp, vp, c_i32, c_i32, c_i32, c_i32, vp, c_f,
                                        vp, vp, vp]),
    "ihip_sparse_attn_decode_cached": (c_i32, [ctypes.POINTER(Shape), Tensor, vp, vp, c_i32, c_i32, c_f, vp, c_f, c_f,
                                               vp, vp, vp, c_sz, vp]),
    "ihip_refresh_due": (c_i32, [c_i32, vp, c_i64, vp]),
    "ihip_cache_update": (c_i32, [vp, vp]),
    "ihip_cache_stats": (c_i32, [vp, vp]),
    "ihip_cache_read_tables": (c_i32, [vp, c_i32, vp, vp]),
    "ihip_cache_geometry": (c_i32, [vp, vp, vp, vp]),
    "ihip_workspace_bytes": (c_sz, [c_i32, ctypes.POINTER(Shape), c_i32, vp, vp]),
    "ihip_profile_enable": (c_i32, [c_i32]),
    "ihip_profile_read": (c_i32, [c_i32, vp, vp, vp]),
    "ihip_mfma_rate": (c_i32, [c_i32, c_i32, vp, vp, vp]),
    "ihip_last_error": (ctypes.c_char_p, []),
    "ihip_version": (c_i32, []),
}

_lib = None


def lib() -> ctypes.CDLL:
    """Loads the in-tree HIP library; raises if it was not built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise IhipError(f"{LIB_PATH} is missing: build it with "
                            "`python -m paper_2502_08910_amd.build` (there is no fallback path)")
        L = ctypes.CDLL(LIB_PATH)
        for name, (res, args) in EXPORTS.items():
            fn = getattr(L, name)
            fn.restype, fn.argtypes = res, args
        _lib = L
    return _lib


def _check(rc: int):
    if rc != 0:
        raise IhipError(f"ihip error {rc}: {lib().ihip_last_error().decode()}")


def _tensor(t: torch.Tensor, name: str) -> Tensor:
    if t.dtype != torch.bfloat16 or t.dim() != 4 or t.stride(3) != 1 or not t.is_cuda:
        raise IhipError(f"{name}: need a 4-d bf16 device tensor with contiguous last dim")
    return Tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _tensor8(t: torch.Tensor, name: str) -> Tensor:
    """FP8 (E4M3) K/V as a uint8 tensor; strides in bytes."""
    if t.dtype != torch.uint8 or t.dim() != 4 or t.stride(3) != 1 or not t.is_cuda:
        raise IhipError(f"{name}: need a 4-d uint8 device tensor with contiguous last dim")
    return Tensor(t.data_ptr(), t.stride(0), t.stride(1), t.stride(2))


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else t.data_ptr()


def _i32(xs: Sequence[int]):
    return (c_i32 * len(xs))(*xs)


def profile_enable(on: bool) -> None:
    _check(lib().ihip_profile_enable(int(on)))


def profile_read(max_entries: int = 64) -> dict:
    """{kernel name: (total ms, launches)} of the launches recorded since the last read."""
    names = (ctypes.c_char_p * max_entries)()
    ms = (ctypes.c_double * max_entries)()
    cnt = (ctypes.c_int64 * max_entries)()
    n = lib().ihip_profile_read(max_entries, names, ms, cnt)
    if n < 0:
        _check(n)
    return {names[i].decode(): (ms[i], cnt[i]) for i in range(n)}


def mfma_rate(kind: int, iters: int = 20000) -> float:
    """Dense bf16 MFMA rate of the current GPU in TFLOP/s (kind 0: 32x32x16, 1: 16x16x32)."""
    scratch = torch.zeros(512, dtype=torch.float32, device="cuda")
    out = ctypes.c_double(0.0)
    _check(lib().ihip_mfma_rate(kind, iters, scratch.data_ptr(), ctypes.byref(out), _stream()))
    return out.value


ROPE_NONE, ROPE_RELATIVE, ROPE_CHUNK_INDEXED, ROPE_STREAMING = 0, 1, 2, 1
POOL_KV_HEAD, POOL_ALL_HEADS = 0, 1


class RopeStruct(ctypes.Structure):
    _fields_ = [("cos", vp), ("sin", vp), ("n_pos", c_i32), ("prune_style", c_i32), ("attn_style", c_i32)]


class Rope:
    """ihip_rope: device fp32 cos / sin tables [n_pos, d/2] and the styles to apply."""

    def __init__(self, cos: torch.Tensor, sin: torch.Tensor, prune_style: int = ROPE_NONE,
                 attn_style: int = ROPE_NONE):
        for t in (cos, sin):
            if t.dtype != torch.float32 or t.dim() != 2 or not t.is_cuda or not t.is_contiguous():
                raise IhipError("rope tables: need contiguous 2-d fp32 device tensors")
        if cos.shape != sin.shape:
            raise IhipError("rope tables: cos and sin differ in shape")
        self.cos, self.sin = cos, sin          # keep the tables alive
        self.c = RopeStruct(cos.data_ptr(), sin.data_ptr(), cos.shape[0], prune_style, attn_style)

    def ref(self):
        return ctypes.byref(self.c)


class PagedStruct(ctypes.Structure):
    _fields_ = [("block_table", vp), ("table_stride", c_i32), ("page_tokens", c_i32)]


class PagedKV:
    """ihip_paged_kv: K / V page pools [n_pages, Hkv, page_tokens, d] (bf16, any strides with a
    contiguous last dim) and the device block table int32 [B, table_stride]."""

    def __init__(self, k_pool: torch.Tensor, v_pool: torch.Tensor, block_table: torch.Tensor):
        if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.dim() != 2 \
                or not block_table.is_contiguous():
            raise IhipError("block_table: need a contiguous int32 device tensor [B, pages]")
        self.k_pool, self.v_pool, self.block_table = k_pool, v_pool, block_table
        self.c = PagedStruct(block_table.data_ptr(), block_table.shape[1], k_pool.shape[2])

    def ref(self):
        return ctypes.byref(self.c)


class DecodeOptions(ctypes.Structure):
    """ihip_decode_options (all zero = the plain decode layer)."""
    _fields_ = [("rope", vp), ("cache", vp), ("paged", vp), ("kv_fp8", c_i32), ("k_scale", c_f), ("v_scale", c_f),
                ("pooling", c_i32), ("first_stage", c_i32), ("stage_starts", vp), ("stage_due", vp)]


class PrefillOptions(ctypes.Structure):
    """ihip_prefill_options (all zero = the plain prefill layer)."""
    _fields_ = [("rope", vp), ("paged", vp), ("pooling", c_i32), ("kv_fp8", c_i32), ("k_scale", c_f), ("v_scale", c_f),
                ("stage_b_q", vp)]


class Layer:
    """Shape of one attention call plus the device seq_lens; the methods are
    the C entry points of the same names."""

    def __init__(self, q: torch.Tensor, k: torch.Tensor, seq_lens: torch.Tensor, b_q: int, n_sink: int,
                 n_stream: int, max_seq_len: Optional[int] = None, b_q_range: int = 0):
        """b_q_range: the first pruning stage's block size when the stages use different ones
        (ihip_shape.b_q_range); 0 = b_q."""
        B, Hq, Tq, d = q.shape
        Hkv = k.shape[1]
        if seq_lens.dtype != torch.int32 or not seq_lens.is_cuda or seq_lens.numel() != B:
            raise IhipError("seq_lens: need an int32 device tensor [B]")
        self.seq_lens = seq_lens
        self.max_seq_len = int(k.shape[2] if max_seq_len is None else max_seq_len)
        if self.max_seq_len > k.shape[2]:
            raise IhipError("max_seq_len exceeds the allocated tokens of K")
        self.shape = Shape(B, Hq, Hkv, d, Tq, b_q, seq_lens.data_ptr(), self.max_seq_len, n_sink, n_stream, b_q_range)
        self.B, self.Hq, self.Hkv, self.d, self.Tq, self.b_q = B, Hq, Hkv, d, Tq, b_q
        self.P = B * Hkv * (Tq // max(b_q, 1))
        self.device = q.device

    # -- helpers ------------------------------------------------------------
    def stage1_slots(self, chunk: int) -> int:
        n = lib().ihip_stage1_slots(ctypes.byref(self.shape), chunk)
        if n < 0:
            raise IhipError(lib().ihip_last_error().decode())
        return n

    def workspace_bytes(self, op: int, chunk_sizes: Sequence[int], keeps: Sequence[int]) -> int:
        n = lib().ihip_workspace_bytes(op, ctypes.byref(self.shape), len(chunk_sizes), _i32(chunk_sizes),
                                       _i32(keeps))
        if n == 0:
            raise IhipError(lib().ihip_last_error().decode())
        return n

    def workspace(self, op: int, chunk_sizes, keeps) -> torch.Tensor:
        return torch.empty(self.workspace_bytes(op, chunk_sizes, keeps), dtype=torch.uint8, device=self.device)

    # -- entry points -------------------------------------------------------
    def prune_stage(self, q, k, chunk: int, parent_starts: Optional[torch.Tensor] = None,
                    parent_chunk: int = 0, want_rep: bool = False, rope: Optional["Rope"] = None,
                    k_scale: Optional[float] = None, paged: Optional["PagedKV"] = None):
        """-> scores fp32 [P, slots], rep int32 [B,Hq,Mq,slots] or None.  k_scale: k holds E4M3 bytes;
        paged: k is ignored, the K pool of `paged` is read through its block table."""
        if parent_starts is None:
            n_parent, slots = 0, self.stage1_slots(chunk)
        else:
            n_parent = parent_starts.shape[-1]
            slots = n_parent * (parent_chunk // chunk)
        scores = torch.empty((self.P, slots), dtype=torch.float32, device=self.device)
        rep = torch.empty((self.B, self.Hq, self.Tq // self.b_q, slots), dtype=torch.int32,
                          device=self.device) if want_rep else None
        if paged is not None:
            _check(lib().ihip_prune_stage_paged(ctypes.byref(self.shape), _tensor(q, "q"),
                                                _tensor(paged.k_pool, "k_pool"), paged.ref(), _ptr(parent_starts),
                                                n_parent, parent_chunk, chunk, slots, _ptr(scores), _ptr(rep),
                                                _stream()))
            return scores, rep
        if k_scale is not None:
            _check(lib().ihip_prune_stage_fp8kv(ctypes.byref(self.shape), _tensor(q, "q"), _tensor8(k, "k"),
                                                _ptr(parent_starts), n_parent, parent_chunk, chunk, slots,
                                                k_scale, _ptr(scores), _ptr(rep), _stream()))
            return scores, rep
        if rope is not None:
            _check(lib().ihip_prune_stage_rope(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                               _ptr(parent_starts), n_parent, parent_chunk, chunk, slots,
                                               rope.ref(), _ptr(scores), _ptr(rep), _stream()))
            return scores, rep
        _check(lib().ihip_prune_stage(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                      _ptr(parent_starts), n_parent, parent_chunk, chunk, slots,
                                      _ptr(scores), _ptr(rep), _stream()))
        return scores, rep

    def subdivide_blocks(self, starts: torch.Tensor, b_q_fine: int) -> torch.Tensor:
        """Kept lists [P, n] of this layer's blocks -> [P * b_q / b_q_fine, n] for blocks of b_q_fine queries."""
        n = starts.shape[-1]
        out = torch.empty((self.P * (self.b_q // b_q_fine), n), dtype=torch.int32, device=self.device)
        _check(lib().ihip_subdivide_blocks(ctypes.byref(self.shape), _ptr(starts), n, b_q_fine, _ptr(out), _stream()))
        return out

    def select_blocks(self, scores: torch.Tensor, chunk: int, keep: int,
                      parent_starts: Optional[torch.Tensor] = None, parent_chunk: int = 0,
                      pooling: Optional[int] = None):
        """-> kept start positions int32 [P, keep], ascending, -1 padded."""
        n_parent = 0 if parent_starts is None else parent_starts.shape[-1]
        out = torch.empty((self.P, keep), dtype=torch.int32, device=self.device)
        if pooling is not None:
            _check(lib().ihip_select_blocks_pooled(ctypes.byref(self.shape), _ptr(scores), scores.shape[-1],
                                                   _ptr(parent_starts), n_parent, parent_chunk, chunk, keep,
                                                   pooling, _ptr(out), _stream()))
            return out
        _check(lib().ihip_select_blocks(ctypes.byref(self.shape), _ptr(scores), scores.shape[-1],
                                        _ptr(parent_starts), n_parent, parent_chunk, chunk, keep,
                                        _ptr(out), _stream()))
        return out

    def _attn(self, fn, op, q, k, v, block_starts, block, sm_scale, want_lse, ws):
        n_blocks = block_starts.shape[-1]
        sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
        out = torch.empty((self.B, self.Hq, self.Tq, self.d), dtype=torch.bfloat16, device=self.device)
        lse = torch.empty((self.B, self.Hq, self.Tq), dtype=torch.float32, device=self.device) \
            if want_lse else None
        if ws is None:
            ws = self.workspace(op, [block], [max(n_blocks, 1)])
        _check(fn(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"), _tensor(v, "v"),
                  _ptr(block_starts), n_blocks, block, sm_scale, _ptr(out), _ptr(lse), _ptr(ws),
                  ws.numel(), _stream()))
        return out, lse

    def sparse_attn_decode(self, q, k, v, block_starts, block, sm_scale=None, want_lse=False, ws=None,
                           rope: Optional["Rope"] = None, kv_scales: Optional[Sequence[float]] = None,
                           paged: Optional["PagedKV"] = None):
        if paged is not None:
            def fn(shape, tq, tk, tv, bs, n_blocks, blk, scale, out, lse, w, w_bytes, stream):
                return lib().ihip_sparse_attn_decode_paged(shape, tq, _tensor(paged.k_pool, "k_pool"),
                                                           _tensor(paged.v_pool, "v_pool"), paged.ref(), bs, n_blocks,
                                                           blk, scale, out, lse, w, w_bytes, stream)
            return self._attn(fn, OP_ATTN_DECODE, q, paged.k_pool, paged.v_pool, block_starts, block, sm_scale,
                              want_lse, ws)
        if kv_scales is not None:
            n_blocks = block_starts.shape[-1]
            sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
            out = torch.empty((self.B, self.Hq, 1, self.d), dtype=torch.bfloat16, device=self.device)
            lse = torch.empty((self.B, self.Hq, 1), dtype=torch.float32, device=self.device) if want_lse else None
            if ws is None:
                ws = self.workspace(OP_ATTN_DECODE, [block], [max(n_blocks, 1)])
            _check(lib().ihip_sparse_attn_decode_fp8kv(ctypes.byref(self.shape), _tensor(q, "q"), _tensor8(k, "k"),
                                                       _tensor8(v, "v"), _ptr(block_starts), n_blocks, block,
                                                       sm_scale, kv_scales[0], kv_scales[1], _ptr(out), _ptr(lse),
                                                       _ptr(ws), ws.numel(), _stream()))
            return out, lse
        if rope is not None:
            def fn(shape, tq, tk, tv, bs, n_blocks, blk, scale, out, lse, w, w_bytes, stream):
                return lib().ihip_sparse_attn_decode_rope(shape, tq, tk, tv, bs, n_blocks, blk, scale, rope.ref(),
                                                          out, lse, w, w_bytes, stream)
            return self._attn(fn, OP_ATTN_DECODE, q, k, v, block_starts, block, sm_scale, want_lse, ws)
        return self._attn(lib().ihip_sparse_attn_decode, OP_ATTN_DECODE, q, k, v, block_starts, block,
                          sm_scale, want_lse, ws)

    def sparse_attn_prefill(self, q, k, v, block_starts, block, sm_scale=None, want_lse=False, ws=None,
                            rope: Optional["Rope"] = None, paged: Optional["PagedKV"] = None,
                            kv_scales: Optional[Sequence[float]] = None):
        if kv_scales is not None:
            if paged is not None:
                raise ValueError("E4M3 page pools go through prefill_layer (ihip_prefill_layer_ex)")
            sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
            out = torch.empty((self.B, self.Hq, self.Tq, self.d), dtype=torch.bfloat16, device=self.device)
            lse = torch.empty((self.B, self.Hq, self.Tq), dtype=torch.float32, device=self.device) if want_lse else None
            _check(lib().ihip_sparse_attn_prefill_fp8kv(
                ctypes.byref(self.shape), _tensor(q, "q"), _tensor8(k, "k"), _tensor8(v, "v"), _ptr(block_starts),
                block_starts.shape[-1], block, sm_scale, kv_scales[0], kv_scales[1],
                rope.ref() if rope is not None else None, _ptr(out), _ptr(lse), None, 0, _stream()))
            return out, lse
        if paged is not None:
            def fn(shape, tq, tk, tv, bs, n_blocks, blk, scale, out, lse, w, w_bytes, stream):
                return lib().ihip_sparse_attn_prefill_paged(shape, tq, tk, tv, paged.ref(), bs, n_blocks, blk, scale,
                                                            rope.ref() if rope is not None else None, out, lse, w,
                                                            w_bytes, stream)
            return self._attn(fn, OP_ATTN_PREFILL, q, paged.k_pool, paged.v_pool, block_starts, block, sm_scale,
                              want_lse, ws)
        if rope is not None:
            def fn(shape, tq, tk, tv, bs, n_blocks, blk, scale, out, lse, w, w_bytes, stream):
                return lib().ihip_sparse_attn_prefill_rope(shape, tq, tk, tv, bs, n_blocks, blk, scale, rope.ref(),
                                                           out, lse, w, w_bytes, stream)
            return self._attn(fn, OP_ATTN_PREFILL, q, k, v, block_starts, block, sm_scale, want_lse, ws)
        return self._attn(lib().ihip_sparse_attn_prefill, OP_ATTN_PREFILL, q, k, v, block_starts, block,
                          sm_scale, want_lse, ws)

    def prune_all(self, q, k, chunk_sizes, keeps, ws=None, out=None):
        """-> last stage's kept block starts int32 [P, keeps[-1]]."""
        if out is None:
            out = torch.empty((self.P, keeps[-1]), dtype=torch.int32, device=self.device)
        if ws is None:
            ws = self.workspace(OP_PRUNE_ALL, chunk_sizes, keeps)
        _check(lib().ihip_prune_all(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                    len(chunk_sizes), _i32(chunk_sizes), _i32(keeps), _ptr(out), _ptr(ws),
                                    ws.numel(), _stream()))
        return out

    def decode_layer(self, q, k, v, chunk_sizes, keeps, sm_scale=None, ws=None, out=None,
                     out_blocks=None, lse=None, rope: Optional["Rope"] = None, pooling: Optional[int] = None,
                     kv_scales: Optional[Sequence[float]] = None, paged: Optional["PagedKV"] = None,
                     cache: Optional["HostKVCache"] = None, stage_starts: Optional[torch.Tensor] = None,
                     first_stage: Optional[int] = None, stage_due: Optional[Sequence[int]] = None):
        """Pruning stages + block-sparse decode attention in one enqueue -> bf16 [B,Hq,1,d].
        paged: k and v are ignored, the pools of `paged` are read through its block table.
        cache: k and v are ignored, the host tier is read.  stage_starts / first_stage: mask caching
        (see decode_layer_masked); stage_due: one flag per stage instead of first_stage (Alg. 4's per-stage
        test).  One variant alone goes to its own entry point, combinations (and the host tier, and
        stage_due) to ihip_decode_layer_ex."""
        sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
        if out is None:
            out = torch.empty((self.B, self.Hq, 1, self.d), dtype=torch.bfloat16, device=self.device)
        if ws is None:
            ws = self.workspace(OP_DECODE_LAYER, chunk_sizes, keeps)
        n_variants = sum(x is not None for x in (rope, pooling, kv_scales, paged, cache, stage_starts))
        if stage_starts is not None and first_stage is None and stage_due is None:
            raise IhipError("decode_layer: stage_starts needs first_stage or stage_due")
        if n_variants > 1 or cache is not None or stage_due is not None:
            # combinations go through the one entry point that takes them all
            opt = DecodeOptions()
            opt.rope = ctypes.cast(rope.ref(), vp) if rope is not None else None
            opt.cache = cache.handle if cache is not None else None
            opt.paged = ctypes.cast(paged.ref(), vp) if paged is not None else None
            if kv_scales is not None:
                opt.kv_fp8, opt.k_scale, opt.v_scale = 1, kv_scales[0], kv_scales[1]
            opt.pooling = POOL_KV_HEAD if pooling is None else pooling
            opt.first_stage = 0 if first_stage is None or stage_due is not None else first_stage
            opt.stage_starts = stage_starts.data_ptr() if stage_starts is not None else None
            due = _i32([int(bool(x)) for x in stage_due]) if stage_due is not None else None   # alive until the call returns
            opt.stage_due = ctypes.cast(due, vp) if due is not None else None
            conv = _tensor8 if kv_scales is not None else _tensor
            if paged is not None:
                tk, tv = conv(paged.k_pool, "k_pool"), conv(paged.v_pool, "v_pool")
            elif cache is not None:
                tk = tv = Tensor(None, 0, 0, 0)
            else:
                tk, tv = conv(k, "k"), conv(v, "v")
            _check(lib().ihip_decode_layer_ex(ctypes.byref(self.shape), _tensor(q, "q"), tk, tv, len(chunk_sizes),
                                              _i32(chunk_sizes), _i32(keeps), sm_scale, ctypes.byref(opt),
                                              _ptr(out), _ptr(lse), _ptr(out_blocks), _ptr(ws), ws.numel(),
                                              _stream()))
            return out
        if stage_starts is not None:
            return self.decode_layer_masked(q, k, v, chunk_sizes, keeps, first_stage, stage_starts, sm_scale, ws,
                                            out, lse)
        if paged is not None:
            _check(lib().ihip_decode_layer_paged(ctypes.byref(self.shape), _tensor(q, "q"),
                                                 _tensor(paged.k_pool, "k_pool"), _tensor(paged.v_pool, "v_pool"),
                                                 paged.ref(), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                 sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks), _ptr(ws),
                                                 ws.numel(), _stream()))
            return out
        if kv_scales is not None:
            _check(lib().ihip_decode_layer_fp8kv(ctypes.byref(self.shape), _tensor(q, "q"), _tensor8(k, "k"),
                                                 _tensor8(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                 sm_scale, kv_scales[0], kv_scales[1], _ptr(out), _ptr(lse),
                                                 _ptr(out_blocks), _ptr(ws), ws.numel(), _stream()))
            return out
        if pooling is not None:
            _check(lib().ihip_decode_layer_pooled(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                                  _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                  pooling, sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks),
                                                  _ptr(ws), ws.numel(), _stream()))
            return out
        if rope is not None:
            _check(lib().ihip_decode_layer_rope(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                                _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                sm_scale, rope.ref(), _ptr(out), _ptr(lse), _ptr(out_blocks),
                                                _ptr(ws), ws.numel(), _stream()))
            return out
        _check(lib().ihip_decode_layer(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                       _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                       sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks), _ptr(ws),
                                       ws.numel(), _stream()))
        return out

    def decode_layer_static(self, q, k, v, chunk_sizes, keeps, out, out_blocks=None, lse=None, sm_scale=None):
        """ihip_decode_layer_static: the decode layer on the library's own static scratch.  `out`
        (bf16 [B,Hq,1,d]) and the optional outputs are the caller's: nothing is allocated here."""
        sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
        _check(lib().ihip_decode_layer_static(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                              _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                              sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks), _stream()))
        return out

    def mask_state(self, keeps) -> torch.Tensor:
        """Device buffer for every stage's cached kept starts (ihip_decode_layer_masked)."""
        n = lib().ihip_mask_state_elems(ctypes.byref(self.shape), len(keeps), _i32(keeps))
        return torch.full((n,), -1, dtype=torch.int32, device=self.device)

    def decode_layer_masked(self, q, k, v, chunk_sizes, keeps, first_stage, stage_starts, sm_scale=None,
                            ws=None, out=None, lse=None):
        """Decode layer that recomputes stages first_stage.. and reuses the cached earlier ones."""
        sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
        if out is None:
            out = torch.empty((self.B, self.Hq, 1, self.d), dtype=torch.bfloat16, device=self.device)
        if ws is None:
            ws = self.workspace(OP_DECODE_LAYER, chunk_sizes, keeps)
        _check(lib().ihip_decode_layer_masked(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                              _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                              first_stage, _ptr(stage_starts), sm_scale, _ptr(out), _ptr(lse),
                                              _ptr(ws), ws.numel(), _stream()))
        return out

    def prefill_layer(self, q, k, v, chunk_sizes, keeps, sm_scale=None, ws=None, out=None,
                      out_blocks=None, lse=None, pooling: Optional[int] = None, rope: Optional["Rope"] = None,
                      paged: Optional["PagedKV"] = None, kv_scales: Optional[Sequence[float]] = None,
                      stage_b_q: Optional[Sequence[int]] = None):
        """Pruning stages + block-sparse prefill attention in one enqueue -> bf16 [B,Hq,Tq,d].
        paged: k and v are ignored.  kv_scales: K and V (or the pools) hold E4M3 bytes.  One variant
        alone goes to its own entry point; paged K/V, E4M3 K/V and combinations to ihip_prefill_layer_ex."""
        sm_scale = 1.0 / math.sqrt(self.d) if sm_scale is None else sm_scale
        if out is None:
            out = torch.empty((self.B, self.Hq, self.Tq, self.d), dtype=torch.bfloat16, device=self.device)
        if ws is None:
            ws = self.workspace(OP_PREFILL_LAYER, chunk_sizes, keeps)
        if paged is not None or kv_scales is not None or stage_b_q is not None or \
                (pooling is not None and rope is not None):
            opt = PrefillOptions()
            sbq = _i32(stage_b_q) if stage_b_q is not None else None      # kept alive until the call returns
            opt.stage_b_q = ctypes.cast(sbq, vp) if sbq is not None else None
            if kv_scales is not None:
                opt.kv_fp8, opt.k_scale, opt.v_scale = 1, kv_scales[0], kv_scales[1]
            conv = _tensor8 if kv_scales is not None else _tensor
            opt.rope = ctypes.cast(rope.ref(), vp) if rope is not None else None
            opt.paged = ctypes.cast(paged.ref(), vp) if paged is not None else None
            opt.pooling = POOL_KV_HEAD if pooling is None else pooling
            tk, tv = (conv(paged.k_pool, "k_pool"), conv(paged.v_pool, "v_pool")) if paged is not None \
                else (conv(k, "k"), conv(v, "v"))
            _check(lib().ihip_prefill_layer_ex(ctypes.byref(self.shape), _tensor(q, "q"), tk, tv, len(chunk_sizes),
                                               _i32(chunk_sizes), _i32(keeps), sm_scale, ctypes.byref(opt),
                                               _ptr(out), _ptr(lse), _ptr(out_blocks), _ptr(ws), ws.numel(),
                                               _stream()))
            return out
        if pooling is not None:
            _check(lib().ihip_prefill_layer_pooled(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                                   _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                   pooling, sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks),
                                                   _ptr(ws), ws.numel(), _stream()))
            return out
        if rope is not None:
            _check(lib().ihip_prefill_layer_rope(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                                 _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                                 sm_scale, rope.ref(), _ptr(out), _ptr(lse), _ptr(out_blocks),
                                                 _ptr(ws), ws.numel(), _stream()))
            return out
        _check(lib().ihip_prefill_layer(ctypes.byref(self.shape), _tensor(q, "q"), _tensor(k, "k"),
                                        _tensor(v, "v"), len(chunk_sizes), _i32(chunk_sizes), _i32(keeps),
                                        sm_scale, _ptr(out), _ptr(lse), _ptr(out_blocks), _ptr(ws),
                                        ws.numel(), _stream()))
        return out


def refresh_due(step: int, refresh: Sequence[int]):
    """ihip_refresh_due: (first due stage or len(refresh), [stage i due at this step])."""
    due = (c_i32 * len(refresh))()
    first = lib().ihip_refresh_due(len(refresh), _i32(refresh), step, due)
    if first < 0:
        _check(first)
    return first, [bool(x) for x in due]


def first_stage_due(step: int, refresh: Sequence[int]) -> int:
    """The first stage Alg. 4's counters make due at this step (ihip_refresh_due); len(refresh) if none."""
    return refresh_due(step, refresh)[0]


class HostKVCache:
    """Host-resident K/V (pinned memory) with the on-GPU hot-block cache.

    host_k / host_v: pinned CPU tensors [B,Hkv,T,d] (torch's pin_memory=True),
    bf16 or -- for an FP8 KV cache -- uint8 holding E4M3 bytes; the banks and
    tables are carved out of one device buffer allocated here through PyTorch
    and kept alive with the handle.

    block_table (device int32 [B, pages per sequence]) + seq_tokens: host_k / host_v are page pools
    [n_pages,Hkv,page_tokens,d] read through the table (ihip_cache_create_paged); seq_tokens is the
    token capacity per sequence."""

    def __init__(self, host_k: torch.Tensor, host_v: torch.Tensor, block_tokens: int, mask_slots: int,
                 sa_slots: int, device="cuda:0", block_table: Optional[torch.Tensor] = None, seq_tokens: int = 0):
        self.fp8 = host_k.dtype in (torch.uint8, torch.float8_e4m3fn)
        for t, name in ((host_k, "host_k"), (host_v, "host_v")):
            if t.dtype != host_k.dtype or (not self.fp8 and t.dtype != torch.bfloat16) or t.dim() != 4 \
                    or t.stride(3) != 1 or t.is_cuda or not t.is_pinned():
                raise IhipError(f"{name}: need a pinned 4-d bf16 (or E4M3 byte) CPU tensor with contiguous last dim")
        self.host_k, self.host_v = host_k, host_v
        B, Hkv, T, _ = host_k.shape
        self.block_table = block_table
        if block_table is not None:
            if block_table.dtype != torch.int32 or not block_table.is_cuda or block_table.dim() != 2 \
                    or block_table.stride(1) != 1:
                raise IhipError("block_table: need a device int32 [B, pages per sequence] tensor")
            B, T = block_table.shape[0], seq_tokens
        size_fn = lib().ihip_cache_device_bytes_fp8 if self.fp8 else lib().ihip_cache_device_bytes
        make_fn = lib().ihip_cache_create_fp8 if self.fp8 else lib().ihip_cache_create
        need = size_fn(B, Hkv, T, block_tokens, mask_slots, sa_slots)
        if need == 0:
            raise IhipError("ihip_cache_device_bytes: bad sizes")
        self.dev_mem = torch.empty(need, dtype=torch.uint8, device=device)
        self.handle = vp()
        hk = Tensor(host_k.data_ptr(), host_k.stride(0), host_k.stride(1), host_k.stride(2))
        hv = Tensor(host_v.data_ptr(), host_v.stride(0), host_v.stride(1), host_v.stride(2))
        with torch.cuda.device(self.dev_mem.device):
            if block_table is not None:
                self._pages = PagedStruct(block_table.data_ptr(), block_table.stride(0), host_k.shape[2])
                _check(lib().ihip_cache_create_paged(ctypes.byref(self.handle), self.dev_mem.data_ptr(), need, hk, hv,
                                                     ctypes.byref(self._pages), 1 if self.fp8 else 0, B, Hkv, T,
                                                     block_tokens, mask_slots, sa_slots, _stream()))
            else:
                _check(make_fn(ctypes.byref(self.handle), self.dev_mem.data_ptr(), need, hk, hv,
                               B, Hkv, T, block_tokens, mask_slots, sa_slots, _stream()))
        self.block_tokens, self.mask_slots, self.sa_slots = block_tokens, mask_slots, sa_slots
        self.n_blocks_total = B * Hkv * ((T + block_tokens - 1) // block_tokens)

    def close(self):
        if self.handle:
            torch.cuda.synchronize()
            lib().ihip_cache_destroy(self.handle)
            self.handle = vp()

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def reset(self):
        _check(lib().ihip_cache_reset(self.handle, _stream()))

    def update(self):
        _check(lib().ihip_cache_update(self.handle, _stream()))

    def stats(self) -> dict:
        s = (ctypes.c_uint64 * 8)()
        _check(lib().ihip_cache_stats(self.handle, s))
        keys = ("hits", "misses", "last_misses", "last_touched")
        return {"mask": dict(zip(keys, s[0:4])), "sa": dict(zip(keys, s[4:8]))}

    def tables(self, bank: int):
        """(page_table [n_blocks_total], slot_block [n_slots]) as int32 numpy arrays."""
        import numpy as np
        pt = np.empty(self.n_blocks_total, np.int32)
        sb = np.empty(self.mask_slots if bank == 0 else self.sa_slots, np.int32)
        _check(lib().ihip_cache_read_tables(self.handle, bank, pt.ctypes.data_as(vp), sb.ctypes.data_as(vp)))
        return pt, sb


def prune_stage_cached(layer: "Layer", q, cache: HostKVCache, chunk: int, parent_starts=None, parent_chunk: int = 0,
                       want_rep: bool = False, rope: Optional["Rope"] = None, k_scale: float = 1.0):
    """ihip_prune_stage_cached -> scores fp32 [P, slots], rep int32 [B,Hq,1,slots] or None."""
    if parent_starts is None:
        n_parent, slots = 0, layer.stage1_slots(chunk)
    else:
        n_parent = parent_starts.shape[-1]
        slots = n_parent * (parent_chunk // chunk)
    scores = torch.empty((layer.P, slots), dtype=torch.float32, device=layer.device)
    rep = torch.empty((layer.B, layer.Hq, 1, slots), dtype=torch.int32, device=layer.device) if want_rep else None
    _check(lib().ihip_prune_stage_cached(ctypes.byref(layer.shape), _tensor(q, "q"), cache.handle, _ptr(parent_starts),
                                         n_parent, parent_chunk, chunk, slots,
                                         rope.ref() if rope is not None else None, k_scale, _ptr(scores), _ptr(rep),
                                         _stream()))
    return scores, rep


def sparse_attn_decode_cached(layer: "Layer", q, cache: HostKVCache, block_starts, block: int, sm_scale=None,
                              want_lse: bool = False, rope: Optional["Rope"] = None,
                              kv_scales: Sequence[float] = (1.0, 1.0)):
    """ihip_sparse_attn_decode_cached -> (out bf16 [B,Hq,1,d], lse or None)."""
    n_blocks = block_starts.shape[-1]
    sm_scale = 1.0 / math.sqrt(layer.d) if sm_scale is None else sm_scale
    out = torch.empty((layer.B, layer.Hq, 1, layer.d), dtype=torch.bfloat16, device=layer.device)
    lse = torch.empty((layer.B, layer.Hq, 1), dtype=torch.float32, device=layer.device) if want_lse else None
    ws = layer.workspace(OP_ATTN_DECODE, [block], [max(n_blocks, 1)])
    _check(lib().ihip_sparse_attn_decode_cached(ctypes.byref(layer.shape), _tensor(q, "q"), cache.handle,
                                                _ptr(block_starts), n_blocks, block, sm_scale,
                                                rope.ref() if rope is not None else None, kv_scales[0], kv_scales[1],
                                                _ptr(out), _ptr(lse), _ptr(ws), ws.numel(), _stream()))
    return out, lse


def decode_layer_cached(layer: "Layer", q, cache: HostKVCache, chunk_sizes, keeps, sm_scale=None, ws=None,
                        out=None, out_blocks=None, lse=None):
    """ihip_decode_layer_cached: the decode layer reading K/V through the host tier."""
    sm_scale = 1.0 / math.sqrt(layer.d) if sm_scale is None else sm_scale
    if out is None:
        out = torch.empty((layer.B, layer.Hq, 1, layer.d), dtype=torch.bfloat16, device=layer.device)
    if ws is None:
        ws = layer.workspace(OP_DECODE_LAYER, chunk_sizes, keeps)
    _check(lib().ihip_decode_layer_cached(ctypes.byref(layer.shape), _tensor(q, "q"), cache.handle,
                                          len(chunk_sizes), _i32(chunk_sizes), _i32(keeps), sm_scale, _ptr(out),
                                          _ptr(lse), _ptr(out_blocks), _ptr(ws), ws.numel(), _stream()))
    return out
