"""CPU oracle of InfiniteHiP's pruning + block-sparse attention path.

TEST INFRASTRUCTURE ONLY: imported by tests, by the smoke check and by the
benchmark's cpu_baseline leg.  It shares no code with the HIP library and the
product package never imports it.

`build()` compiles ihip_oracle.c with gcc; `lib()` loads the result.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ihip_oracle.c")
_SO = os.path.join(_HERE, "libihip_oracle.so")
_lib = None


def build(force: bool = True) -> str:
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-std=c99", "-ffp-contract=off", "-shared", "-fPIC",
                               "-o", _SO, _SRC, "-lm"])
    return _SO


class Rope(ctypes.Structure):
    _fields_ = [("cos", ctypes.c_void_p), ("sin", ctypes.c_void_p), ("n_pos", ctypes.c_int32)]


class Tensors(ctypes.Structure):
    _fields_ = [("Q", ctypes.c_void_p), ("K", ctypes.c_void_p), ("V", ctypes.c_void_p),
                ("B", ctypes.c_int32), ("Hq", ctypes.c_int32), ("Hkv", ctypes.c_int32),
                ("d", ctypes.c_int32), ("Tq", ctypes.c_int32), ("T_alloc", ctypes.c_int64),
                ("kv_fp8", ctypes.c_int32), ("k_scale", ctypes.c_float), ("v_scale", ctypes.c_float)]


def lib():
    global _lib
    if _lib is None:
        build(force=False)
        L = ctypes.CDLL(_SO)
        P = ctypes.POINTER
        c_i32, c_i64, c_f, c_d, vp = (ctypes.c_int32, ctypes.c_int64, ctypes.c_float,
                                      ctypes.c_double, ctypes.c_void_p)
        L.orc_score.restype = c_f
        L.orc_score.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64]
        L.orc_select_rep.restype = None
        L.orc_select_rep.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, c_i32, c_i32,
                                     c_i32, P(c_i64), P(c_f), vp]
        L.orc_prune_stage.restype = None
        L.orc_prune_stage.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i32, vp, vp,
                                      c_i32, c_i32, vp, vp, vp]
        L.orc_topk.restype = c_i32
        L.orc_topk.argtypes = [c_i32, vp, c_i32, vp]
        L.orc_sparse_attention.restype = None
        L.orc_sparse_attention.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, c_i64,
                                           c_i64, c_i32, vp, vp, c_d, vp, vp]
        L.orc_e4m3_to_f32.restype = c_f
        L.orc_e4m3_to_f32.argtypes = [ctypes.c_uint8]
        L.orc_score_rope.restype = c_f
        L.orc_score_rope.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, P(Rope), vp, c_i64]
        L.orc_select_rep_rope.restype = None
        L.orc_select_rep_rope.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, c_i32, c_i32,
                                          P(Rope), c_i32, vp, c_i64, P(c_i64), vp]
        L.orc_prune_stage_rope.restype = None
        L.orc_prune_stage_rope.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, c_i32, vp, vp,
                                           c_i32, P(Rope), c_i32, c_i64, vp, vp, vp]
        L.orc_sparse_attention_rope.restype = None
        L.orc_sparse_attention_rope.argtypes = [P(Tensors), c_i32, c_i32, c_i64, c_i32, c_i64, c_i64,
                                                c_i64, c_i32, vp, vp, c_d, P(Rope), vp, vp]
        _lib = L
    return _lib


from .pipeline import Oracle, RopeSpec, StageResult, ProblemResult  # noqa: E402,F401
from .lru import LruBank  # noqa: E402,F401
