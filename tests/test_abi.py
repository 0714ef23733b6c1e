"""The C-ABI library loads and exports every symbol the header declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", h)).read() for h in ("ihip.h", "ihip_measure.h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ihip_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def built_lib():
    import paper_2502_08910_amd as pkg
    if not os.path.exists(pkg.LIB_PATH):
        from paper_2502_08910_amd.build import build
        build(verbose=False)
    return pkg


def test_header_symbols_are_exported(built_lib):
    syms = declared_symbols()
    assert {"ihip_prune_stage", "ihip_select_blocks", "ihip_sparse_attn_decode",
            "ihip_sparse_attn_prefill"} <= set(syms)
    L = ctypes.CDLL(built_lib.LIB_PATH)
    for s in syms:
        assert hasattr(L, s), s
    assert set(built_lib.binding.EXPORTS) == set(syms)


def test_version_and_error_text(built_lib):
    L = built_lib.lib()
    assert L.ihip_version() >= 100
    assert isinstance(L.ihip_last_error(), bytes)


def test_argument_checks_need_no_gpu(built_lib):
    # every check happens before anything is enqueued
    from paper_2502_08910_amd.binding import Shape, Tensor
    L = built_lib.lib()
    s = Shape(1, 32, 8, 64, 1, 1, 1, 100, 4, 4)             # d = 64: unsupported
    t = Tensor(256, 0, 0, 128)
    rc = L.ihip_prune_stage(ctypes.byref(s), t, t, None, 0, 0, 16, 10, 256, None, None)
    assert rc == -4 and b"128" in L.ihip_last_error()
    s = Shape(1, 32, 8, 128, 1, 1, 1, 100, 4, 4)
    assert L.ihip_prune_stage(ctypes.byref(s), t, t, None, 0, 0, 24, 10, 256, None, None) == -1   # chunk not 2^n
    assert L.ihip_prune_stage(ctypes.byref(s), t, t, None, 0, 0, 16, 2, 256, None, None) == -1    # too few slots
    assert L.ihip_stage1_slots(ctypes.byref(s), 16) == 6
    s2 = Shape(1, 32, 8, 128, 1, 1, 1, 100, 4, 0)           # n_stream < b_q
    assert L.ihip_select_blocks(ctypes.byref(s2), 256, 6, None, 0, 0, 16, 2, 256, None) == -1
    rc = L.ihip_sparse_attn_decode(ctypes.byref(s), t, t, t, 256, 4, 4, 1.0, 256, None, 256, 16, None)
    assert rc == -2 and b"workspace" in L.ihip_last_error()
    one = (ctypes.c_int32 * 1)(16)
    assert L.ihip_workspace_bytes(99, ctypes.byref(s), 1, one, one) == 0


def test_static_scratch_limit_needs_no_gpu(built_lib):
    """ihip_decode_layer_static refuses a plan beyond its array before it touches the device."""
    from paper_2502_08910_amd.binding import Shape, Tensor
    L = built_lib.lib()
    s = Shape(64, 32, 8, 128, 1, 1, 1, 1 << 20, 128, 1024, 0)       # batch 64 x 1M keys: ~ 33 MiB of scores
    t = Tensor(256, 0, 0, 128)
    chunks = (ctypes.c_int32 * 2)(256, 16)
    keeps = (ctypes.c_int32 * 2)(256, 256)
    rc = L.ihip_decode_layer_static(ctypes.byref(s), t, t, t, 2, chunks, keeps, 1.0, 256, None, None, None)
    assert rc == -2 and b"static" in L.ihip_last_error()
    need = L.ihip_workspace_bytes(4, ctypes.byref(s), 2, chunks, keeps)
    assert need > (8 << 20)


def test_argument_checks_of_the_variants_need_no_gpu(built_lib):
    """Dynamic RoPE, FP8 K/V, paged K/V and pooled selection: what they refuse, before any launch."""
    from paper_2502_08910_amd.binding import Shape, Tensor, RopeStruct, PagedStruct
    L = built_lib.lib()
    s = Shape(1, 32, 8, 128, 1, 1, 1, 4096, 128, 1024)      # decode, 4096 keys
    t = Tensor(256, 0, 0, 128)
    slots = L.ihip_stage1_slots(ctypes.byref(s), 64)
    # rope: NULL struct, NULL tables, unknown style, table too short for the relative style
    assert L.ihip_prune_stage_rope(ctypes.byref(s), t, t, None, 0, 0, 64, slots, None, 256, None, None) == -1
    r = RopeStruct(None, None, 4096, 1, 1)
    assert L.ihip_prune_stage_rope(ctypes.byref(s), t, t, None, 0, 0, 64, slots, ctypes.byref(r), 256, None, None) == -1
    r = RopeStruct(256, 256, 4096, 7, 1)
    assert L.ihip_prune_stage_rope(ctypes.byref(s), t, t, None, 0, 0, 64, slots, ctypes.byref(r), 256, None, None) == -1
    r = RopeStruct(256, 256, 1025, 1, 1)                     # needs n_stream + 2 = 1026 rows
    assert L.ihip_prune_stage_rope(ctypes.byref(s), t, t, None, 0, 0, 64, slots, ctypes.byref(r), 256, None, None) == -1
    assert b"1026" in L.ihip_last_error()
    # chunked prefill: the chunk-indexed style needs max_chunks + n_stream table rows; the attention
    # checks the table too
    sp = Shape(1, 32, 8, 128, 64, 64, 1, 4096, 128, 1024)
    r = RopeStruct(256, 256, slots + 1024 - 1, 2, 1)
    rc = L.ihip_prune_stage_rope(ctypes.byref(sp), t, t, None, 0, 0, 64, slots, ctypes.byref(r), 256, None, None)
    assert rc == -1
    f = ctypes.c_float
    assert L.ihip_sparse_attn_prefill_rope(ctypes.byref(sp), t, t, t, 256, 16, 16, f(0.1), None, 256, None, None, 0,
                                           None) == -1
    r = RopeStruct(256, 256, 128 + 256 + 1024 - 1, 1, 1)     # needs n_sink + n_blocks*block + n_stream rows
    assert L.ihip_sparse_attn_prefill_rope(ctypes.byref(sp), t, t, t, 256, 16, 16, f(0.1), ctypes.byref(r), 256,
                                           None, None, 0, None) == -1
    assert b"1408" in L.ihip_last_error()
    assert L.ihip_prefill_layer_rope(ctypes.byref(sp), t, t, t, 0, None, None, f(0.1), None, 256, None, None, None,
                                     0, None) == -1
    # fp8: scales must be positive and finite; rows 16-byte aligned in bytes
    assert L.ihip_prune_stage_fp8kv(ctypes.byref(s), t, t, None, 0, 0, 64, slots, f(0.0), 256, None, None) == -1
    assert L.ihip_prune_stage_fp8kv(ctypes.byref(s), t, t, None, 0, 0, 64, slots, f(float("inf")), 256, None, None) == -1
    t8 = Tensor(256, 0, 0, 136)
    assert L.ihip_prune_stage_fp8kv(ctypes.byref(s), t, t8, None, 0, 0, 64, slots, f(1.0), 256, None, None) == -1
    # paged: NULL table, page size not a power of two, table too short
    assert L.ihip_prune_stage_paged(ctypes.byref(s), t, t, None, None, 0, 0, 64, slots, 256, None, None) == -1
    pg = PagedStruct(256, 256, 24)
    assert L.ihip_prune_stage_paged(ctypes.byref(s), t, t, ctypes.byref(pg), None, 0, 0, 64, slots, 256, None, None) == -1
    pg = PagedStruct(256, 100, 16)                           # covers 1600 < 4096 tokens
    assert L.ihip_prune_stage_paged(ctypes.byref(s), t, t, ctypes.byref(pg), None, 0, 0, 64, slots, 256, None, None) == -1
    # the combined entry point: NULL options, bad scales, a stage offset without state, host tier + pages
    from paper_2502_08910_amd.binding import DecodeOptions
    i32 = (ctypes.c_int32 * 1)
    ex = lambda opt: L.ihip_decode_layer_ex(ctypes.byref(s), t, t, t, 1, i32(64), i32(8), f(0.1), opt, 256, None,  # noqa: E731
                                            None, 256, 1 << 30, None)
    assert ex(None) == -1
    o = DecodeOptions(); o.kv_fp8, o.k_scale, o.v_scale = 1, -1.0, 1.0
    assert ex(ctypes.byref(o)) == -1
    o = DecodeOptions(); o.first_stage = 1
    assert ex(ctypes.byref(o)) == -1
    assert b"first_stage" in L.ihip_last_error()
    o = DecodeOptions(); o.pooling = 9
    assert ex(ctypes.byref(o)) == -1
    # the combined prefill entry point: NULL options, bad scales; E4M3 attention alone: bad scales
    from paper_2502_08910_amd.binding import PrefillOptions
    exp = lambda opt: L.ihip_prefill_layer_ex(ctypes.byref(sp), t, t, t, 1, i32(64), i32(8), f(0.1), opt, 256,  # noqa: E731
                                              None, None, 256, 1 << 30, None)
    assert exp(None) == -1
    po = PrefillOptions(); po.kv_fp8, po.k_scale, po.v_scale = 1, 1.0, 0.0
    assert exp(ctypes.byref(po)) == -1
    assert b"scales" in L.ihip_last_error()
    po = PrefillOptions(); po.pooling = 9
    assert exp(ctypes.byref(po)) == -1
    assert L.ihip_sparse_attn_prefill_fp8kv(ctypes.byref(sp), t, t, t, 256, 8, 16, f(0.1), f(-1.0), f(1.0), None,
                                            256, None, None, 0, None) == -1
    # pooling rule
    assert L.ihip_select_blocks_pooled(ctypes.byref(s), 256, slots, None, 0, 0, 64, 8, 5, 256, None) == -1


def test_a_plain_c_client_links_and_runs(built_lib, tmp_path):
    """gcc -std=c99 compiles tests/c_client/client.c against include/ihip.h, links it with the built
    library and runs it: version, slot and workspace arithmetic and an argument check from C."""
    import os
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(built_lib.LIB_PATH)
    exe = str(tmp_path / "client")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-pedantic", "-I", os.path.join(root, "include"),
                           os.path.join(root, "tests", "c_client", "client.c"), "-o", exe,
                           "-L", libdir, "-l:libihip.so", "-Wl,-rpath," + libdir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([exe], check=True, capture_output=True, text=True, timeout=120).stdout.splitlines()
    assert out[0] == "version 100"
    assert out[1] == "stage1_slots 4092"               # ceil((1048576 - 1024 - 128) / 256)
    assert int(out[2].split()[1]) >= 64 * 4092 * 4     # at least the first stage's scores
    assert out[3].startswith("null tensor rc -1: ihip_prune_stage: q.ptr is NULL")
    assert out[4] == "d=64 rc -1"
