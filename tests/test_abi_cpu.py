"""The C-ABI library loads and exports every symbol include/specexit.h declares (no GPU work)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2509_24248_amd", "libspecexit.so")
HEADER = os.path.join(ROOT, "include", "specexit.h")


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(specexit_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_stage_calls():
    names = declared_symbols()
    for n in ("specexit_draft_step", "specexit_verify_attn", "specexit_lmhead_argmax", "specexit_accept_exit"):
        assert n in names


@pytest.mark.skipif(not os.path.exists(LIB), reason="libspecexit.so not built")
def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(LIB)
    for n in declared_symbols():
        assert hasattr(lib, n), n
    lib.specexit_version.restype = ctypes.c_uint32
    assert lib.specexit_version() >= 0x00010000


@pytest.mark.skipif(not os.path.exists(LIB), reason="libspecexit.so not built")
def test_binding_matches_header_and_validates_on_the_host():
    from paper_2509_24248_amd import binding as sx
    assert sorted(sx.EXPORTS) == declared_symbols()
    # struct sizes the binding sends equal what the library was compiled with: a wrong size is rejected
    cfg = sx.exit_cfg()
    cfg.struct_size = 4
    rc = sx.LIB.specexit_accept_exit(ctypes.byref(cfg), 1, 2, *([None] * 6), 0, *([None] * 10), 0, None)
    assert rc == sx.EINVAL and b"ABI size" in sx.LIB.specexit_last_error()
    # argument validation happens before any launch: no GPU is needed to see these errors
    assert sx.specexit_lmhead_argmax_workspace_bytes(sx.BF16, 0, 2560, 151936, 0) == 0
    assert sx.specexit_lmhead_argmax_workspace_bytes(sx.BF16, 7, 2560, 151936, 0) > 0
    rc = sx.LIB.specexit_lmhead_argmax(sx.BF16, 500, 2560, 151936, 0, *([None] * 7), 0, 0, None)
    assert rc == sx.EINVAL and b"outside 1..144" in sx.LIB.specexit_last_error()
    kv = sx.KVView()
    kv.struct_size = ctypes.sizeof(sx.KVView)
    kv.layout, kv.dtype, kv.n_kv_heads, kv.head_dim, kv.k, kv.v, kv.l_max = 0, 1, 8, 96, 256, 256, 128
    assert sx.specexit_verify_attn_workspace_bytes(kv, 1, 7, 32) == 0
    assert "head_dim" in sx.last_error()
    kv.head_dim = 128
    assert sx.specexit_verify_attn_workspace_bytes(kv, 1, 7, 32) > 0
    assert sx.specexit_verify_attn_workspace_bytes(kv, 1, 65, 32) == 0
    assert sx.specexit_verify_attn_workspace_bytes(kv, 1, 7, 30) == 0


@pytest.mark.skipif(not os.path.exists(LIB), reason="libspecexit.so not built")
def test_generic_workspace_query_agrees_with_the_per_call_queries():
    from paper_2509_24248_amd import binding as sx
    kv = sx.KVView()
    kv.struct_size = ctypes.sizeof(sx.KVView)
    kv.layout, kv.dtype, kv.n_kv_heads, kv.head_dim, kv.k, kv.v, kv.l_max = 0, 1, 8, 128, 256, 256, 4200
    desc = sx.model_desc(sx.BF16, 2560, 32, 8, 128, 9728, 151936)
    for B in (1, 5):
        a = sx.specexit_workspace_bytes(sx.OP_DRAFT_STEP, sx.draft_query(desc, kv), B, 1)
        assert a == sx.specexit_draft_step_workspace_bytes(desc, kv, B) > 0
        a = sx.specexit_workspace_bytes(sx.OP_DRAFT_TREE_LEVEL, sx.draft_query(desc, kv, top_b=3), B, 4)
        assert a == sx.specexit_draft_tree_level_workspace_bytes(desc, kv, B, 4, 3) > 0
        a = sx.specexit_workspace_bytes(sx.OP_VERIFY_ATTN, sx.attn_query(kv, 32), B, 7)
        assert a == sx.specexit_verify_attn_workspace_bytes(kv, B, 7, 32) > 0
        a = sx.specexit_workspace_bytes(sx.OP_LMHEAD_ARGMAX, sx.lmhead_query(sx.BF16, 2560, 151936), B, 7)
        assert a == sx.specexit_lmhead_argmax_workspace_bytes(sx.BF16, B * 7, 2560, 151936, 0) > 0
    assert sx.specexit_workspace_bytes(sx.OP_ACCEPT_EXIT, None, 4, 7) == 0
    assert sx.specexit_workspace_bytes(sx.OP_KV_COMPACT, None, 4, 7) == 0
    assert sx.specexit_workspace_bytes(99, None, 4, 7) == 0 and "unknown op" in sx.last_error()
    assert sx.specexit_workspace_bytes(sx.OP_VERIFY_ATTN, None, 4, 7) == 0          # missing descriptor
    q = sx.attn_query(kv, 32)
    q.struct_size = 4
    assert sx.specexit_workspace_bytes(sx.OP_VERIFY_ATTN, q, 4, 7) == 0             # another ABI size
    # shapes one call cannot split are refused on the host
    assert sx.specexit_verify_attn_workspace_bytes(kv, 2000, 7, 32) == 0 and "1024 sequences" in sx.last_error()
    kv.l_max = 4
    assert sx.specexit_verify_attn_workspace_bytes(kv, 1, 7, 32) == 0 and "fewer than the block" in sx.last_error()
