"""Host-side checks of the C ABI that need no GPU: exported symbols, status strings, argument
validation that happens before any kernel launch."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "decoquant.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"\b(dq_[a-z0-9_]+)\s*\(", text)
    return sorted(set(names))


def test_library_exports_every_declared_symbol(dq):
    declared = _declared_functions()
    assert "dq_attn_decode" in declared and "dq_compress_kv" in declared
    assert sorted(declared) == sorted(dq.EXPORTED_SYMBOLS)
    for name in declared:
        assert hasattr(dq.lib, name), name


def test_status_strings_and_version(dq):
    assert dq.version() >= 1
    assert dq.status_string(0) == "ok"
    assert "workspace" in dq.status_string(-2)
    assert "invalid" in dq.status_string(-1)


def test_workspace_queries_validate_the_format(dq):
    good = dq.Format(4, 128, 128, 16, 8, 128).c()
    assert dq.lib.dq_decode_workspace_bytes(C.byref(good), 8, 32, 32, 4096) > 0
    assert dq.lib.dq_compress_workspace_bytes(C.byref(good), 4, 40) == 256 + 4 * 40 * 2 * 128 * 128 * 4
    for bad in [dq.Format(3, 128, 128, 16, 8, 128), dq.Format(4, 128, 128, 16, 4, 128),
                dq.Format(4, 96, 128, 16, 8, 128), dq.Format(4, 128, 128, 16, 8, 100),
                dq.Format(4, 128, 256, 16, 16, 128)]:
        c = bad.c()
        assert dq.lib.dq_decode_workspace_bytes(C.byref(c), 8, 32, 32, 4096) == 0
        assert dq.lib.dq_compress_workspace_bytes(C.byref(c), 4, 40) == 0
    # q_heads must be a multiple of kv_heads
    assert dq.lib.dq_decode_workspace_bytes(C.byref(good), 8, 30, 8, 4096) == 0


def test_entry_points_reject_null_pointers_before_touching_the_gpu(dq):
    good = dq.Format(4, 128, 128, 16, 8, 128).c()
    st = dq.lib.dq_attn_decode(C.byref(good), None, None, 32, None, 4096, 0.0, None, None, None, 0, 0, None)
    assert st == -1
    st = dq.lib.dq_compress_kv(C.byref(good), None, None, None, 128, None, None, None, 0, None)
    assert st == -1
    st = dq.lib.dq_quantize_pack(C.byref(good), None, 128, 0, None, None, None)
    assert st == -1
    assert dq.lib.dq_stream_read(None, 16, None, None) == -1
    assert dq.lib.dq_workspace_init(None, 16, None) == -1
