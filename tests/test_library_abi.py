"""Host-side checks of the C ABI that need no GPU: exported symbols, status strings, argument
validation that happens before any kernel launch."""
import ctypes as C
import os
import re
import subprocess
import sys

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
    assert dq.version() == dq.ABI_VERSION == 6
    assert dq.status_string(0) == "ok"
    assert "workspace" in dq.status_string(-2)
    assert "invalid" in dq.status_string(-1)
    assert "limit" in dq.status_string(-4)


def test_workspace_queries_validate_the_format(dq):
    good = dq.Format(4, 128, 128, 16, 8, 128).c()
    assert dq.lib.dq_decode_workspace_bytes(C.byref(good), 8, 32, 32, 4096) > 0
    # header + fp32 large tensors + one status word per block (padded to 256 bytes)
    assert dq.lib.dq_compress_workspace_bytes(C.byref(good), 4, 40) == 256 + 4 * 40 * 2 * 128 * 128 * 4 + 1280
    for bad in [dq.Format(3, 128, 128, 16, 8, 128), dq.Format(4, 128, 128, 16, 4, 128),
                dq.Format(4, 96, 128, 16, 8, 128), dq.Format(4, 128, 128, 16, 8, 100),
                dq.Format(4, 128, 256, 16, 16, 128), dq.Format(4, 128, 128, 16, 8, 128, 4),
                dq.Format(4, 128, 128, 16, 8, 128, 1, 2), dq.Format(4, 128, 128, 16, 8, 128, 1, 0, 3),
                dq.Format(4, 128, 128, 16, 8, 128, 8, 0, 2), dq.Format(4, 128, 128, 16, 8, 128, 1, 0, 4),
                dq.Format(4, 128, 128, 16, 8, 128, 1, 0, 0)]:
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


def test_decode_rejects_a_small_workspace_and_bad_sizes_before_launching(dq):
    good = dq.Format(4, 128, 128, 16, 8, 128).c()

    class FakeCache(C.Structure):
        _fields_ = [("p", C.c_void_p * 8), ("batch", C.c_int32), ("kv_heads", C.c_int32), ("cap", C.c_int32)]

    fake = FakeCache()
    for i in range(8):
        fake.p[i] = 0x1000          # never dereferenced: the checks below fail first
    fake.batch, fake.kv_heads, fake.cap = 2, 4, 8
    need = dq.lib.dq_decode_workspace_bytes(C.byref(good), 2, 4, 4, 1024)
    ptr = C.c_void_p(0x1000)
    cache_p = C.cast(C.byref(fake), C.POINTER(type(dq.Cache.__init__.__globals__["_CCache"]())))
    # workspace one byte short
    st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, need - 1, 0, None)
    assert st == -2
    # max_seq_len beyond the cache capacity (8 blocks x 128 tokens)
    st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1025, 0.0, ptr, None, ptr, need, 0, None)
    assert st == -1
    # q_heads not a multiple of kv_heads
    st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 6, ptr, 1024, 0.0, ptr, None, ptr, need, 0, None)
    assert st == -1
    # more (sequence, query head) pairs than one launch takes
    fake.batch = (1 << 22) + 1
    big = dq.lib.dq_decode_workspace_bytes(C.byref(good), (1 << 22) + 1, 4, 4, 1024)
    st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, big, 0, None)
    assert st == -1
    fake.batch = 2
    # an fp16 tail of more rows than a call takes
    tail_t = dq.Cache.__init__.__globals__["_CTail"]
    for cap, want in ((1024, -2), (1025, -1), (0, -1)):      # a fitting one gets as far as the workspace check
        tail = tail_t(0x1000, 0x1000, 0x1000, cap)
        st = dq.lib.dq_attn_decode_tail(C.byref(good), cache_p, ptr, 4, ptr, 1024, C.byref(tail), 0.0, ptr, None,
                                        ptr, need - 1 if want == -2 else need, 0, None)
        assert st == want, (cap, st)
    # both force flags
    st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, need, 3, None)
    assert st == -1
    # launch-shape overrides in the flags word: more splits than the library has, a wave count it
    # does not build, an order of units it does not know, a bit that means nothing
    for bad in (dq.decode_flags(splits=65), dq.decode_flags(waves=3), dq.decode_flags(unit_map=6), 1 << 4, 1 << 24):
        st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, need, bad, None)
        assert st == -1, hex(bad)
    for fine in (dq.decode_flags(splits=64, waves=8, unit_map=5), dq.decode_flags(dq.DECODE_FORCE_GENERIC, splits=1, waves=4)):
        st = dq.lib.dq_attn_decode(C.byref(good), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, need - 1, fine, None)
        assert st == -2, hex(fine)     # accepted as far as the workspace check
    # compress: t_new out of range, workspace too small
    cneed = dq.lib.dq_compress_workspace_bytes(C.byref(good), 2, 4)
    st = dq.lib.dq_compress_kv(C.byref(good), cache_p, ptr, ptr, 129, ptr, None, ptr, cneed, None)
    assert st == -1
    st = dq.lib.dq_compress_kv(C.byref(good), cache_p, ptr, ptr, 128, ptr, None, ptr, cneed - 1, None)
    assert st == -2
    # the flagged variant: unknown flag bits, then the same size checks
    for bad in (4, 1 << 12, dq.compress_flags(waves=3), dq.compress_flags(waves=8)):
        st = dq.lib.dq_compress_kv_ex(C.byref(good), cache_p, ptr, ptr, 128, ptr, None, ptr, cneed, bad, None)
        assert st == -1, hex(bad)
    st = dq.lib.dq_compress_kv_ex(C.byref(good), cache_p, ptr, ptr, 128, ptr, None, ptr, cneed - 1,
                                  dq.compress_flags(keep_large=False, waves=2, plain=True), None)
    assert st == -2
    st = dq.lib.dq_compress_kv_ex(C.byref(good), cache_p, ptr, ptr, 128, ptr, None, ptr, cneed - 1, 1, None)
    assert st == -2
    # several blocks per call: the workspace grows with the number of blocks; more blocks than the cache holds
    assert dq.lib.dq_compress_blocks_workspace_bytes(C.byref(good), 2, 4, 128) == cneed
    bneed = dq.lib.dq_compress_blocks_workspace_bytes(C.byref(good), 2, 4, 300)
    assert bneed == 256 + 2 * 4 * 3 * 2 * 128 * 128 * 4 + 256
    st = dq.lib.dq_compress_kv_blocks(C.byref(good), cache_p, ptr, ptr, 300, ptr, None, ptr, bneed - 1, None)
    assert st == -2
    st = dq.lib.dq_compress_kv_blocks(C.byref(good), cache_p, ptr, ptr, 8 * 128 + 1, ptr, None, ptr, 1 << 40, None)
    assert st == -1
    assert dq.lib.dq_compress_blocks_workspace_bytes(C.byref(good), 2, 4, 0) == 0
    # three local tensors need the two extra arrays
    three = dq.Format(4, 128, 128, 16, 8, 128, 8).c()
    fake.p[6] = 0
    fake.p[7] = 0
    need3 = dq.lib.dq_decode_workspace_bytes(C.byref(three), 2, 4, 4, 1024)
    assert need3 == need
    st = dq.lib.dq_attn_decode(C.byref(three), cache_p, ptr, 4, ptr, 1024, 0.0, ptr, None, ptr, need3, 0, None)
    assert st == -1
    st = dq.lib.dq_compress_kv(C.byref(three), cache_p, ptr, ptr, 128, ptr, None, ptr, cneed, None)
    assert st == -1
    # the entry point without a workspace: more (sequence, query head) pairs than its scratch memory holds
    fake.p[6] = 0x1000
    fake.p[7] = 0x1000
    fake.batch = 129
    st = dq.lib.dq_attn_decode_static(C.byref(good), cache_p, ptr, 4, ptr, 1024, None, 0.0, ptr, None, 0, None)
    assert st == -4
    fake.batch = 2
    # the device-side cache policy: a state with a null pointer, row counts outside [1, block_tokens], unknown
    # flags, a workspace one byte short (all before anything is launched)
    class State(C.Structure):
        _fields_ = [("p", C.c_void_p * 4)]

    state = State()
    for i in range(4):
        state.p[i] = 0x1000
    aneed = dq.lib.dq_cache_append_workspace_bytes(C.byref(good), 2, 4)
    assert aneed == cneed + 256                                   # four int32 per sequence, padded to 256 bytes
    append = lambda st_p, n, ws_bytes, flags: dq.lib.dq_cache_append(   # noqa: E731
        C.byref(good), cache_p, st_p, ptr, ptr, n, None, ptr, ws_bytes, flags, None)
    assert append(C.byref(state), 0, aneed, 0) == -1
    assert append(C.byref(state), 129, aneed, 0) == -1
    assert append(C.byref(state), 1, aneed, 2) == -1
    assert append(C.byref(state), 1, aneed - 1, 0) == -2
    assert append(None, 1, aneed, 0) == -1
    state.p[2] = 0
    assert append(C.byref(state), 1, aneed, 0) == -1
    big_block = dq.Format(4, 128, 128, 16, 8, 2048).c()           # a tail of more rows than a decode call takes
    assert dq.lib.dq_cache_append_workspace_bytes(C.byref(big_block), 2, 4) == 0
    # quantize_pack: rows not a multiple of 128
    st = dq.lib.dq_quantize_pack(C.byref(good), ptr, 100, 0, ptr, ptr, None)
    assert st == -1


def test_library_depends_on_the_hip_runtime_only(dq):
    """The boundary is a plain C ABI: the shared library must not pull in torch, Python or any
    other framework (PyTorch only provides device memory and streams on the caller's side)."""
    import subprocess
    from paper_2405_12591_amd import build as B
    out = subprocess.run(["readelf", "-d", B.LIB_PATH], capture_output=True, text=True, check=True).stdout
    needed = [line.split("[")[1].split("]")[0] for line in out.splitlines() if "NEEDED" in line]
    assert any("amdhip64" in n for n in needed), needed
    for n in needed:
        assert not any(bad in n.lower() for bad in ("torch", "python", "c10", "caffe", "rccl", "nccl")), needed


def test_public_header_is_plain_c():
    """include/decoquant.h must be usable from C: no C++ in the declarations."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    header = os.path.join(os.path.dirname(os.path.dirname(os.path.abspath(__file__))), "include", "decoquant.h")
    proc = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c", header],
                          capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr


def test_a_plain_c_program_links_and_calls_the_library(dq, tmp_path):
    """tests/c/abi_host.c: compiled with gcc against include/decoquant.h, linked to the built library,
    run on the host (it makes no call that reaches the GPU)."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no C compiler here")
    from paper_2405_12591_amd import build as B
    lib_dir = os.path.dirname(B.LIB_PATH)
    exe = str(tmp_path / "abi_host")
    proc = subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", os.path.join(ROOT, "tests", "c", "abi_host.c"),
                           "-I", os.path.join(ROOT, "include"), "-L", lib_dir, "-ldecoquant",
                           "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib", "-L/opt/rocm/lib", "-o", exe],
                          capture_output=True, text=True)
    assert proc.returncode == 0, proc.stderr
    run = subprocess.run([exe], capture_output=True, text=True)
    assert run.returncode == 0 and "abi ok" in run.stdout, run.stdout + run.stderr


def test_a_missing_library_is_an_error_not_a_fall_back(tmp_path):
    """With the library path pointing at nothing the package raises as soon as it is imported: there is no other path."""
    code = ("try:\n"
            "    import paper_2405_12591_amd as dq\n"
            "    dq.decode_mfma_supported(dq.Format(4, 128, 128, 16, 8, 128), 1, 1)\n"
            "except Exception as e:\n"
            "    print(type(e).__name__, e)\n"
            "    raise SystemExit(7)\n")
    env = dict(os.environ, DQ_LIBRARY_PATH=str(tmp_path / "nothing_here.so"))
    r = subprocess.run([sys.executable, "-c", code], cwd=ROOT, env=env, capture_output=True, text=True, timeout=300)
    assert r.returncode == 7, (r.stdout, r.stderr)
    assert r.stdout.startswith("DQError") and "missing" in r.stdout


def test_the_package_does_not_know_the_oracle():
    """The product path and the oracle share no code: no source file of the package names the oracle's module."""
    pkg = os.path.join(ROOT, "paper_2405_12591_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip", ".c", ".cpp")):
                text = open(os.path.join(dirpath, f), encoding="utf-8").read()
                assert "oracle" not in text.lower(), os.path.join(dirpath, f)
    text = open(os.path.join(ROOT, "oracle", "decoquant_oracle.py"), encoding="utf-8").read()
    assert "paper_2405_12591_amd" not in text and "ctypes" not in text
