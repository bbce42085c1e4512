"""The C-ABI library loads, exports every symbol include/quantspec.h declares, and rejects bad
arguments before touching the GPU (so these checks run on a host without one)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2502_10424_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build()
    return binding


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "quantspec.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(qs_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported(B):
    lib = B.lib()
    declared = _declared_symbols()
    assert set(declared) == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert B.qs_version() >= 100
    assert B.qs_strerror(0) == "ok" and "NULL" in B.qs_strerror(B.QS_ERR_NULL)
    assert "unknown" in B.qs_strerror(-99)


def test_planner_settings_travel_in_the_descriptor(B):
    """compute_units and flags are validated like any other field, and the workspace size follows from the
    descriptor alone (the library keeps no settings of its own)."""
    w_default = B.qs_workspace_bytes(_fake_cache(B), 1)
    w_small = B.qs_workspace_bytes(_fake_cache(B, compute_units=1), 1)
    assert 0 < w_small < w_default                          # fewer compute units: fewer chunks per unit
    # the workspace covers either way of dealing the groups out
    assert B.qs_workspace_bytes(_fake_cache(B, compute_units=1, flags=B.QS_FLAG_FIXED_RANGES), 1) == w_small
    assert B.qs_workspace_bytes(_fake_cache(B), 1) == w_default
    assert B.qs_workspace_bytes(_fake_cache(B, compute_units=-1), 1) == 0
    assert B.qs_workspace_bytes(_fake_cache(B, flags=2), 1) == 0
    lib = B.lib()
    for bad in (dict(compute_units=-1), dict(compute_units=1 << 20), dict(flags=0x10)):
        c = _fake_cache(B, **bad)
        assert lib.qs_quantize_flush(ctypes.byref(c), 128, None) == B.QS_ERR_RANGE


def test_static_scratch_entry_validates_before_touching_the_gpu(B):
    lib = B.lib()
    c = _fake_cache(B)
    q, out = 0x50000, 0x60000
    assert lib.qs_attn_static(ctypes.byref(c), q, 1, 2, out, 0.1, None, None) == B.QS_ERR_RANGE        # verify flag
    assert lib.qs_attn_static(ctypes.byref(c), q, 2, 0, out, 0.1, None, None) == B.QS_ERR_UNSUPPORTED  # draft: one query
    assert lib.qs_attn_static(ctypes.byref(c), None, 1, 0, out, 0.1, None, None) == B.QS_ERR_NULL
    assert lib.qs_attn_static(ctypes.byref(c), q, 17, 1, out, 0.1, None, None) == B.QS_ERR_UNSUPPORTED
    big = _fake_cache(B, batch=256, n_q_heads=64, n_kv_heads=8)
    nq, nb = np.full(256, 512, np.int32), np.full(256, 256, np.int32)
    big.n_quant = nq.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    big.n_buf = nb.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    assert B.qs_workspace_bytes(big, 16) > B.QS_STATIC_WS_BYTES
    assert lib.qs_attn_static(ctypes.byref(big), q, 16, 1, out, 0.1, None, None) == B.QS_ERR_WORKSPACE


def test_w4_validation_without_gpu(B):
    """The 4-bit weight layer's calls check sizes, pointers and alignment before anything is enqueued."""
    lib = B.lib()
    assert B.qs_w4_bytes(4096, 4096) == 256 * 32 * 1088
    for n_out, n_in in ((0, 128), (16, 0), (24, 128), (16, 64), (16, 32768 + 128), (-16, 128)):
        assert B.qs_w4_bytes(n_out, n_in) == 0
    good = B.qs_w4(32, 256, 0x10000)
    x, y = 0x20000, 0x30000
    assert lib.qs_w4_linear(ctypes.byref(good), x, 0, y, None) == B.QS_ERR_SHAPE
    assert lib.qs_w4_linear(ctypes.byref(good), x, 17, y, None) == B.QS_ERR_SHAPE
    assert lib.qs_w4_linear(ctypes.byref(good), None, 1, y, None) == B.QS_ERR_NULL
    assert lib.qs_w4_linear(ctypes.byref(good), x, 1, None, None) == B.QS_ERR_NULL
    assert lib.qs_w4_linear(ctypes.byref(good), x + 2, 1, y, None) == B.QS_ERR_ALIGN
    assert lib.qs_w4_quantize(ctypes.byref(good), None, None) == B.QS_ERR_NULL
    assert lib.qs_w4_quantize(ctypes.byref(good), x + 8, None) == B.QS_ERR_ALIGN
    assert lib.qs_w4_linear(None, x, 1, y, None) == B.QS_ERR_NULL
    for bad in (B.qs_w4(24, 256, 0x10000), B.qs_w4(32, 192, 0x10000), B.qs_w4(32, 65536, 0x10000)):
        assert lib.qs_w4_linear(ctypes.byref(bad), x, 1, y, None) == B.QS_ERR_SHAPE
        assert lib.qs_w4_export(ctypes.byref(bad), None, None, None, None) == B.QS_ERR_SHAPE
    assert lib.qs_w4_quantize(ctypes.byref(B.qs_w4(32, 256, None)), x, None) == B.QS_ERR_NULL
    assert lib.qs_w4_quantize(ctypes.byref(B.qs_w4(32, 256, 0x10004)), x, None) == B.QS_ERR_ALIGN


def _fake_cache(B, **over):
    """A descriptor with plausible, never-dereferenced device addresses (validation only)."""
    c = B.qs_cache()
    c.batch, c.n_q_heads, c.n_kv_heads, c.head_dim, c.group, c.q_cap, c.buf_cap = 2, 8, 2, 128, 128, 1024, 264
    for i, name in enumerate(("upper", "lower",
                              "k_buf", "v_buf")):
        setattr(c, name, 0x10000 * (i + 1))
    nq = np.array([512, 1024], np.int32)
    nb = np.array([256, 130], np.int32)
    c.n_quant = nq.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    c.n_buf = nb.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))
    c._keep = (nq, nb)
    for k, v in over.items():
        setattr(c, k, v)
    return c


def test_workspace_bytes(B):
    c = _fake_cache(B)
    w1, w5 = B.qs_workspace_bytes(c, 1), B.qs_workspace_bytes(c, 5)
    assert w1 > 0 and w5 == 5 * w1 and w1 % (130 * 4) == 0
    assert B.qs_workspace_bytes(_fake_cache(B, head_dim=64), 1) == 0          # group 128 does not divide 64
    assert B.qs_workspace_bytes(_fake_cache(B, head_dim=96, group=32), 1) == 0
    w64 = B.qs_workspace_bytes(_fake_cache(B, head_dim=64, group=32), 1)
    assert w64 > 0 and w64 % (66 * 4) == 0
    assert B.qs_workspace_bytes(_fake_cache(B, head_dim=256, group=64), 1) % (258 * 4) == 0
    assert B.qs_workspace_bytes(c, 0) == 0 and B.qs_workspace_bytes(c, 17) == 0


def test_validation_errors_without_gpu(B):
    lib = B.lib()
    ws = 1 << 30

    def draft(c, q=0x200000, out=0x300000, wsp=0x400000, wsb=ws):
        return lib.qs_attn_draft(ctypes.byref(c), q, out, 0.1, wsp, wsb, None, None)

    def verify(c, nq):
        return lib.qs_attn_verify(ctypes.byref(c), 0x200000, nq, 0x300000, 0.1, 0x400000, ws, None, None)

    assert lib.qs_attn_draft(None, 0x200000, 0x300000, 0.1, 0x400000, ws, None, None) == B.QS_ERR_NULL
    assert draft(_fake_cache(B, upper=None)) == B.QS_ERR_NULL
    assert draft(_fake_cache(B, q_cap=0, upper=None, lower=None)) == B.QS_ERR_RANGE   # planes optional, but n_quant > 0
    assert draft(_fake_cache(B), q=None) == B.QS_ERR_NULL
    assert draft(_fake_cache(B, n_q_heads=7)) == B.QS_ERR_SHAPE
    assert draft(_fake_cache(B, q_cap=1000)) == B.QS_ERR_SHAPE
    assert draft(_fake_cache(B, head_dim=64)) == B.QS_ERR_UNSUPPORTED          # whole groups per token row only
    assert draft(_fake_cache(B, head_dim=96, group=32)) == B.QS_ERR_UNSUPPORTED
    assert draft(_fake_cache(B, group=16)) == B.QS_ERR_UNSUPPORTED
    assert draft(_fake_cache(B, head_dim=256, group=256)) == B.QS_ERR_UNSUPPORTED
    c = _fake_cache(B, head_dim=64, group=32); c._keep[0][0] = 96            # a multiple of the group of 32
    assert draft(c, wsb=0) == B.QS_ERR_WORKSPACE                                 # i.e. everything else was accepted
    c = _fake_cache(B, head_dim=64, group=64); c._keep[0][0] = 96
    assert draft(c) == B.QS_ERR_RANGE
    assert draft(_fake_cache(B, batch=257)) == B.QS_ERR_UNSUPPORTED
    assert draft(_fake_cache(B, lower=0x10008)) == B.QS_ERR_ALIGN
    assert draft(_fake_cache(B), q=0x200004) == B.QS_ERR_ALIGN
    assert draft(_fake_cache(B), wsp=None) == B.QS_ERR_WORKSPACE
    assert draft(_fake_cache(B), wsb=16) == B.QS_ERR_WORKSPACE
    for bad in (0.0, -0.1, float("inf"), float("nan")):
        assert lib.qs_attn_draft(ctypes.byref(_fake_cache(B)), 0x200000, 0x300000, bad, 0x400000, ws, None, None) == B.QS_ERR_RANGE
    assert verify(_fake_cache(B), 0) == B.QS_ERR_UNSUPPORTED
    assert verify(_fake_cache(B), 17) == B.QS_ERR_UNSUPPORTED
    c = _fake_cache(B); c._keep[0][0] = 100            # n_quant not a multiple of 128
    assert draft(c) == B.QS_ERR_RANGE
    c = _fake_cache(B); c._keep[0][1] = 2048           # n_quant > q_cap
    assert draft(c) == B.QS_ERR_RANGE
    c = _fake_cache(B); c._keep[1][0] = 300            # n_buf > buf_cap
    assert draft(c) == B.QS_ERR_RANGE
    c = _fake_cache(B); c._keep[1][1] = 3              # fewer buffer tokens than queries
    assert verify(c, 5) == B.QS_ERR_RANGE
    # flush: multiple of 128, within the buffer, within capacity
    fl = lambda c, n: lib.qs_quantize_flush(ctypes.byref(c), n, None)
    assert fl(_fake_cache(B), 100) == B.QS_ERR_RANGE
    assert fl(_fake_cache(B), 256) == B.QS_ERR_RANGE       # sequence 1 has only 130 buffered tokens
    c = _fake_cache(B); c._keep[1][1] = 256
    assert fl(c, 128) == B.QS_ERR_RANGE                    # sequence 1 is already at q_cap
    assert fl(_fake_cache(B), 0) == B.QS_OK
    pf = lambda c, n, stride: lib.qs_quantize_prefill(ctypes.byref(c), 0x500000, 0x600000, stride, n, None)
    assert pf(_fake_cache(B), 128, 64) == B.QS_ERR_RANGE
    assert pf(_fake_cache(B), 1024, 1024) == B.QS_ERR_RANGE
    # append: sources present and aligned, room for n_new rows in every sequence's buffer
    ap = lambda c, n, k=0x500000, v=0x600000: lib.qs_append(ctypes.byref(c), k, v, n, None)
    assert ap(_fake_cache(B), 1, k=None) == B.QS_ERR_NULL
    assert ap(_fake_cache(B), 1, v=0x600008) == B.QS_ERR_ALIGN
    assert ap(_fake_cache(B), -1) == B.QS_ERR_RANGE
    assert ap(_fake_cache(B), 9) == B.QS_ERR_RANGE           # sequence 0 holds 256 of 264 rows
    assert ap(_fake_cache(B), 0) == B.QS_OK
    assert lib.qs_export_codes(ctypes.byref(_fake_cache(B)), 2, 0, 128, None, None, None, None, None, None, None, None, None) == B.QS_ERR_RANGE
    assert lib.qs_export_codes(ctypes.byref(_fake_cache(B)), 0, 0, 100, None, None, None, None, None, None, None, None, None) == B.QS_ERR_RANGE


def test_header_is_plain_c_and_library_works_without_python(B, tmp_path):
    """include/quantspec.h compiles as C99 and a C program drives the library through dlopen."""
    import shutil
    import subprocess
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    exe = str(tmp_path / "abi_check")
    src = os.path.join(ROOT, "tests", "c_abi", "abi_check.c")
    subprocess.run([cc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
                    src, "-o", exe, "-ldl"], check=True)
    B.lib()
    out = subprocess.run([exe, B.LIB_PATH], check=True, capture_output=True, text=True)
    assert out.stdout.strip() == "ok"


def test_validation_paths_under_sanitizers(B, tmp_path):
    """The host side of the API layer (argument validation, planning, sizing) built with AddressSanitizer
    and UndefinedBehaviorSanitizer - host code only, the device code objects are the ordinary ones - and
    driven by the same C program."""
    import shutil
    import subprocess
    from paper_2502_10424_amd import build
    hipcc = build.hipcc()
    clang = os.path.join(os.path.dirname(os.path.realpath(hipcc)), "..", "lib", "llvm", "bin", "clang")
    if not os.path.exists(clang):
        clang = shutil.which("amdclang") or shutil.which("clang")
    if clang is None:
        pytest.skip("no clang for the sanitizer runtime")
    objs = [os.path.join(build.CSRC, n) for n in ("qs_attn.o", "qs_flush.o", "qs_w4.o")]
    if not all(os.path.exists(o) for o in objs):
        build.build()
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-sanitize-recover=undefined"]
    host_san = [x for f in san for x in ("-Xarch_host", f)]
    api_o, lib, exe = str(tmp_path / "qs_api_san.o"), str(tmp_path / "libquantspec_san.so"), str(tmp_path / "abi_check_san")
    subprocess.run([hipcc, *build.COMMON, "-O1", "-g", *host_san, "-c", os.path.join(build.CSRC, "qs_api.hip"), "-o", api_o],
                   check=True, capture_output=True)
    subprocess.run([hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-fsanitize=address", "-fsanitize=undefined",
                    "-shared-libsan", "-o", lib, api_o, *objs], check=True, capture_output=True)
    subprocess.run([clang, "-std=c99", "-g", *san, "-shared-libsan", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "c_abi", "abi_check.c"), "-o", exe, "-ldl"], check=True, capture_output=True)
    rt = subprocess.run([clang, "-print-file-name=libclang_rt.asan-x86_64.so"], check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.pathsep.join([os.path.dirname(rt.stdout.strip()), "/opt/rocm/lib", env.get("LD_LIBRARY_PATH", "")])
    # the HIP runtime's own allocations at load time are not ours to judge; link order: a preloaded library may come first
    env["ASAN_OPTIONS"] = "detect_leaks=0:verify_asan_link_order=0"
    out = subprocess.run([exe, lib], env=env, capture_output=True, text=True)
    assert out.returncode == 0 and out.stdout.strip() == "ok", out.stderr[-2000:]


def test_missing_library_fails_loudly(B, monkeypatch):
    monkeypatch.setattr(B, "_lib", None)
    monkeypatch.setattr(B, "LIB_PATH", "/nonexistent/libquantspec.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        B.lib()
