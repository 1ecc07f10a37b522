"""CPU-side checks of the C-ABI library: it loads, exports every function that
include/f8.h declares, and rejects bad arguments on the host before any launch
(so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_2410_06511_amd import f8

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "f8.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(f8_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    names = declared_functions()
    assert len(names) >= 10 and "f8_linear_fwd" in names and "f8_gemm" in names
    raw = C.CDLL(f8.LIB_PATH)
    for n in names:
        assert hasattr(raw, n), n
    assert sorted(f8.EXPORTS) == names            # the binding covers exactly the header


def test_status_strings():
    assert f8.status_string(0) == "ok"
    for code in range(1, 7):
        assert len(f8.status_string(code)) > 5
    assert f8.status_string(99) == "unknown status"


def test_workspace_size_grows_with_columns():
    a, b = f8.workspace_bytes(8192, 4096), f8.workspace_bytes(8192, 16384)
    assert a >= 8192 and b >= a and b % 256 == 0
    assert f8.workspace_bytes(0, 0) >= 8192


FAKE = 0x10000  # a 16-byte aligned non-NULL address that is never dereferenced on these paths


def test_argument_errors_are_reported_before_any_launch():
    l = f8.lib()
    ws = f8.workspace_bytes(64, 64)
    # NULL pointers
    assert l.f8_amax(None, 16, 16, 16, 0, FAKE, FAKE, ws, None) == 1
    assert l.f8_amax(FAKE, 16, 16, 16, 0, None, FAKE, ws, None) == 1
    # shapes: not a multiple of 16, negative, ld < cols
    assert l.f8_amax(FAKE, 15, 16, 16, 0, FAKE, FAKE, ws, None) == 2
    assert l.f8_amax(FAKE, 16, -16, 16, 0, FAKE, FAKE, ws, None) == 2
    assert l.f8_amax(FAKE, 16, 32, 16, 0, FAKE, FAKE, ws, None) == 2
    # alignment
    assert l.f8_amax(FAKE + 8, 16, 16, 16, 0, FAKE, FAKE, ws, None) == 3
    # enums
    assert l.f8_amax(FAKE, 16, 16, 16, 7, FAKE, FAKE, ws, None) == 4
    assert l.f8_scale(FAKE, 4, 5, FAKE, FAKE, None) == 4
    # workspace
    assert l.f8_amax(FAKE, 16, 16, 16, 0, FAKE, None, 0, None) == 5
    assert l.f8_amax(FAKE, 16, 16, 16, 2, FAKE, FAKE, 16, None) == 5
    # cast: needs at least one output, ld_out_t >= rows
    assert l.f8_cast(FAKE, 16, 16, 16, FAKE, 0, 0, None, 0, None, 0, None) == 1
    assert l.f8_cast(FAKE, 32, 16, 16, FAKE, 0, 0, None, 0, FAKE, 16, None) == 2
    assert l.f8_cast(FAKE, 16, 16, 16, None, 0, 0, FAKE, 16, None, 0, None) == 1
    # gemm: colwise is not a GEMM mode; K not a multiple of 16; ld too small
    assert l.f8_gemm(0, 16, 16, 16, FAKE, 0, 16, FAKE, 0, 16, FAKE, FAKE, 2, FAKE, 16, None, None) == 4
    assert l.f8_gemm(0, 16, 16, 24, FAKE, 0, 32, FAKE, 0, 32, FAKE, FAKE, 0, FAKE, 16, None, None) == 2
    assert l.f8_gemm(1, 16, 32, 16, FAKE, 0, 16, FAKE, 0, 16, FAKE, FAKE, 0, FAKE, 32, None, None) == 2
    assert l.f8_gemm(0, 16, 16, 16, None, 0, 16, FAKE, 0, 16, FAKE, FAKE, 0, FAKE, 16, None, None) == 1
    # linear: bad descriptor / missing saved buffers / workspace
    d = f8.linear_desc(32, 32, 32)
    sv = f8.SavedStruct()
    assert l.f8_linear_fwd(None, FAKE, FAKE, FAKE, C.byref(sv), FAKE, 1 << 20, None) == 1
    assert l.f8_linear_fwd(C.byref(d), FAKE, FAKE, FAKE, C.byref(sv), FAKE, 1 << 20, None) == 1
    bad = f8.linear_desc(32, 32, 30)
    assert l.f8_linear_fwd(C.byref(bad), FAKE, FAKE, FAKE, C.byref(sv), FAKE, 1 << 20, None) == 2
    bad = f8.LinearDesc(32, 32, 32, 2, 0)
    assert l.f8_linear_bwd(C.byref(bad), FAKE, C.byref(sv), FAKE, FAKE, FAKE, 1 << 20, None) == 4
    # the same checks behind the entry points that take a scratch buffer or no product
    assert l.f8_gemm_ws(0, 16, 16, 24, FAKE, 0, 32, FAKE, 0, 32, FAKE, FAKE, 0, FAKE, 16, None, FAKE, 1 << 20, None) == 2
    assert l.f8_gemm_ws(2, 16, 16, 16, FAKE, 0, 16, FAKE, 0, 8, FAKE, FAKE, 0, FAKE, 16, None, None, 0, None) == 2
    assert l.f8_gemm_ws(3, 16, 16, 16, FAKE, 0, 16, FAKE, 0, 16, FAKE, FAKE, 0, FAKE, 16, None, None, 0, None) == 4
    assert l.f8_linear_fwd_quantise(None, FAKE, FAKE, C.byref(sv), FAKE, 1 << 20, None) == 1
    assert l.f8_linear_fwd_quantise(C.byref(d), FAKE, None, C.byref(sv), FAKE, 1 << 20, None) == 1
    assert l.f8_linear_fwd_quantise(C.byref(d), FAKE + 4, FAKE, C.byref(sv), FAKE, 1 << 20, None) == 3
    assert l.f8_linear_fwd_noalloc(C.byref(bad), FAKE, FAKE, FAKE, C.byref(sv), None) == 4
    assert l.f8_probe_mfma(2, FAKE, 1 << 20, 1, None, FAKE, None, None) == 4
    assert l.f8_probe_mfma(0, FAKE, 3 << 18, 1, None, FAKE, None, None) == 2
    assert l.f8_probe_copy(FAKE, FAKE, 24, None) == 2
    assert l.f8_probe_clock(None, None) == 1


def test_block_entry_points_reject_bad_arguments_before_any_launch():
    l = f8.lib()
    # rope: no output; head dimension not a multiple of 8 / too large; pitch smaller than the row; sequence length 0
    assert l.f8_rope(FAKE, 128, 16, 16, 1, 128, 500000.0, 0, None, 0, None, None, None) == 1
    assert l.f8_rope(FAKE, 128, 16, 16, 1, 12, 500000.0, 0, FAKE, 128, None, None, None) == 2
    assert l.f8_rope(FAKE, 512, 16, 16, 1, 512, 500000.0, 0, FAKE, 512, None, None, None) == 2
    assert l.f8_rope(FAKE, 64, 16, 16, 1, 128, 500000.0, 0, FAKE, 128, None, None, None) == 2
    assert l.f8_rope(FAKE, 128, 16, 0, 1, 128, 500000.0, 0, FAKE, 128, None, None, None) == 2
    assert l.f8_rope(FAKE + 2, 128, 16, 16, 1, 128, 500000.0, 0, FAKE, 128, None, None, None) == 3
    # transpose, add
    assert l.f8_transpose_bf16(FAKE, 16, 16, 20, FAKE, None) == 2
    assert l.f8_transpose_bf16(FAKE, 32, 16, 32, None, None) == 1
    assert l.f8_add(FAKE, FAKE, 12, FAKE, None) == 2
    assert l.f8_add(FAKE, None, 16, FAKE, None) == 1
    # rmsnorm backward: neither output; dg without workspace
    assert l.f8_rmsnorm_bwd(FAKE, FAKE, FAKE, FAKE, 16, 16, None, None, None, 0, None) == 1
    assert l.f8_rmsnorm_bwd(FAKE, FAKE, FAKE, FAKE, 16, 16, FAKE, FAKE, None, 0, None) == 5
    assert l.f8_rmsnorm_bwd(FAKE, FAKE, FAKE, FAKE, 16, 24, FAKE, None, None, 0, None) == 2
    # attention: head dimension, sequence length, head grouping, pitches, workspace of the grouped backward
    fwd = lambda B, S, Hq, Hkv, hd, ldq=4096, ldk=1024, vt=FAKE: l.f8_sdpa_fwd(FAKE, ldq, FAKE, ldk, vt, B, S, Hq, Hkv, hd, FAKE, 4096, FAKE, None, None)
    assert fwd(1, 64, 32, 8, 64) == 2
    assert fwd(1, 60, 32, 8, 128) == 2
    assert fwd(1, 64, 32, 5, 128) == 2
    assert fwd(1, 64, 32, 8, 128, ldq=2048) == 2
    assert fwd(1, 64, 32, 8, 128, vt=None) == 1
    assert f8.sdpa_bwd_workspace_bytes(1, 8192, 32, 8, 128) == 2 * 8192 * 4096 * 4
    assert f8.sdpa_bwd_workspace_bytes(1, 8192, 8, 8, 128) == 0
    bwd = lambda ws, nbytes: l.f8_sdpa_bwd(FAKE, 4096, FAKE, FAKE, 1024, FAKE, FAKE, 1024, FAKE, 4096, FAKE, 4096, FAKE, FAKE,
                                           1, 64, 32, 8, 128, FAKE, 4096, FAKE, 1024, FAKE, 1024, FAKE, None, ws, nbytes, None)
    assert bwd(None, 0) == 5
    assert bwd(FAKE, 1024) == 5


def test_binding_raises_with_message():
    with pytest.raises(f8.F8Error) as e:
        f8._check(5)
    assert "workspace" in str(e.value)


def test_missing_library_fails_loudly(monkeypatch):
    """There is no fallback path: without the built HIP library every call raises."""
    monkeypatch.setattr(f8, "_lib", None)
    monkeypatch.setattr(f8, "LIB_PATH", "/nonexistent/libf8.so")
    import pytest
    with pytest.raises(RuntimeError, match="is missing"):
        f8.lib()
    with pytest.raises(RuntimeError, match="is missing"):
        f8.workspace_bytes(16, 16)
