"""Host-only checks of the C-ABI library: it loads, exports every symbol that
include/mv.h declares, and rejects bad configurations before any device call."""
import ctypes
import os
import re

import pytest

from paper_2011_06495_amd import binding as B
from paper_2011_06495_amd import build as mv_build

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        mv_build.build_lib()
    return B.load()


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "mv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mv_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(lib):
    names = declared_symbols()
    assert set(names) == set(B.ABI_SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_config_struct_layout():
    assert ctypes.sizeof(B.mv_config) == 56
    assert B.mv_config.d.offset == 16 and B.mv_config.workspace.offset == 40


def test_workspace_bytes_and_invalid_configs(lib):
    good = B.make_config(16, 11173962, 11174)
    n = B.mv_workspace_bytes(good)
    assert 0 < n < 200 * 1024 * 1024
    assert B.mv_workspace_bytes(B.make_config(32, 25557032, 25557, B.MV_BF16)) > n
    bad = [B.make_config(0, 100, 10), B.make_config(256, 100, 10), B.make_config(4, 0, 1),
           B.make_config(4, 100, 0), B.make_config(4, 100, 101), B.make_config(4, 1 << 31, 10),
           B.make_config(4, 100, 10, grad_dtype=7), B.make_config(4, 100, 10, reduce=2),
           B.make_config(4, 100, 10, device=-1)]
    wrong_size = B.make_config(4, 100, 10)
    wrong_size.struct_size = 48
    reserved = B.make_config(4, 100, 10)
    reserved.flags = 2
    for cfg in bad + [wrong_size, reserved]:
        assert B.mv_workspace_bytes(cfg) == 0
        h = ctypes.c_void_p()
        assert lib.mv_begin(ctypes.byref(cfg), ctypes.byref(h)) == B.MV_ERR_INVALID_ARG
        assert not h.value
    assert lib.mv_begin(None, ctypes.byref(ctypes.c_void_p())) == B.MV_ERR_INVALID_ARG
    assert lib.mv_begin(ctypes.byref(good), None) == B.MV_ERR_INVALID_ARG
    # a caller workspace that is too small or misaligned is refused on the host
    small = B.make_config(4, 100000, 100, workspace=4096, workspace_bytes=16)
    assert lib.mv_begin(ctypes.byref(small), ctypes.byref(ctypes.c_void_p())) == B.MV_ERR_INVALID_ARG
    odd = B.make_config(4, 100000, 100, workspace=4097, workspace_bytes=1 << 30)
    assert lib.mv_begin(ctypes.byref(odd), ctypes.byref(ctypes.c_void_p())) == B.MV_ERR_INVALID_ARG


def test_null_context_calls(lib):
    assert lib.mv_vote_step(None, 0, 0, 0, 0, 0, 0, 0, 0, 0) == B.MV_ERR_INVALID_ARG
    assert lib.mv_end(None) == B.MV_ERR_INVALID_ARG
    assert lib.mv_set_profiling(None, 1) == B.MV_ERR_INVALID_ARG
    lib.mv_release(None)


def test_status_strings_and_kernel_names(lib):
    seen = {B.status_string(s) for s in range(6)}
    assert len(seen) == 6 and "ok" in seen
    assert B.status_string(99) == "unknown status"
    names = B.kernel_names()
    assert len(names) == lib.mv_kernel_count() and "mv_stream_collect" in names
    assert lib.mv_kernel_name(-1) == b"" and lib.mv_kernel_name(100) == b""
