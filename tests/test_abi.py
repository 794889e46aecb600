"""CPU-only checks of the boundary: the built library loads, exports every function the header
declares, the binding covers each of them, and argument errors are caught on the host."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "espn.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(espn_[a-z_0-9]+)\s*\(", text)))


@pytest.fixture(scope="module")
def lib():
    from paper_2312_05417_amd import binding, build
    if not os.path.exists(binding.LIB_PATH):
        build.build_library(verbose=False)
    return binding.lib()


def test_header_declares_the_path():
    names = declared_functions()
    for must in ("espn_table_load", "espn_table_free", "espn_score", "espn_topk", "espn_rerank"):
        assert must in names


def test_every_declared_symbol_is_exported_and_bound(lib):
    from paper_2312_05417_amd import binding
    for name in declared_functions():
        assert hasattr(lib, name), "library does not export " + name
        assert name in binding.SIGNATURES, "binding has no signature for " + name
    assert sorted(binding.SIGNATURES) == declared_functions()


def test_status_strings(lib):
    from paper_2312_05417_amd import binding
    assert binding.status_string(0) == "ok"
    assert len({binding.status_string(i) for i in range(9)}) == 9


def test_host_side_argument_errors_need_no_gpu(lib):
    from paper_2312_05417_amd import binding as bd
    h = ctypes.c_void_p()
    off = (ctypes.c_int64 * 3)(0, 2, 1)
    good = (ctypes.c_int64 * 3)(0, 1, 2)
    assert lib.espn_table_load(None, off, 2, 32, 0, 0, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_load(None, None, 2, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG
    assert lib.espn_table_load(None, good, -1, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG
    assert lib.espn_table_load(None, good, 2, 12, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG
    assert lib.espn_table_load(None, good, 2, 32, 7, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG
    assert lib.espn_table_load(16, off, 2, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_OFFSETS
    assert "decrease" in bd.last_error()
    bad0 = (ctypes.c_int64 * 2)(1, 2)
    assert lib.espn_table_load(16, bad0, 1, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_OFFSETS
    assert lib.espn_table_load(None, good, 2, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG   # rows but no emb
    assert lib.espn_table_load(24, good, 2, 32, 0, 0, ctypes.byref(h)) == bd.ESPN_ERR_ARG     # misaligned
    assert not h.value
    assert lib.espn_topk(None, None, 1, 4, 5, None, None, None) == bd.ESPN_ERR_SHAPE
    assert lib.espn_topk(None, None, 1, 4, 2, None, None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_topk(None, None, -1, 4, 2, None, None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_score(None, None, None, 1, 32, 4, None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_rerank(None, None, None, 1, 32, 4, 2, None, None, None, 0, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_check(None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_free(None) == bd.ESPN_OK


def test_workspace_bytes(lib):
    assert lib.espn_workspace_bytes(64, 1000) == 256000
    assert lib.espn_workspace_bytes(1, 1) == 256
    assert lib.espn_workspace_bytes(0, 1000) == 256
    assert lib.espn_workspace_bytes(3, 100) % 256 == 0 and lib.espn_workspace_bytes(3, 100) >= 1200


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2312_05417_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libespn.so"))
    with pytest.raises(ImportError):
        binding.lib()
