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


def test_header_is_plain_c_and_links_from_c(lib, tmp_path):
    """The header compiles as strict C99 and as C++, and a C program that includes it links against the
    library and gets sane answers from the calls that need no GPU."""
    import subprocess
    from paper_2312_05417_amd import binding
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c", HEADER])
    subprocess.check_call(["g++", "-std=c++11", "-pedantic", "-Wall", "-Werror", "-fsyntax-only", "-x", "c++", HEADER])
    src = tmp_path / "use_espn.c"
    src.write_text('''
#include <stdio.h>
#include <string.h>
#include "espn.h"
int main(void) {
    if (espn_workspace_bytes(64, 1000) != 256000u + 512000u) return 1;
    if (espn_batch_threshold(2.0e9, 0.5, 1.0e6) != 1000.0) return 2;
    if (strcmp(espn_status_string(ESPN_ERR_SHAPE), "inconsistent sizes") != 0) return 3;
    if (espn_topk(NULL, NULL, 1, 4, 5, NULL, NULL, NULL) != ESPN_ERR_SHAPE) return 4;
    if (strstr(espn_last_error(), "k = 5") == NULL) return 5;
    if (espn_table_free(NULL) != ESPN_OK) return 6;
    puts("ok");
    return 0;
}
''')
    exe = tmp_path / "use_espn"
    libdir = os.path.dirname(binding.LIB_PATH)
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.dirname(HEADER), str(src), "-o", str(exe),
                           "-L", libdir, "-l:libespn.so", "-Wl,-rpath," + libdir])
    assert subprocess.check_output([str(exe)]).decode().strip() == "ok"


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
    assert len({binding.status_string(i) for i in range(8)}) == 8
    assert binding.status_string(8) == "unknown status"


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
    assert lib.espn_rerank_noalloc(None, None, None, 1, 32, 4, 2, None, None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_rerank_batches(None, 2, None, None, 1, 32, 4, 2, None, None, None, 0, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_sample(None, None, 1, 4, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_check(None, None) == bd.ESPN_ERR_ARG
    assert lib.espn_table_free(None) == bd.ESPN_OK


def test_workspace_bytes(lib):
    # the scores (4 bytes per pair) and the lists in id order (8 bytes per pair), each rounded up to 256 bytes
    assert lib.espn_workspace_bytes(64, 1000) == 256000 + 512000
    assert lib.espn_workspace_bytes(1, 1) == 256 + 256
    assert lib.espn_workspace_bytes(0, 1000) == 256
    assert lib.espn_workspace_bytes(3, 100) % 256 == 0 and lib.espn_workspace_bytes(3, 100) >= 3600


def test_batches_workspace_bytes_without_a_table(lib):
    # no table: the size for one batch (the sizes for a table's queues are checked on the GPU)
    assert lib.espn_batches_workspace_bytes(None, 5, 64, 32, 1000, 10) == lib.espn_workspace_bytes(64, 1000)


def test_the_benchmark_probes_are_a_library_of_their_own(lib):
    """bench.py's plain-read and plain-copy kernels are not exported by the product library."""
    from paper_2312_05417_amd import benchprobe
    assert not hasattr(lib, "espn_stream_read_probe") and not hasattr(lib, "espn_bench_stream_read")
    probe = benchprobe.lib()
    assert hasattr(probe, "espn_bench_stream_read") and hasattr(probe, "espn_bench_copy")
    assert probe.espn_bench_stream_read(None, 16, None, None) == 1          # bad argument, found on the host
    assert probe.espn_bench_copy(None, None, 0, None) == 0


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    from paper_2312_05417_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "libespn.so"))
    with pytest.raises(ImportError):
        binding.lib()
