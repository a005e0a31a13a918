"""The C-ABI library loads and exports every symbol include/gnn.h declares (no GPU needed)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2412_06354_amd", "libgnn_mi355x.so")


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "gnn.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gnn_[a-z0-9_]+)\s*\(", text)))


@pytest.fixture(scope="module")
def handle():
    if not os.path.exists(LIB):
        from paper_2412_06354_amd import build
        build.build(verbose=False)
    return ctypes.CDLL(LIB)


def test_header_declares_the_five_named_calls():
    names = declared_symbols()
    for must in ("gnn_build_csr", "gnn_propagate", "gnn_gcnconv", "gnn_segment_softmax", "gnn_graph_pool"):
        assert must in names


def test_every_declared_symbol_is_exported(handle):
    for name in declared_symbols():
        assert hasattr(handle, name), name


def test_binding_signatures_cover_the_header():
    pytest.importorskip("torch")
    from paper_2412_06354_amd import binding
    assert sorted(binding.SIGNATURES) == declared_symbols()


def test_status_strings(handle):
    handle.gnn_status_string.restype = ctypes.c_char_p
    seen = {handle.gnn_status_string(c) for c in range(10)}
    assert len(seen) == 10 and handle.gnn_status_string(0) == b"ok"
    assert handle.gnn_status_string(99) == b"unknown status"


def test_host_side_argument_errors_need_no_gpu(handle):
    # These are rejected before any HIP call is made.
    out = ctypes.c_void_p()
    f = handle.gnn_build_csr
    f.restype = ctypes.c_int
    f.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p,
                  ctypes.POINTER(ctypes.c_void_p)]
    assert f(None, None, 0, 0, None, ctypes.byref(out)) == 2          # N <= 0
    assert f(None, None, 5, 3, None, ctypes.byref(out)) == 1          # NULL edge arrays
    assert f(None, None, 1 << 31, 3, None, ctypes.byref(out)) == 2    # too many edges
    assert f(None, None, 0, 3, None, None) == 1                       # NULL out pointer
    handle.gnn_gcnconv_workspace_bytes.restype = ctypes.c_size_t
    handle.gnn_gcnconv_workspace_bytes.argtypes = [ctypes.c_int32, ctypes.c_int32]
    assert handle.gnn_gcnconv_workspace_bytes(1000, 128) >= 1000 * 128 * 4   # the projected rows
    p = handle.gnn_propagate
    p.restype = ctypes.c_int
    assert p(None, None, 4, None, 1, 0, 0, 0, None, None) == 1        # NULL graph
    for name in ("gnn_graph_build_edge_route", "gnn_graph_reserve"):
        fn = getattr(handle, name)
        fn.restype = ctypes.c_int
    assert handle.gnn_graph_build_edge_route(None, None) == 1          # NULL graph
    assert handle.gnn_graph_reserve(None, ctypes.c_int32(64), ctypes.c_int32(8)) == 1
    for name in ("gnn_edge_data_to_csr", "gnn_edge_data_to_coo"):
        fn = getattr(handle, name)
        fn.restype = ctypes.c_int
        fn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        assert fn(None, None, 1, None, None) == 1                      # NULL graph
    ws = handle.gnn_graph_pool_workspace_bytes
    ws.restype = ctypes.c_size_t
    ws.argtypes = [ctypes.c_int32, ctypes.c_int32, ctypes.c_int32]
    assert ws(1000, 10, 64) == 0                                       # small graphs: no workspace, one block per graph
    assert ws(1_000_000, 1, 64) >= (1_000_000 // 1024) * 64 * 4        # a part per about 1 024 nodes
    pw = handle.gnn_graph_pool_ws
    pw.restype = ctypes.c_int
    pw.argtypes = [ctypes.c_void_p, ctypes.c_int32, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32, ctypes.c_int,
                   ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
    assert pw(None, 1_000_000, 1, None, 64, 0, None, None, 0, None) == 1   # a workspace is needed and missing
    bb = handle.gnn_build_csr_batch
    bb.restype = ctypes.c_int
    assert bb(0, None, None, None, 5, None, None) == 1                 # NULL handle array


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    pytest.importorskip("torch")
    from paper_2412_06354_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", str(tmp_path / "absent.so"))
    with pytest.raises(RuntimeError, match="is missing"):
        binding.lib()


def test_product_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2412_06354_amd")
    for dirpath, _, files in os.walk(pkg):
        for name in files:
            if name.endswith((".py", ".hip", ".h", ".cpp")):
                text = open(os.path.join(dirpath, name)).read()
                assert "import oracle" not in text and "from oracle" not in text and "gnn_oracle" not in text, name
    for name in ("__init__.py", "gnn_oracle.c"):
        text = open(os.path.join(ROOT, "oracle", name)).read()
        assert "paper_2412_06354_amd" not in text and "libgnn_mi355x" not in text, name


def test_header_is_plain_c_and_the_library_links_from_c(tmp_path):
    """include/gnn.h compiles as strict C99 and a C program linked against the library runs its host-side checks."""
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    lib_dir = os.path.join(root, "paper_2412_06354_amd")
    if not os.path.exists(os.path.join(lib_dir, "libgnn_mi355x.so")):
        pytest.skip("library not built")
    src = tmp_path / "use_abi.c"
    src.write_text(r"""
#include <stdio.h>
#include <string.h>
#include "gnn.h"
int main(void)
{
    gnn_graph *g = NULL;
    if (strcmp(gnn_status_string(GNN_OK), "ok") != 0) return 1;
    if (gnn_build_csr(NULL, NULL, 5, 3, NULL, &g) != GNN_ERR_NULL || g != NULL) return 2;
    if (gnn_build_csr(NULL, NULL, 0, 0, NULL, &g) != GNN_ERR_BAD_SIZE) return 3;
    if (gnn_propagate(NULL, NULL, 4, NULL, 1, GNN_EDGE_ORDER_COO, GNN_MSG_COPY_XJ, GNN_AGGR_SUM, NULL, NULL) != GNN_ERR_NULL) return 4;
    if (gnn_graph_pool_workspace_bytes(100, 1, 8) != 0) return 5;
    if (gnn_graph_destroy(NULL) != GNN_OK) return 6;
    puts("c abi ok");
    return 0;
}
""")
    exe = tmp_path / "use_abi"
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"),
                           str(src), "-o", str(exe), "-L", lib_dir, "-lgnn_mi355x",
                           "-Wl,-rpath," + lib_dir, "-Wl,-rpath,/opt/rocm/lib"])
    out = subprocess.run([str(exe)], capture_output=True, text=True, timeout=120)
    assert out.returncode == 0 and "c abi ok" in out.stdout, (out.returncode, out.stdout, out.stderr)
