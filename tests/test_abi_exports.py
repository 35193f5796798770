"""The C-ABI library loads (no GPU needed) and exports every function include/gss.h declares."""
import ctypes
import os
import re

from paper_2406_17918_amd import gss

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "gss.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gss_[a-z_]+)\s*\(", text)) - {"gss_alloc_fn", "gss_free_fn"})


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(gss.EXPORTS) == set(names)
    lib = gss.load_library()
    for n in names:
        assert getattr(lib, n) is not None
    assert b"gfx950" in lib.gss_version()


def test_struct_sizes_match_the_header_layout():
    # natural C layout of the structs in gss.h on x86-64
    assert ctypes.sizeof(gss.gss_relation) == 40
    assert ctypes.sizeof(gss.gss_graph) == 32
    assert ctypes.sizeof(gss.gss_config) == 80
    assert ctypes.sizeof(gss.gss_block_nodes) == 16
    assert ctypes.sizeof(gss.gss_block_edges) == 24
    assert ctypes.sizeof(gss.gss_blocks) == 40


def test_host_side_argument_checks_need_no_device():
    lib = gss.load_library()
    h = ctypes.c_void_p()
    assert lib.gss_create(None, None, ctypes.byref(h)) == gss.GSS_ERR_INVALID_ARG
    assert lib.gss_create(None, None, None) == gss.GSS_ERR_INVALID_ARG
    nn = (ctypes.c_int64 * 1)(10)
    rel = (gss.gss_relation * 1)(gss.gss_relation(0, 0, 0, 1, 0, None))
    g = gss.gss_graph(1, nn, 1, rel)
    for k, layers, mode, period in [(0, 1, 0, 1), (65, 1, 0, 1), (4, 0, 0, 1), (4, 9, 0, 1), (4, 1, 7, 1), (4, 1, 0, 0)]:
        cfg = gss.gss_config(k, mode, layers, 0.0, period, 0, None, gss.ALLOC_FN(0), gss.FREE_FN(0), None)
        assert lib.gss_create(ctypes.byref(g), ctypes.byref(cfg), ctypes.byref(h)) == gss.GSS_ERR_INVALID_ARG
    bad = gss.gss_graph(1, nn, 1, (gss.gss_relation * 1)(gss.gss_relation(0, 3, 0, 1, 0, None)))
    cfg = gss.gss_config(4, 0, 1, 0.0, 1, 0, None, gss.ALLOC_FN(0), gss.FREE_FN(0), None)
    assert lib.gss_create(ctypes.byref(bad), ctypes.byref(cfg), ctypes.byref(h)) == gss.GSS_ERR_INVALID_GRAPH
    assert lib.gss_step(None, None, 0, 0, None, 1, 0, None) == gss.GSS_ERR_INVALID_ARG
    assert lib.gss_destroy(None) == gss.GSS_OK
    assert lib.gss_last_error(None) == b"create: invalid graph"     # NULL handle: why this thread's last create failed


def test_missing_library_is_an_error_not_a_fallback(monkeypatch, tmp_path):
    # the product path has no CPU route: without the built library every entry point of the binding raises
    monkeypatch.setattr(gss, "_lib", None)
    monkeypatch.setattr(gss, "LIB_PATH", str(tmp_path / "libgss.so"))
    import pytest
    with pytest.raises(RuntimeError, match="no fallback"):
        gss.load_library()


def test_product_path_and_oracle_do_not_know_each_other():
    # the oracle is test infrastructure: nothing in the package names it, and the oracle names nothing of the package
    pkg = os.path.join(ROOT, "paper_2406_17918_amd")
    for base, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")) and "synth" not in base:
                text = open(os.path.join(base, f)).read()
                assert "gsso" not in text and "import oracle" not in text and "from oracle" not in text, f
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2406_17918_amd" not in text and "gss.h" not in text and "libgss.so" not in text, f
