"""The C-ABI library loads and exports every entry point the header declares (no compute calls: no GPU here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "piperag.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(piperag_[a-z_0-9]+)\s*\(", text)))


def library():
    from paper_2403_05676_amd import build, binding
    if not os.path.exists(binding.lib_path()):
        build.build()
    return ctypes.CDLL(binding.lib_path())


def test_header_declares_the_three_north_star_entry_points():
    names = declared_symbols()
    for must in ("piperag_ivf_load", "piperag_ivfpq_search", "piperag_latency_profile"):
        assert must in names
    assert len(names) >= 15


def test_library_exports_every_declared_symbol():
    lib = library()
    for name in declared_symbols():
        assert hasattr(lib, name), f"{name} is declared in piperag.h but not exported"


def test_binding_covers_every_declared_symbol():
    from paper_2403_05676_amd import binding
    src = open(binding.__file__).read()
    for name in declared_symbols():
        assert name in src, f"the Python binding does not call {name}"
    binding.load_library()          # sets argtypes for every symbol; raises if one is missing


def test_error_paths_without_gpu():
    lib = library()
    lib.piperag_last_error.restype = ctypes.c_char_p
    assert lib.piperag_ivfpq_search(None, None, 1, 1, 1, None, None, None) == -1
    assert b"NULL" in lib.piperag_last_error()
    out = ctypes.c_void_p()
    assert lib.piperag_ivf_load(b"/nonexistent/file", ctypes.byref(ctypes.create_string_buffer(64)), ctypes.byref(out)) == -4
    assert lib.piperag_ivf_ntotal(None) == -1
    for setter in (lib.piperag_set_scan_streaming, lib.piperag_set_graph_replay, lib.piperag_set_stage_timing):
        assert setter(None, 1) == -1


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2403_05676_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("no CPU fallback", ""), f"{f} mentions the oracle"
