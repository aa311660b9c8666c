"""The C-ABI library loads and exports every function include/subgen.h declares (no compute, no GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "subgen.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(subgen_[a-z_]+)\s*\(", text)))


def test_header_declares_the_four_core_calls():
    names = declared_functions()
    for core in ["subgen_create", "subgen_update", "subgen_attend", "subgen_ingest_prefix", "subgen_step"]:
        assert core in names


def test_library_exports_every_declared_symbol():
    from paper_2402_06082_amd import binding
    path = binding.lib_path()
    assert path.exists(), "build the library first (python -m paper_2402_06082_amd.build)"
    lib = ctypes.CDLL(str(path))
    names = declared_functions()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTS) == names
    assert binding.strerror(0) == "ok" and binding.strerror(-1) == "invalid argument"


def test_binding_struct_sizes_match_the_header_layout():
    # natural C layout of the three structs in the header (x86-64)
    from paper_2402_06082_amd import binding
    assert ctypes.sizeof(binding.subgen_opts) == 64
    assert ctypes.sizeof(binding.subgen_stats_t) == 56
    assert ctypes.sizeof(binding.subgen_state_view) == 144
