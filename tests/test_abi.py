"""The C-ABI library loads and exports every symbol the header declares
(no compute: this runs without a GPU)."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "rsd.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(rsd_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2501_19324_amd import binding

    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = binding.load_library()
    names = declared_symbols()
    assert len(names) >= 14
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(binding.EXPORTED_SYMBOLS) == names
    # the build with the table checks exports the same interface
    import ctypes
    dbg = ctypes.CDLL(os.path.join(os.path.dirname(binding.LIB_PATH), "librsd_debug.so"))
    for n in names:
        assert hasattr(dbg, n), n


def test_missing_library_fails_loudly(tmp_path):
    from paper_2501_19324_amd import binding

    with pytest.raises(RuntimeError):
        binding.load_library(str(tmp_path / "nope.so"))
    binding.load_library(binding.LIB_PATH)


def test_struct_layouts_match_header_sizes():
    import ctypes as C
    from paper_2501_19324_amd import binding as b

    assert C.sizeof(b._Shape) == 40 and C.sizeof(b._Weights) == 16
    assert C.sizeof(b._Params) == 48 + 24 + 16 and b._Params.bon_n.offset == 84
    assert C.sizeof(b._StepOut) == 88 and C.sizeof(b._GenOut) == 24 + 8 + 40 + 24 and C.sizeof(b._BonOut) == 72
