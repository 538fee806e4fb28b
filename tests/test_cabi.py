"""The C-ABI library loads and exports every function include/tasc.h declares (no compute calls)."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "tasc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(tasc_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_four_entry_points():
    names = declared_functions()
    for n in ("tasc_ngram_build", "tasc_draft", "tasc_verify_step", "tasc_generate"):
        assert n in names


def test_library_exports_every_declared_symbol():
    import paper_2602_24174_amd as T
    if not os.path.exists(T.LIB_PATH):
        pytest.skip("libtasc.so not built (run __graft_entry__.build())")
    lib = ctypes.CDLL(T.LIB_PATH)
    missing = [n for n in declared_functions() if not hasattr(lib, n)]
    assert not missing, missing
    assert sorted(T.EXPORTS) == declared_functions()


def test_binding_structs_match_header_sizes():
    import paper_2602_24174_amd as T
    assert ctypes.sizeof(T.ModelDesc) == 11 * 4
    assert ctypes.sizeof(T.SpecParams) == 16
    assert ctypes.sizeof(T.NgramStats) == 8 + 4 * 9 * 8 + 16
    assert ctypes.sizeof(T.GenStats) == 4 * 8 + 16 * 8 + 16 + 8
