"""CPU-side checks of the C-ABI library: it loads, and it exports every function that
include/gsplit.h declares (no compute calls: there is no GPU here)."""
import ctypes
import os
import re

import pytest

from conftest import ROOT


def _declared():
    text = open(os.path.join(ROOT, "include", "gsplit.h")).read()
    return sorted(set(re.findall(r"GSPLIT_API[^;(]*?\b(gsplit_\w+)\s*\(", text)))


def _lib_path():
    from paper_2303_13775_amd import LIB_PATH
    if not os.path.exists(LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    return LIB_PATH


def test_header_declares_the_four_hot_path_calls():
    names = _declared()
    for n in ("gsplit_sample_split", "gsplit_gather_features", "gsplit_sage_fwd", "gsplit_sage_bwd"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = ctypes.CDLL(_lib_path())
    for n in _declared():
        assert hasattr(lib, n), n


def test_binding_lists_the_same_names():
    from paper_2303_13775_amd import EXPORTS
    assert sorted(EXPORTS) == _declared()


def test_product_path_has_no_oracle_or_cpu_fallback():
    pkg = os.path.join(ROOT, "paper_2303_13775_amd")
    for dirpath, _, files in os.walk(pkg):
        if "_build" in dirpath:
            continue
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower().replace("no oracle", ""), f


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2303_13775_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(ImportError):
        b.load_library()
