"""The C-ABI library loads without a GPU and exports every symbol the public header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "ckks_mi355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ckks_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    import paper_2604_03425_amd as pkg
    lib = ctypes.CDLL(pkg.library_path())
    names = declared_functions()
    assert len(names) >= 11
    for n in names:
        assert hasattr(lib, n), n
    assert set(pkg.exported_symbols()) == set(names)


def test_binding_has_no_cpu_fallback():
    src = open(os.path.join(ROOT, "paper_2604_03425_amd", "binding.py")).read()
    assert "oracle" not in src.replace("no CPU fallback", "")
    import paper_2604_03425_amd as pkg
    for n in declared_functions():
        if n.startswith("ckks_ctx") or n == "ckks_last_error" or n.startswith("ckks_prof_") or n == "ckks_tune_set":
            continue
        assert hasattr(pkg, n), n
