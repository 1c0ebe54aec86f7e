"""CPU-side checks of the boundary: the library loads and exports every symbol the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "dp_step.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(dp_step\w*)\s*\(", src)))


def test_header_symbols_are_exported():
    from paper_2010_09063_amd import EXPORTS, LIB_PATH
    if not os.path.exists(LIB_PATH):
        from paper_2010_09063_amd.build import build_library
        build_library()
    lib = ctypes.CDLL(LIB_PATH)
    names = _declared()
    assert names and set(names) == set(EXPORTS)
    for n in names:
        assert hasattr(lib, n), n


def test_strerror_without_gpu():
    from paper_2010_09063_amd import load_library
    L = load_library()
    assert L.dp_step_strerror(0) == b"ok"
    assert b"invalid" in L.dp_step_strerror(-1)
    assert L.dp_step_num_params(None) == 0


def test_product_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2010_09063_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".h", ".hip")):
                txt = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in txt.lower() or f == "dp_step.py" and "oracle" not in txt.lower(), f
