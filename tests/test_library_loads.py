"""CPU-side checks of the boundary: the shared library loads and exports every symbol essa.h declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "essa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(essa_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_are_exported():
    import paper_2507_04453_amd as essa
    names = _declared_symbols()
    assert len(names) >= 20
    lib = ctypes.CDLL(essa.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    assert sorted(essa.EXPORTED_SYMBOLS) == names
    assert "gfx950" in essa.essa_version()


def test_no_oracle_in_the_product_path():
    """The package must not import the oracle (and the oracle must not import the package)."""
    for base, other in (("paper_2507_04453_amd", "oracle"), ("oracle", "paper_2507_04453_amd")):
        for dirpath, _, files in os.walk(os.path.join(ROOT, base)):
            for f in files:
                if f.endswith((".py", ".hip", ".cpp", ".h")):
                    src = open(os.path.join(dirpath, f)).read()
                    assert ("import " + other) not in src and ("from " + other) not in src, (f, other)
