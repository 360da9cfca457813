"""CPU check: the C-ABI library loads and exports every symbol the header declares."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "pie_mi355.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(pie_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    from paper_2510_24051_amd import lib_path, load_library
    assert os.path.exists(lib_path()), "build the library first (python -m paper_2510_24051_amd.build)"
    lib = load_library()
    names = declared_symbols()
    assert len(names) >= 18
    for n in names:
        assert hasattr(lib, n), f"{n} declared in include/pie_mi355.h but not exported"
    raw = ctypes.CDLL(lib_path())
    for n in names:
        getattr(raw, n)


def test_create_fails_cleanly_on_bad_arguments_without_gpu_work():
    from paper_2510_24051_amd import load_library
    lib = load_library()
    out = ctypes.c_void_p()
    assert lib.pie_create(None, None, None, ctypes.byref(out)) == -1  # PIE_EINVAL before any HIP call
    assert b"null" in lib.pie_last_error(None)
    assert lib.pie_destroy(None) == 0


def test_product_package_never_imports_the_oracle():
    pkg = os.path.join(ROOT, "paper_2510_24051_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f"{f} mentions the oracle"
