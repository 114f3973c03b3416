"""The C-ABI library loads and exports every symbol include/spconv.h declares
(no compute calls: this runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "spconv.h")).read()
    return sorted(set(re.findall(r"SPCONV_API\s+[\w\s\*]+?\b(spconv_\w+)\s*\(", text)))


def test_header_declares_the_boundary():
    names = _declared()
    for must in ("spconv_build_kmap", "spconv_fwd", "spconv_dgrad", "spconv_wgrad", "spconv_tune",
                 "spconv_kmap_destroy", "spconv_kmap_export"):
        assert must in names


def test_library_exports_every_declared_symbol():
    import paper_2311_12862_amd as sp
    lib = ctypes.CDLL(sp.lib_path())
    for name in _declared():
        assert hasattr(lib, name), name
    assert sp.load_library().spconv_version() >= 100
    assert sp.load_library().spconv_strerror(-2).decode().startswith("coordinate")


def test_python_binding_mirrors_the_c_names():
    import paper_2311_12862_amd as sp
    for name in ("build_kmap", "fwd", "dgrad", "wgrad", "tune"):
        assert callable(getattr(sp, name))


def test_argument_errors_need_no_gpu():
    import paper_2311_12862_amd as sp
    lib = sp.load_library()
    out = ctypes.c_void_p()
    assert lib.spconv_build_kmap(None, -1, 3, 1, 0, None, ctypes.byref(out)) == -1
    assert lib.spconv_build_kmap(None, 5, 3, 1, 0, None, ctypes.byref(out)) == -1
    assert lib.spconv_build_kmap(None, 0, 2, 1, 0, None, ctypes.byref(out)) == -1
    assert lib.spconv_kmap_sizes(None, None, None, None) == -1
    assert lib.spconv_fwd(None, None, None, 64, 64, 1, None, None, None) == -1
