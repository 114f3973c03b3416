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
    for name in ("build_kmap", "fwd", "dgrad", "wgrad", "tune", "tune_group", "set_allocator", "ew", "copy_cols"):
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
    assert lib.spconv_fwd_noalloc(None, None, None, 64, 64, 1, None, None, None) == -1
    for K, stride, transposed in ((4, 1, 0), (5, 2, 0), (5, 1, 1), (7, 1, 0), (3, 0, 0), (3, 65, 0), (3, 1, 2), (2, 1, 0), (2, 3, 0)):
        assert lib.spconv_build_kmap(None, 0, K, stride, transposed, None, ctypes.byref(out)) == -1, (K, stride)
        assert lib.spconv_build_kmap_async(None, 0, K, stride, transposed, None, ctypes.byref(out)) == -1
    assert lib.spconv_build_kmap(None, 0, 3, 1, 0, None, None) == -1
    assert lib.spconv_kmap_transpose(None, None, ctypes.byref(out)) == -1 and out.value is None
    assert lib.spconv_kmap_transpose(None, None, None) == -1
    assert lib.spconv_kmap_pointwise(None, 0, None, ctypes.byref(out)) == -1 and out.value is None
    assert lib.spconv_kmap_pointwise(None, 0, None, None) == -1
    assert lib.spconv_kmap_status(None, None) == -1
    assert lib.spconv_dgrad(None, None, None, 64, 64, 1, None, None, None) == -1
    assert lib.spconv_wgrad(None, None, None, 64, 64, 1, None, None, None) == -1
    assert lib.spconv_tune(None, 64, 64, 1, 0, 1, None, None, None) == -1
    assert lib.spconv_tune_group(None, None, 0, 1, 0, 1, None, None, None, None, None) == -1
    assert lib.spconv_ew(9, None, None, None, 4, 1, None) == -1
    assert lib.spconv_ew(0, None, None, None, 0, 1, None) == 0          # nothing to do
    assert lib.spconv_copy_cols(None, 8, 4, None, 8, 0, 8, 4, 1, None) == -1   # columns past the row
    alloc = ctypes.CFUNCTYPE(ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p)(lambda n, s, u: None)
    assert lib.spconv_set_allocator(ctypes.cast(alloc, ctypes.c_void_p), None, None) == -1   # both or neither
    assert lib.spconv_set_allocator(None, None, None) == 0
    lib.spconv_kmap_destroy(None)                                        # a no-op
