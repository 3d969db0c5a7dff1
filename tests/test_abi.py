"""The C-ABI library loads on a machine without a GPU and exports every function the header
declares (no compute is called here)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "cachemir.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(cm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function():
    path = os.path.join(ROOT, "paper_2602_11470_amd", "libcachemir.so")
    assert os.path.exists(path), "build first: python -m paper_2602_11470_amd.build"
    lib = ctypes.CDLL(path)
    names = _declared()
    assert len(names) >= 45
    missing = [n for n in names if not hasattr(lib, n)]
    assert not missing, missing
    lib.cm_strerror.restype = ctypes.c_char_p
    assert lib.cm_strerror(0) == b"ok" and b"key" in lib.cm_strerror(-4)


def test_binding_covers_the_header():
    from paper_2602_11470_amd import binding
    assert sorted(binding.EXPORTS) == _declared()


def test_invalid_arguments_are_rejected_without_a_gpu():
    from paper_2602_11470_amd import binding as B
    h = ctypes.c_void_p()
    bad = B.cm_params(1000, 5, 1, 1, 50, 40, 60, 0, 2.0 ** 40, 3.2)       # ring degree not supported
    assert B.lib.cm_ctx_create(ctypes.byref(bad), ctypes.byref(h)) == -1
    assert B.lib.cm_ctx_create(None, ctypes.byref(h)) == -1
    assert B.lib.cm_ct_words(None, 0, 2) == 0
