"""The C-ABI library loads and exports every entry point that include/imunpack.h declares
(no compute calls: runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
LIB = os.path.join(ROOT, "paper_2403_07339_amd", "libimunpack.so")
HEADER = os.path.join(ROOT, "include", "imunpack.h")


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(imunpack_[a-z0-9_]+)\s*\(", text)))


def built_library():
    if not os.path.exists(LIB):
        from paper_2403_07339_amd import build
        build.build()
    return ctypes.CDLL(LIB)


def test_header_declares_the_five_path_calls():
    names = declared_functions()
    for f in ("imunpack_quantize", "imunpack_plan", "imunpack_unpack", "imunpack_gemm", "imunpack_recombine"):
        assert f in names


def test_library_exports_every_declared_symbol():
    lib = built_library()
    for f in declared_functions():
        assert hasattr(lib, f), f


def test_strerror_and_argument_validation_without_gpu():
    lib = built_library()
    lib.imunpack_strerror.restype = ctypes.c_char_p
    assert lib.imunpack_strerror(0) == b"ok"
    assert b"invalid" in lib.imunpack_strerror(-1)
    # null pointers are rejected on the host before any HIP call
    lib.imunpack_plan_dims.restype = ctypes.c_int
    assert lib.imunpack_plan_dims(None, None, None, None, None) == -1
    lib.imunpack_plan_destroy.restype = ctypes.c_int
    assert lib.imunpack_plan_destroy(None) == 0


def test_binding_matches_header():
    import importlib
    text = open(os.path.join(ROOT, "paper_2403_07339_amd", "binding.py")).read()
    for f in declared_functions():
        assert f in text, f"binding.py does not wrap {f}"
    importlib.import_module("paper_2403_07339_amd.workloads")
