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


def test_entry_points_reject_bad_arguments_on_the_host():
    """Every entry point checks its arguments before the first HIP call, so these return EINVAL (-1)
    on a machine without a GPU; the pointers passed are never dereferenced."""
    lib = built_library()
    EINVAL = -1
    i64, i32, f32, f64, vp = ctypes.c_int64, ctypes.c_int, ctypes.c_float, ctypes.c_double, ctypes.c_void_p
    fake = vp(0x1000)   # a non-null address that must not be touched
    lib.imunpack_quantize.restype = ctypes.c_int
    lib.imunpack_quantize.argtypes = [vp, i64, i64, i64, i64, f32, i32, vp, i64, vp, vp, vp]
    assert lib.imunpack_quantize(None, 4, 4, 4, 1, 1.0, 8, fake, 4, None, None, None) == EINVAL      # no input
    assert lib.imunpack_quantize(fake, 4, 4, 4, 1, 1.0, 9, fake, 4, None, None, None) == EINVAL      # b > 8
    assert lib.imunpack_quantize(fake, 4, 4, 4, 1, 1.0, 1, fake, 4, None, None, None) == EINVAL      # b < 2
    assert lib.imunpack_quantize(fake, 4, 4, 4, 1, 0.0, 8, fake, 4, None, None, None) == EINVAL      # step 0
    assert lib.imunpack_quantize(fake, 4, 4, 4, 1, float("nan"), 8, fake, 4, None, None, None) == EINVAL
    assert lib.imunpack_quantize(fake, 4, 4, 4, 1, 1.0, 8, fake, 3, None, None, None) == EINVAL      # ldq < cols
    assert lib.imunpack_quantize(fake, -1, 4, 4, 1, 1.0, 8, fake, 4, None, None, None) == EINVAL
    assert lib.imunpack_quantize(fake, 4, 4, 0, 1, 1.0, 8, fake, 4, None, None, None) == EINVAL      # stride 0
    assert lib.imunpack_quantize(fake, 4, 4, 4, -1, 1.0, 8, fake, 4, None, None, None) == EINVAL     # negative stride
    lib.imunpack_quantize_pair.restype = ctypes.c_int
    lib.imunpack_quantize_pair.argtypes = [vp, i64, i64, i64, f32, vp, i64, vp, vp, i64, i64, i64, f32, vp, i64, vp, i64, i32, vp, vp]
    pair = lambda A=fake, n=4, sa_c=1, sc_a=1.0, QB=fake, ldqb=4, b=8: lib.imunpack_quantize_pair(
        A, n, 4, sa_c, sc_a, fake, 4, None, fake, 4, 4, 1, 1.0, QB, ldqb, None, 4, b, None, None)
    assert pair(A=None) == EINVAL and pair(QB=None) == EINVAL and pair(b=9) == EINVAL and pair(sc_a=0.0) == EINVAL
    assert pair(ldqb=3) == EINVAL and pair(n=-1) == EINVAL and pair(sa_c=0) == EINVAL
    lib.imunpack_scan.restype = ctypes.c_int
    lib.imunpack_scan.argtypes = [vp, i64, i64, i64, i32, vp, vp]
    assert lib.imunpack_scan(None, 4, 4, 4, 8, None, None) == EINVAL
    assert lib.imunpack_scan(fake, 4, 4, 3, 8, None, None) == EINVAL
    lib.imunpack_percentile.restype = ctypes.c_int
    lib.imunpack_percentile.argtypes = [vp, i64, i64, i64, i64, f64, vp, vp, vp, vp]
    for p in (0.0, -5.0, 100.0001, float("nan")):
        assert lib.imunpack_percentile(fake, 4, 4, 4, 1, p, fake, None, fake, None) == EINVAL
    assert lib.imunpack_percentile(fake, 0, 4, 4, 1, 95.0, fake, None, fake, None) == EINVAL         # empty
    assert lib.imunpack_percentile(fake, 4, 4, 0, 1, 95.0, fake, None, fake, None) == EINVAL         # stride 0
    assert lib.imunpack_percentile(fake, 1 << 20, 1 << 20, 1 << 20, 1, 95.0, fake, None, fake, None) == EINVAL  # >= 2^32
    assert lib.imunpack_percentile(fake, 4, 4, 4, 1, 95.0, fake, None, None, None) == EINVAL         # no workspace
    lib.imunpack_plan.restype = ctypes.c_int
    lib.imunpack_plan.argtypes = [vp, i64, i64, i64, vp, i64, i64, i32, i32, i32, vp, vp, vp, vp]
    handle = vp(None)
    ref = ctypes.byref(handle)
    assert lib.imunpack_plan(fake, 4, 4, 4, fake, 4, 4, 8, 3, 0, None, None, ref, None) == EINVAL    # unknown strategy
    assert lib.imunpack_plan(fake, 4, 4, 4, fake, 4, 4, 8, 0, -1, None, None, ref, None) == EINVAL
    assert lib.imunpack_plan(fake, 4, 4, 3, fake, 4, 4, 8, 0, 0, None, None, ref, None) == EINVAL    # lda < d
    assert lib.imunpack_plan(fake, 4, 4, 4, fake, 4, 4, 12, 0, 0, None, None, ref, None) == EINVAL   # b
    assert lib.imunpack_plan(fake, 1 << 25, 4, 4, fake, 4, 4, 8, 0, 0, None, None, ref, None) == EINVAL  # too many rows
    assert lib.imunpack_plan(fake, 4, 4, 4, fake, 4, 4, 8, 0, 0, None, None, None, None) == EINVAL   # nowhere to put the plan
    assert handle.value is None
    for name, nargs in (("imunpack_unpacked_bytes", 4), ("imunpack_unpack", 8), ("imunpack_unpack_canonical", 6),
                        ("imunpack_gemm", 11), ("imunpack_recombine", 8), ("imunpack_plan_export", 10),
                        ("imunpack_plan_bounds", 2), ("imunpack_plan_layout", 2), ("imunpack_plan_set_digits", 2),
                        ("imunpack_plan_keep_weights", 2)):
        fn = getattr(lib, name)
        fn.restype = ctypes.c_int
        fn.argtypes = None
        if name == "imunpack_gemm":
            args = [None, fake, fake, None, fake, fake, i64(4), f32(1.0), f32(1.0), i32(1), None]
        elif name == "imunpack_recombine":
            args = [None, fake, f32(1.0), f32(1.0), fake, fake, i64(4), None]
        else:
            args = [None] + [fake] * (nargs - 1)
        assert fn(*args) == EINVAL, name                                                             # no plan
    lib.imunpack_plan_fusable.restype = ctypes.c_int
    assert lib.imunpack_plan_fusable(None) == 0
    lib.imunpack_price.restype = ctypes.c_int
    lib.imunpack_price.argtypes = [vp, i64, vp, i64, i64, i32, vp, vp, vp, vp, vp, vp]
    assert lib.imunpack_price(None, 4, None, 4, 4, 8, fake, fake, fake, fake, fake, None) == EINVAL
    lib.imunpack_rtn_step.restype = ctypes.c_int
    lib.imunpack_rtn_step.argtypes = [vp, i64, i64, i64, i64, f64, f32, vp, vp, vp, vp]
    assert lib.imunpack_rtn_step(fake, 4, 4, 4, 1, 95.0, 0.0, fake, None, fake, None) == EINVAL      # beta 0
    assert lib.imunpack_rtn_step(fake, 4, 4, 4, 1, 95.0, 31.0, None, None, fake, None) == EINVAL     # nowhere to put the step
    lib.imunpack_gemm_batched.restype = ctypes.c_int
    lib.imunpack_gemm_batched.argtypes = [vp, i64, i64, i64, vp, i64, i64, i64, i64, i64, i64, i64, f64, f32, f32, i32, i32,
                                          i32, vp, i64, i64, vp, vp]
    bctx = vp(None)
    bref = ctypes.byref(bctx)
    assert lib.imunpack_gemm_batched(fake, 16, 4, 1, fake, 16, 4, 1, 2, 4, 4, 4, 95.0, 31.0, 31.0, 8, 0, 0, fake, 16, 3, bref, None) == EINVAL   # ldc < h
    assert lib.imunpack_gemm_batched(fake, 16, 4, 0, fake, 16, 4, 1, 2, 4, 4, 4, 95.0, 31.0, 31.0, 8, 0, 0, fake, 16, 4, bref, None) == EINVAL   # stride 0
    assert lib.imunpack_gemm_batched(fake, 16, 4, 1, fake, 16, 4, 1, 2, 4, 4, 4, 95.0, 31.0, 31.0, 8, 0, 5, fake, 16, 4, bref, None) == EINVAL   # strategy
    assert lib.imunpack_gemm_batched(fake, 16, 4, 1, fake, 16, 4, 1, 2, 4, 4, 4, 0.0, 31.0, 31.0, 8, 0, 0, fake, 16, 4, bref, None) == EINVAL    # p
    assert lib.imunpack_gemm_batched(fake, 16, 4, 1, fake, 16, 4, 1, 2, 4, 4, 4, 95.0, 31.0, 31.0, 8, 0, 0, fake, 16, 4, None, None) == EINVAL   # no context slot
    assert bctx.value is None
    lib.imunpack_batch_destroy.restype = ctypes.c_int
    assert lib.imunpack_batch_destroy(None) == 0
    lib.imunpack_diag_mfma_peak.restype = ctypes.c_int
    lib.imunpack_diag_mfma_peak.argtypes = [i32, i32, vp, vp]
    assert lib.imunpack_diag_mfma_peak(0, 10, None, None) == EINVAL
    assert lib.imunpack_diag_mfma_peak(10, 0, None, None) == EINVAL
    lib.imunpack_diag_copy.restype = ctypes.c_int
    lib.imunpack_diag_copy.argtypes = [vp, vp, ctypes.c_int64, vp]
    assert lib.imunpack_diag_copy(None, fake, 1 << 20, None) == EINVAL
    assert lib.imunpack_diag_copy(fake, fake, (1 << 20) + 16, None) == EINVAL    # not whole bands of 64 rows
    assert lib.imunpack_diag_copy(fake, fake, 0, None) == EINVAL


def test_layers_reject_operands_that_do_not_form_a_product():
    """The batched A B^T of the attention layer checks its shapes before anything reaches the library
    (runs without a GPU: the check comes first)."""
    import pytest
    import torch
    from paper_2403_07339_amd import attention, linear
    cfg = linear.QuantConfig()
    for a, b in (((2, 3, 8, 5), (2, 3, 7, 4)), ((2, 3, 8, 5), (3, 2, 7, 5)), ((8, 5), (1, 7, 5))):
        with pytest.raises(ValueError):
            attention.quantized_bmm(torch.zeros(a), torch.zeros(b), 31.0, 31.0, cfg)
    assert cfg.b == 8 and cfg.p == 95.0
