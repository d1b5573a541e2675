"""Thin ctypes binding of libimunpack.so: argument marshalling only.

Function names and argument order follow ``include/imunpack.h``.  PyTorch is used for device
memory and streams; every step of the path runs in the library's HIP kernels.  Importing this
module raises if the library has not been built (``python -m paper_2403_07339_amd.build``); there
is no CPU fallback.
"""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import torch

ROW, COL, BOTH = 0, 1, 2
OK, EINVAL, ERANGE, ENOMEM, EHIP, ESMALL = 0, -1, -2, -3, -4, -5

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("IMUNPACK_LIB") or os.path.join(_HERE, "libimunpack.so")
if not os.path.exists(LIB_PATH):
    raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2403_07339_amd.build`")
_lib = C.CDLL(LIB_PATH)

EXPORTS = [
    "imunpack_quantize", "imunpack_scan", "imunpack_plan", "imunpack_plan_dims", "imunpack_plan_export",
    "imunpack_plan_destroy", "imunpack_unpacked_bytes", "imunpack_unpack", "imunpack_unpack_canonical",
    "imunpack_gemm", "imunpack_recombine", "imunpack_strerror", "imunpack_last_hip_error",
    "imunpack_plan_fusable", "imunpack_plan_bounds", "imunpack_diag_mfma_peak", "imunpack_diag_clock_probe", "imunpack_diag_copy", "imunpack_price",
    "imunpack_percentile", "imunpack_percentile_static", "imunpack_plan_layout", "imunpack_rtn_step",
    "imunpack_gemm_batched", "imunpack_batch_destroy", "imunpack_quantize_pair", "imunpack_plan_set_digits",
    "imunpack_plan_digits", "imunpack_plan_keep_weights", "imunpack_plan_weights_reused",
]
DIGITS_INT8, DIGITS_FP6 = 0, 1


class _Stats(C.Structure):
    _fields_ = [("rowcnt", C.c_void_p), ("colcnt", C.c_void_p), ("rowmax", C.c_void_p), ("colmax", C.c_void_p),
                ("ob", C.c_void_p), ("ob_cap", C.c_int64), ("ob_count", C.c_void_p)]


_vp, _i64, _i32, _f32 = C.c_void_p, C.c_int64, C.c_int, C.c_float
_lib.imunpack_quantize.argtypes = [_vp, _i64, _i64, _i64, _i64, _f32, _i32, _vp, _i64, C.POINTER(_Stats), _vp, _vp]
_lib.imunpack_quantize_pair.argtypes = [_vp, _i64, _i64, _i64, _f32, _vp, _i64, C.POINTER(_Stats),
                                        _vp, _i64, _i64, _i64, _f32, _vp, _i64, C.POINTER(_Stats), _i64, _i32, _vp, _vp]
_lib.imunpack_scan.argtypes = [_vp, _i64, _i64, _i64, _i32, C.POINTER(_Stats), _vp]
_lib.imunpack_plan.argtypes = [_vp, _i64, _i64, _i64, _vp, _i64, _i64, _i32, _i32, _i32,
                               C.POINTER(_Stats), C.POINTER(_Stats), C.POINTER(_vp), _vp]
_lib.imunpack_plan_dims.argtypes = [_vp, C.POINTER(_i64), C.POINTER(_i64), C.POINTER(_i64), C.POINTER(C.c_int32)]
_lib.imunpack_plan_export.argtypes = [_vp] + [_vp] * 8 + [C.POINTER(_i64)]
_lib.imunpack_plan_destroy.argtypes = [_vp]
_lib.imunpack_unpacked_bytes.argtypes = [_vp, C.POINTER(C.c_size_t), C.POINTER(C.c_size_t), C.POINTER(C.c_size_t)]
_lib.imunpack_rtn_step.argtypes = [_vp, _i64, _i64, _i64, _i64, C.c_double, _f32, _vp, _vp, _vp, _vp]
_lib.imunpack_gemm_batched.argtypes = [_vp, _i64, _i64, _i64, _vp, _i64, _i64, _i64, _i64, _i64, _i64, _i64, C.c_double,
                                       _f32, _f32, _i32, _i32, _i32, _vp, _i64, _i64, C.POINTER(_vp), _vp]
_lib.imunpack_batch_destroy.argtypes = [_vp]
_lib.imunpack_plan_layout.argtypes = [_vp, C.POINTER(_i64)]
_lib.imunpack_plan_set_digits.argtypes = [_vp, _i32]
_lib.imunpack_plan_digits.argtypes = [_vp]
_lib.imunpack_plan_keep_weights.argtypes = [_vp, _i32]
_lib.imunpack_plan_weights_reused.argtypes = [_vp]
_lib.imunpack_unpack.argtypes = [_vp, _vp, _i64, _vp, _i64, _vp, _vp, _vp]
_lib.imunpack_unpack_canonical.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp]
_lib.imunpack_gemm.argtypes = [_vp, _vp, _vp, _vp, _vp, _vp, _i64, _f32, _f32, _i32, _vp]
_lib.imunpack_recombine.argtypes = [_vp, _vp, _f32, _f32, _vp, _vp, _i64, _vp]
_lib.imunpack_strerror.argtypes = [_i32]
_lib.imunpack_strerror.restype = C.c_char_p
_lib.imunpack_plan_fusable.argtypes = [_vp]
_lib.imunpack_percentile.argtypes = [_vp, _i64, _i64, _i64, _i64, C.c_double, _vp, _vp, _vp, _vp]
_lib.imunpack_percentile_static.argtypes = [_vp, _i64, _i64, _i64, _i64, C.c_double, _vp, _vp, _vp]
_lib.imunpack_plan_bounds.argtypes = [_vp, C.POINTER(C.c_uint64)]
_lib.imunpack_diag_mfma_peak.argtypes = [_i32, _i32, C.POINTER(_i64), _vp]
_lib.imunpack_diag_clock_probe.argtypes = [_vp]
_lib.imunpack_diag_copy.argtypes = [_vp, _vp, _i64, _vp]
_lib.imunpack_price.argtypes = [C.POINTER(_Stats), _i64, C.POINTER(_Stats), _i64, _i64, _i32, _vp, C.POINTER(_i64),
                                C.POINTER(C.c_double), C.POINTER(_i32), C.POINTER(_i32), _vp]
for _name in EXPORTS:
    if _name != "imunpack_strerror":
        getattr(_lib, _name).restype = C.c_int


class ImunpackError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _lib.imunpack_strerror(code).decode()
        if code == EHIP:
            msg += f" (hipError {_lib.imunpack_last_hip_error()})"
        super().__init__(f"{where}: {msg} [{code}]")


def _check(code: int, where: str):
    if code != OK:
        raise ImunpackError(code, where)


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t):
    return None if t is None else t.data_ptr()


@dataclass
class Stats:
    """OB count and largest magnitude per row and per column of an integer operand (device int32)."""
    rowcnt: torch.Tensor
    colcnt: torch.Tensor
    rowmax: torch.Tensor
    colmax: torch.Tensor
    ob: torch.Tensor | None = None        # [3, ob_cap] int32: rows | cols | values of the OB entries
    ob_count: torch.Tensor | None = None  # [1] int32

    @staticmethod
    def empty(rows: int, cols: int, device, ob_cap: int = 0) -> "Stats":
        """ob_cap > 0 also allocates the OB entry list that UnpackBoth plans from."""
        buf = torch.empty(2 * (rows + cols), dtype=torch.int32, device=device)
        st = Stats(buf[:rows], buf[rows:rows + cols], buf[rows + cols:2 * rows + cols], buf[2 * rows + cols:])
        if ob_cap > 0:
            st.ob = torch.empty((3, ob_cap), dtype=torch.int32, device=device)
            st.ob_count = torch.zeros(1, dtype=torch.int32, device=device)
        return st

    @staticmethod
    def default_ob_cap(rows: int, cols: int) -> int:
        return max(4096, rows * cols // 64)

    def _c(self) -> _Stats:
        return _Stats(self.rowcnt.data_ptr(), self.colcnt.data_ptr(), self.rowmax.data_ptr(), self.colmax.data_ptr(),
                      self.ob.data_ptr() if self.ob is not None else None,
                      self.ob.shape[1] if self.ob is not None else 0,
                      self.ob_count.data_ptr() if self.ob_count is not None else None)


PERCENTILE_WORKSPACE_BYTES = 16384


def imunpack_percentile(X: torch.Tensor, p: float, alpha: torch.Tensor | None = None,
                        status: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """alpha_p(X): the p-th percentile of the magnitudes of X (the k-th smallest |x|, k = ceil(p N / 100)).
    X: 2-D fp32 device tensor, any positive strides.  Returns (alpha, status), one-element device tensors."""
    assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
    if alpha is None:
        alpha = torch.empty(1, dtype=torch.float32, device=X.device)
    if status is None:
        status = torch.empty(1, dtype=torch.int32, device=X.device)
    if workspace is None:
        workspace = torch.empty(PERCENTILE_WORKSPACE_BYTES, dtype=torch.uint8, device=X.device)
    assert workspace.numel() * workspace.element_size() >= PERCENTILE_WORKSPACE_BYTES
    _check(_lib.imunpack_percentile(X.data_ptr(), X.shape[0], X.shape[1], X.stride(0), X.stride(1), float(p),
                                    alpha.data_ptr(), status.data_ptr(), workspace.data_ptr(), _stream()),
           "imunpack_percentile")
    return alpha, status


def imunpack_percentile_static(X: torch.Tensor, p: float, alpha: torch.Tensor, status: torch.Tensor | None = None):
    """imunpack_percentile on the library's own fixed scratch array: the call allocates nothing, so the
    caller passes the one-element outputs.  Returns (alpha, status)."""
    assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
    assert alpha.is_cuda and alpha.dtype == torch.float32 and alpha.numel() >= 1
    _check(_lib.imunpack_percentile_static(X.data_ptr(), X.shape[0], X.shape[1], X.stride(0), X.stride(1), float(p),
                                           alpha.data_ptr(), _ptr(status), _stream()),
           "imunpack_percentile_static")
    return alpha, status


def imunpack_quantize(X: torch.Tensor, scale: float, b: int, Q: torch.Tensor | None = None,
                      stats: Stats | None = None, status: torch.Tensor | None = None,
                      want_stats: bool = True, want_ob_list: bool = False):
    """Q = rint(X / scale) (int32, row-major) fused with the heavy-hitter scan.  X: 2-D fp32 device
    tensor, any strides.  Returns (Q, stats, status)."""
    assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
    rows, cols = X.shape
    if Q is None:
        Q = torch.empty((rows, cols), dtype=torch.int32, device=X.device)
    if stats is None and want_stats:
        stats = Stats.empty(rows, cols, X.device, Stats.default_ob_cap(rows, cols) if want_ob_list else 0)
    if status is None:
        status = torch.empty(1, dtype=torch.int32, device=X.device)
    cs = stats._c() if stats is not None else None
    _check(_lib.imunpack_quantize(X.data_ptr(), rows, cols, X.stride(0), X.stride(1), float(scale), b,
                                  Q.data_ptr(), Q.stride(0), C.byref(cs) if cs else None,
                                  status.data_ptr(), _stream()), "imunpack_quantize")
    return Q, stats, status


def imunpack_quantize_pair(A: torch.Tensor, B: torch.Tensor, scale_a: float, scale_b: float, b: int,
                           Qa: torch.Tensor | None = None, Qb: torch.Tensor | None = None,
                           stats_a: Stats | None = None, stats_b: Stats | None = None,
                           status: torch.Tensor | None = None, want_ob_list=(False, False)):
    """imunpack_quantize for both operands of A B^T (A: n x d, B: h x d) with fewer launches.
    Returns (Qa, Qb, stats_a, stats_b, status) with status[0] for A and status[1] for B."""
    assert A.is_cuda and B.is_cuda and A.dtype == torch.float32 and B.dtype == torch.float32
    assert A.dim() == 2 and B.dim() == 2 and A.shape[1] == B.shape[1]
    (n, d), h = A.shape, B.shape[0]
    if Qa is None:
        Qa = torch.empty((n, d), dtype=torch.int32, device=A.device)
    if Qb is None:
        Qb = torch.empty((h, d), dtype=torch.int32, device=A.device)
    if stats_a is None:
        stats_a = Stats.empty(n, d, A.device, Stats.default_ob_cap(n, d) if want_ob_list[0] else 0)
    if stats_b is None:
        stats_b = Stats.empty(h, d, A.device, Stats.default_ob_cap(h, d) if want_ob_list[1] else 0)
    if status is None:
        status = torch.empty(2, dtype=torch.int32, device=A.device)
    ca, cb = stats_a._c(), stats_b._c()
    _check(_lib.imunpack_quantize_pair(A.data_ptr(), n, A.stride(0), A.stride(1), float(scale_a), Qa.data_ptr(), Qa.stride(0),
                                       C.byref(ca), B.data_ptr(), h, B.stride(0), B.stride(1), float(scale_b), Qb.data_ptr(),
                                       Qb.stride(0), C.byref(cb), d, b, status.data_ptr(), _stream()),
           "imunpack_quantize_pair")
    return Qa, Qb, stats_a, stats_b, status


def imunpack_scan(Q: torch.Tensor, b: int, stats: Stats | None = None) -> Stats:
    assert Q.is_cuda and Q.dtype == torch.int32 and Q.dim() == 2 and Q.stride(1) == 1
    rows, cols = Q.shape
    if stats is None:
        stats = Stats.empty(rows, cols, Q.device)
    cs = stats._c()
    _check(_lib.imunpack_scan(Q.data_ptr(), rows, cols, Q.stride(0), b, C.byref(cs), _stream()), "imunpack_scan")
    return stats


class Plan:
    """Owns an imunpack_plan_t; re-planning through the same object reuses its device buffers."""

    def __init__(self):
        self._h = _vp(None)
        self.n = self.d = self.h = 0

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def destroy(self):
        if self._h and self._h.value:
            _lib.imunpack_plan_destroy(self._h)
            self._h = _vp(None)

    @property
    def handle(self):
        return self._h

    def dims(self):
        n_u, d_u, h_u, ng = _i64(), _i64(), _i64(), C.c_int32()
        _check(_lib.imunpack_plan_dims(self._h, C.byref(n_u), C.byref(d_u), C.byref(h_u), C.byref(ng)),
               "imunpack_plan_dims")
        return n_u.value, d_u.value, h_u.value, ng.value

    def unpack_ratio(self) -> float:
        n_u, d_u, h_u, _ = self.dims()
        return (n_u * d_u * h_u) / (self.n * self.d * self.h)

    def export(self):
        """Canonical plan as host int32 tensors: rowA_src, rowA_exp, rowB_src, rowB_exp, col_src, col_exp."""
        return self.export_all()[:6]

    def export_all(self):
        """export() plus col_parent (d') and the sequence of splits, one row (call, kind, index) each."""
        n_u, d_u, h_u, _ = self.dims()
        n_ops = (n_u - self.n) + (h_u - self.h) + (d_u - self.d)
        outs = [torch.empty(k, dtype=torch.int32) for k in (n_u, n_u, h_u, h_u, d_u, d_u, d_u)]
        ops = torch.empty((n_ops, 3), dtype=torch.int32)
        got = _i64(-1)
        _check(_lib.imunpack_plan_export(self._h, *[o.data_ptr() for o in outs], ops.data_ptr(), C.byref(got)),
               "imunpack_plan_export")
        assert got.value == n_ops
        return outs + [ops]

    def unpacked_bytes(self):
        a, b_, w = C.c_size_t(), C.c_size_t(), C.c_size_t()
        _check(_lib.imunpack_unpacked_bytes(self._h, C.byref(a), C.byref(b_), C.byref(w)), "imunpack_unpacked_bytes")
        return a.value, b_.value, w.value

    def set_digits(self, fmt: int):
        """DIGITS_INT8 or DIGITS_FP6 (b <= 4): the storage format of the digits from the next unpack on."""
        _check(_lib.imunpack_plan_set_digits(self._h, int(fmt)), "imunpack_plan_set_digits")

    def digits(self) -> int:
        return int(_lib.imunpack_plan_digits(self._h))

    def keep_weights(self, keep: bool = True):
        """Promise that B (integers, statistics, OB list) is the same in every later plan on this object."""
        _check(_lib.imunpack_plan_keep_weights(self._h, 1 if keep else 0), "imunpack_plan_keep_weights")

    def weights_reused(self) -> bool:
        return bool(_lib.imunpack_plan_weights_reused(self._h))

    def layout(self):
        """((rows, stored columns, row pitch in bytes) of the A store, the same of B_eu)."""
        v = (_i64 * 6)()
        _check(_lib.imunpack_plan_layout(self._h, v), "imunpack_plan_layout")
        return (int(v[0]), int(v[1]), int(v[2])), (int(v[3]), int(v[4]), int(v[5]))

    def fusable(self) -> bool:
        return bool(_lib.imunpack_plan_fusable(self._h))

    def bounds(self):
        """(bound_A, bound_B): the largest weighted L1 row norm of A_ue and of B_eu that the last unpack measured."""
        out = (C.c_uint64 * 2)()
        _check(_lib.imunpack_plan_bounds(self._h, out), "imunpack_plan_bounds")
        return int(out[0]), int(out[1])


def imunpack_plan(A: torch.Tensor, B: torch.Tensor, b: int, strategy_a: int, strategy_b: int,
                  stats_a: Stats | None = None, stats_b: Stats | None = None, plan: Plan | None = None) -> Plan:
    """Plans Unpack(A, B, I, b, strategy_a) then Unpack(B_e, A_u, S_u, b, strategy_b).  A: n x d, B: h x d int32."""
    assert A.is_cuda and B.is_cuda and A.dtype == torch.int32 and B.dtype == torch.int32
    assert A.stride(1) == 1 and B.stride(1) == 1 and A.shape[1] == B.shape[1]
    if plan is None:
        plan = Plan()
    ca = stats_a._c() if stats_a is not None else None
    cb = stats_b._c() if stats_b is not None else None
    _check(_lib.imunpack_plan(A.data_ptr(), A.shape[0], A.shape[1], A.stride(0), B.data_ptr(), B.shape[0],
                              B.stride(0), b, strategy_a, strategy_b, C.byref(ca) if ca else None,
                              C.byref(cb) if cb else None, C.byref(plan._h), _stream()), "imunpack_plan")
    plan.n, plan.d, plan.h = A.shape[0], A.shape[1], B.shape[0]
    return plan


def imunpack_unpack(plan: Plan, A: torch.Tensor, B: torch.Tensor, A_ue: torch.Tensor | None = None,
                    B_eu: torch.Tensor | None = None):
    """Writes the int8 operands in the plan's physical layout; returns (A_ue, B_eu) as flat int8 buffers."""
    ba, bb, _ = plan.unpacked_bytes()
    if A_ue is None:
        A_ue = torch.empty(ba, dtype=torch.int8, device=A.device)
    if B_eu is None:
        B_eu = torch.empty(bb, dtype=torch.int8, device=A.device)
    assert A_ue.numel() >= ba and B_eu.numel() >= bb
    _check(_lib.imunpack_unpack(plan.handle, A.data_ptr(), A.stride(0), B.data_ptr(), B.stride(0),
                                A_ue.data_ptr(), B_eu.data_ptr(), _stream()), "imunpack_unpack")
    return A_ue, B_eu


def imunpack_unpack_canonical(plan: Plan, A_ue: torch.Tensor, B_eu: torch.Tensor):
    """Test aid: the unpacked operands in the paper's order, dense (n' x d', h' x d') int8."""
    n_u, d_u, h_u, _ = plan.dims()
    Ac = torch.empty((n_u, d_u), dtype=torch.int8, device=A_ue.device)
    Bc = torch.empty((h_u, d_u), dtype=torch.int8, device=A_ue.device)
    _check(_lib.imunpack_unpack_canonical(plan.handle, A_ue.data_ptr(), B_eu.data_ptr(), Ac.data_ptr(),
                                          Bc.data_ptr(), _stream()), "imunpack_unpack_canonical")
    return Ac, Bc


def imunpack_gemm(plan: Plan, A_ue: torch.Tensor, B_eu: torch.Tensor, scale_a: float, scale_b: float,
                  C_int: torch.Tensor | None = None, C_fp: torch.Tensor | None = None,
                  workspace: torch.Tensor | None = None, fuse: bool = True):
    """int8 MFMA GEMM; with fuse=True also recombines and dequantises into C_int / C_fp."""
    ldc = 0
    for t in (C_int, C_fp):
        if t is not None:
            assert t.stride(1) == 1
            ldc = t.stride(0)
    if C_int is not None and C_fp is not None:
        assert C_int.stride(0) == C_fp.stride(0)
    _check(_lib.imunpack_gemm(plan.handle, A_ue.data_ptr(), B_eu.data_ptr(), _ptr(workspace), _ptr(C_int),
                              _ptr(C_fp), ldc, float(scale_a), float(scale_b), 1 if fuse else 0, _stream()),
           "imunpack_gemm")


def imunpack_recombine(plan: Plan, workspace: torch.Tensor, scale_a: float, scale_b: float,
                       C_int: torch.Tensor | None = None, C_fp: torch.Tensor | None = None):
    ldc = 0
    for t in (C_int, C_fp):
        if t is not None:
            ldc = t.stride(0)
    _check(_lib.imunpack_recombine(plan.handle, workspace.data_ptr(), float(scale_a), float(scale_b),
                                   _ptr(C_int), _ptr(C_fp), ldc, _stream()), "imunpack_recombine")


def exact_int_gemm(A_fp: torch.Tensor, B_fp: torch.Tensor, scale_a: float, scale_b: float, b: int,
                   strategy_a: int, strategy_b: int, want_int: bool = True, want_fp: bool = True,
                   plan: Plan | None = None, fuse: bool = True):
    """The whole hot path: quantize -> plan -> unpack -> GEMM (+ recombine, dequantise).
    Returns (C_int or None, C_fp or None, plan)."""
    dev = A_fp.device
    Aq, Bq, sa, sb, st = imunpack_quantize_pair(A_fp, B_fp, scale_a, scale_b, b,
                                                want_ob_list=(strategy_a == BOTH, strategy_b == BOTH))
    plan = imunpack_plan(Aq, Bq, b, strategy_a, strategy_b, sa, sb, plan)
    A_ue, B_eu = imunpack_unpack(plan, Aq, Bq)
    n, h = A_fp.shape[0], B_fp.shape[0]
    C_int = torch.empty((n, h), dtype=torch.int64, device=dev) if want_int else None
    C_fp = torch.empty((n, h), dtype=torch.float32, device=dev) if want_fp else None
    ws = None
    if not fuse or not plan.fusable():
        ws = torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device=dev)
    if fuse:
        imunpack_gemm(plan, A_ue, B_eu, scale_a, scale_b, C_int, C_fp, ws, fuse=True)
    else:
        imunpack_gemm(plan, A_ue, B_eu, scale_a, scale_b, None, None, ws, fuse=False)
        imunpack_recombine(plan, ws, scale_a, scale_b, C_int, C_fp)
    if int(st.amax().item()):
        raise ImunpackError(ERANGE, "imunpack_quantize status")
    return C_int, C_fp, plan


def imunpack_rtn_step(X: torch.Tensor, p: float, beta: float, step: torch.Tensor | None = None,
                      status: torch.Tensor | None = None, workspace: torch.Tensor | None = None):
    """The RTN step alpha_p(X) / (0.5 beta) of Eq. (quantized_A), formed on the device.  Returns (step, status),
    one-element device tensors; nothing is read back."""
    assert X.is_cuda and X.dtype == torch.float32 and X.dim() == 2
    if step is None:
        step = torch.empty(1, dtype=torch.float32, device=X.device)
    if status is None:
        status = torch.empty(1, dtype=torch.int32, device=X.device)
    if workspace is None:
        workspace = torch.empty(PERCENTILE_WORKSPACE_BYTES, dtype=torch.uint8, device=X.device)
    _check(_lib.imunpack_rtn_step(X.data_ptr(), X.shape[0], X.shape[1], X.stride(0), X.stride(1), float(p), float(beta),
                                  step.data_ptr(), status.data_ptr(), workspace.data_ptr(), _stream()), "imunpack_rtn_step")
    return step, status


class BatchContext:
    """Owns an imunpack_batch_t: the buffers that imunpack_gemm_batched reuses from call to call."""

    def __init__(self):
        self._h = _vp(None)

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass

    def destroy(self):
        if self._h and self._h.value:
            _lib.imunpack_batch_destroy(self._h)
            self._h = _vp(None)


def _as_batch(t: torch.Tensor):
    """[..., rows, cols] as (base tensor, batch count, batch stride) when the leading dimensions collapse
    into one stride (they do for contiguous tensors and their transposes), else None."""
    lead = t.shape[:-2]
    count = 1
    for s_ in lead:
        count *= s_
    if count <= 1:
        return count, 0
    stride = None
    expect = None
    for size, st in zip(reversed(lead), reversed(t.stride()[:-2])):
        if size == 1:
            continue
        if stride is None:
            stride, expect = st, st * size
        elif st != expect:
            return None
        else:
            expect = st * size
    return count, stride


def imunpack_gemm_batched(A: torch.Tensor, B: torch.Tensor, p: float, beta_a: float, beta_b: float, b: int,
                          strategy_a: int, strategy_b: int, out: torch.Tensor | None = None,
                          ctx: BatchContext | None = None) -> torch.Tensor:
    """A B^T over the leading dimensions on the exact integer path: A [..., n, d], B [..., h, d] fp32 device
    tensors with equal leading shapes and any strides (transposed views are passed as they are); every
    matrix pair is quantised with its own percentile steps.  Returns [..., n, h] fp32."""
    assert A.is_cuda and B.is_cuda and A.dtype == torch.float32 and B.dtype == torch.float32
    assert A.dim() >= 2 and A.shape[:-2] == B.shape[:-2] and A.shape[-1] == B.shape[-1]
    n, d, h = A.shape[-2], A.shape[-1], B.shape[-2]
    if out is None:
        out = torch.empty(*A.shape[:-2], n, h, dtype=torch.float32, device=A.device)
    assert out.is_contiguous() and out.shape == (*A.shape[:-2], n, h)
    ba, bb = _as_batch(A), _as_batch(B)
    if ba is None or bb is None:   # leading dimensions that do not collapse: one call per leading index
        for i in range(A.shape[0]):
            imunpack_gemm_batched(A[i], B[i], p, beta_a, beta_b, b, strategy_a, strategy_b, out[i], ctx)
        return out
    if ctx is None:
        ctx = _default_batch_context()
    _check(_lib.imunpack_gemm_batched(A.data_ptr(), ba[1], A.stride(-2), A.stride(-1), B.data_ptr(), bb[1], B.stride(-2),
                                      B.stride(-1), ba[0], n, d, h, float(p), float(beta_a), float(beta_b), b, strategy_a,
                                      strategy_b, out.data_ptr(), n * h, h, C.byref(ctx._h), _stream()),
           "imunpack_gemm_batched")
    return out


_BATCH_CTX = None


def _default_batch_context() -> BatchContext:
    global _BATCH_CTX
    if _BATCH_CTX is None:
        _BATCH_CTX = BatchContext()
    return _BATCH_CTX


def imunpack_diag_mfma_peak(workgroups: int, iters: int) -> int:
    """Launches the register-resident int8 MFMA loop on the current stream; returns the integer
    operations it performs (the caller times the stream)."""
    ops = _i64(0)
    _check(_lib.imunpack_diag_mfma_peak(int(workgroups), int(iters), C.byref(ops), _stream()), "imunpack_diag_mfma_peak")
    return int(ops.value)


def imunpack_diag_copy(src: torch.Tensor, dst: torch.Tensor) -> int:
    """Streams src to dst (contiguous device tensors of equal byte size, a multiple of 1 MiB) with the
    library's copy kernel on the current stream; returns the bytes moved (read + written)."""
    assert src.is_cuda and dst.is_cuda and src.is_contiguous() and dst.is_contiguous()
    nbytes = src.numel() * src.element_size()
    assert nbytes == dst.numel() * dst.element_size()
    _check(_lib.imunpack_diag_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream()), "imunpack_diag_copy")
    return 2 * nbytes


def imunpack_diag_clock_probe(ticks: torch.Tensor | None) -> None:
    """ticks: two int64 on the device that the first workgroup of every later fused GEMM launch fills
    with {shader clock cycles, 100 MHz ticks} of its loop over K; None switches the probe off."""
    if ticks is not None:
        assert ticks.is_cuda and ticks.dtype == torch.int64 and ticks.is_contiguous() and ticks.numel() >= 2
    _check(_lib.imunpack_diag_clock_probe(_ptr(ticks)), "imunpack_diag_clock_probe")


PRICE_WORKSPACE_BYTES = 64


def imunpack_price(stats_a: Stats, n: int, stats_b: Stats, h: int, d: int, b: int,
                   workspace: torch.Tensor | None = None):
    """Prices the four pairs of one-axis strategies from the scan statistics (no unpacking).  Returns
    (dims, ratios, best): dims[(sA, sB)] = (n', d', h'), ratios[(sA, sB)] = r, best = the pair with
    the smallest r."""
    dims = (_i64 * 12)()
    ratios = (C.c_double * 4)()
    ba, bb = _i32(0), _i32(0)
    ca, cb = stats_a._c(), stats_b._c()
    if workspace is None:
        workspace = torch.empty(PRICE_WORKSPACE_BYTES // 8, dtype=torch.int64, device=stats_a.rowmax.device)
    _check(_lib.imunpack_price(C.byref(ca), n, C.byref(cb), h, d, b, workspace.data_ptr(), dims, ratios, C.byref(ba), C.byref(bb),
                               _stream()), "imunpack_price")
    pairs = [(ROW, ROW), (ROW, COL), (COL, ROW), (COL, COL)]
    return ({p: tuple(int(dims[3 * q + c]) for c in range(3)) for q, p in enumerate(pairs)},
            {p: float(ratios[q]) for q, p in enumerate(pairs)}, (int(ba.value), int(bb.value)))
