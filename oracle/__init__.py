"""IM-Unpack CPU oracle (test infrastructure, not product code).

ctypes front end of ``imunpack_oracle.c``: a plain CPU implementation of the
exact low-bit integer GEMM of arXiv 2403.07339 (RTN quantisation of Sec. 2,
Algorithms 1-5 and the Pi / S bookkeeping of Sec. 4).  Only ``tests/``, the
smoke check and the ``cpu_baseline`` leg of ``bench.py`` may import this
package.  It shares nothing with the HIP library.
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess
from dataclasses import dataclass

import numpy as np

ROW, COL, BOTH = 0, 1, 2

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "imunpack_oracle.c")
_LIB = os.path.join(_HERE, "liboracle.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (no fast-math, no FMA contraction)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fno-fast-math", "-ffp-contract=off",
               "-fPIC", "-shared", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def lib():
    global _lib
    if _lib is None:
        L = C.CDLL(build())
        i32p, i64p, f32p, f64p, i8p = (C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                                       C.POINTER(C.c_float), C.POINTER(C.c_double),
                                       C.POINTER(C.c_int8))
        L.orc_rtn_quantize.argtypes = [f32p, C.c_int64, C.c_float, i32p]
        L.orc_rtn_quantize.restype = C.c_int
        L.orc_int_gemm.argtypes = [i32p, C.c_int64, C.c_int64, i32p, C.c_int64, i64p]
        L.orc_int_gemm.restype = None
        L.orc_int_gemm_at.argtypes = [i32p, C.c_int64, i32p, i64p, i64p, C.c_int64, i64p]
        L.orc_int_gemm_at.restype = None
        L.orc_dequantize.argtypes = [i64p, C.c_int64, C.c_float, C.c_float, f64p]
        L.orc_dequantize.restype = None
        L.orc_num_threads.restype = C.c_int
        L.orc_digit.argtypes = [C.c_int32, C.c_int32, C.c_int]
        L.orc_digit.restype = C.c_int32
        L.orc_unpack.argtypes = [i32p, C.c_int64, C.c_int64, i32p, C.c_int64, i64p,
                                 C.c_int, C.c_int, C.c_int]
        L.orc_unpack.restype = C.c_void_p
        L.orc_unpack_pair.argtypes = [i32p, C.c_int64, C.c_int64, i32p, C.c_int64,
                                      C.c_int, C.c_int, C.c_int, C.c_int]
        L.orc_unpack_pair.restype = C.c_void_p
        L.orc_result_dims.argtypes = [C.c_void_p, i64p, i64p, i64p]
        L.orc_result_dims.restype = None
        L.orc_result_copy.argtypes = [C.c_void_p, i32p, i32p, i64p, i64p, i64p, i64p, i64p]
        L.orc_result_copy.restype = None
        L.orc_result_copy_i8.argtypes = [C.c_void_p, i8p, i8p]
        L.orc_result_copy_i8.restype = None
        L.orc_result_copy_meta.argtypes = [C.c_void_p, i64p, i64p, i64p, i64p, i64p]
        L.orc_result_copy_meta.restype = None
        L.orc_result_num_ops.argtypes = [C.c_void_p]
        L.orc_result_num_ops.restype = C.c_int64
        L.orc_result_copy_trace.argtypes = [C.c_void_p, i64p, i64p]
        L.orc_result_copy_trace.restype = None
        L.orc_result_max_abs.argtypes = [C.c_void_p]
        L.orc_result_max_abs.restype = C.c_int32
        L.orc_result_free.argtypes = [C.c_void_p]
        L.orc_result_free.restype = None
        L.orc_scaled_matmul.argtypes = [i32p, C.c_int64, C.c_int64, i32p, C.c_int64, i64p, i64p]
        L.orc_scaled_matmul.restype = None
        L.orc_apply_pi.argtypes = [i64p, C.c_int64, C.c_int64, i64p, i64p, i64p, i64p,
                                   C.c_int64, C.c_int64, i64p]
        L.orc_apply_pi.restype = None
        L.orc_unpacked_product_at.argtypes = [C.c_void_p, i64p, i64p, C.c_int64, i64p]
        L.orc_unpacked_product_at.restype = None
        _lib = L
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


# ---------------------------------------------------------------- Sec. 2
def rtn_quantize(x: np.ndarray, scale) -> tuple[np.ndarray, int]:
    """A_q = round(x / scale), element by element (Sec. 2, Eq. quantized_A). Returns (q, status)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    q = np.empty(x.shape, dtype=np.int32)
    st = lib().orc_rtn_quantize(_p(x, C.c_float), x.size, C.c_float(float(np.float32(scale))),
                                _p(q, C.c_int32))
    return q, int(st)


def int_gemm(A: np.ndarray, B: np.ndarray) -> np.ndarray:
    """C = A B^T in int64 by the triple loop (Sec. 1, Eq. gemm). A: n x d, B: h x d."""
    A, B = _i32(A), _i32(B)
    n, d = A.shape
    h, d2 = B.shape
    assert d == d2
    Cm = np.empty((n, h), dtype=np.int64)
    lib().orc_int_gemm(_p(A, C.c_int32), n, d, _p(B, C.c_int32), h, _p(Cm, C.c_int64))
    return Cm


def int_gemm_at(A: np.ndarray, B: np.ndarray, rows, cols) -> np.ndarray:
    """The same dot products at the listed (row, col) output positions only."""
    A, B = _i32(A), _i32(B)
    rows, cols = _i64(rows), _i64(cols)
    out = np.empty(rows.shape, dtype=np.int64)
    lib().orc_int_gemm_at(_p(A, C.c_int32), A.shape[1], _p(B, C.c_int32),
                          _p(rows, C.c_int64), _p(cols, C.c_int64), rows.size, _p(out, C.c_int64))
    return out


def dequantize(Cm: np.ndarray, scale_a, scale_b) -> np.ndarray:
    """C_fp = scale_a * scale_b * C_int in binary64 (Sec. 2, Eq. quantized_gemm)."""
    Cm = _i64(Cm)
    out = np.empty(Cm.shape, dtype=np.float64)
    lib().orc_dequantize(_p(Cm, C.c_int64), Cm.size, C.c_float(float(np.float32(scale_a))),
                         C.c_float(float(np.float32(scale_b))), _p(out, C.c_double))
    return out


def num_threads() -> int:
    return int(lib().orc_num_threads())


# ---------------------------------------------------------------- Sec. 4
def digit(v: int, s: int, i: int) -> int:
    """m(v, s, i) of Eq. (mod)."""
    return int(lib().orc_digit(int(v), int(s), int(i)))


@dataclass
class Unpacked:
    """A_ue (n' x d'), B_eu (h' x d'), diag(S_uu) (d'), Pi_A and Pi_B as (source row, weight) per column."""
    A: np.ndarray
    B: np.ndarray
    S: np.ndarray
    piA_src: np.ndarray
    piA_w: np.ndarray
    piB_src: np.ndarray
    piB_w: np.ndarray


class UnpackHandle:
    """Owns a C-side result; lets large results be inspected without dense int32 copies."""

    def __init__(self, ptr):
        self._ptr = ptr
        n_u, d_u, h_u = C.c_int64(), C.c_int64(), C.c_int64()
        lib().orc_result_dims(ptr, C.byref(n_u), C.byref(d_u), C.byref(h_u))
        self.n_u, self.d_u, self.h_u = n_u.value, d_u.value, h_u.value

    def dense(self) -> Unpacked:
        A = np.empty((self.n_u, self.d_u), dtype=np.int32)
        B = np.empty((self.h_u, self.d_u), dtype=np.int32)
        S, pas, paw, pbs, pbw = self._meta_arrays()
        lib().orc_result_copy(self._ptr, _p(A, C.c_int32), _p(B, C.c_int32), _p(S, C.c_int64),
                              _p(pas, C.c_int64), _p(paw, C.c_int64), _p(pbs, C.c_int64),
                              _p(pbw, C.c_int64))
        return Unpacked(A, B, S, pas, paw, pbs, pbw)

    def _meta_arrays(self):
        return (np.empty(self.d_u, dtype=np.int64), np.empty(self.n_u, dtype=np.int64),
                np.empty(self.n_u, dtype=np.int64), np.empty(self.h_u, dtype=np.int64),
                np.empty(self.h_u, dtype=np.int64))

    def meta(self):
        """(S, piA_src, piA_w, piB_src, piB_w) without the operands."""
        S, pas, paw, pbs, pbw = self._meta_arrays()
        lib().orc_result_copy_meta(self._ptr, _p(S, C.c_int64), _p(pas, C.c_int64),
                                   _p(paw, C.c_int64), _p(pbs, C.c_int64), _p(pbw, C.c_int64))
        return S, pas, paw, pbs, pbw

    def trace(self):
        """(col_parent, ops): col_parent[c] = the column that column c was appended for (-1 for the d
        columns the first Unpack call started from); ops = one row (call, kind, index) per split in the
        order they were made: call 0 / 1 = the first / second Unpack of Sec. 4 'Combining everything',
        kind 0 = a row split (Alg. 1 l.4-6, Alg. 4 l.7-9), 1 = a column split (Alg. 2 l.4-7, Alg. 4
        l.11-14), index = the split row / column at that moment."""
        col_parent = np.empty(self.d_u, dtype=np.int64)
        ops = np.empty((int(lib().orc_result_num_ops(self._ptr)), 3), dtype=np.int64)
        lib().orc_result_copy_trace(self._ptr, _p(col_parent, C.c_int64), _p(ops, C.c_int64))
        return col_parent, ops

    def col_src(self):
        """The original column each unpacked column descends from (col_parent followed to its root)."""
        parent, _ = self.trace()
        src = np.arange(self.d_u, dtype=np.int64)
        for c in range(self.d_u):          # a parent always has a smaller index
            if parent[c] >= 0:
                src[c] = src[parent[c]]
        return src

    def operands_i8(self):
        """A_ue, B_eu as int8 (check max_abs() <= 127 first)."""
        A = np.empty((self.n_u, self.d_u), dtype=np.int8)
        B = np.empty((self.h_u, self.d_u), dtype=np.int8)
        lib().orc_result_copy_i8(self._ptr, _p(A, C.c_int8), _p(B, C.c_int8))
        return A, B

    def max_abs(self) -> int:
        return int(lib().orc_result_max_abs(self._ptr))

    def product_at(self, rows, cols) -> np.ndarray:
        """sum_{R->i, Q->j, c} Pi_A[i,R] Pi_B[j,Q] S[c] A_ue[R,c] B_eu[Q,c] at the listed (i, j)."""
        rows, cols = _i64(rows), _i64(cols)
        out = np.empty(rows.shape, dtype=np.int64)
        lib().orc_unpacked_product_at(self._ptr, _p(rows, C.c_int64), _p(cols, C.c_int64),
                                      rows.size, _p(out, C.c_int64))
        return out

    def close(self):
        if self._ptr:
            lib().orc_result_free(self._ptr)
            self._ptr = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def unpack_handle(A, B, b: int, strategy: int, S=None, recount: bool = False) -> UnpackHandle:
    """Alg. 5 applied once: unpack A with partner B and diagonal S (None = I)."""
    A, B = _i32(A), _i32(B)
    n, d = A.shape
    h = B.shape[0]
    assert B.shape[1] == d
    sp = None
    if S is not None:
        S = _i64(S)
        assert S.shape == (d,)
        sp = _p(S, C.c_int64)
    ptr = lib().orc_unpack(_p(A, C.c_int32), n, d, _p(B, C.c_int32), h, sp, b, strategy, int(recount))
    return UnpackHandle(ptr)


def unpack(A, B, b: int, strategy: int, S=None, recount: bool = False) -> Unpacked:
    return unpack_handle(A, B, b, strategy, S, recount).dense()


def unpack_pair_handle(A, B, b: int, strategy_a: int, strategy_b: int, recount: bool = False) -> UnpackHandle:
    """Sec. 4 'Combining everything': Unpack(A, B, I, b, s_A) then Unpack(B_e, A_u, S_u, b, s_B)."""
    A, B = _i32(A), _i32(B)
    n, d = A.shape
    h = B.shape[0]
    assert B.shape[1] == d
    ptr = lib().orc_unpack_pair(_p(A, C.c_int32), n, d, _p(B, C.c_int32), h, b,
                                strategy_a, strategy_b, int(recount))
    return UnpackHandle(ptr)


def unpack_pair(A, B, b: int, strategy_a: int, strategy_b: int, recount: bool = False) -> Unpacked:
    return unpack_pair_handle(A, B, b, strategy_a, strategy_b, recount).dense()


def scaled_matmul(A, B, S) -> np.ndarray:
    """Alg. 3: one product per distinct diagonal entry of S, scaled and summed (int64)."""
    A, B, S = _i32(A), _i32(B), _i64(S)
    n, d = A.shape
    h = B.shape[0]
    out = np.empty((n, h), dtype=np.int64)
    lib().orc_scaled_matmul(_p(A, C.c_int32), n, d, _p(B, C.c_int32), h, _p(S, C.c_int64),
                            _p(out, C.c_int64))
    return out


def apply_pi(C_u, piA_src, piA_w, piB_src, piB_w, n: int, h: int) -> np.ndarray:
    """Pi_A C_u Pi_B^T as an index-add (Sec. 4, 'Reconstructing A')."""
    C_u = _i64(C_u)
    out = np.empty((n, h), dtype=np.int64)
    lib().orc_apply_pi(_p(C_u, C.c_int64), C_u.shape[0], C_u.shape[1],
                       _p(_i64(piA_src), C.c_int64), _p(_i64(piA_w), C.c_int64),
                       _p(_i64(piB_src), C.c_int64), _p(_i64(piB_w), C.c_int64), n, h,
                       _p(out, C.c_int64))
    return out


def exact_gemm_via_unpack(A, B, b: int, strategy_a: int, strategy_b: int) -> np.ndarray:
    """The whole integer path through the unpacked operands (small inputs only)."""
    n, h = A.shape[0], B.shape[0]
    u = unpack_pair(A, B, b, strategy_a, strategy_b)
    C_u = scaled_matmul(u.A, u.B, u.S)
    return apply_pi(C_u, u.piA_src, u.piA_w, u.piB_src, u.piB_w, n, h)


def percentile_alpha(x: np.ndarray, p: float) -> np.float32:
    """alpha_p(A) of Sec. 2 (the sentence after Eq. (quantized_A)): the p-th percentile of the
    magnitudes, i.e. the smallest magnitude a such that at least p % of the entries of A lie in
    [-a, a].  Written out: sort the magnitudes; with N entries the answer is the k-th smallest,
    k = ceil(p N / 100) (at least 1).  No interpolation: the paper only asks for a value that
    p % of the entries fall within, and an order statistic is the smallest such value."""
    a = np.sort(np.abs(np.asarray(x, dtype=np.float32)).ravel())
    if a.size == 0 or not (0.0 < p <= 100.0):
        raise ValueError("empty matrix or p outside (0, 100]")
    k = min(a.size, max(1, math.ceil(p * float(a.size) / 100.0)))
    return np.float32(a[k - 1])


def rtn_step(alpha, beta) -> np.float32:
    """Eq. (quantized_A): A_q = round((0.5 beta / alpha_p(A)) A): beta integers cover
    [-alpha_p, alpha_p], so one RTN step is alpha_p / (0.5 beta) (formed once, in binary32)."""
    return np.float32(np.float32(alpha) / np.float32(0.5 * float(beta)))
