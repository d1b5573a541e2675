"""Pins for the CPU oracle: each test checks it against something the paper or the
mathematics fixes (printed values, closed forms, invariants, library routines, brute force),
never against itself.  No GPU needed."""
import itertools
import math
import os

import numpy as np
import pytest
import torch

import oracle
from oracle import BOTH, COL, ROW

STRATS = (ROW, COL, BOTH)


def read_kv(path):
    out = {}
    for line in open(path):
        line = line.strip()
        if line and not line.startswith("#"):
            k, v = line.split("=")
            out[k.strip()] = int(v)
    return out


def dense_pi(src, w, n):
    """Pi as the paper defines it: n x n', column t has the single non-zero w[t] at row src[t]."""
    P = np.zeros((n, len(src)), dtype=object)
    for t, (i, wt) in enumerate(zip(src, w)):
        P[int(i), t] = int(wt)
    return P


def obj(M):
    return np.array(M, dtype=object)


def rand_int_matrix(rng, rows, cols, s, p_ob=0.15, depth=3):
    """Mostly in-bound entries, a fraction of out-of-bound ones up to s**depth."""
    M = rng.integers(-(s - 1), s, size=(rows, cols))
    mask = rng.random((rows, cols)) < p_ob
    big = rng.integers(-(s ** depth), s ** depth + 1, size=(rows, cols))
    return np.where(mask, big, M).astype(np.int32)


# ------------------------------------------------------------------ Sec. 2
def test_rtn_ties_are_half_to_even():
    x = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 3.5, 0.49999997, -0.0, 7.0], dtype=np.float32)
    q, st = oracle.rtn_quantize(x, 1.0)
    assert st == 0
    assert q.tolist() == [0, 2, 2, 0, -2, -2, 4, 0, 0, 7]


def test_rtn_matches_ieee_division_then_rint():
    # numpy's float32 division is the correctly rounded IEEE one and np.rint rounds half to even
    rng = np.random.default_rng(0)
    for scale in (np.float32(0.0314159), np.float32(1.0 / 3.0), np.float32(7.25e-4)):
        x = (rng.standard_normal(200_000) * 3).astype(np.float32)
        # add exact ties k + 0.5 in units of the step where representable
        ties = (np.arange(-500, 500, dtype=np.float32) + np.float32(0.5)) * scale
        x = np.concatenate([x, ties])
        want = np.rint(x / scale).astype(np.int64)
        q, st = oracle.rtn_quantize(x, scale)
        assert st == 0
        assert np.array_equal(q.astype(np.int64), want)


def test_rtn_is_nearest_integer_and_unclipped():
    # |q - x/scale| <= 1/2 in exact arithmetic up to the rounding of the quotient; large values survive
    x = np.array([1e6, -3.0e7, 12345.678, 2.0e9], dtype=np.float32)
    q, st = oracle.rtn_quantize(x, 1.0)
    assert st == 0 and q.tolist() == [1000000, -30000000, 12346, 2000000000]
    _, st = oracle.rtn_quantize(np.array([3.0e9], dtype=np.float32), 1.0)
    assert st == 1
    _, st = oracle.rtn_quantize(np.array([np.nan], dtype=np.float32), 1.0)
    assert st == 1
    _, st = oracle.rtn_quantize(np.array([np.inf], dtype=np.float32), 1.0)
    assert st == 1


def test_int_gemm_matches_library_matmul():
    rng = np.random.default_rng(1)
    A = rng.integers(-70000, 70000, size=(37, 53)).astype(np.int32)
    B = rng.integers(-70000, 70000, size=(29, 53)).astype(np.int32)
    want = torch.from_numpy(A.astype(np.int64)) @ torch.from_numpy(B.astype(np.int64)).t()
    assert np.array_equal(oracle.int_gemm(A, B), want.numpy())
    # a transposed-operand mistake would fail on this asymmetric case
    A1 = np.array([[1, 2, 3]], dtype=np.int32)
    B1 = np.array([[1, 0, 0], [0, 10, 0], [0, 0, 100], [1, 1, 1]], dtype=np.int32)
    assert oracle.int_gemm(A1, B1).tolist() == [[1, 20, 300, 6]]
    rows = np.array([0, 0, 36, 17])
    cols = np.array([0, 28, 28, 5])
    assert np.array_equal(oracle.int_gemm_at(A, B, rows, cols), want.numpy()[rows, cols])


def test_int_gemm_no_32bit_wrap():
    A = np.full((1, 2), 2_000_000_000, dtype=np.int32)
    B = np.full((1, 2), -2_000_000_000, dtype=np.int32)
    assert oracle.int_gemm(A, B)[0, 0] == -2 * 2_000_000_000 * 2_000_000_000


def test_dequantize_closed_form():
    Cm = np.array([[0, 1, -3], [2**40, -(2**52) - 1, 7]], dtype=np.int64)
    sa, sb = np.float32(0.125), np.float32(0.0078125)  # powers of two: the product is exact
    got = oracle.dequantize(Cm, sa, sb)
    want = Cm.astype(np.float64) / 1024.0
    assert np.array_equal(got, want)
    sa, sb = np.float32(0.1), np.float32(0.3)
    got = oracle.dequantize(Cm, sa, sb)
    want = np.float64(sa) * np.float64(sb) * Cm.astype(np.float64)
    assert np.allclose(got, want, rtol=1e-15, atol=0)


def test_quantized_gemm_approximates_real_gemm():
    # Eq. (quantized_gemm): the dequantised integer product approximates A B^T; error bounded by the
    # rounding of each entry by at most half a step.
    rng = np.random.default_rng(2)
    A = rng.standard_normal((16, 64)).astype(np.float32)
    B = rng.standard_normal((8, 64)).astype(np.float32)
    sa, sb = np.float32(0.01), np.float32(0.02)
    Aq, _ = oracle.rtn_quantize(A, sa)
    Bq, _ = oracle.rtn_quantize(B, sb)
    Cf = oracle.dequantize(oracle.int_gemm(Aq, Bq), sa, sb)
    exact = A.astype(np.float64) @ B.astype(np.float64).T
    bound = (np.abs(A).astype(np.float64).sum(1)[:, None] * (sb / 2) +
             np.abs(B).astype(np.float64).sum(1)[None, :] * (sa / 2) + 64 * sa * sb / 4) * 1.001
    assert (np.abs(Cf - exact) <= bound).all()


# ------------------------------------------------------------------ digits
@pytest.mark.parametrize("b", range(2, 9))
def test_digits_reconstruct_and_stay_in_bound(b, golden_dir):
    s = 1 << (b - 1)
    rows = [tuple(map(int, l.split())) for l in open(os.path.join(golden_dir, "paper_sec4_ranges.txt"))
            if l.strip() and not l.startswith("#")]
    lo, hi = next((r[2], r[3]) for r in rows if r[0] == b)
    assert next(r[1] for r in rows if r[0] == b) == s
    edge = []
    for k in range(1, 32 // (b - 1) + 1):
        p = s ** k
        if p < 2 ** 31:
            edge += [p - 1, p, p + 1, -(p - 1), -p, -(p + 1)]
    edge += [2 ** 31 - 1, -(2 ** 31 - 1), 0, 1, -1]
    sweep = list(range(-(1 << 13), (1 << 13) + 1)) if b < 8 else list(range(-(1 << 17), (1 << 17) + 1, 7))
    for v in edge + sweep:
        if abs(v) >= 2 ** 31:
            continue
        total, i, nd = 0, 0, 0
        while True:
            dgt = oracle.digit(v, s, i)
            assert lo <= dgt <= hi
            # sign-magnitude reading of floor/mod, written with bit operations
            want = (1 if v >= 0 else -1) * ((abs(v) >> ((b - 1) * i)) & (s - 1))
            assert dgt == want
            total += dgt * s ** i
            i += 1
            if abs(v) < s ** i:
                break
        assert total == v
        # the number of digits is that of |v| in base s
        nd = i
        assert s ** (nd - 1) <= max(abs(v), 1) < s ** nd or (v == 0 and nd == 1)


def test_paper_scalar_example(golden_dir):
    g = read_kv(os.path.join(golden_dir, "paper_sec4_scalar_example.txt"))
    b, s = g["bit_width"], g["base"]
    assert s == 1 << (b - 1)
    # any 32-bit magnitude needs at most five base-128 digits, and the largest ones need exactly five
    for v in (2 ** 31 - 1, -(2 ** 31 - 1), 128 ** 4, -(128 ** 4)):
        nz = [i for i in range(8) if oracle.digit(v, s, i) != 0 or i == 0]
        assert max(nz) + 1 == g["digits_for_32bit"]
        assert oracle.digit(v, s, 5) == 0
    # one multiplication of two such numbers = 25 low-bit multiplications, under every strategy pair
    A = np.array([[2 ** 31 - 1]], dtype=np.int32)
    B = np.array([[-(128 ** 4) - 77]], dtype=np.int32)
    for sa, sb in itertools.product(STRATS, STRATS):
        u = oracle.unpack_pair(A, B, b, sa, sb)
        n_u, d_u = u.A.shape
        h_u = u.B.shape[0]
        assert n_u * d_u * h_u == g["multiplications"], (sa, sb)
        assert oracle.exact_gemm_via_unpack(A, B, b, sa, sb)[0, 0] == int(A[0, 0]) * int(B[0, 0])
    u = oracle.unpack_pair(A, B, b, ROW, ROW)
    assert u.A.shape == (5, 1) and u.B.shape == (5, 1)
    u = oracle.unpack_pair(A, B, b, COL, COL)
    assert u.A.shape == (1, 25) and u.B.shape == (1, 25)
    u = oracle.unpack_pair(A, B, b, ROW, COL)
    assert u.A.shape == (5, 5) and u.B.shape == (1, 5)


def test_two_bit_digits_are_ternary():
    rng = np.random.default_rng(3)
    A = rng.integers(-40, 41, size=(5, 6)).astype(np.int32)
    B = rng.integers(-40, 41, size=(4, 6)).astype(np.int32)
    for sa, sb in itertools.product(STRATS, STRATS):
        u = oracle.unpack_pair(A, B, 2, sa, sb)
        assert set(np.unique(u.A)) <= {-1, 0, 1} and set(np.unique(u.B)) <= {-1, 0, 1}
        assert np.array_equal(oracle.exact_gemm_via_unpack(A, B, 2, sa, sb), oracle.int_gemm(A, B))


# ------------------------------------------------------------------ Alg. 1
@pytest.mark.parametrize("b", [2, 3, 5, 8])
def test_unpack_row_reconstructs_A(b):
    rng = np.random.default_rng(10 + b)
    s = 1 << (b - 1)
    A = rand_int_matrix(rng, 9, 7, s)
    B = rng.integers(-(s - 1), s, size=(4, 7)).astype(np.int32)
    u = oracle.unpack(A, B, b, ROW)
    n = A.shape[0]
    assert np.abs(u.A).max() <= s - 1                              # every entry In-Bound
    P = dense_pi(u.piA_src, u.piA_w, n)
    assert all(np.count_nonzero(P[:, t]) == 1 for t in range(P.shape[1]))
    assert np.array_equal(P @ obj(u.A), obj(A))                    # A = Pi_A A_u
    assert np.array_equal(u.B, B) and (u.S == 1).all()              # partner and S pass through
    assert np.array_equal(P[:, :n], np.eye(n, dtype=object))        # Pi starts as I
    for t in range(n, P.shape[1]):
        w = int(u.piA_w[t])
        assert w > 1 and s ** round(np.log(w) / np.log(s)) == w      # weights are powers of s


def levels_of(maxabs, s):
    L = 1
    while maxabs >= s ** L:
        L += 1
    return L


@pytest.mark.parametrize("b", [2, 4, 8])
def test_unpack_row_order_is_level_major(b):
    """The FIFO loop of Alg. 1 has a closed form: slots 0..n-1 keep digit 0, then the digit-1
    rows of all rows with >= 2 digits in ascending source index, then the digit-2 rows, ..."""
    rng = np.random.default_rng(20 + b)
    s = 1 << (b - 1)
    A = rand_int_matrix(rng, 12, 5, s, p_ob=0.12, depth=4)
    B = np.zeros((1, 5), dtype=np.int32)
    u = oracle.unpack(A, B, b, ROW)
    L = [levels_of(int(np.abs(A[i]).max()), s) for i in range(A.shape[0])]
    src, w, rows = list(range(A.shape[0])), [1] * A.shape[0], []
    sgn = np.sign(A).astype(np.int64)
    mag = np.abs(A).astype(np.int64)
    rows = [sgn[i] * (mag[i] % s) for i in range(A.shape[0])]
    for lvl in range(1, max(L)):
        for i in range(A.shape[0]):
            if L[i] > lvl:
                src.append(i)
                w.append(s ** lvl)
                rows.append(sgn[i] * ((mag[i] // s ** lvl) % s))
    assert u.piA_src.tolist() == src
    assert u.piA_w.tolist() == w
    assert np.array_equal(u.A, np.array(rows))


# ------------------------------------------------------------------ Alg. 2 + Alg. 3
@pytest.mark.parametrize("b", [2, 3, 5, 8])
def test_unpack_column_identity(b):
    rng = np.random.default_rng(30 + b)
    s = 1 << (b - 1)
    A = rand_int_matrix(rng, 6, 8, s)
    B = rng.integers(-500, 500, size=(5, 8)).astype(np.int32)     # partner may hold anything
    u = oracle.unpack(A, B, b, COL)
    assert np.abs(u.A).max() <= s - 1
    assert u.A.shape[0] == 6 and u.B.shape[0] == 5 and u.A.shape[1] == u.B.shape[1] == len(u.S)
    want = obj(A) @ obj(B).T
    assert np.array_equal(obj(u.A) @ np.diag(obj(u.S)) @ obj(u.B).T, want)   # A B^T = A_u S_u B_e^T
    assert np.array_equal(oracle.scaled_matmul(u.A, u.B, u.S), want.astype(np.int64))
    assert (u.piA_src == np.arange(6)).all() and (u.piA_w == 1).all()          # Pi_A = I
    # every new column of B_e is a copy of an original column; S holds powers of s
    d = A.shape[1]
    for c in range(d, u.B.shape[1]):
        assert any(np.array_equal(u.B[:, c], B[:, k]) for k in range(d))
    for v in u.S:
        k = 0
        while s ** k < v:
            k += 1
        assert s ** k == v


def test_unpack_column_order_with_given_S():
    """Alg. 2 with a non-identity S input (as in the second application of Alg. 5): the child of
    column i carries s * S[i,i]; children are appended in FIFO order."""
    b, s = 4, 8
    A = np.array([[9, 1, 70], [2, -8, 3]], dtype=np.int32)   # col0: 2 digits, col1: 2 digits, col2: 3 digits
    B = np.array([[1, 2, 3]], dtype=np.int32)
    S = np.array([1, 8, 64], dtype=np.int64)
    u = oracle.unpack(A, B, b, COL, S=S)
    assert u.S.tolist() == [1, 8, 64, 8, 64, 512, 4096]
    assert u.B.tolist() == [[1, 2, 3, 1, 2, 3, 3]]
    assert u.A.tolist() == [[1, 1, 6, 1, 0, 0, 1], [2, 0, 3, 0, -1, 0, 0]]


def test_scaled_matmul_is_A_diagS_Bt():
    rng = np.random.default_rng(4)
    A = rng.integers(-127, 128, size=(7, 11)).astype(np.int32)
    B = rng.integers(-127, 128, size=(6, 11)).astype(np.int32)
    S = np.array([128 ** int(k) for k in rng.integers(0, 4, size=11)], dtype=np.int64)
    want = obj(A) @ np.diag(obj(S)) @ obj(B).T
    assert np.array_equal(obj(oracle.scaled_matmul(A, B, S)), want)


def test_apply_pi_is_the_matrix_product():
    rng = np.random.default_rng(5)
    C_u = rng.integers(-10 ** 6, 10 ** 6, size=(7, 5)).astype(np.int64)
    pa_src, pa_w = np.array([0, 1, 2, 1, 1, 0, 2]), np.array([1, 1, 1, 8, 64, 8, 8])
    pb_src, pb_w = np.array([0, 1, 0, 0, 1]), np.array([1, 1, 8, 64, 8])
    want = dense_pi(pa_src, pa_w, 3) @ obj(C_u) @ dense_pi(pb_src, pb_w, 2).T
    got = oracle.apply_pi(C_u, pa_src, pa_w, pb_src, pb_w, 3, 2)
    assert np.array_equal(obj(got), want)


# ------------------------------------------------------------------ Alg. 4
@pytest.mark.parametrize("b", [2, 3, 4, 8])
def test_unpack_both_identity(b):
    rng = np.random.default_rng(40 + b)
    s = 1 << (b - 1)
    for trial in range(6):
        A = rand_int_matrix(rng, 7, 6, s, p_ob=0.2, depth=3)
        B = rng.integers(-300, 300, size=(5, 6)).astype(np.int32)
        u = oracle.unpack(A, B, b, BOTH)
        assert np.abs(u.A).max() <= s - 1
        P = dense_pi(u.piA_src, u.piA_w, 7)
        want = obj(A) @ obj(B).T
        # A B^T = Pi_A A_u S_u B_e^T
        assert np.array_equal(P @ obj(u.A) @ np.diag(obj(u.S)) @ obj(u.B).T, want)
        # bookkeeping variant: recount every step
        u2 = oracle.unpack(A, B, b, BOTH, recount=True)
        for f in ("A", "B", "S", "piA_src", "piA_w"):
            assert np.array_equal(getattr(u, f), getattr(u2, f))


def test_unpack_both_paper_failure_cases():
    """Sec. 4, 'Are we done?' / 'Are we done yet?': heavy hitters in one column are cheap for
    column unpacking and expensive for row unpacking; heavy hitters in one row plus one column
    are best handled by splitting exactly that row and that column."""
    b, s = 8, 128
    left = np.ones((4, 4), dtype=np.int32)
    left[:, 1] = 1000
    B = np.ones((3, 4), dtype=np.int32)
    assert oracle.unpack(left, B, b, ROW).A.shape == (8, 4)
    assert oracle.unpack(left, B, b, COL).A.shape == (4, 5)
    ub = oracle.unpack(left, B, b, BOTH)
    assert ub.A.shape == (4, 5)                     # column count 4 beats every row count 1
    right = np.ones((4, 4), dtype=np.int32)
    right[1, :] = 1000
    right[:, 1] = 1000
    assert oracle.unpack(right, B, b, ROW).A.shape == (8, 4)
    assert oracle.unpack(right, B, b, COL).A.shape == (4, 8)
    ub = oracle.unpack(right, B, b, BOTH)
    assert ub.A.shape == (5, 5)                     # second row and second column
    # order: counts are 4 and 4, the tie goes to the row (c0 >= c1); then the column (count 3)
    assert ub.piA_src.tolist() == [0, 1, 2, 3, 1] and ub.piA_w.tolist() == [1, 1, 1, 1, 128]
    assert ub.S.tolist() == [1, 1, 1, 1, 128]
    want = right.copy()
    want[1, :] = 1000 % 128
    want[:, 1] = 1000 % 128
    exp = np.zeros((5, 5), dtype=np.int32)
    exp[:4, :4] = want
    exp[4, :4] = 1000 // 128                         # new row: floor(row 1 / s)
    exp[[0, 2, 3], 4] = 1000 // 128                  # new column: floor(col 1 / s) of rows still OB
    assert np.array_equal(ub.A, exp)


def test_unpack_both_tie_breaks_and_single_entry():
    b = 8
    A = np.zeros((3, 3), dtype=np.int32)
    A[1, 2] = 300
    B = np.arange(6, dtype=np.int32).reshape(2, 3)
    u = oracle.unpack(A, B, b, BOTH)                 # c0 = c1 = 1 -> row
    assert u.A.shape == (4, 3) and u.B.shape == (2, 3)
    assert oracle.unpack(A, B, b, ROW).A.shape == (4, 3)
    assert oracle.unpack(A, B, b, COL).A.shape == (3, 4)
    # two rows with the same top count: the lower index is split first
    A = np.zeros((3, 2), dtype=np.int32)
    A[2, 0] = 300
    A[0, 1] = 400
    u = oracle.unpack(A, B[:, :2].copy(), b, BOTH)
    assert u.piA_src.tolist() == [0, 1, 2, 0, 2]
    # nothing OB: identity, unpack ratio 1
    A = np.full((3, 3), 127, dtype=np.int32)
    A[0, 0] = -127
    for st in STRATS:
        u = oracle.unpack(A, B, b, st)
        assert np.array_equal(u.A, A) and np.array_equal(u.B, B) and (u.S == 1).all()
    # -128 is out of bound for b = 8 although a byte could hold it
    A[0, 0] = -128
    assert oracle.unpack(A, B, b, ROW).A.shape == (4, 3)


def test_unpack_both_counts_follow_current_matrix():
    """An entry with three digits keeps its column/row out-of-bound after one split, so the
    greedy must look at the grown matrix, not the original one."""
    b, s = 4, 8
    A = np.array([[500, 9, 0], [0, 9, 0], [0, 9, 1]], dtype=np.int32)
    B = np.eye(3, dtype=np.int32)
    u = oracle.unpack(A, B, b, BOTH)
    # counts: rows (2,1,1), cols (1,3,0): column 1 first (3 > 2); then row 0 (count 1, tie -> row),
    # whose child row holds 62 (still OB) -> split again; child holds 7.
    assert u.S.tolist() == [1, 1, 1, 8]
    assert u.piA_src.tolist() == [0, 1, 2, 0, 0]
    assert u.piA_w.tolist() == [1, 1, 1, 8, 64]
    assert u.A.tolist() == [[4, 1, 0, 1], [0, 1, 0, 1], [0, 1, 1, 1], [6, 0, 0, 0], [7, 0, 0, 0]]


# ------------------------------------------------------------------ Alg. 5 / composition
@pytest.mark.parametrize("b", [2, 4, 8])
def test_pair_identity_all_strategy_pairs(b):
    rng = np.random.default_rng(50 + b)
    s = 1 << (b - 1)
    for sa, sb in itertools.product(STRATS, STRATS):
        A = rand_int_matrix(rng, 6, 7, s, p_ob=0.15, depth=3)
        B = rand_int_matrix(rng, 5, 7, s, p_ob=0.15, depth=3)
        u = oracle.unpack_pair(A, B, b, sa, sb)
        assert np.abs(u.A).max() <= s - 1 and np.abs(u.B).max() <= s - 1
        PA = dense_pi(u.piA_src, u.piA_w, 6)
        PB = dense_pi(u.piB_src, u.piB_w, 5)
        want = obj(A) @ obj(B).T
        got = PA @ obj(u.A) @ np.diag(obj(u.S)) @ obj(u.B).T @ PB.T
        assert np.array_equal(got, want), (sa, sb)
        assert np.array_equal(obj(oracle.exact_gemm_via_unpack(A, B, b, sa, sb)), want)
        assert np.array_equal(oracle.int_gemm(A, B), want.astype(np.int64))
        h = oracle.unpack_pair_handle(A, B, b, sa, sb)
        rows, cols = np.array([0, 5, 3]), np.array([4, 0, 2])
        assert np.array_equal(h.product_at(rows, cols), want.astype(np.int64)[rows, cols])
        assert h.max_abs() == max(np.abs(u.A).max(), np.abs(u.B).max())
        # strategies are independent: ROW leaves the contraction size alone, COL leaves the rows alone
        if sa == ROW and sb == ROW:
            assert u.A.shape[1] == 7
        if sa == COL and sb == COL:
            assert u.A.shape[0] == 6 and u.B.shape[0] == 5


def test_pair_col_col_structure():
    """A first, then B on the already widened B_e: S exponents add, and A_ue repeats A_u's columns."""
    b, s = 8, 128
    A = np.array([[300, 1]], dtype=np.int32)
    B = np.array([[2, 3], [40000, 5]], dtype=np.int32)
    u = oracle.unpack_pair(A, B, b, COL, COL)
    # phase 1: A col 0 splits -> A_u = [44, 1, 2], B_e = [[2,3,2],[40000,5,40000]], S = [1,1,128]
    # phase 2 on B_e: col 0 (40000: 3 digits) and its copy col 2 split, in FIFO order
    assert u.S.tolist() == [1, 1, 128, 128, 128 * 128, 128 ** 2, 128 ** 3]
    assert u.A.tolist() == [[44, 1, 2, 44, 2, 44, 2]]
    assert u.B.tolist() == [[2, 3, 2, 0, 0, 0, 0], [64, 5, 64, 56, 56, 2, 2]]


def test_copy_out_accessors_match_the_pinned_dense_copy():
    """The two copy-outs the GPU parity tests read the oracle through (int8 operands, Pi / S without
    the operands) against hand-worked values and against dense(), which the identities above pin: on
    non-square shapes (a row-stride or cast slip would show), every strategy pair, and a matrix whose
    storage has grown past its first capacity (row stride != column count inside the oracle)."""
    b, s = 8, 128
    A = np.array([[300, 1]], dtype=np.int32)
    B = np.array([[2, 3], [40000, 5]], dtype=np.int32)
    h = oracle.unpack_pair_handle(A, B, b, COL, COL)     # the hand-worked case of test_pair_col_col_structure
    a8, b8 = h.operands_i8()
    assert a8.dtype == np.int8 and b8.dtype == np.int8
    assert a8.tolist() == [[44, 1, 2, 44, 2, 44, 2]]
    assert b8.tolist() == [[2, 3, 2, 0, 0, 0, 0], [64, 5, 64, 56, 56, 2, 2]]
    S, pas, paw, pbs, pbw = h.meta()
    assert S.tolist() == [1, 1, 128, 128, 128 * 128, 128 ** 2, 128 ** 3]
    assert pas.tolist() == [0] and paw.tolist() == [1] and pbs.tolist() == [0, 1] and pbw.tolist() == [1, 1]
    h.close()
    # negative digits survive the cast; Pi of a row split (hand-worked: -300 = -(2*128 + 44))
    h = oracle.unpack_pair_handle(np.array([[-300, 7], [5, -6]], dtype=np.int32),
                                  np.array([[1, 2], [3, 4], [-129, 0]], dtype=np.int32), b, ROW, ROW)
    a8, b8 = h.operands_i8()
    assert a8.tolist() == [[-44, 7], [5, -6], [-2, 0]]
    assert b8.tolist() == [[1, 2], [3, 4], [-1, 0], [-1, 0]]
    S, pas, paw, pbs, pbw = h.meta()
    assert S.tolist() == [1, 1]
    assert pas.tolist() == [0, 1, 0] and paw.tolist() == [1, 1, 128]
    assert pbs.tolist() == [0, 1, 2, 2] and pbw.tolist() == [1, 1, 1, 128]
    h.close()
    rng = np.random.default_rng(2024)
    for bb in (2, 4, 8):
        ss = 1 << (bb - 1)
        for sa, sb in itertools.product(STRATS, STRATS):
            Am = rand_int_matrix(rng, 9, 13, ss, p_ob=0.3, depth=4)     # grows well past the first capacity
            Bm = rand_int_matrix(rng, 5, 13, ss, p_ob=0.3, depth=4)
            h = oracle.unpack_pair_handle(Am, Bm, bb, sa, sb)
            u = h.dense()
            a8, b8 = h.operands_i8()
            assert a8.shape == u.A.shape and b8.shape == u.B.shape
            assert np.array_equal(a8.astype(np.int32), u.A) and np.array_equal(b8.astype(np.int32), u.B)
            for got, want in zip(h.meta(), (u.S, u.piA_src, u.piA_w, u.piB_src, u.piB_w)):
                assert got.dtype == np.int64 and np.array_equal(got, want)
            assert (h.n_u, h.d_u, h.h_u) == (u.A.shape[0], u.A.shape[1], u.B.shape[0])
            h.close()


def _replay_split_trace(A, B, b, sa, sb, ops):
    """Applies the recorded splits one by one with numpy on Python integers, checking at every step that
    the split is the one the algorithm in charge must make at that moment.  Returns the final
    (first operand, second operand, diag S, column parents)."""
    s = 1 << (b - 1)
    M = [obj(A), obj(B)]                     # M[0]: the operand of the first Unpack call, M[1]: of the second
    S = [1] * A.shape[1]
    parent = [-1] * A.shape[1]
    last_fifo = {0: -1, 1: -1}
    trunc_div = np.vectorize(lambda v: int(abs(v) // s) * (1 if v >= 0 else -1), otypes=[object])
    for call, kind, idx in ops.tolist():
        X, P = M[call], M[1 - call]          # the matrix being unpacked and its partner
        strat = sa if call == 0 else sb
        ob = np.abs(X) >= s
        rc, cc = ob.sum(1), ob.sum(0)
        if strat == BOTH:                    # Alg. 4: top count, rows on c0 >= c1, lowest index among equals
            c0, c1 = rc.max(), cc.max()
            assert max(c0, c1) > 0
            if c0 >= c1:
                assert kind == 0 and idx == int(np.argmax(rc))
            else:
                assert kind == 1 and idx == int(np.argmax(cc))
        else:                                # Alg. 1 / 2: one visit per row / column in index order, split iff OB
            assert kind == (0 if strat == ROW else 1)
            assert idx > last_fifo[call]
            skipped = range(last_fifo[call] + 1, idx)
            assert not any((rc if kind == 0 else cc)[t] for t in skipped)
            assert (rc if kind == 0 else cc)[idx] > 0
            last_fifo[call] = idx
        if kind == 0:
            row = X[idx].copy()
            q = trunc_div(row)
            X[idx] = row - s * q
            M[call] = np.vstack([X, q[None, :]])
        else:
            col = X[:, idx].copy()
            q = trunc_div(col)
            X[:, idx] = col - s * q
            M[call] = np.hstack([X, q[:, None]])
            M[1 - call] = np.hstack([P, P[:, idx:idx + 1]])
            S.append(s * S[idx])
            parent.append(idx)
    return M[0], M[1], S, parent


@pytest.mark.parametrize("b", [2, 4, 8])
def test_split_trace_replays_to_the_same_result(b):
    """The recorded sequence of splits and the column parents: replayed step by step they give the
    oracle's own unpacked operands and S, each step is the one its algorithm prescribes on the
    replayed state, and nothing Out-of-Bound is left at the end (so the sequence is complete)."""
    rng = np.random.default_rng(900 + b)
    s = 1 << (b - 1)
    for sa, sb in itertools.product(STRATS, STRATS):
        A = rand_int_matrix(rng, 6, 8, s, p_ob=0.2, depth=3)
        B = rand_int_matrix(rng, 7, 8, s, p_ob=0.2, depth=3)
        h = oracle.unpack_pair_handle(A, B, b, sa, sb)
        u = h.dense()
        parent, ops = h.trace()
        assert all(c0 <= c1 for c0, c1 in zip(ops[:-1, 0], ops[1:, 0]))     # the first call's splits come first
        Au, Bu, S, par = _replay_split_trace(A, B, b, sa, sb, ops)
        assert np.array_equal(Au, obj(u.A)) and np.array_equal(Bu, obj(u.B))
        assert S == [int(x) for x in u.S] and par == parent.tolist()
        assert np.abs(u.A).max() < s and np.abs(u.B).max() < s
        # a column's parent holds the digit below it: S[c] = s * S[parent], and col_src follows the chain
        src = h.col_src()
        for c in range(len(par)):
            assert src[c] == (c if par[c] < 0 else src[par[c]])
        h.close()


def test_column_parents_name_the_duplicated_partner_column():
    """Alg. 2 line 6 / Alg. 4 line 13: the partner receives a copy of the split column, so after one
    Unpack call column c of B_e equals column col_src[c] of B, whatever the strategy."""
    rng = np.random.default_rng(31)
    for b, strat in itertools.product((3, 8), (COL, BOTH)):
        s = 1 << (b - 1)
        A = rand_int_matrix(rng, 12, 9, s, p_ob=0.25, depth=4)
        A[:, 2] = s * s + 1                 # a column with more OB entries than any row: UnpackBoth splits it
        B = rng.integers(-1000, 1000, size=(4, 9)).astype(np.int32)
        h = oracle.unpack_handle(A, B, b, strat)
        u = h.dense()
        src = h.col_src()
        assert u.B.shape[1] == u.A.shape[1] > 9
        assert np.array_equal(u.B, B[:, src])
        assert set(src[:9].tolist()) == set(range(9)) and src[:9].tolist() == list(range(9))
        h.close()
    # hand-worked: the COL/COL example above
    h = oracle.unpack_pair_handle(np.array([[300, 1]], dtype=np.int32), np.array([[2, 3], [40000, 5]], dtype=np.int32),
                                  8, COL, COL)
    parent, ops = h.trace()
    assert parent.tolist() == [-1, -1, 0, 0, 2, 3, 4] and h.col_src().tolist() == [0, 1, 0, 0, 0, 0, 0]
    assert ops.tolist() == [[0, 1, 0], [1, 1, 0], [1, 1, 2], [1, 1, 3], [1, 1, 4]]
    h.close()


def test_brute_force_tiny_matrices():
    """All 2x2 A over a value set that straddles every digit boundary, a few partners,
    all nine strategy pairs, b in {2,3,4}: exact product, In-Bound digits, termination."""
    for b in (2, 3, 4):
        s = 1 << (b - 1)
        vals = sorted({-s * s, -s - 1, -s, -1, 0, 1, s - 1, s, s * s, s * s + 1})
        partners = [np.array([[s * s + 1, -s], [1, s - 1], [-(s ** 3), 0]], dtype=np.int32),
                    np.array([[1, -1]], dtype=np.int32)]
        for entries in itertools.product(vals, repeat=4):
            A = np.array(entries, dtype=np.int32).reshape(2, 2)
            if b == 4 and (entries[0] + entries[3]) % 3:      # thin the largest sweep
                continue
            for Bm in partners:
                want = A.astype(np.int64) @ Bm.astype(np.int64).T
                for sa, sb in itertools.product(STRATS, STRATS):
                    h = oracle.unpack_pair_handle(A, Bm, b, sa, sb)
                    assert h.max_abs() <= s - 1
                    rr, cc = np.divmod(np.arange(want.size), want.shape[1])
                    assert np.array_equal(h.product_at(rr, cc), want.ravel())
                    h.close()


def test_brute_force_2x3_sample():
    rng = np.random.default_rng(7)
    for b in (2, 3, 4):
        s = 1 << (b - 1)
        vals = np.array(sorted({-s * s, -s - 1, -s, -1, 0, 1, s - 1, s, s * s, s * s + 1}))
        for _ in range(300):
            A = rng.choice(vals, size=(2, 3)).astype(np.int32)
            Bm = rng.choice(vals, size=(3, 3)).astype(np.int32)
            want = A.astype(np.int64) @ Bm.astype(np.int64).T
            for sa, sb in itertools.product(STRATS, STRATS):
                assert np.array_equal(oracle.exact_gemm_via_unpack(A, Bm, b, sa, sb), want)


def test_unpack_ratio_definition():
    """r = n'd'h' / (n d h) (Sec. 4.2); 1 when nothing is out of bound; a single two-digit
    entry costs one extra row (ROW) or one extra column (COL)."""
    b = 8
    A = np.ones((4, 5), dtype=np.int32)
    B = np.ones((3, 5), dtype=np.int32)
    u = oracle.unpack_pair(A, B, b, BOTH, BOTH)
    assert u.A.shape == (4, 5) and u.B.shape == (3, 5)
    A[2, 3] = 200
    u = oracle.unpack_pair(A, B, b, ROW, ROW)
    assert (u.A.shape[0], u.A.shape[1], u.B.shape[0]) == (5, 5, 3)
    u = oracle.unpack_pair(A, B, b, COL, ROW)
    assert (u.A.shape[0], u.A.shape[1], u.B.shape[0]) == (4, 6, 3)


# ---------------------------------------------------------------------------------------------
# alpha_p and the RTN step of Sec. 2 (Eq. (quantized_A))
# ---------------------------------------------------------------------------------------------
@pytest.mark.parametrize("N", [1, 2, 7, 100, 1000, 4097])
@pytest.mark.parametrize("p", [0.01, 1.0, 50.0, 95.0, 99.5, 100.0])
def test_percentile_is_the_smallest_covering_magnitude(N, p):
    """Brute force on the definition: at least p % of the entries lie in [-alpha, alpha], and no
    smaller magnitude of the matrix does that."""
    rng = np.random.default_rng(N * 1000 + int(p * 100))
    x = (rng.standard_normal(N) * rng.choice([1.0, 30.0], N, p=[0.97, 0.03])).astype(np.float32)
    x[rng.integers(0, N, max(1, N // 10))] = x[0]          # ties
    a = oracle.percentile_alpha(x.reshape(1, -1), p)
    mags = np.abs(x)
    need = p * N / 100.0
    assert (mags <= a).sum() >= need
    assert a in mags
    smaller = mags[mags < a]
    if smaller.size:
        assert (mags <= smaller.max()).sum() < need


def test_percentile_closed_forms():
    # a permutation of +-1..N: the k-th smallest magnitude is k
    for N in (10, 100, 1001):
        rng = np.random.default_rng(N)
        x = (rng.permutation(N) + 1).astype(np.float32) * rng.choice([-1.0, 1.0], N).astype(np.float32)
        for p in (10.0, 33.3, 95.0, 100.0):
            assert oracle.percentile_alpha(x.reshape(-1, 1), p) == np.float32(math.ceil(p * N / 100.0))
    # p = 100 is the largest magnitude; a tiny p the smallest; the sign and the order do not matter
    x = np.array([[3.0, -7.5, 0.25], [-0.125, 2.0, 7.0]], dtype=np.float32)
    assert oracle.percentile_alpha(x, 100.0) == np.float32(7.5)
    assert oracle.percentile_alpha(x, 1e-9) == np.float32(0.125)
    assert oracle.percentile_alpha(-x.T[::-1], 50.0) == oracle.percentile_alpha(x, 50.0) == np.float32(2.0)
    # all equal: that value for every p
    assert oracle.percentile_alpha(np.full((5, 5), -2.5, np.float32), 37.0) == np.float32(2.5)
    # large normal sample: the 95th percentile of |N(0, sigma)| is 1.95996 sigma
    z = np.random.default_rng(0).standard_normal(1 << 20).astype(np.float32) * np.float32(0.02)
    assert abs(float(oracle.percentile_alpha(z.reshape(1024, -1), 95.0)) / 0.02 - 1.95996) < 0.01
    with pytest.raises(ValueError):
        oracle.percentile_alpha(x, 0.0)
    with pytest.raises(ValueError):
        oracle.percentile_alpha(x, 100.5)


def test_rtn_step_covers_the_percentile_range_with_beta_integers():
    """Eq. (quantized_A): with the step alpha_p / (0.5 beta), a value of magnitude alpha_p rounds to
    0.5 beta in magnitude, so [-alpha_p, alpha_p] maps onto the beta integers around zero (beta odd:
    -(beta-1)/2 .. (beta-1)/2 after rounding half to even at the two ends is not required here, only
    the range) and p % of the entries round into it."""
    rng = np.random.default_rng(5)
    x = rng.standard_normal((64, 257)).astype(np.float32) * np.float32(0.3)
    for beta in (15, 31, 255):
        for p in (95.0, 99.0):
            a = oracle.percentile_alpha(x, p)
            step = oracle.rtn_step(a, beta)
            assert step == np.float32(np.float32(a) / np.float32(0.5 * beta))
            q, st = oracle.rtn_quantize(x, step)
            assert st == 0
            lim = math.floor(0.5 * beta + 0.5)   # round(0.5 beta) in magnitude at most
            inside = (np.abs(q) <= lim).sum()
            assert inside >= p * x.size / 100.0
            # the entry that defines alpha_p lands on +-round(0.5 beta) up to the rounding of the step
            ia = np.argmin(np.abs(np.abs(x) - a))
            assert abs(abs(int(q.ravel()[ia])) - 0.5 * beta) <= 0.5 + 1e-3
