"""GPU parity: every stage of the HIP path against the CPU oracle, element by element, through the
C ABI.  Integer results must match bit for bit; the dequantised fp32 output must be within 1e-6
relative of the oracle's fp64 value."""
import itertools

import numpy as np
import pytest
import torch

import oracle
from paper_2403_07339_amd import workloads

pytestmark = pytest.mark.gpu

ROW, COL, BOTH = 0, 1, 2
STRATS = (ROW, COL, BOTH)
REL_TOL = 1e-6  # relative error allowed on the dequantised fp32 output


@pytest.fixture(scope="module")
def imu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_07339_amd import binding
    return binding


def dev(x):
    return x.to("cuda")


def oracle_quant(x: torch.Tensor, scale):
    q, st = oracle.rtn_quantize(x.contiguous().numpy(), scale)
    assert st == 0
    return q


def np_stats(q, s):
    a = np.abs(q.astype(np.int64))
    ob = a >= s
    return ob.sum(1), ob.sum(0), a.max(1), a.max(0)


# ------------------------------------------------------------------ quantize + scan
@pytest.mark.parametrize("shape", [(64, 256), (200, 1000), (77, 130), (1, 5), (513, 260), (300, 64)])
@pytest.mark.parametrize("b", [8, 4])
def test_quantize_and_scan(imu, shape, b):
    g = torch.Generator().manual_seed(shape[0] * 1000 + shape[1] + b)
    x = torch.randn(shape, generator=g) * 3
    x[torch.rand(shape, generator=g) < 0.01] *= 100
    # exact ties in units of the step
    scale = float(np.float32(0.0371))
    x.view(-1)[: min(64, x.numel())] = (torch.arange(min(64, x.numel())) - 20 + 0.5) * np.float32(scale)
    s = 1 << (b - 1)
    want = oracle_quant(x, scale)
    Q, st, status = imu.imunpack_quantize(dev(x), scale, b)
    assert int(status.item()) == 0
    assert np.array_equal(Q.cpu().numpy(), want)
    rc, cc, rm, cm = np_stats(want, s)
    assert np.array_equal(st.rowcnt.cpu().numpy(), rc) and np.array_equal(st.colcnt.cpu().numpy(), cc)
    assert np.array_equal(st.rowmax.cpu().numpy(), rm) and np.array_equal(st.colmax.cpu().numpy(), cm)
    st2 = imu.imunpack_scan(Q, b)
    for f in ("rowcnt", "colcnt", "rowmax", "colmax"):
        assert torch.equal(getattr(st, f), getattr(st2, f))
    # transposed view (unit stride down the rows) and a general strided view
    xt = dev(x.t().contiguous()).t()
    Qt, stt, _ = imu.imunpack_quantize(xt, scale, b)
    assert np.array_equal(Qt.cpu().numpy(), want)
    assert np.array_equal(stt.colmax.cpu().numpy(), cm) and np.array_equal(stt.rowcnt.cpu().numpy(), rc)
    wide = dev(torch.zeros(shape[0], 2 * shape[1]))
    wide[:, ::2] = dev(x)
    Qs, sts, _ = imu.imunpack_quantize(wide[:, ::2], scale, b)
    assert np.array_equal(Qs.cpu().numpy(), want)
    assert np.array_equal(sts.colcnt.cpu().numpy(), cc) and np.array_equal(sts.rowmax.cpu().numpy(), rm)


@pytest.mark.parametrize("n,h,d,b", [(200, 333, 520, 8), (70, 64, 256, 4), (1, 129, 4, 8), (130, 131, 130, 8), (64, 1, 256, 8)])
def test_quantize_pair_matches_the_oracle_for_both_operands(imu, n, h, d, b):
    """Both operands of a product in one call (one clearing launch, one launch over the rows of both when
    both take the fast path; d = 130 takes the general path): integers, all four statistics, the OB lists
    and the two status flags against the oracle's RTN (Sec. 2, Eq. quantized_A) and the IB/OB definition
    (Sec. 4); a NaN in B raises only B's flag."""
    g = torch.Generator().manual_seed(n + 31 * h + d + b)
    xa, xb = torch.randn((n, d), generator=g) * 2, torch.randn((h, d), generator=g)
    xa[torch.rand((n, d), generator=g) < 0.02] *= 150.0
    xb[torch.rand((h, d), generator=g) < 0.01] *= 90.0
    sa, sb = float(np.float32(0.0371)), float(np.float32(0.0113))
    s = 1 << (b - 1)
    sta = imu.Stats.empty(n, d, "cuda", ob_cap=max(1, n * d))
    stb = imu.Stats.empty(h, d, "cuda", ob_cap=max(1, h * d))
    Qa, Qb, sta, stb, status = imu.imunpack_quantize_pair(dev(xa), dev(xb), sa, sb, b, stats_a=sta, stats_b=stb)
    assert status.cpu().tolist() == [0, 0]
    for x, scale, Q, st in ((xa, sa, Qa, sta), (xb, sb, Qb, stb)):
        if x.shape[0] == 0:
            continue
        want = oracle_quant(x, scale)
        assert np.array_equal(Q.cpu().numpy(), want)
        rc, cc, rm, cm = np_stats(want, s)
        assert np.array_equal(st.rowcnt.cpu().numpy(), rc) and np.array_equal(st.colcnt.cpu().numpy(), cc)
        assert np.array_equal(st.rowmax.cpu().numpy(), rm) and np.array_equal(st.colmax.cpu().numpy(), cm)
        ii, jj = np.nonzero(np.abs(want.astype(np.int64)) >= s)
        n_ob = int(st.ob_count.item())
        assert n_ob == len(ii)
        ob = st.ob[:, :n_ob].cpu().numpy()
        assert sorted(zip(ob[0].tolist(), ob[1].tolist(), ob[2].tolist())) == sorted(zip(ii.tolist(), jj.tolist(), want[ii, jj].tolist()))
    if h > 0:
        xb[h // 2, d // 3] = float("nan")
        *_, status = imu.imunpack_quantize_pair(dev(xa), dev(xb), sa, sb, b)
        assert status.cpu().tolist() == [0, 1]


def test_quantize_pair_with_operands_of_different_layouts(imu):
    """One operand row-major, the other a transposed view (as in a backward GEMM): the pair call runs them
    through their own kernels, one after the other, with the same results."""
    g = torch.Generator().manual_seed(5)
    xa, xb = torch.randn((256, 384), generator=g) * 4, torch.randn((128, 384), generator=g) * 4
    xa[torch.rand((256, 384), generator=g) < 0.01] *= 80.0
    sa, sb, b = float(np.float32(0.05)), float(np.float32(0.03)), 8
    A_d, B_t = dev(xa), dev(xb.t().contiguous()).t()          # B: unit stride down its rows
    Qa, Qb, sta, stb, status = imu.imunpack_quantize_pair(A_d, B_t, sa, sb, b, want_ob_list=(True, True))
    assert status.cpu().tolist() == [0, 0]
    for x, scale, Q, st in ((xa, sa, Qa, sta), (xb, sb, Qb, stb)):
        want = oracle_quant(x, scale)
        assert np.array_equal(Q.cpu().numpy(), want)
        rc, cc, rm, cm = np_stats(want, 1 << (b - 1))
        assert np.array_equal(st.rowcnt.cpu().numpy(), rc) and np.array_equal(st.colcnt.cpu().numpy(), cc)
        assert np.array_equal(st.rowmax.cpu().numpy(), rm) and np.array_equal(st.colmax.cpu().numpy(), cm)
        assert int(st.ob_count.item()) == int(rc.sum())


@pytest.mark.parametrize("shape,b,frac", [((300, 520), 8, 0.01), ((132, 260), 4, 0.2), ((1024, 384), 8, 0.0005),
                                          ((256, 256), 2, 0.9)])
def test_ob_entry_list_for_every_input_layout(imu, shape, b, frac):
    """The OB entry list (row, column, value of every entry with |q| >= s, in any order) that UnpackBoth
    plans from, for a row-major operand, a transposed view (the tiled transposing kernel) and a view with
    neither stride 1: the same set as the definition gives, each entry once."""
    g = torch.Generator().manual_seed(shape[0] + 7 * shape[1] + b)
    x = torch.randn(shape, generator=g)
    x[torch.rand(shape, generator=g) < frac] *= 300.0
    scale = float(np.float32(0.021))
    s = 1 << (b - 1)
    want = oracle_quant(x, scale)
    ii, jj = np.nonzero(np.abs(want.astype(np.int64)) >= s)
    want_set = sorted(zip(ii.tolist(), jj.tolist(), want[ii, jj].tolist()))
    wide = dev(torch.zeros(shape[0], 3 * shape[1]))
    wide[:, 1::3] = dev(x)
    for view in (dev(x), dev(x.t().contiguous()).t(), wide[:, 1::3]):
        st = imu.Stats.empty(shape[0], shape[1], view.device, ob_cap=shape[0] * shape[1])  # room for every entry
        Q, st, status = imu.imunpack_quantize(view, scale, b, stats=st)
        assert int(status.item()) == 0 and np.array_equal(Q.cpu().numpy(), want)
        n_ob = int(st.ob_count.item())
        assert n_ob == len(want_set) <= st.ob.shape[1]
        ob = st.ob[:, :n_ob].cpu().numpy()
        assert sorted(zip(ob[0].tolist(), ob[1].tolist(), ob[2].tolist())) == want_set


@pytest.mark.parametrize("scale,lo_exp,negate", [(1.0, 21, False), (0.75, 21, True), (0.0371, -3, False)])
def test_quantize_every_float_of_two_binades(imu, scale, lo_exp, negate):
    """Every binary32 value of two adjacent binades (2 x 2^23 bit patterns) through the quantizer: the
    division must be the correctly rounded one and the rounding half-to-even for each of them.  With
    step 1 the binades [2^21, 2^23) hold every tie k + 0.5 up to 2^22; steps 0.75 and 0.0371 make
    nearly every quotient inexact, so a reciprocal-multiply or a fused form would show."""
    scale = float(np.float32(scale))
    lo = np.float32(2.0 ** lo_exp).view(np.uint32)
    bits = np.arange(int(lo), int(lo) + (1 << 24), dtype=np.uint32)
    if negate:
        bits = bits | np.uint32(0x80000000)
    x = bits.view(np.float32).reshape(4096, 4096)
    assert np.isfinite(x).all() and np.abs(x).min() == np.float32(2.0 ** lo_exp)
    want, st = oracle.rtn_quantize(x, scale)
    assert st == 0
    Q, _, status = imu.imunpack_quantize(dev(torch.from_numpy(x)), scale, 8, want_stats=False)
    assert int(status.item()) == 0
    assert np.array_equal(Q.cpu().numpy(), want)
    # the transposing path runs the same arithmetic on the same values
    Qt, _, status = imu.imunpack_quantize(dev(torch.from_numpy(x)).t(), scale, 8, want_stats=False)
    assert int(status.item()) == 0
    assert np.array_equal(Qt.cpu().numpy(), want.T)


def test_quantize_flags_bad_input(imu):
    x = torch.ones(8, 8)
    x[3, 4] = float("nan")
    _, _, status = imu.imunpack_quantize(dev(x), 1.0, 8)
    assert int(status.item()) == 1
    x[3, 4] = 3.0e9
    Q, _, status = imu.imunpack_quantize(dev(x), 1.0, 8)
    assert int(status.item()) == 1 and int(Q[3, 4].item()) == 0
    x[3, 4] = 2.0e9
    Q, _, status = imu.imunpack_quantize(dev(x), 1.0, 8)
    assert int(status.item()) == 0 and int(Q[3, 4].item()) == 2000000000
    with pytest.raises(imu.ImunpackError):
        imu.imunpack_quantize(dev(x), 0.0, 8)
    with pytest.raises(imu.ImunpackError):
        imu.imunpack_quantize(dev(x), 1.0, 9)


# ------------------------------------------------------------------ plan + operands + product
def check_against_oracle(imu, Aq, Bq, b, sa, sb, scale_a=0.013, scale_b=0.0021, full_product=True, fp6=False):
    """Aq, Bq: int32 numpy.  Compares plan, unpacked operands, int64 product (fused and un-fused)
    and the fp32 output with the oracle.  fp6: the digits are stored as 6-bit floating-point codes."""
    n, h = Aq.shape[0], Bq.shape[0]
    s = 1 << (b - 1)
    hnd = oracle.unpack_pair_handle(Aq, Bq, b, sa, sb)
    S, pas, paw, pbs, pbw = hnd.meta()
    assert hnd.max_abs() <= s - 1
    A_d, B_d = dev(torch.from_numpy(Aq)), dev(torch.from_numpy(Bq))
    plan = imu.imunpack_plan(A_d, B_d, b, sa, sb)
    n_u, d_u, h_u, ng = plan.dims()
    assert (n_u, d_u, h_u) == (hnd.n_u, hnd.d_u, hnd.h_u)
    ra_s, ra_e, rb_s, rb_e, c_s, c_e, c_par, ops = [t.numpy().astype(np.int64) for t in plan.export_all()]
    want_parent, want_ops = hnd.trace()
    assert np.array_equal(c_s, hnd.col_src()) and np.array_equal(c_par, want_parent)
    assert np.array_equal(ops, want_ops)          # every split, in the order Alg. 1 / 2 / 4 make them
    assert np.array_equal(ra_s, pas) and np.array_equal(s ** ra_e.astype(object), paw.astype(object))
    assert np.array_equal(rb_s, pbs) and np.array_equal(s ** rb_e.astype(object), pbw.astype(object))
    assert np.array_equal(s ** c_e.astype(object), S.astype(object))
    assert ng == len(np.unique(S))
    if fp6:
        plan.set_digits(imu.DIGITS_FP6)
    assert plan.digits() == (imu.DIGITS_FP6 if fp6 else imu.DIGITS_INT8)
    A_ue, B_eu = imu.imunpack_unpack(plan, A_d, B_d)
    Ac, Bc = imu.imunpack_unpack_canonical(plan, A_ue, B_eu)
    oa, ob = hnd.operands_i8()
    assert np.array_equal(Ac.cpu().numpy(), oa)
    assert np.array_equal(Bc.cpu().numpy(), ob)
    # B_eu is stored in full and its padding (and the zero columns beside columns of A it has no copy
    # for) must be zero: total magnitude is preserved.  Of A_ue every column of A_u is stored once (the
    # repeated columns are read from there), plus a few gathered copies: never more than A_ue holds.
    (ra, wa, pa), (rb, wb, pb) = plan.layout()
    assert A_ue.numel() == ra * pa == plan.unpacked_bytes()[0] and B_eu.numel() == rb * pb == plan.unpacked_bytes()[1]
    if fp6:  # 96 bytes per 128 columns; a zero digit is the code 0, so the number of non-zero bits bounds the padding
        assert pa >= wa * 3 // 4 and pb >= wb * 3 // 4
        nz_b = int((B_eu.view(rb, pb)[:, :wb * 3 // 4] != 0).sum().item())
        assert nz_b <= int((ob != 0).sum())  # every stored non-zero byte holds bits of a non-zero digit...
        assert nz_b * 2 >= int((ob != 0).sum())  # ... and a byte holds bits of at most two digits
    else:
        stored_b = B_eu.view(rb, pb)[:, :wb].to(torch.int64)
        assert int(stored_b.abs().sum().item()) == int(np.abs(ob.astype(np.int64)).sum())
        stored_a = A_ue.view(ra, pa)[:, :wa].to(torch.int64)
        assert int(stored_a.abs().sum().item()) <= int(np.abs(oa.astype(np.int64)).sum())
    assert wa <= wb and wa % 128 == 0 and wb % 128 == 0
    check_bounds(plan, oa, ob, S, s, fp6)
    want = oracle.int_gemm(Aq, Bq)
    want_fp = oracle.dequantize(want, scale_a, scale_b)
    ws = torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
    results = []
    # un-fused: GEMM into the int64 workspace, then recombine
    C_int = torch.full((n, h), -7, dtype=torch.int64, device="cuda")
    C_fp = torch.full((n, h), -7.0, dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, scale_a, scale_b, None, None, ws, fuse=False)
    imu.imunpack_recombine(plan, ws, scale_a, scale_b, C_int, C_fp)
    results.append(("unfused", C_int, C_fp))
    # fused (falls back to the un-fused kernels by itself when the int32 bound does not hold)
    C_int2 = torch.full((n, h), -7, dtype=torch.int64, device="cuda")
    C_fp2 = torch.full((n, h), -7.0, dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, scale_a, scale_b, C_int2, C_fp2, ws, fuse=True)
    results.append(("fused" if plan.fusable() else "fused->fallback", C_int2, C_fp2))
    # fp32 output alone: the fused epilogue may then add the digit levels up in binary64 instead of
    # int64, which must not change a single bit of the result
    C_fp3 = torch.full((n, h), -7.0, dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, scale_a, scale_b, None, C_fp3, ws, fuse=True)
    assert torch.equal(C_fp3, C_fp2), "fp32-only output differs from the fp32 + int64 call"
    for name, ci, cf in results:
        assert np.array_equal(ci.cpu().numpy(), want), name
        got = cf.cpu().numpy().astype(np.float64)
        err = np.abs(got - want_fp)
        assert (err <= REL_TOL * np.abs(want_fp)).all(), name
    hnd.close()
    return plan


def check_bounds(plan, oa, ob, S, s, fp6=False):
    """The accumulator bounds the scatter measured against their definition, evaluated on the
    oracle's unpacked operands: max over rows of sum_c S[c] |digit|; and the path they select."""
    w = np.array([int(x) for x in S], dtype=object)
    want = []
    for m in (oa, ob):
        if m.size == 0:
            want.append(0)
            continue
        rows = (np.abs(m.astype(np.int64)).astype(object) * w[None, :]).sum(1)
        want.append(int(max(rows)))
    got = plan.bounds()
    for g, t in zip(got, want):
        assert g == t if t < (1 << 44) else g >= (1 << 44), (got, want)
    m = min(want)
    assert plan.fusable() == (m < (1 << 40) and m * (s - 1) < (1 << (24 if fp6 else 31)))


def rand_ints(rng, rows, cols, s, p_ob, depth):
    M = rng.integers(-(s - 1), s, size=(rows, cols))
    mask = rng.random((rows, cols)) < p_ob
    big = rng.integers(-(s ** depth), s ** depth + 1, size=(rows, cols))
    return np.where(mask, big, M).astype(np.int32)


@pytest.mark.parametrize("sa,sb", list(itertools.product(STRATS, STRATS)))
@pytest.mark.parametrize("b", [8, 4, 2])
def test_small_random_all_strategies(imu, sa, sb, b):
    rng = np.random.default_rng(100 * b + 10 * sa + sb)
    s = 1 << (b - 1)
    depth = 3 if b > 2 else 5
    Aq = rand_ints(rng, 70, 90, s, 0.03, depth)
    Bq = rand_ints(rng, 50, 90, s, 0.03, depth)
    check_against_oracle(imu, Aq, Bq, b, sa, sb)


@pytest.mark.parametrize("kind", ["scattered", "channels", "rows", "heavy", "clean", "deep"])
@pytest.mark.parametrize("sa,sb", [(BOTH, BOTH), (ROW, COL), (COL, ROW), (COL, COL)])
def test_structured_multi_tile(imu, kind, sa, sb):
    """Shapes that span several GEMM tiles with ragged tails, heavy hitters laid out as in the
    paper's workloads (a few channels, scattered entries, heavy tails)."""
    w = workloads.small(7, 300, 330, 270, kind=kind, b=8)
    Aq = oracle_quant(w.A, w.scale_a)
    Bq = oracle_quant(w.B, w.scale_b)
    check_against_oracle(imu, Aq, Bq, 8, sa, sb, w.scale_a, w.scale_b)


@pytest.mark.parametrize("sa,sb", [(ROW, COL), (BOTH, BOTH), (COL, COL), (COL, ROW), (BOTH, ROW)])
@pytest.mark.parametrize("b", [4, 3, 2])
def test_six_bit_floating_point_digits(imu, sa, sb, b):
    """b <= 4 (Sec. 4.2, low bit widths): the digits stored as e2m3 codes and multiplied by the
    f8f6f4 matrix instruction give the same unpacked operands (decoded) and the same product, bit for bit."""
    rng = np.random.default_rng(1000 * b + 10 * sa + sb)
    s = 1 << (b - 1)
    Aq = rand_ints(rng, 150, 300, s, 0.05, 3 if b > 2 else 5)
    Bq = rand_ints(rng, 270, 300, s, 0.05, 3 if b > 2 else 5)
    check_against_oracle(imu, Aq, Bq, b, sa, sb, fp6=True)


def test_six_bit_digits_fused_path_and_format_rules(imu):
    """A case whose accumulator bound stays below 2^24 runs the fused 6-bit kernel (Horner step as a
    multiplication by a power of two in binary32); the format is refused for b > 4, and a plan object
    that asked for it goes back to int8 when it is re-planned with b > 4."""
    rng = np.random.default_rng(77)
    b, s = 4, 8
    Aq = rand_ints(rng, 300, 700, s, 0.02, 2)
    Bq = rand_ints(rng, 520, 700, s, 0.02, 2)
    plan = check_against_oracle(imu, Aq, Bq, b, COL, COL, fp6=True)
    assert plan.fusable() and plan.digits() == imu.DIGITS_FP6 and plan.dims()[3] >= 2
    # a second unpack of the same plan into fresh buffers (the row norms are cleared and measured again)
    A_d, B_d = dev(torch.from_numpy(Aq)), dev(torch.from_numpy(Bq))
    bounds = plan.bounds()
    A6, B6 = imu.imunpack_unpack(plan, A_d, B_d)
    assert plan.bounds() == bounds
    C = torch.empty((Aq.shape[0], Bq.shape[0]), dtype=torch.int64, device="cuda")
    imu.imunpack_gemm(plan, A6, B6, 1.0, 1.0, C, None, None, fuse=True)
    assert np.array_equal(C.cpu().numpy(), oracle.int_gemm(Aq, Bq))
    A8 = rand_ints(rng, 64, 128, 128, 0.02, 2)
    B8 = rand_ints(rng, 64, 128, 128, 0.02, 2)
    imu.imunpack_plan(dev(torch.from_numpy(A8)), dev(torch.from_numpy(B8)), 8, ROW, ROW, plan=plan)
    assert plan.digits() == imu.DIGITS_INT8
    with pytest.raises(imu.ImunpackError):
        plan.set_digits(imu.DIGITS_FP6)
    with pytest.raises(imu.ImunpackError):
        plan.set_digits(7)
    imu.imunpack_plan(dev(torch.from_numpy(Aq)), dev(torch.from_numpy(Bq)), b, COL, COL, plan=plan)
    assert plan.digits() == imu.DIGITS_FP6          # the request stayed with the plan object
    plan.set_digits(imu.DIGITS_INT8)
    assert plan.digits() == imu.DIGITS_INT8


@pytest.mark.parametrize("sa,sb", [(BOTH, BOTH), (ROW, BOTH), (COL, BOTH), (BOTH, COL), (ROW, COL), (COL, ROW), (BOTH, ROW)])
def test_keep_weights_takes_the_second_operand_over_only_when_it_may(imu, sa, sb):
    """Keep-weights mode (Sec. 4.2: weights unpacked once): with B fixed, a plan call reuses B's unpacking
    exactly when the column slots of A's unpacking are those of the call before.  Every call's plan (every
    split in order), unpacked operands and product are compared with the oracle's, reused or not."""
    rng = np.random.default_rng(4242 + 3 * sa + sb)
    b, s = 8, 128
    n, d, h = 150, 300, 270
    Bq = rand_ints(rng, h, d, s, 0.02, 2)
    def make_A(cols, seed):
        r = np.random.default_rng(seed)
        A = r.integers(-(s - 1), s, size=(n, d)).astype(np.int32)
        for c in cols:                                  # heavy columns: the column splits of A's unpacking
            A[:, c] = r.integers(s, s * s, size=n).astype(np.int32) * r.choice([-1, 1], size=n)
        if sa == ROW:
            A[r.integers(0, n, 5), :] = r.integers(-(s * s - 1), s * s, size=(5, d)).astype(np.int32)
        return A
    B_d = dev(torch.from_numpy(Bq))
    plan = imu.Plan()
    buf_a = torch.empty(8 << 20, dtype=torch.int8, device="cuda")
    buf_b = torch.empty(8 << 20, dtype=torch.int8, device="cuda")
    seq = [((3, 77, 200), 1, False),     # first call in this mode: B is unpacked
           ((3, 77, 200), 2, True),      # other values, same heavy columns: the same column slots
           ((3, 77, 200), 3, True),
           ((5, 77, 201), 4, False),     # other columns split: B is unpacked again
           ((5, 77, 201), 5, True),
           ((3, 77, 200), 6, False)]
    if sa == ROW:                        # no column of A is ever split: always the same column slots
        seq = [(c, k, i > 0) for i, (c, k, _) in enumerate(seq)]
    for i, (cols, seed, want_reuse) in enumerate(seq):
        Aq = make_A(cols, seed)
        A_d = dev(torch.from_numpy(Aq))
        imu.imunpack_plan(A_d, B_d, b, sa, sb, plan=plan)
        if i == 0:
            assert not plan.weights_reused()
            plan.keep_weights(True)      # from the next call on
            imu.imunpack_plan(A_d, B_d, b, sa, sb, plan=plan)
            assert not plan.weights_reused()
        else:
            assert plan.weights_reused() == want_reuse, (i, cols)
        hnd = oracle.unpack_pair_handle(Aq, Bq, b, sa, sb)
        assert plan.dims()[:3] == (hnd.n_u, hnd.d_u, hnd.h_u)
        got = [t.numpy().astype(np.int64) for t in plan.export_all()]
        S, pas, paw, pbs, pbw = hnd.meta()
        want_parent, want_ops = hnd.trace()
        assert np.array_equal(got[0], pas) and np.array_equal(got[2], pbs) and np.array_equal(got[4], hnd.col_src())
        assert np.array_equal(got[6], want_parent) and np.array_equal(got[7], want_ops)
        assert np.array_equal(s ** got[5].astype(object), S.astype(object))
        # the same two buffers in every call: with B's unpacking taken over, B_eu is left as the unpack before wrote it
        ba, bb, bw = plan.unpacked_bytes()
        assert ba <= buf_a.numel() and bb <= buf_b.numel()
        A_ue, B_eu = imu.imunpack_unpack(plan, A_d, B_d, buf_a, buf_b)
        Ac, Bc = imu.imunpack_unpack_canonical(plan, A_ue, B_eu)
        oa, ob = hnd.operands_i8()
        assert np.array_equal(Ac.cpu().numpy(), oa) and np.array_equal(Bc.cpu().numpy(), ob)
        check_bounds(plan, oa, ob, S, s)
        C = torch.empty((n, h), dtype=torch.int64, device="cuda")
        ws = torch.empty(bw // 8, dtype=torch.int64, device="cuda")
        imu.imunpack_gemm(plan, A_ue, B_eu, 1.0, 1.0, C, None, ws, fuse=True)
        assert np.array_equal(C.cpu().numpy(), oracle.int_gemm(Aq, Bq)), i
        if i == 2:  # a second unpack of the same plan measures the row norms again: nothing may be left out then
            imu.imunpack_unpack(plan, A_d, B_d, buf_a, buf_b)
            check_bounds(plan, oa, ob, S, s)
        hnd.close()
    plan.keep_weights(False)
    imu.imunpack_plan(A_d, B_d, b, sa, sb, plan=plan)
    assert not plan.weights_reused()


@pytest.mark.parametrize("b", [3, 5, 6, 7])
def test_other_bit_widths(imu, b):
    w = workloads.small(11, 130, 200, 140, kind="scattered", b=b)
    Aq = oracle_quant(w.A, w.scale_a)
    Bq = oracle_quant(w.B, w.scale_b)
    check_against_oracle(imu, Aq, Bq, b, BOTH, COL, w.scale_a, w.scale_b)
    check_against_oracle(imu, Aq, Bq, b, ROW, BOTH, w.scale_a, w.scale_b)


def test_degenerate_shapes(imu):
    rng = np.random.default_rng(5)
    for (n, d, h) in [(1, 1, 1), (1, 300, 1), (257, 1, 3), (2, 65, 600)]:
        Aq = rand_ints(rng, n, d, 128, 0.1, 3)
        Bq = rand_ints(rng, h, d, 128, 0.1, 3)
        for sa, sb in [(ROW, ROW), (COL, COL), (BOTH, BOTH)]:
            check_against_oracle(imu, Aq, Bq, 8, sa, sb)
    # the scalar example of Sec. 4: five base-128 digits each, 25 low-bit multiplications
    Aq = np.array([[2 ** 31 - 1]], dtype=np.int32)
    Bq = np.array([[-(128 ** 4) - 77]], dtype=np.int32)
    for sa, sb in itertools.product(STRATS, STRATS):
        plan = check_against_oracle(imu, Aq, Bq, 8, sa, sb)
        n_u, d_u, h_u, _ = plan.dims()
        assert n_u * d_u * h_u == 25


def test_plan_object_is_reusable(imu):
    rng = np.random.default_rng(9)
    plan = None
    for (n, d, h, sa, sb) in [(40, 50, 30, BOTH, BOTH), (300, 100, 80, ROW, COL), (40, 50, 30, COL, BOTH)]:
        Aq = rand_ints(rng, n, d, 128, 0.05, 3)
        Bq = rand_ints(rng, h, d, 128, 0.05, 3)
        A_d, B_d = dev(torch.from_numpy(Aq)), dev(torch.from_numpy(Bq))
        plan = imu.imunpack_plan(A_d, B_d, 8, sa, sb, plan=plan)
        hnd = oracle.unpack_pair_handle(Aq, Bq, 8, sa, sb)
        assert plan.dims()[:3] == (hnd.n_u, hnd.d_u, hnd.h_u)
        A_ue, B_eu = imu.imunpack_unpack(plan, A_d, B_d)
        C_int = torch.empty((n, h), dtype=torch.int64, device="cuda")
        ws = torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
        imu.imunpack_gemm(plan, A_ue, B_eu, 1.0, 1.0, C_int, None, ws, fuse=True)
        assert np.array_equal(C_int.cpu().numpy(), oracle.int_gemm(Aq, Bq))


def test_end_to_end_config1(imu):
    """Workload 1 (256 x 256 x 256, scattered heavy hitters, UnpackBoth on both operands) through the
    whole path, full comparison of every stage."""
    w = workloads.make(1)
    Aq = oracle_quant(w.A, w.scale_a)
    Bq = oracle_quant(w.B, w.scale_b)
    Qa, _, _ = imu.imunpack_quantize(dev(w.A), w.scale_a, w.b)
    Qb, _, _ = imu.imunpack_quantize(dev(w.B), w.scale_b, w.b)
    assert np.array_equal(Qa.cpu().numpy(), Aq) and np.array_equal(Qb.cpu().numpy(), Bq)
    check_against_oracle(imu, Aq, Bq, w.b, w.strategy_a, w.strategy_b, w.scale_a, w.scale_b)
    C_int, C_fp, plan = imu.exact_int_gemm(dev(w.A), dev(w.B), w.scale_a, w.scale_b, w.b, w.strategy_a,
                                           w.strategy_b)
    want = oracle.int_gemm(Aq, Bq)
    assert np.array_equal(C_int.cpu().numpy(), want)
    ref = oracle.dequantize(want, w.scale_a, w.scale_b)
    assert (np.abs(C_fp.cpu().numpy().astype(np.float64) - ref) <= REL_TOL * np.abs(ref)).all()


def test_run_to_run_determinism(imu):
    """All outputs are integers (the fp32 one is a function of an integer), atomics only add
    integers, so every stage must reproduce itself bit for bit, whatever the thread timing."""
    g = torch.Generator().manual_seed(3)
    A = torch.randn(600, 1100, generator=g) * 2
    B = torch.randn(520, 1100, generator=g)
    B[torch.randperm(520, generator=g)[:6], :] *= 60          # heavy-hitter rows: one big row batch
    A[torch.rand(A.shape, generator=g) < 0.004] *= 90         # scattered heavy hitters
    sa, sb = workloads.rtn_scale(A), workloads.rtn_scale(B)
    A_d, B_d = dev(A), dev(B)
    plan = imu.Plan()
    first = None
    for _ in range(12):
        Qa, st_a, _ = imu.imunpack_quantize(A_d, sa, 8, want_ob_list=True)
        Qb, st_b, _ = imu.imunpack_quantize(B_d, sb, 8, want_ob_list=True)
        imu.imunpack_plan(Qa, Qb, 8, BOTH, BOTH, st_a, st_b, plan)
        A_ue, B_eu = imu.imunpack_unpack(plan, Qa, Qb)
        C_int = torch.empty((600, 520), dtype=torch.int64, device="cuda")
        ws = None if plan.fusable() else torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
        imu.imunpack_gemm(plan, A_ue, B_eu, sa, sb, C_int, None, ws, fuse=True)
        cur = [Qa, Qb, torch.tensor(plan.dims()), torch.cat(plan.export()), A_ue.clone(), B_eu.clone(), C_int]
        if first is None:
            first = [t.clone() for t in cur]
            want = oracle.int_gemm(oracle_quant(A, sa), oracle_quant(B, sb))
            assert np.array_equal(C_int.cpu().numpy(), want)
        else:
            for a, b in zip(first, cur):
                assert a.shape == b.shape and torch.equal(a, b)


def test_fused_launch_before_the_bounds_are_known(imu):
    """imunpack_unpack leaves the accumulator bounds in flight and a fused imunpack_gemm goes out
    guarded before the host has them.  On data whose shifted group sum does not fit int32 the guarded
    launch must write nothing: without a workspace the call reports ERANGE, with one it falls back to
    the un-fused path and the result is exact."""
    rng = np.random.default_rng(5)
    Aq = rng.integers(-(1 << 22), 1 << 22, size=(96, 320)).astype(np.int32)
    Bq = rng.integers(-(1 << 22), 1 << 22, size=(80, 320)).astype(np.int32)
    want = oracle.int_gemm(Aq, Bq)
    Qa, Qb = torch.from_numpy(Aq).cuda(), torch.from_numpy(Bq).cuda()
    plan = imu.imunpack_plan(Qa, Qb, 8, ROW, COL)   # a new plan object guesses "fused"
    A_ue, B_eu = imu.imunpack_unpack(plan, Qa, Qb)
    C_int = torch.full(want.shape, -7, dtype=torch.int64, device="cuda")
    with pytest.raises(imu.ImunpackError) as err:
        imu.imunpack_gemm(plan, A_ue, B_eu, 1.0, 1.0, C_int, None, None, fuse=True)
    assert err.value.code == imu.ERANGE
    assert not plan.fusable()
    assert bool((C_int == -7).all()), "the guarded launch must not have written anything"
    plan2 = imu.imunpack_plan(Qa, Qb, 8, ROW, COL)
    A2, B2 = imu.imunpack_unpack(plan2, Qa, Qb)
    ws = torch.empty(plan2.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
    imu.imunpack_gemm(plan2, A2, B2, 1.0, 1.0, C_int, None, ws, fuse=True)   # guarded launch, then the fallback
    assert np.array_equal(C_int.cpu().numpy(), want)


def test_streaming_copy_copies(imu):
    """The copy kernel behind the benchmark's measured HBM rate moves every byte (3 MiB: three bands)."""
    g = torch.Generator().manual_seed(3)
    src = torch.randint(-2 ** 31, 2 ** 31 - 1, (3 << 18,), dtype=torch.int32, generator=g).to("cuda")
    dst = torch.zeros_like(src)
    assert imu.imunpack_diag_copy(src, dst) == 2 * (3 << 20)
    assert torch.equal(src, dst)
    with pytest.raises(imu.ImunpackError):
        imu.imunpack_diag_copy(src[:1000], dst[:1000])


def test_clock_probe_reports_a_plausible_clock_and_leaves_the_result_alone(imu):
    """While the probe is set a fused GEMM writes {shader cycles, 100 MHz ticks} of its first workgroup's
    loop over K; the product is the same with and without it, and nothing is written once it is off."""
    rng = np.random.default_rng(11)
    Aq = rng.integers(-300, 300, size=(300, 4096)).astype(np.int32)
    Bq = rng.integers(-300, 300, size=(260, 4096)).astype(np.int32)
    want = oracle.int_gemm(Aq, Bq)
    Qa, Qb = torch.from_numpy(Aq).cuda(), torch.from_numpy(Bq).cuda()
    plan = imu.imunpack_plan(Qa, Qb, 8, ROW, COL)
    A_ue, B_eu = imu.imunpack_unpack(plan, Qa, Qb)
    assert plan.fusable()
    C_int = torch.empty(want.shape, dtype=torch.int64, device="cuda")
    ticks = torch.zeros(2, dtype=torch.int64, device="cuda")
    imu.imunpack_diag_clock_probe(ticks)
    try:
        imu.imunpack_gemm(plan, A_ue, B_eu, 1.0, 1.0, C_int, None, None, fuse=True)
        torch.cuda.synchronize()
    finally:
        imu.imunpack_diag_clock_probe(None)
    assert np.array_equal(C_int.cpu().numpy(), want)
    cyc, wall = ticks.tolist()
    assert cyc > 0 and wall > 0
    assert 300.0 < 100.0 * cyc / wall < 3000.0, (cyc, wall)
    ticks.zero_()
    imu.imunpack_gemm(plan, A_ue, B_eu, 1.0, 1.0, C_int, None, None, fuse=True)
    torch.cuda.synchronize()
    assert ticks.tolist() == [0, 0]
    assert np.array_equal(C_int.cpu().numpy(), want)


@pytest.mark.parametrize("kind,b", [("scattered", 8), ("channels", 8), ("heavy", 4), ("deep", 8), ("clean", 8), ("rows", 3)])
def test_price_matches_unpacked_sizes(imu, kind, b):
    """Sec. 4.2: the sizes n', d', h' (and so the unpack ratio r) that imunpack_price reads off the scan
    statistics equal those of the oracle's literal UnpackRow / UnpackColumn for all four pairs, and
    the pair it picks has the smallest r."""
    w = workloads.small(seed=21, n=150, d=260, h=90, kind=kind, b=b)
    Aq, _ = oracle.rtn_quantize(w.A.numpy(), w.scale_a)
    Bq, _ = oracle.rtn_quantize(w.B.numpy(), w.scale_b)
    Qa, Qb = torch.from_numpy(Aq).cuda(), torch.from_numpy(Bq).cuda()
    st_a, st_b = imu.imunpack_scan(Qa, b), imu.imunpack_scan(Qb, b)
    dims, ratios, best = imu.imunpack_price(st_a, w.n, st_b, w.h, w.d, b)
    want_r = {}
    for pair in dims:
        hnd = oracle.unpack_pair_handle(Aq, Bq, b, pair[0], pair[1])
        assert dims[pair] == (hnd.n_u, hnd.d_u, hnd.h_u), pair
        want_r[pair] = hnd.n_u * hnd.d_u * hnd.h_u / (w.n * w.d * w.h)
        assert abs(ratios[pair] - want_r[pair]) <= 1e-12 * want_r[pair]
        hnd.close()
    assert want_r[best] == min(want_r.values())
    # and the planner agrees with the price of the chosen pair
    plan = imu.imunpack_plan(Qa, Qb, b, best[0], best[1], st_a, st_b)
    assert plan.dims()[:3] == (dims[best][0], dims[best][1], dims[best][2])


@pytest.mark.parametrize("shape", [(1, 1), (3, 5), (64, 256), (200, 1000), (77, 130), (513, 260), (2048, 2048)])
@pytest.mark.parametrize("p", [0.5, 50.0, 95.0, 99.9, 100.0])
def test_percentile_matches_the_order_statistic(imu, shape, p):
    """alpha_p on the device is the oracle's order statistic, bit for bit (it is an entry of the
    matrix): heavy-tailed values with ties, infinities and zeros, row-major and transposed views."""
    g = torch.Generator().manual_seed(shape[0] * 7919 + shape[1] + int(p * 10))
    x = torch.randn(shape, generator=g) * 0.02
    x[torch.rand(shape, generator=g) < 0.01] *= 50.0
    flat = x.view(-1)
    n = flat.numel()
    if n > 8:
        flat[torch.randint(0, n, (max(1, n // 7),), generator=g)] = float(flat[0])      # ties
        flat[torch.randint(0, n, (max(1, n // 50),), generator=g)] = 0.0
        flat[1] = float("inf")
        flat[2] = -float("inf")
    want = oracle.percentile_alpha(x.numpy(), p)
    for view in (x.to("cuda"), x.t().contiguous().to("cuda").t()):           # unit column stride / unit row stride
        alpha, status = imu.imunpack_percentile(view, p)
        assert int(status.item()) == 0
        got = alpha.cpu().numpy()[0]
        assert got == want or (np.isinf(got) and np.isinf(want)), (got, want)
    # a view with neither stride 1 and an odd row pitch (scalar path)
    wide = torch.zeros((shape[0], 2 * shape[1] + 1), device="cuda")
    wide[:, 0:2 * shape[1]:2] = x.to("cuda")
    alpha, status = imu.imunpack_percentile(wide[:, 0:2 * shape[1]:2], p)
    assert alpha.cpu().numpy()[0] == want or np.isinf(want)


def test_percentile_flags_nan_and_rejects_bad_arguments(imu):
    x = torch.randn(33, 70, device="cuda")
    alpha, status = imu.imunpack_percentile(x, 95.0)
    assert int(status.item()) == 0
    x[5, 6] = float("nan")
    alpha, status = imu.imunpack_percentile(x, 95.0)
    assert int(status.item()) == 1
    for bad in (0.0, -1.0, 100.5, float("nan")):
        with pytest.raises(imu.ImunpackError) as err:
            imu.imunpack_percentile(x, bad)
        assert err.value.code == imu.EINVAL


def test_percentile_step_feeds_the_quantizer(imu):
    """Eq. (quantized_A) end to end: alpha_95 on the device, the step alpha / (0.5 beta), RTN on the
    device; equal to the oracle's chain on the same matrix."""
    g = torch.Generator().manual_seed(11)
    x = torch.randn((300, 520), generator=g) * 0.05
    x[:, 17] *= 40.0
    for beta in (15, 255):
        alpha, _ = imu.imunpack_percentile(x.to("cuda"), 95.0)
        a = alpha.cpu().numpy()[0]
        assert a == oracle.percentile_alpha(x.numpy(), 95.0)
        step = oracle.rtn_step(a, beta)
        Q, _, flag = imu.imunpack_quantize(x.to("cuda"), float(step), 8)
        want, st = oracle.rtn_quantize(x.numpy(), step)
        assert st == 0 and int(flag.item()) == 0
        assert np.array_equal(Q.cpu().numpy(), want)


def _oracle_matmul(A, B, p, beta_a, beta_b):
    """A B^T through the oracle: alpha_p, RTN step, RTN, exact int64 GEMM, fp64 dequantisation."""
    sa = oracle.rtn_step(oracle.percentile_alpha(A, p), beta_a)
    sb = oracle.rtn_step(oracle.percentile_alpha(B, p), beta_b)
    Aq, fa = oracle.rtn_quantize(np.ascontiguousarray(A), sa)
    Bq, fb = oracle.rtn_quantize(np.ascontiguousarray(B), sb)
    assert fa == 0 and fb == 0
    return oracle.dequantize(oracle.int_gemm(Aq, Bq), sa, sb)


@pytest.mark.parametrize("b,strategies", [(8, (BOTH, BOTH)), (5, (ROW, COL)), (4, (COL, ROW))])
def test_linear_layer_forward_and_backward(imu, b, strategies):
    """The three GEMMs of a linear layer (Sec. 3) against the oracle chain on the same operands:
    Y = X W^T, grad_X = grad_Y W, grad_W = grad_Y^T X, each within 1e-6 relative of the exactly
    dequantised integer product (the transposed operands go through the strided quantize path)."""
    from paper_2403_07339_amd import linear
    g = torch.Generator().manual_seed(100 + b)
    n, d, h = 200, 320, 136
    x = torch.randn((n, d), generator=g)
    x[:, 7] *= 30.0                                     # an outlier channel
    cfg = linear.QuantConfig(beta_x=31.0, beta_w=31.0, beta_g=255.0, p=95.0, b=b,
                             strategy_a=strategies[0], strategy_b=strategies[1])
    layer = linear.IMUnpackLinear(d, h, bias=True, cfg=cfg, device="cuda")
    with torch.no_grad():
        w = torch.randn((h, d), generator=g) * 0.05
        w[torch.rand((h, d), generator=g) < 0.002] *= 25.0
        layer.weight.copy_(w)
        layer.bias.copy_(torch.randn(h, generator=g))
    xg = x.to("cuda").requires_grad_(True)
    y = layer(xg)
    gy = torch.randn((n, h), generator=g) * 1e-3
    gy[torch.rand((n, h), generator=g) < 0.01] *= 40.0   # heavy-tailed gradient
    y.backward(gy.to("cuda"))
    xn, wn, gn = x.numpy(), w.numpy(), gy.numpy()
    bias = layer.bias.detach().cpu().numpy().astype(np.float64)
    want_c = _oracle_matmul(xn, wn, 95.0, 31.0, 31.0)
    want_gx = _oracle_matmul(gn, wn.T, 95.0, 255.0, 31.0)
    want_gw = _oracle_matmul(gn.T, xn.T, 95.0, 255.0, 31.0)
    # the product is rounded to fp32 once, the bias addition once more: both relative to their own operands
    got_y = y.detach().cpu().numpy().astype(np.float64)
    assert (np.abs(got_y - (want_c + bias)) <= 2 * REL_TOL * (np.abs(want_c) + np.abs(bias)[None, :])).all()
    for got, want in ((xg.grad, want_gx), (layer.weight.grad, want_gw)):
        got = got.detach().cpu().numpy().astype(np.float64)
        assert (np.abs(got - want) <= REL_TOL * np.abs(want)).all()
    assert np.allclose(layer.bias.grad.cpu().numpy(), gn.sum(0), rtol=1e-5, atol=1e-6)
    # and the quantised layer tracks the fp32 one to within the RTN error of beta = 31 / 255
    ref = torch.nn.functional.linear(x, w, layer.bias.detach().cpu())
    rel = (y.detach().cpu() - ref).norm() / ref.norm()
    assert float(rel) < 0.15


@pytest.mark.parametrize("b,strategies", [(8, (BOTH, BOTH)), (4, (ROW, COL))])
def test_attention_gemms_forward_and_backward(imu, b, strategies):
    """The six GEMMs of self-attention (Sec. 3), two sequences x three heads, each against the oracle
    chain on the very operands the module fed it (the softmax between them is fp32 arithmetic outside
    the GEMMs, so the intermediates are taken from the module's trace):
    P = Q K^T, O = M V, grad_M = grad_O V^T, grad_V = M^T grad_O, grad_Q = grad_P K, grad_K = grad_P^T Q."""
    from paper_2403_07339_amd import attention, linear
    g = torch.Generator().manual_seed(300 + b)
    lead, T, dh = (2, 3), 72, 40
    q = torch.randn((*lead, T, dh), generator=g)
    k = torch.randn((*lead, T, dh), generator=g)
    v = torch.randn((*lead, T, dh), generator=g)
    k[..., 5] *= 12.0                                     # an outlier channel in the keys
    cfg = linear.QuantConfig(beta_x=31.0, beta_w=31.0, beta_g=255.0, p=95.0, b=b,
                             strategy_a=strategies[0], strategy_b=strategies[1])
    trace = {}
    attn = attention.IMUnpackAttention(cfg, trace)
    qd, kd, vd = (t.to("cuda").requires_grad_(True) for t in (q, k, v))
    out = attn(qd, kd, vd)
    go = torch.randn((*lead, T, dh), generator=g) * 1e-2
    go[torch.rand(go.shape, generator=g) < 0.01] *= 30.0
    out.backward(go.to("cuda"))
    assert out.shape == (*lead, T, dh) and set(trace) == {"P", "M", "O", "grad_M", "grad_P"}
    t = {name: val.detach().cpu().numpy() for name, val in trace.items()}
    gq, gk, gv = (x.grad.detach().cpu().numpy() for x in (qd, kd, vd))
    qn, kn, vn, gon = q.numpy(), k.numpy(), v.numpy(), go.numpy()
    bx, bg = 31.0, 255.0

    def close(got, want):
        return (np.abs(got.astype(np.float64) - want) <= REL_TOL * np.abs(want)).all()

    assert np.array_equal(t["O"], out.detach().cpu().numpy())
    for i in range(lead[0]):
        for j in range(lead[1]):
            M, gP = t["M"][i, j], t["grad_P"][i, j]
            assert close(t["P"][i, j], _oracle_matmul(qn[i, j], kn[i, j], 95.0, bx, bx))
            assert close(t["O"][i, j], _oracle_matmul(M, vn[i, j].T, 95.0, bx, bx))
            assert close(t["grad_M"][i, j], _oracle_matmul(gon[i, j], vn[i, j], 95.0, bg, bx))
            assert close(gv[i, j], _oracle_matmul(M.T, gon[i, j].T, 95.0, bx, bg))
            assert close(gq[i, j], _oracle_matmul(gP, kn[i, j].T, 95.0, bg, bx))
            assert close(gk[i, j], _oracle_matmul(gP.T, qn[i, j].T, 95.0, bg, bx))
    # the fp32 steps between the GEMMs, and the whole against fp32 attention
    scale = 1.0 / np.sqrt(dh)
    Mref = torch.softmax(trace["P"].cpu() * scale, -1).numpy()
    assert np.allclose(t["M"], Mref, rtol=1e-5, atol=1e-7)
    gPref = (t["grad_M"] - (t["grad_M"] * t["M"]).sum(-1, keepdims=True)) * t["M"] * scale
    assert np.allclose(t["grad_P"], gPref, rtol=1e-4, atol=1e-8)
    ref = torch.nn.functional.scaled_dot_product_attention(q, k, v)
    rel = (out.detach().cpu() - ref).norm() / ref.norm()
    assert float(rel) < 0.2


@pytest.mark.parametrize("seed", list(range(24)))
def test_random_shapes_strategies_and_densities(imu, seed):
    """Seeded sweep over what the other cases fix: ragged shapes from one row to a few tiles, every
    bit width, every strategy pair, OB densities from none to most entries, up to five digits, heavy
    rows / heavy columns / scattered entries mixed."""
    rng = np.random.default_rng(9000 + seed)
    b = int(rng.integers(2, 9))
    s = 1 << (b - 1)
    n, d, h = (int(rng.integers(1, 520)) for _ in range(3))
    sa, sb = int(rng.integers(0, 3)), int(rng.integers(0, 3))
    depth = int(rng.integers(1, 6 if b <= 4 else 4))
    p_ob = float(rng.choice([0.0, 0.001, 0.02, 0.3, 0.9]))
    Aq = rand_ints(rng, n, d, s, p_ob, depth)
    Bq = rand_ints(rng, h, d, s, float(rng.choice([0.0, 0.005, 0.1])), depth)
    if rng.random() < 0.5 and d > 2:      # heavy columns of A (outlier channels)
        Aq[:, rng.integers(0, d, 2)] = rng.integers(-(s ** depth), s ** depth + 1, size=(n, 2)).astype(np.int32)
    if rng.random() < 0.5 and h > 2:      # heavy rows of B
        Bq[rng.integers(0, h, 2), :] = rng.integers(-(s ** depth), s ** depth + 1, size=(2, d)).astype(np.int32)
    check_against_oracle(imu, Aq, Bq, b, sa, sb)


def test_rtn_step_on_the_device(imu):
    """alpha_p / (0.5 beta) formed on the device against the oracle's order statistic and binary32 division;
    the fall-backs for a mostly-zero and an all-zero matrix (largest magnitude, then 1)."""
    g = torch.Generator().manual_seed(11)
    x = torch.randn((300, 260), generator=g) * 0.7
    x[torch.rand(x.shape, generator=g) < 0.01] *= 90.0
    xd = dev(x)
    for p, beta, view, view_d in ((95.0, 31.0, x, xd), (99.0, 255.0, x.t(), xd.t()), (50.0, 15.0, x[:, ::2], xd[:, ::2])):
        step, status = imu.imunpack_rtn_step(view_d, p, beta)
        want = oracle.rtn_step(oracle.percentile_alpha(view.contiguous().numpy(), p), beta)
        assert int(status.item()) == 0
        assert step.cpu().numpy().view(np.uint32)[0] == np.float32(want).view(np.uint32)
    sparse = torch.zeros((64, 64))
    sparse[3, 5] = -7.5                                    # the 95th percentile of the magnitudes is 0
    step, _ = imu.imunpack_rtn_step(dev(sparse), 95.0, 31.0)
    assert step.item() == float(np.float32(7.5) / np.float32(15.5))
    step, _ = imu.imunpack_rtn_step(dev(torch.zeros((64, 64))), 95.0, 31.0)
    assert step.item() == 1.0


@pytest.mark.parametrize("b,strategies", [(8, (BOTH, BOTH)), (4, (ROW, COL)), (6, (COL, BOTH))])
def test_gemm_batched_matches_the_oracle_chain_per_item(imu, b, strategies):
    """imunpack_gemm_batched: five products of one shape in one call, operands passed as strided views (one
    of them transposed), each against the oracle chain percentile -> step -> RTN -> exact int64 GEMM -> fp64
    dequantisation on that item's own operands; a second call on the same context with a smaller shape."""
    g = torch.Generator().manual_seed(500 + b)
    ctx = imu.BatchContext()
    for batch, n, d, h in ((5, 48, 72, 56), (2, 17, 40, 9)):
        a = torch.randn((batch, n, d), generator=g)
        a[:, :, 3] *= 25.0
        bt = torch.randn((batch, d, h), generator=g) * 0.03          # stored d x h: B_i is its transpose
        bt[torch.rand(bt.shape, generator=g) < 0.004] *= 30.0
        A_d, B_d = dev(a), dev(bt).transpose(-1, -2)
        out = imu.imunpack_gemm_batched(A_d, B_d, 95.0, 31.0, 63.0, b, strategies[0], strategies[1], ctx=ctx)
        assert out.shape == (batch, n, h)
        got = out.cpu().numpy().astype(np.float64)
        for i in range(batch):
            want = _oracle_matmul(a[i].numpy(), bt[i].t().contiguous().numpy(), 95.0, 31.0, 63.0)
            assert (np.abs(got[i] - want) <= REL_TOL * np.abs(want)).all(), i
    with pytest.raises(imu.ImunpackError):                           # a NaN in one item is reported
        bad = a.clone()
        bad[1, 2, 3] = float("nan")
        imu.imunpack_gemm_batched(dev(bad), B_d, 95.0, 31.0, 63.0, b, strategies[0], strategies[1], ctx=ctx)
    ctx.destroy()
