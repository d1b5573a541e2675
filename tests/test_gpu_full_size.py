"""Full-size parity on the benchmark workloads (2-5; workload 1 is covered element by element in
test_gpu_parity.py), in the launch configuration bench.py times: caller-provided statistics and OB
lists from the fused quantize pass, fused GEMM epilogue.

Compared in full: the quantized integers, the unpack plan and both unpacked int8 operands in the
paper's order (the CPU oracle unpacks the full operands in seconds), the int64 product and the fp32
output, from the fused launch and from the un-fused path (the oracle's triple loop takes a few seconds
per workload on the host cores)."""
import numpy as np
import pytest
import torch

import oracle
from paper_2403_07339_amd import workloads

pytestmark = pytest.mark.gpu
REL_TOL = 1e-6


@pytest.fixture(scope="module")
def imu():
    if not torch.cuda.is_available():
        pytest.skip("no GPU")
    from paper_2403_07339_amd import binding
    return binding


@pytest.mark.parametrize("index", [2, 3, 4, 5])
def test_workload_full_size(imu, index):
    w = workloads.make(index)
    s = 1 << (w.b - 1)
    print(f"workload {index}: {w.name}", flush=True)
    Aq, sta = oracle.rtn_quantize(w.A.contiguous().numpy(), w.scale_a)
    Bq, stb = oracle.rtn_quantize(w.B.contiguous().numpy(), w.scale_b)
    assert sta == 0 and stb == 0
    A_d, B_d = w.A.to("cuda"), w.B.to("cuda")          # workload 4 keeps its transposed strides
    Qa, st_a, fa = imu.imunpack_quantize(A_d, w.scale_a, w.b, want_ob_list=w.strategy_a == imu.BOTH)
    Qb, st_b, fb = imu.imunpack_quantize(B_d, w.scale_b, w.b, want_ob_list=w.strategy_b == imu.BOTH)
    assert int(fa.item()) == 0 and int(fb.item()) == 0
    assert np.array_equal(Qa.cpu().numpy(), Aq) and np.array_equal(Qb.cpu().numpy(), Bq)
    for st, q in ((st_a, Aq), (st_b, Bq)):
        a = np.abs(q.astype(np.int64))
        assert np.array_equal(st.rowcnt.cpu().numpy(), (a >= s).sum(1))
        assert np.array_equal(st.colcnt.cpu().numpy(), (a >= s).sum(0))
        assert np.array_equal(st.rowmax.cpu().numpy(), a.max(1))
        assert np.array_equal(st.colmax.cpu().numpy(), a.max(0))
        if st.ob is not None:
            cnt = int(st.ob_count.item())
            assert cnt == int((a >= s).sum()) and cnt <= st.ob.shape[1]
            ob = st.ob[:, :cnt].cpu().numpy()
            assert np.array_equal(q[ob[0], ob[1]], ob[2])
            assert len(np.unique(ob[0].astype(np.int64) * q.shape[1] + ob[1])) == cnt

    hnd = oracle.unpack_pair_handle(Aq, Bq, w.b, w.strategy_a, w.strategy_b)
    assert hnd.max_abs() <= s - 1
    plan = imu.imunpack_plan(Qa, Qb, w.b, w.strategy_a, w.strategy_b, st_a, st_b)
    n_u, d_u, h_u, ng = plan.dims()
    assert (n_u, d_u, h_u) == (hnd.n_u, hnd.d_u, hnd.h_u)
    S, pas, paw, pbs, pbw = hnd.meta()
    ra_s, ra_e, rb_s, rb_e, c_s, c_e, c_par, ops = [t.numpy().astype(np.int64) for t in plan.export_all()]
    want_parent, want_ops = hnd.trace()
    assert np.array_equal(c_s, hnd.col_src()) and np.array_equal(c_par, want_parent)
    assert np.array_equal(ops, want_ops)          # every split, in the order Alg. 1 / 2 / 4 make them
    assert np.array_equal(ra_s, pas) and np.array_equal(s ** ra_e.astype(object), paw.astype(object))
    assert np.array_equal(rb_s, pbs) and np.array_equal(s ** rb_e.astype(object), pbw.astype(object))
    assert np.array_equal(s ** c_e.astype(object), S.astype(object))
    assert ng == len(np.unique(S))

    A_ue, B_eu = imu.imunpack_unpack(plan, Qa, Qb)
    Ac, Bc = imu.imunpack_unpack_canonical(plan, A_ue, B_eu)
    oa, ob_ = hnd.operands_i8()
    assert np.array_equal(Ac.cpu().numpy(), oa)
    assert np.array_equal(Bc.cpu().numpy(), ob_)
    # the accumulator bounds: max over rows of sum_c S[c] |digit|, on the oracle's operands
    S64 = S.astype(np.int64)
    for got, m in zip(plan.bounds(), (oa, ob_)):
        want_b = max(int((np.abs(m[r0:r0 + 1024].astype(np.int64)) * S64[None, :]).sum(1).max())
                     for r0 in range(0, m.shape[0], 1024))
        assert got == want_b
    del Ac, Bc, oa, ob_

    assert plan.fusable(), "the benchmark workloads are expected to take the fused path"
    C_int = torch.empty((w.n, w.h), dtype=torch.int64, device="cuda")
    C_fp = torch.empty((w.n, w.h), dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, w.scale_a, w.scale_b, C_int, C_fp, None, fuse=True)
    # the whole int64 product, element by element, against the oracle's triple loop
    want = oracle.int_gemm(Aq, Bq)
    got = C_int.cpu().numpy()
    assert got.shape == want.shape and np.array_equal(got, want)
    del got
    # the fp32 output against the oracle's fp64 dequantisation, in full (row bands keep the host copies small)
    C_fp_h = C_fp.cpu().numpy()
    for r0 in range(0, w.n, 2048):
        ref64 = oracle.dequantize(want[r0:r0 + 2048], w.scale_a, w.scale_b)
        assert (np.abs(C_fp_h[r0:r0 + 2048].astype(np.float64) - ref64) <= REL_TOL * np.abs(ref64)).all()
    del C_fp_h
    # the product identity through the oracle's own unpacked operands, at a few positions
    rng = np.random.default_rng(index)
    rows, cols = rng.integers(0, w.n, 64), rng.integers(0, w.h, 64)
    assert np.array_equal(hnd.product_at(rows, cols), want[rows, cols])
    # the un-fused path (one launch per diagonal entry of S into the int64 unpacked product, then the
    # recombination kernel) against the oracle as well
    ws = torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
    C2 = torch.full((w.n, w.h), -1, dtype=torch.int64, device="cuda")
    C2_fp = torch.full((w.n, w.h), float("nan"), dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, w.scale_a, w.scale_b, None, None, ws, fuse=False)
    imu.imunpack_recombine(plan, ws, w.scale_a, w.scale_b, C2, C2_fp)
    assert np.array_equal(C2.cpu().numpy(), want)
    assert torch.equal(C2_fp, C_fp)          # the same single rounding of the same integers
    if w.b <= 4:
        # the same workload with the digits stored as 6-bit floating-point codes (Sec. 4.2, low bit widths):
        # decoded operands against the oracle's, then the fused launch on the f8f6f4 matrix instruction
        plan.set_digits(imu.DIGITS_FP6)
        A6, B6 = imu.imunpack_unpack(plan, Qa, Qb)
        assert A6.numel() * 4 == A_ue.numel() * 3 or A6.numel() < A_ue.numel()
        Ac, Bc = imu.imunpack_unpack_canonical(plan, A6, B6)
        oa, ob_ = hnd.operands_i8()
        assert np.array_equal(Ac.cpu().numpy(), oa) and np.array_equal(Bc.cpu().numpy(), ob_)
        del Ac, Bc, oa, ob_
        assert plan.fusable(), "workload 5 is expected to stay below 2^24 in the binary32 accumulators"
        C6 = torch.full((w.n, w.h), -1, dtype=torch.int64, device="cuda")
        C6_fp = torch.full((w.n, w.h), float("nan"), dtype=torch.float32, device="cuda")
        imu.imunpack_gemm(plan, A6, B6, w.scale_a, w.scale_b, C6, C6_fp, None, fuse=True)
        assert np.array_equal(C6.cpu().numpy(), want) and torch.equal(C6_fp, C_fp)
        C6.fill_(-1)
        imu.imunpack_gemm(plan, A6, B6, w.scale_a, w.scale_b, None, None, ws, fuse=False)
        imu.imunpack_recombine(plan, ws, w.scale_a, w.scale_b, C6, None)
        assert np.array_equal(C6.cpu().numpy(), want)
        del A6, B6, C6, C6_fp
        plan.set_digits(imu.DIGITS_INT8)
    del ws, C2, C2_fp, want
    # every fp32 output is the rounded dequantisation of its own int64 (checked on the device in fp64)
    ref = C_int.to(torch.float64) * (float(np.float32(w.scale_a)) * float(np.float32(w.scale_b)))
    err = (C_fp.to(torch.float64) - ref).abs()
    assert bool((err <= REL_TOL * ref.abs()).all())
    del ref, err, C_int
    # the launch bench.py times asks for the fp32 output alone (the epilogue may then add digit levels
    # up in binary64): the same bits
    C_fp_only = torch.empty((w.n, w.h), dtype=torch.float32, device="cuda")
    imu.imunpack_gemm(plan, A_ue, B_eu, w.scale_a, w.scale_b, None, C_fp_only, None, fuse=True)
    assert torch.equal(C_fp_only, C_fp)
    hnd.close()


def test_percentile_full_size(imu):
    """alpha_95 of the two operands of the benchmark workload, against the sorted magnitudes."""
    w = workloads.make(3)
    for X in (w.A, w.B):
        alpha, status = imu.imunpack_percentile(X.to("cuda"), 95.0)
        assert int(status.item()) == 0
        assert alpha.cpu().numpy()[0] == oracle.percentile_alpha(X.numpy(), 95.0)


def test_more_rows_than_a_launch_dimension(imu):
    """70 000 rows: more row blocks than one grid dimension holds in the quantize, scatter and
    recombine launches.  Quantised integers, plan sizes and both unpacked operands in full; the
    product at sampled positions and through the column-sum identity."""
    n, d, h, b = 70001, 256, 384, 8
    g = torch.Generator().manual_seed(77)
    A = torch.randn((n, d), generator=g)
    A[:, 5] *= 60.0
    A[torch.rand((n, d), generator=g) < 0.0005] *= 300.0
    B = torch.randn((h, d), generator=g) * 0.02
    B[torch.rand((h, d), generator=g) < 0.002] *= 40.0
    sa, sb = float(4 * A.std() / 127), float(4 * B.std() / 127)
    Aq, fa = oracle.rtn_quantize(A.numpy(), sa)
    Bq, fb = oracle.rtn_quantize(B.numpy(), sb)
    assert fa == 0 and fb == 0
    for strat_a, strat_b in ((imu.BOTH, imu.BOTH), (imu.ROW, imu.COL)):
        Qa, st_a, f1 = imu.imunpack_quantize(A.to("cuda"), sa, b, want_ob_list=strat_a == imu.BOTH)
        Qb, st_b, f2 = imu.imunpack_quantize(B.to("cuda"), sb, b, want_ob_list=strat_b == imu.BOTH)
        assert int(f1.item()) == 0 and int(f2.item()) == 0
        assert np.array_equal(Qa.cpu().numpy(), Aq) and np.array_equal(Qb.cpu().numpy(), Bq)
        hnd = oracle.unpack_pair_handle(Aq, Bq, b, strat_a, strat_b)
        plan = imu.imunpack_plan(Qa, Qb, b, strat_a, strat_b, st_a, st_b)
        n_u, d_u, h_u, _ = plan.dims()
        assert (n_u, d_u, h_u) == (hnd.n_u, hnd.d_u, hnd.h_u)
        A_ue, B_eu = imu.imunpack_unpack(plan, Qa, Qb)
        Ac, Bc = imu.imunpack_unpack_canonical(plan, A_ue, B_eu)
        oa, ob_ = hnd.operands_i8()
        assert np.array_equal(Ac.cpu().numpy(), oa) and np.array_equal(Bc.cpu().numpy(), ob_)
        del Ac, Bc, oa, ob_
        C_int = torch.empty((n, h), dtype=torch.int64, device="cuda")
        C_fp = torch.empty((n, h), dtype=torch.float32, device="cuda")
        ws = None if plan.fusable() else torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
        imu.imunpack_gemm(plan, A_ue, B_eu, sa, sb, C_int, C_fp, ws, fuse=True)
        rng = np.random.default_rng(3)
        rows = np.concatenate([rng.integers(0, n, 2000), [0, n - 1, 65535, 65536]])
        cols = np.concatenate([rng.integers(0, h, 2000), [0, h - 1, 1, 2]])
        want = oracle.int_gemm_at(Aq, Bq, rows, cols)
        ri, ci = torch.from_numpy(rows).cuda(), torch.from_numpy(cols).cuda()
        assert np.array_equal(C_int[ri, ci].cpu().numpy(), want)
        want_fp = oracle.dequantize(want, sa, sb)
        got_fp = C_fp[ri, ci].cpu().numpy().astype(np.float64)
        assert (np.abs(got_fp - want_fp) <= REL_TOL * np.abs(want_fp)).all()
        total = int(C_int.sum().item())
        assert total == int((Aq.astype(np.int64).sum(0).astype(object) * Bq.astype(np.int64).sum(0).astype(object)).sum())
        # the un-fused path too (its recombine launch has one block row per source row)
        ws2 = torch.empty(plan.unpacked_bytes()[2] // 8, dtype=torch.int64, device="cuda")
        C2 = torch.full((n, h), -1, dtype=torch.int64, device="cuda")
        imu.imunpack_gemm(plan, A_ue, B_eu, sa, sb, None, None, ws2, fuse=False)
        imu.imunpack_recombine(plan, ws2, sa, sb, C2, None)
        assert bool((C2 == C_int).all())
        hnd.close()
