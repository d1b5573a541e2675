#!/usr/bin/env python3
"""Benchmark of the exact low-bit integer GEMM hot path on one MI355X.

One step = one pass of the whole path over one seeded synthetic GEMM already resident in HBM:
RTN-quantize A and B (fused heavy-hitter scan) -> unpack plan -> digit scatter -> int8 MFMA GEMM with
the recombination and dequantisation fused into its epilogue (fp32 output).  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 1..5] [--no-cpu-baseline] [--steps-only]

Roofline figures are algorithmic bytes or operations per launch divided by the launch durations measured
here with events on the stream the kernels run on; the HBM traffic beside them comes from the tracked
rocprofv3 summary ``profiles/bench_workload<k>_kernels.json`` (written by
``python -m paper_2403_07339_amd.profile_summary``), if there is one for the workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0   # MI355X dense int8 MFMA peak, 5.0 POP/s
FP6_PEAK_TOPS = 10100.0   # dense fp6 / fp4 MFMA peak, 10.1 PFLOP/s
HBM_PEAK_GBS = 8000.0     # MI355X HBM3E peak


def profiled_traffic(workload: int, digits: str = "int8"):
    """HBM bytes per launch by kernel from the tracked rocprofv3 summary of this workload's step
    (FETCH_SIZE + WRITE_SIZE, each scaled by a plain copy of known size), or {} if none is there."""
    path = os.path.join(ROOT, "profiles", f"bench_workload{workload}{'_fp6' if digits == 'fp6' else ''}_kernels.json")
    if not os.path.exists(path):
        return {}, None
    doc = json.load(open(path))
    out = {}
    for k in doc.get("kernels", []):
        if k.get("hbm_read_bytes") is None or k.get("hbm_written_bytes") is None:
            continue
        key = k["kernel"].split("<")[0]
        out[key] = out.get(key, 0.0) + k["hbm_read_bytes"] + k["hbm_written_bytes"]   # operands A and B: two launches
    return out, os.path.relpath(path, ROOT)


def cpu_baseline(w, budget_rows: int = 4096):
    """The CPU oracle (unchanged, untuned) on a bounded sample of the same workload: RTN of both
    operands, the unpack of the full operands (Alg. 5), then the naive int64 GEMM and the fp64
    dequantisation of the sampled rows of A against all of B."""
    import oracle
    rows = min(budget_rows, w.n)
    A = w.A.contiguous().numpy()
    B = w.B.contiguous().numpy()
    t0 = time.perf_counter()
    Aq, _ = oracle.rtn_quantize(A, w.scale_a)
    Bq, _ = oracle.rtn_quantize(B, w.scale_b)
    t1 = time.perf_counter()
    hnd = oracle.unpack_pair_handle(Aq, Bq, w.b, w.strategy_a, w.strategy_b)
    hnd.close()
    t2 = time.perf_counter()
    C = oracle.int_gemm(Aq[:rows], Bq)
    _ = oracle.dequantize(C, w.scale_a, w.scale_b)
    t3 = time.perf_counter()
    # scaled to the metric's unit: the sampled rows' share of the quantize/unpack time plus their GEMM
    dt = (t2 - t0) * rows / w.n + (t3 - t2)
    ops = 2.0 * rows * w.d * w.h
    return {"value": ops / dt / 1e12, "unit": "TOPS", "cores": oracle.num_threads(), "kind": "oracle",
            "sample": f"RTN of A and B {t1 - t0:.1f} s, unpack of both operands {t2 - t1:.1f} s, naive int64 GEMM + "
                      f"fp64 dequantise of the first {rows} of {w.n} rows of A against all of B {t3 - t2:.1f} s"}


def measure_extras(torch, imu, workloads, w, Qa, Qb, st_a, st_b, status, A, B, C_fp, args):
    """Untimed side measurements reported beside the headline: the two quantize calls on their own, this
    library's GEMM on the original shape with operands clipped to int8 (what one pays without
    exactness), and the measured peaks of the matrix cores and of a device-to-device copy."""
    def timed(fn, reps):
        fn()
        torch.cuda.synchronize()
        a, b = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        a.record()
        for _ in range(reps):
            fn()
        b.record()
        torch.cuda.synchronize()
        return a.elapsed_time(b) / reps
    res = {}
    res["quant_a_ms"] = timed(lambda: imu.imunpack_quantize(A, w.scale_a, w.b, Qa, st_a, status[0:1]), 10)
    res["quant_b_ms"] = timed(lambda: imu.imunpack_quantize(B, w.scale_b, w.b, Qb, st_b, status[1:2]), 10)
    lim = (1 << (w.b - 1)) - 1
    Qa_c, Qb_c = Qa.clamp(-lim, lim), Qb.clamp(-lim, lim)
    plain = imu.imunpack_plan(Qa_c, Qb_c, w.b, imu.ROW, imu.ROW)
    A8, B8 = imu.imunpack_unpack(plain, Qa_c, Qb_c)
    assert plain.unpack_ratio() == 1.0 and plain.fusable()
    res["plain_gemm_ms"] = timed(lambda: imu.imunpack_gemm(plain, A8, B8, w.scale_a, w.scale_b, None, C_fp, None,
                                                           fuse=True), 10)
    del plain, A8, B8, Qa_c, Qb_c
    ops = [0]
    def peak():
        ops[0] = imu.imunpack_diag_mfma_peak(256 * 4, 4000)
    ms = timed(peak, 3)
    res["mfma_peak_tops"] = ops[0] / ms / 1e9
    # ---- "Mix" (Sec. 4.2): every pair of strategies is priced by its unpack ratio r -- the four
    # one-axis pairs from the scan statistics alone, the pairs with UnpackBoth by planning with it --
    # and, because equal r does not mean equal time (split rows cost the GEMM epilogue, UnpackBoth
    # costs the planner), the pairs whose r is within 25 % of the smallest are run and the fastest kept.
    names = workloads.STRATEGY_NAMES
    _, ratios, _ = imu.imunpack_price(st_a, w.n, st_b, w.h, w.d, w.b)
    mix_plan = imu.Plan()
    # UnpackBoth is a sequential greedy (Alg. 4; the paper itself uses it for weights at load time only):
    # on an operand where more than 1 % of the entries are out of bound its planner alone takes far
    # longer than the whole step of any other pair, so such pairs are neither planned nor timed here.
    s_ob = 1 << (w.b - 1)
    dense_ob = {0: float((Qa.abs() >= s_ob).float().mean().item()) > 0.01,
                1: float((Qb.abs() >= s_ob).float().mean().item()) > 0.01}
    # the OB entry lists that UnpackBoth plans from, for the operands it is tried on
    mst_a = st_a if (st_a.ob is not None or dense_ob[0]) else imu.Stats.empty(w.n, w.d, A.device, imu.Stats.default_ob_cap(w.n, w.d))
    mst_b = st_b if (st_b.ob is not None or dense_ob[1]) else imu.Stats.empty(w.h, w.d, A.device, imu.Stats.default_ob_cap(w.h, w.d))
    imu.imunpack_quantize(A, w.scale_a, w.b, Qa, mst_a, status[0:1])
    imu.imunpack_quantize(B, w.scale_b, w.b, Qb, mst_b, status[1:2])
    configured = (w.strategy_a, w.strategy_b)
    all_r = {}
    for sa in (imu.ROW, imu.COL, imu.BOTH):
        for sb in (imu.ROW, imu.COL, imu.BOTH):
            if (sa, sb) in ratios:
                all_r[(sa, sb)] = ratios[(sa, sb)]
            elif (sa, sb) != configured and ((sa == imu.BOTH and dense_ob[0]) or (sb == imu.BOTH and dense_ob[1])):
                all_r[(sa, sb)] = None
            else:
                imu.imunpack_plan(Qa, Qb, w.b, sa, sb, mst_a, mst_b, mix_plan)
                all_r[(sa, sb)] = mix_plan.unpack_ratio()
    res["priced_r"] = {f"{names[p[0]]}/{names[p[1]]}": r for p, r in all_r.items()}
    known = {p: r for p, r in all_r.items() if r is not None}
    rmin = min(known.values())
    cands = sorted((p for p, r in known.items() if r <= 1.25 * rmin and p != configured), key=lambda p: known[p])[:4]
    cands.append(configured)
    mix = {"A": None, "B": None, "ws": None}

    def mix_step(pair):
        imu.imunpack_quantize(A, w.scale_a, w.b, Qa, mst_a, status[0:1])
        imu.imunpack_quantize(B, w.scale_b, w.b, Qb, mst_b, status[1:2])
        imu.imunpack_plan(Qa, Qb, w.b, pair[0], pair[1], mst_a, mst_b, mix_plan)
        ba, bb, bw = mix_plan.unpacked_bytes()
        if mix["A"] is None or mix["A"].numel() < ba:
            mix["A"] = torch.empty(ba, dtype=torch.int8, device=A.device)
        if mix["B"] is None or mix["B"].numel() < bb:
            mix["B"] = torch.empty(bb, dtype=torch.int8, device=A.device)
        imu.imunpack_unpack(mix_plan, Qa, Qb, mix["A"], mix["B"])
        if not mix_plan.fusable() and (mix["ws"] is None or mix["ws"].numel() < bw // 8):
            mix["ws"] = torch.empty(bw // 8, dtype=torch.int64, device=A.device)
        imu.imunpack_gemm(mix_plan, mix["A"], mix["B"], w.scale_a, w.scale_b, None, C_fp, mix["ws"], fuse=True)

    timed_ms = {}
    for pair in cands:
        for _ in range(3):
            mix_step(pair)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            mix_step(pair)
        torch.cuda.synchronize()
        timed_ms[pair] = (time.perf_counter() - t0) * 1e3 / 5
    best = min(timed_ms, key=timed_ms.get)
    res["mix_timed_ms"] = {f"{names[p[0]]}/{names[p[1]]}": t for p, t in timed_ms.items()}
    res["priced_best"] = f"{names[best[0]]}/{names[best[1]]}"
    res["mix_ms"] = timed_ms[best]
    res["mix_r"] = known[best]
    mix_plan.destroy()
    del mix, mst_a, mst_b
    src = torch.empty(1 << 28, dtype=torch.float32, device="cuda")
    dst = torch.empty_like(src)
    ms = timed(lambda: dst.copy_(src), 5)
    res["torch_copy_gbps"] = 2 * src.numel() * 4 / ms / 1e6
    ms = timed(lambda: imu.imunpack_diag_copy(src, dst), 5)   # the library's own streaming copy: the better reference
    res["copy_gbps"] = max(res["torch_copy_gbps"], 2 * src.numel() * 4 / ms / 1e6)
    del src, dst
    torch.cuda.empty_cache()
    return res


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", type=int, default=3)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--with-int64", action="store_true", help="also write the int64 product (parity output)")
    ap.add_argument("--digits", choices=["int8", "fp6"], default="int8",
                    help="storage of the digits: fp6 (e2m3 codes on the f8f6f4 matrix instruction) needs b <= 4")
    ap.add_argument("--steps-only", action="store_true",
                    help="only the warm-up and the timed steps, no side measurements: the command the profiles are taken with")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="run only a plain elementwise copy of 1 GiB (read 1 GiB, write 1 GiB), five times: the "
                         "known-size kernel that hardware traffic counters are scaled by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1",
              file=sys.stderr)
        sys.exit(2)

    import torch
    from paper_2403_07339_amd import binding as imu
    from paper_2403_07339_amd import workloads

    torch.cuda.set_device(0)
    if args.calibrate_copy:
        src = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        dst = torch.empty_like(src)
        for _ in range(5):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy_bytes_read": src.numel() * 4, "calibrate_copy_bytes_written": dst.numel() * 4}))
        return
    w = workloads.make(args.workload)
    A, B = w.A.to("cuda"), w.B.to("cuda")          # strided views keep their strides
    n, d, h = w.n, w.d, w.h
    dev = A.device

    # buffers reused by every step (allocation is not part of the path)
    Qa = torch.empty((n, d), dtype=torch.int32, device=dev)
    Qb = torch.empty((h, d), dtype=torch.int32, device=dev)
    st_a = imu.Stats.empty(n, d, dev, imu.Stats.default_ob_cap(n, d) if w.strategy_a == imu.BOTH else 0)
    st_b = imu.Stats.empty(h, d, dev, imu.Stats.default_ob_cap(h, d) if w.strategy_b == imu.BOTH else 0)
    status = torch.zeros(2, dtype=torch.int32, device=dev)
    C_fp = torch.empty((n, h), dtype=torch.float32, device=dev)
    C_int = torch.empty((n, h), dtype=torch.int64, device=dev) if args.with_int64 else None
    plan = imu.Plan()
    bufs = {"A": None, "B": None, "ws": None}
    ev = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]

    fp6 = args.digits == "fp6"
    assert not fp6 or w.b <= 4, "--digits fp6 needs a workload with b <= 4"
    mfma_peak = FP6_PEAK_TOPS if fp6 else INT8_PEAK_TOPS

    def step(marks=None, quantize_b=True, c_int=C_int):
        def mark(i):
            if marks is not None:
                marks[i].record()
        mark(0)
        if quantize_b:
            imu.imunpack_quantize_pair(A, B, w.scale_a, w.scale_b, w.b, Qa, Qb, st_a, st_b, status)
        else:
            imu.imunpack_quantize(A, w.scale_a, w.b, Qa, st_a, status[0:1])
        mark(1)
        imu.imunpack_plan(Qa, Qb, w.b, w.strategy_a, w.strategy_b, st_a, st_b, plan)
        if fp6 and plan.digits() != imu.DIGITS_FP6:
            plan.set_digits(imu.DIGITS_FP6)   # stays with the plan object from here on
        mark(2)
        ba, bb, bw = plan.unpacked_bytes()
        if bufs["A"] is None or bufs["A"].numel() < ba:
            bufs["A"] = torch.empty(ba, dtype=torch.int8, device=dev)
        if bufs["B"] is None or bufs["B"].numel() < bb:
            bufs["B"] = torch.empty(bb, dtype=torch.int8, device=dev)
        imu.imunpack_unpack(plan, Qa, Qb, bufs["A"], bufs["B"])
        mark(3)
        mark(4)
        # The fused launch goes out before the host knows whether it is exact; only if it was not (and
        # no workspace was at hand for the fallback) does the call report ERANGE.
        try:
            imu.imunpack_gemm(plan, bufs["A"], bufs["B"], w.scale_a, w.scale_b, c_int, C_fp, bufs["ws"], fuse=True)
        except imu.ImunpackError as e:
            if e.code != imu.ERANGE:
                raise
            bufs["ws"] = torch.empty(bw // 8, dtype=torch.int64, device=dev)
            imu.imunpack_gemm(plan, bufs["A"], bufs["B"], w.scale_a, w.scale_b, c_int, C_fp, bufs["ws"], fuse=True)
        mark(5)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    assert int(status.sum().item()) == 0, "quantize reported NaN/Inf/overflow"
    ms_step = dt * 1e3 / args.steps
    # The stage times come from the same number of steps run once more with HIP events between the stages
    # (recording six events costs a step about 20 us, so the timed steps above carry none).
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(ev[k])
    torch.cuda.synchronize()
    ms_step_marked = (time.perf_counter() - t0) * 1e3 / args.steps
    stage_ms = [sum(e[i].elapsed_time(e[i + 1]) for e in ev) / args.steps for i in range(5)]
    n_u, d_u, h_u, ng = plan.dims()
    ba, bb, _ = plan.unpacked_bytes()
    (_, wa, _), (_, wb, _) = plan.layout()
    gemm_ms = stage_ms[4]
    gemm_ops = 2.0 * n_u * d_u * h_u
    achieved = gemm_ops / (gemm_ms * 1e-3) / 1e12
    value = w.ops / (ms_step * 1e-3) / 1e12
    traffic, traffic_file = profiled_traffic(args.workload, args.digits)
    # algorithmic bytes per launch of the memory-bound passes: quantize + scan moves 4 B in and 4 B out
    # per element; the scatter reads 4 B per source element and owes 1 B per element of the unpacked
    # operands (n' d' + h' d'), of which it stores fewer (repeated columns of A_ue are not stored)
    q_bytes = 8.0 * (n * d + h * d)
    u_bytes = 4.0 * (n * d + h * d) + (n_u + h_u) * d_u
    def hbm_entry(kernels, alg_bytes, ms, extra=None):
        got = [traffic[k] for k in kernels if k in traffic]
        e = {"bound": "hbm", "kernels": kernels, "achieved": alg_bytes / ms / 1e6, "peak": HBM_PEAK_GBS, "unit": "GB/s",
             "frac": alg_bytes / ms / 1e6 / HBM_PEAK_GBS, "algorithmic_bytes": alg_bytes,
             "traffic": sum(got) if got else None, "ms": ms}
        if extra:
            e.update(extra)
        return e
    out = {
        "metric": "effective int GEMM TOPS (2*n*d*h of the original GEMM / end-to-end time)",
        "value": value, "unit": "TOPS", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "int8 digits, int32 accumulate, int64 recombine", "data": "synthetic",
        "config": {"workload": w.name, "n": n, "d": d, "h": h, "b": w.b,
                   "strategy": f"{workloads.STRATEGY_NAMES[w.strategy_a]}/{workloads.STRATEGY_NAMES[w.strategy_b]}",
                   "outputs": "fp32" + ("+int64" if args.with_int64 else ""), "digits": args.digits},
        "frac_of_int8_peak": value / INT8_PEAK_TOPS,
        "unpack": {"n_u": n_u, "d_u": d_u, "h_u": h_u, "groups": ng,
                   "ratio_r": (n_u * d_u * h_u) / (n * d * h), "fused_epilogue": bool(plan.fusable()),
                   "stored_bytes": {"A_store": ba, "B_eu": bb, "A_ue_if_materialised": plan.layout()[0][0] * wb},
                   "stored_columns": {"A_store": wa, "B_eu": wb}},
        "stage_ms": {"quantize+scan": stage_ms[0], "plan": stage_ms[1], "scatter": stage_ms[2],
                     "gemm+recombine+dequant": gemm_ms, "host_gap": ms_step_marked - sum(stage_ms),
                     "step_with_event_marks": ms_step_marked},
        "roofline": {"bound": "mfma", "kernel": "gemm_f6_kernel<0>" if fp6 else "gemm_i8_kernel<0>", "achieved": achieved,
                     "peak": mfma_peak, "unit": "TOP/s", "frac": achieved / mfma_peak,
                     "traffic": traffic.get("gemm_f6_kernel" if fp6 else "gemm_i8_kernel"), "ms": gemm_ms, "ops": gemm_ops,
                     "algorithmic_bytes": float(ba + bb + 4 * n * h + (8 * n * h if args.with_int64 else 0))},
        "roofline_passes": {
            "quantize+scan": hbm_entry(["qscan_vec_pair_kernel", "qscan_vec_kernel", "qscan_tr_kernel", "qscan_tile_kernel", "zero_lists_kernel"],
                                       q_bytes, stage_ms[0]),
            "scatter": hbm_entry(["scatter_kernel", "fixup_kernel", "bound_kernel"], u_bytes, stage_ms[2],
                                 {"stored_and_read_bytes": 4.0 * (n * d + h * d) + ba + bb}),
        },
        "traffic_source": traffic_file,
    }
    if args.steps_only:
        print(json.dumps(out))
        return
    # Second figure: B is a weight matrix whose quantised integers and statistics are kept from one step
    # to the next (the paper unpacks weights when they are loaded, Sec. 4.2); its plan and scatter depend
    # on A's column splits here and stay in the step.
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(None, quantize_b=False)
    torch.cuda.synchronize()
    ms_step_wq = (time.perf_counter() - t0) * 1e3 / args.steps
    # ... and with the plan told that B stays what it is (imunpack_plan_keep_weights): UnpackBoth's greedy
    # on B is run again only when the column splits of A differ from the step before
    plan.keep_weights(True)
    for _ in range(2):
        step(None, quantize_b=False)
    torch.cuda.synchronize()
    reused = plan.weights_reused()
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(None, quantize_b=False)
    torch.cuda.synchronize()
    ms_step_keep = (time.perf_counter() - t0) * 1e3 / args.steps
    ev_k = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
    for k in range(args.steps):     # once more with marks, for the stage times
        step(ev_k[k], quantize_b=False)
    torch.cuda.synchronize()
    plan_keep_ms = sum(e[1].elapsed_time(e[2]) for e in ev_k) / args.steps
    scatter_keep_ms = sum(e[2].elapsed_time(e[3]) for e in ev_k) / args.steps
    plan.keep_weights(False)
    step()
    torch.cuda.synchronize()
    # Third figure: the step that also writes the int64 product the parity tests are defined on.
    if C_int is None:
        C64 = torch.empty((n, h), dtype=torch.int64, device=dev)
        for _ in range(2):
            step(None, True, C64)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(None, True, C64)
        torch.cuda.synchronize()
        ms_step_i64 = (time.perf_counter() - t0) * 1e3 / args.steps
        del C64
        out["with_int64_output"] = {"ms_per_step": ms_step_i64, "value": w.ops / (ms_step_i64 * 1e-3) / 1e12, "unit": "TOPS",
                                    "note": "same step writing the int64 product beside the fp32 output; not the headline value"}
    # The clock the matrix cores run at inside the step's own GEMM (its first workgroup times its loop
    # over K with the shader clock and with the constant 100 MHz clock): the power limit holds it below
    # the 2.4 GHz of the published peak.
    clock_mhz = None
    if plan.fusable():
        ticks = torch.zeros(2, dtype=torch.int64, device=dev)
        imu.imunpack_diag_clock_probe(ticks)
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        imu.imunpack_diag_clock_probe(None)
        cyc, wall = ticks.tolist()
        clock_mhz = 100.0 * cyc / wall if wall > 0 else None
    # b <= 4 (Sec. 4.2, low bit widths): the same step with the digits stored as 6-bit floating-point codes and
    # multiplied by the f8f6f4 matrix instruction; the configuration itself asks for int8, so this is a side figure
    if w.b <= 4 and not fp6:
        step()                                  # a plan to hang the request on
        plan.set_digits(imu.DIGITS_FP6)         # stays with the plan object through the re-planning of every step
        for _ in range(3):
            step()
        torch.cuda.synchronize()
        ev6 = [[torch.cuda.Event(enable_timing=True) for _ in range(6)] for _ in range(args.steps)]
        t0 = time.perf_counter()
        for k in range(args.steps):
            step(ev6[k])
        torch.cuda.synchronize()
        ms6 = (time.perf_counter() - t0) * 1e3 / args.steps
        gemm6 = sum(e[4].elapsed_time(e[5]) for e in ev6) / args.steps
        out["fp6_digits_step"] = {"ms_per_step": ms6, "value": w.ops / (ms6 * 1e-3) / 1e12, "unit": "TOPS",
                                  "gemm_ms": gemm6, "gemm_kernel": "gemm_f6_kernel<0>",
                                  "gemm_frac_of_fp6_peak": gemm_ops / (gemm6 * 1e-3) / 1e12 / FP6_PEAK_TOPS,
                                  "stored_bytes": dict(zip(("A_store", "B_eu"), plan.unpacked_bytes()[:2])),
                                  "note": "same step, digits as e2m3 codes (96 bytes per 128 columns) on "
                                          "v_mfma_f32_32x32x64_f8f6f4; results bit-identical; not the headline value"}
        plan.set_digits(imu.DIGITS_INT8)
        step()
        torch.cuda.synchronize()
    extra = measure_extras(torch, imu, workloads, w, Qa, Qb, st_a, st_b, status, A, B, C_fp, args)
    if clock_mhz:
        out["roofline"]["clock_mhz_in_k_loop"] = clock_mhz
        out["roofline"]["frac_of_peak_at_that_clock"] = achieved / (mfma_peak * clock_mhz / 2400.0)
    out["weights_prequantized"] = {"ms_per_step": ms_step_wq, "value": w.ops / (ms_step_wq * 1e-3) / 1e12, "unit": "TOPS",
                                   "note": "same step with the RTN integers and scan statistics of B kept from an "
                                           "earlier step (weights are quantised once); not the headline value",
                                   "keep_weights": {"ms_per_step": ms_step_keep, "value": w.ops / (ms_step_keep * 1e-3) / 1e12,
                                                    "plan_ms": plan_keep_ms, "scatter_ms": scatter_keep_ms,
                                                    "unpacking_of_B_reused": bool(reused),
                                                    "note": "and the plan in keep-weights mode: B's unpacking, its layouts and "
                                                            "B_eu itself are taken over while the column splits of A stay the same"}}
    out["unpack"]["time_ratio_vs_plain_int8_gemm"] = ms_step / extra["plain_gemm_ms"]
    out["unpack"]["priced_r_all_pairs"] = extra["priced_r"]   # Sec. 4.2, "Mix": r of all nine strategy pairs
    out["priced_best_pair_step"] = {"strategy": extra["priced_best"], "ms_per_step": extra["mix_ms"],
                                    "value": w.ops / (extra["mix_ms"] * 1e-3) / 1e12, "unit": "TOPS",
                                    "ratio_r": extra["mix_r"], "timed_ms_of_candidates": extra["mix_timed_ms"],
                                    "note": "the whole step (both operands quantised) with the strategy pair that is "
                                            "fastest among those whose unpack ratio is within 25 % of the smallest "
                                            "(the configured pair always takes part); not the headline value, whose "
                                            "strategies are the configuration's"}
    out["plain_int8_gemm"] = {"ms": extra["plain_gemm_ms"], "TOPS": w.ops / extra["plain_gemm_ms"] / 1e9,
                              "note": "this library's GEMM on the original shape, operands clipped to int8 (not exact)"}
    out["stage_ms"]["quantize+scan A"] = extra["quant_a_ms"]
    out["stage_ms"]["quantize+scan B"] = extra["quant_b_ms"]
    out["measured_peaks"] = {"int8_mfma_TOPS": extra["mfma_peak_tops"], "copy_GBps": extra["copy_gbps"],
                             "torch_copy_GBps": extra["torch_copy_gbps"],
                             "gemm_frac_of_measured_mfma": achieved / extra["mfma_peak_tops"],
                             "note": "register-resident v_mfma_i32_32x32x32_i8 loop, 4 waves per SIMD; device-to-device "
                                     "copy of 1 GiB (read + written bytes): the faster of torch's copy and the library's "
                                     "streaming copy (64 rows x 1 KiB per workgroup, non-temporal loads and stores)"}
    for name in ("quantize+scan", "scatter"):
        out["roofline_passes"][name]["frac_of_measured_copy"] = out["roofline_passes"][name]["achieved"] / extra["copy_gbps"]
    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(w)
    print(json.dumps(out))


if __name__ == "__main__":
    main()
