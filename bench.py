#!/usr/bin/env python3
"""Benchmark of the ozimmu hot path on one MI355X.

A "step" is one ozimmu_dgemm call: scale extraction, splitting of A and B into s int8 slices,
and the fused int8-MFMA GEMM with the binary64 accumulation, on synthetic inputs that are
resident in HBM before the timed region.  Prints ONE JSON line.

  value      effective FP64 TFLOP/s = 2 m n k / (time per step)
  roofline   fused GEMM kernel alone: int8 op/s = 2 m n k * s(s+1)/2 / (HIP-event time of the
             kernel, recorded on its stream during the timed region) against the int8 MFMA peak
  cpu_baseline  the CPU oracle, timed on a bounded sample (a block of rows of A times a block of
             columns of B, full k) of the same inputs
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

INT8_PEAK_TOPS = 5000.0          # MI355X dense int8 MFMA, published
HBM_PEAK_GBS = 8000.0


class PowerSampler:
    """Board power of GPU 0 from the driver's hwmon file (microwatts), read every few milliseconds by a thread
    while a timed loop runs.  Context for the roofline fraction: the GEMM kernels run at the board's power cap,
    which is what sets their clock.  Reports nothing where the file is not readable."""

    def __init__(self):
        import glob
        hw = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_input"))
        cap = sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/power1_cap"))
        self.path = hw[0] if hw else None
        self.cap_w = None
        try:
            self.cap_w = int(open(cap[0]).read()) / 1e6 if cap else None
        except (OSError, ValueError):
            pass
        self.samples = []
        self._stop = False
        self._thread = None

    def _loop(self):
        while not self._stop:
            try:
                self.samples.append((time.perf_counter(), int(open(self.path).read())))
            except (OSError, ValueError):
                pass
            time.sleep(0.004)

    def start(self):
        import threading
        self.samples = []
        self._stop = False
        if self.path:
            self._thread = threading.Thread(target=self._loop, daemon=True)
            self._thread.start()
        self.t0 = time.perf_counter()

    def stop(self):
        t1 = time.perf_counter()
        self._stop = True
        if self._thread:
            self._thread.join()
            self._thread = None
        # the reading is a moving average over some hundred milliseconds: only the second half of the interval is
        # used, and nothing is reported for an interval too short for the average to settle
        lo = self.t0 + 0.5 * (t1 - self.t0)
        w = [p / 1e6 for (t, p) in self.samples if lo <= t <= t1 and p > 0]
        if not w or t1 - self.t0 < 0.25:
            return None
        return {"avg_W": sum(w) / len(w), "max_W": max(w), "cap_W": self.cap_w, "samples": len(w),
                "source": "hwmon power1_input sampled during the timed steps"}


def error_measures(C, A, B, Cref):
    """Normwise measure eq. (err_higham) with alpha=1, beta=0, and max componentwise relative
    error eq. (fwd-err-def-mat), both against a binary64 reference product."""
    import torch
    k = A.shape[1]
    diff = C - Cref
    normwise = (torch.linalg.norm(diff) / ((k + 2) ** 0.5 * torch.linalg.norm(A) * torch.linalg.norm(B))).item()
    denom = Cref.abs()
    comp = (diff.abs() / denom)[denom > 0].max().item()
    return normwise, comp


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="pow2_scaled_8192")
    ap.add_argument("--slices", type=int, default=7)
    ap.add_argument("--no-sweep", action="store_true",
                    help="skip the per-slice-count sweep of the workload (the `sweep` array of the output)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-sample", type=int, default=1536, help="rows of A and columns of B in the oracle sample")
    ap.add_argument("--calibration-copy", action="store_true",
                    help="also run one plain 1 GiB device copy (a known amount of HBM traffic) so that "
                         "rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE readings can be scaled")
    ap.add_argument("--traffic-bytes", type=float, default=None,
                    help="HBM bytes per GEMM launch from rocprofv3 --pmc runs (see profiles/)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (the method needs no exchange when C is tiled "
              "over GPUs: every row of A and column of B carries its own scale); --gpus must be 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch
    from paper_2506_11277_amd import ozimmu, workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    ozimmu.lib()   # fails loudly if the HIP library is missing

    cfg = workloads.CONFIGS[args.workload]
    m, n, k = cfg["m"], cfg["n"], cfg["k"]
    A, B = cfg["gen"]()
    dA, dB = ozimmu.to_colmajor(A), ozimmu.to_colmajor(B)
    C = ozimmu.colmajor_empty(m, n)
    flops = 2.0 * m * n * k

    power = PowerSampler()

    def run(s, steps, warmup):
        ws = ozimmu.alloc_workspace(m, n, k, s)
        for _ in range(warmup):
            ozimmu.dgemm(dA, dB, s, C=C, workspace=ws)
        ozimmu.check(ws)
        torch.cuda.synchronize()
        ozimmu.profile_start(steps)
        power.start()
        t0 = time.perf_counter()
        for _ in range(steps):
            ozimmu.dgemm(dA, dB, s, C=C, workspace=ws)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        watts = power.stop()
        calls, phases = ozimmu.profile_stop()
        assert calls == steps
        phases["kernel"] = ozimmu.last_gemm_kernel()       # written by the launcher that ran
        return dt, phases, watts

    s = args.slices
    dt, phases, watts = run(s, args.steps, args.warmup)
    pairs = s * (s + 1) // 2
    gemm_s = phases["gemm"] * 1e-3
    int8_tops = flops * pairs / gemm_s / 1e12
    split_bytes = (8.0 + s) * (m * k + k * n)
    scales_bytes = 8.0 * (m * k + k * n)

    # bytes beyond the L2s per GEMM launch, per slice count, from the rocprofv3 --pmc runs summarised under
    # profiles/ (null for a slice count or workload that has not been measured)
    measured = {}
    tfile = os.path.join(ROOT, "paper_2506_11277_amd", "measured_traffic.json")
    if os.path.exists(tfile):
        measured = json.load(open(tfile))
    traffic = args.traffic_bytes
    if traffic is None:
        traffic = measured.get(f"{args.workload}:{s}")

    out = {
        "metric": "effective FP64 TFLOP/s (2mnk/t) vs slices s; % of int8 MFMA peak",
        "value": flops / dt / 1e12,
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": dt * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "i8",
        "data": "synthetic",
        "config": {"workload": args.workload, "m": m, "n": n, "k": k, "slices": s, "slice_pairs": pairs},
        "roofline": {
            "kernel": phases.pop("kernel"),
            "bound": "mfma",
            "achieved": int8_tops,
            "peak": INT8_PEAK_TOPS,
            "unit": "TOP/s",
            "frac": int8_tops / INT8_PEAK_TOPS,
            "traffic": traffic,
            "ms": phases["gemm"],
        },
        "phases_ms": phases,
        "board_power": watts,
        "hbm_kernels": {
            "scales_GBs": scales_bytes / (phases["scales"] * 1e-3) / 1e9 if phases["scales"] > 0 else None,
            "split_GBs": split_bytes / (phases["split"] * 1e-3) / 1e9 if phases["split"] > 0 else None,
            "peak_GBs": HBM_PEAK_GBS,
        },
    }

    if args.calibration_copy:
        src = torch.empty(1 << 27, dtype=torch.float64, device="cuda").fill_(1.0)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        ozimmu.calibration_copy(dst, src)      # calibration_copy_kernel: exactly 1 GiB read, 1 GiB written
        torch.cuda.synchronize()
        del src, dst

    # context: native binary64 GEMM of the vendor library on the same tensors, and accuracy
    Cref = torch.matmul(dA, dB)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    reps = 3
    for _ in range(reps):
        Cref = torch.matmul(dA, dB)
    torch.cuda.synchronize()
    t_native = (time.perf_counter() - t0) / reps
    ozimmu.dgemm(dA, dB, s, C=C)
    normwise, comp = error_measures(C, dA, dB, Cref)
    out["native_dgemm"] = {"tflops": flops / t_native / 1e12, "ms": t_native * 1e3, "library": "rocBLAS/hipBLASLt via torch.matmul"}
    out["error_vs_native"] = {"normwise_err_higham": normwise, "max_componentwise": comp}

    # the two accuracy variants at the same slice count: round-to-nearest slices, levels of 3 diagonals
    variants = {}
    ws2 = ozimmu.alloc_workspace(m, n, k, s)
    for name, splitting, q in (("nearest_slices", ozimmu.SPLIT_NEAREST, 1),
                               ("levels_of_3_diagonals", ozimmu.SPLIT_TRUNCATE, min(3, ozimmu.max_level_diagonals(k, s, s)))):
        ozimmu.dgemm3(dA, dB, s, s, False, splitting, q, C=C, workspace=ws2)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(3):
            ozimmu.dgemm3(dA, dB, s, s, False, splitting, q, C=C, workspace=ws2)
        torch.cuda.synchronize()
        tv = (time.perf_counter() - t0) / 3
        nw, cw = error_measures(C, dA, dB, Cref)
        variants[name] = {"ms_per_step": tv * 1e3, "tflops_effective": flops / tv / 1e12,
                          "normwise_err_higham": nw, "max_componentwise": cw}
    out["variants"] = variants
    del ws2

    # context: what the matrix cores sustain with nothing else running, and the vendor's int8 GEMM
    def settled(fn, seconds=0.3):
        # median over repeated launches: one launch of 10 ms right after other work reads low while the power
        # controller settles
        vals, t_end = [], time.perf_counter() + seconds
        while not vals or time.perf_counter() < t_end:
            vals.append(fn())
        return sorted(vals)[len(vals) // 2]

    out["int8_mfma_sustained_TOPs"] = {
        "constant_operands": settled(lambda: ozimmu.measure_int8_ceiling(False)),
        "random_operands": settled(lambda: ozimmu.measure_int8_ceiling(True)),
        "random_operands_16x16x64": settled(lambda: ozimmu.measure_int8_ceiling(True, shape16=True)),
        "random_operand_tile": settled(lambda: ozimmu.measure_int8_ceiling(2)),
        "random_operand_tile_16x16x64": settled(lambda: ozimmu.measure_int8_ceiling(2, shape16=True)),
        "what": "register-only v_mfma_i32_32x32x32_i8 loop (entries named 16x16x64: v_mfma_i32_16x16x64_i8); operand "
                "tile: consecutive instructions read different random operands, as in a GEMM; median of the launches "
                "of 0.3 s"}
    out["int8_mfma_with_data_movement_TOPs"] = {
        "lds_reads_only": settled(lambda: ozimmu.measure_int8_with_traffic(4, 0)),
        "lds_dma_only": settled(lambda: ozimmu.measure_int8_with_traffic(0, 3)),
        "ratios_of_7_slices": settled(lambda: ozimmu.measure_int8_with_traffic(4, 3)),
        "ratios_of_9_slices": settled(lambda: ozimmu.measure_int8_with_traffic(3, 2)),
        "what": "the random-operand-tile 16x16x64 loop with, per wavefront, 4 (3) operand registers re-read from LDS "
                "per 16 matrix instructions and 3 (2) LDS-DMA copies of 1 KiB from an L2-resident buffer per 32: the "
                "data movement of the fused kernel for 7 (9) slices with no barrier, no wait on the data, no split "
                "stage, no epilogue and no HBM traffic; median of the launches of 0.3 s"}
    try:
        ia = torch.randint(-127, 128, (m, k), dtype=torch.int8, device="cuda")
        ib = torch.randint(-127, 128, (n, k), dtype=torch.int8, device="cuda").t()
        torch._int_mm(ia, ib)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(5):
            torch._int_mm(ia, ib)
        torch.cuda.synchronize()
        t_i8 = (time.perf_counter() - t0) / 5
        out["native_int8_gemm"] = {"tops": flops / t_i8 / 1e12, "ms": t_i8 * 1e3,
                                   "what": "one int8 GEMM of the same shape, random entries, torch._int_mm (hipBLASLt)"}
        del ia, ib
    except Exception as exc:  # context only
        out["native_int8_gemm"] = {"error": str(exc)[:200]}

    if not args.no_sweep:
        # the metric is a curve over the slice count: every s of the workload, each timed like the headline
        sweep = []
        for ss in cfg["s"]:
            # at least 0.4 s of steps per slice count, so that the board-power reading has settled
            dts, _, _ = run(ss, 3, 2)
            nsteps = min(500, max(5, args.steps // 2, int(0.4 / dts) + 1))
            dts, ph, pw = run(ss, nsteps, 0)
            pp = ss * (ss + 1) // 2
            ozimmu.dgemm(dA, dB, ss, C=C)
            nw, cw = error_measures(C, dA, dB, Cref)
            tops = flops * pp / (ph["gemm"] * 1e-3) / 1e12
            sweep.append({"s": ss, "steps": nsteps, "ms_per_step": dts * 1e3, "tflops_effective": flops / dts / 1e12,
                          "kernel": ph["kernel"], "gemm_ms": ph["gemm"], "scales_ms": ph["scales"],
                          "split_ms": ph["split"], "int8_tops": tops, "frac_int8_peak": tops / INT8_PEAK_TOPS,
                          "traffic": measured.get(f"{args.workload}:{ss}"),
                          "board_power_W": pw["avg_W"] if pw else None,
                          "normwise_err": nw, "max_componentwise_err": cw})
        out["sweep"] = sweep
        tol = 2.0 ** -53
        est = ozimmu.estimate_slices(dA, dB, tol)
        out["estimator"] = {"tol": tol, "s": est[0], "status": est[1], "kappa_A": est[2], "kappa_B": est[3]}

        # The badly scaled product of the paper's accuracy experiment (Sect. 5): A = Abar D, B = D^-1 Bbar, entries of
        # Abar, Bbar uniform in (1, 2), D geometric with condition number kappa_D, rows of A and columns of B rotated.
        # Here at 4096^3, kappa_D = 1e20: time and error for the slice counts of that experiment and for the
        # estimate; the error is measured against the vendor's binary64 product, relative to |A||B|.
        nb, kd = 4096, 1e20
        Ab, Bb = workloads.diag_scaled(nb, kd, 1005)
        dAb, dBb = ozimmu.to_colmajor(Ab), ozimmu.to_colmajor(Bb)
        del Ab, Bb
        ref_b = torch.matmul(dAb, dBb)
        absprod = torch.matmul(dAb.abs(), dBb.abs())
        est_b = ozimmu.estimate_slices(dAb, dBb, tol)
        rows = []
        for ss in sorted({8, 12, 16, 18, min(est_b[0], 32)}):
            wsb = ozimmu.alloc_workspace(nb, nb, nb, ss)
            Cb = ozimmu.dgemm(dAb, dBb, ss, workspace=wsb)
            torch.cuda.synchronize()
            t0 = time.perf_counter()
            for _ in range(5):
                ozimmu.dgemm(dAb, dBb, ss, C=Cb, workspace=wsb)
            torch.cuda.synchronize()
            tb = (time.perf_counter() - t0) / 5
            rows.append({"s": ss, "ms_per_step": tb * 1e3, "tflops_effective": 2.0 * nb ** 3 / tb / 1e12,
                         "kernel": ozimmu.last_gemm_kernel(),
                         "max_err_rel_absprod": ((Cb - ref_b).abs() / absprod).max().item()})
            del wsb, Cb
        out["badly_scaled"] = {"workload": f"diag_scaled n={nb} kappa_D={kd:g} rotated", "estimator_s": est_b[0],
                               "kappa_A": est_b[2], "kappa_B": est_b[3], "runs": rows,
                               "reference": "torch.matmul in binary64 (its own error is of the order n u |A||B|)"}
        del dAb, dBb, ref_b, absprod

    if not args.no_cpu_baseline:
        from oracle import oracle
        ms_ = min(args.cpu_sample, m)
        ns_ = min(args.cpu_sample, n)
        As = np.asfortranarray(A[:ms_, :])
        Bs = np.asfortranarray(B[:, :ns_])
        t0 = time.perf_counter()
        Cs = oracle.dgemm(As, Bs, s)
        t_cpu = time.perf_counter() - t0
        ozimmu.dgemm(dA, dB, s, C=C)
        same = bool(np.array_equal(C[:ms_, :ns_].cpu().numpy(), Cs))
        out["cpu_baseline"] = {
            "value": 2.0 * ms_ * ns_ * k / t_cpu / 1e12,
            "unit": "TFLOP/s",
            "cores": oracle.num_threads(),
            "kind": "oracle",
            "sample": f"C[0:{ms_}, 0:{ns_}] = A[0:{ms_}, :] B[:, 0:{ns_}] with full k={k}, s={s}: {t_cpu:.2f} s",
            "gpu_matches_oracle_on_sample": same,
        }

    print(json.dumps(out))


if __name__ == "__main__":
    main()
