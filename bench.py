#!/usr/bin/env python3
"""Benchmark of libstrassen_tc on one MI355X.

Workload: the square fp64 GEMM-shaped contraction C[i,j] += A[i,k] * B[k,j] with m = n = k = 16384 (the largest
single-GPU case of the second benchmark configuration), seeded uniform[-1,1) data, generalized column-major.
A step is one pass of the whole hot path on inputs resident in HBM: tc_plan (bundle classification, scatter and
block scatter vectors, Strassen schedule), tc_contract (operand sums, gather, FP64 matrix-core tiles,
multi-destination update) and tc_destroy, for the headline mode: one-level Strassen in the ABC variant of the paper
(operand sums formed while tiles are staged, every product added to its blocks of C from registers, no temporaries).
The other modes (classical, AB, Naive, two-level, and the HYBRID variant that stores the first-level operand sums)
are timed the same way and listed under config.modes.

Prints ONE JSON line: effective GFLOPS = 2 m n k / t (classical flop count for every mode), the roofline figure of
the fused kernel (all launches of the headline mode together, and per kernel family = number of blocks in the operand
sums of A and B), the same against the measured MFMA-only ceiling, and the CPU oracle timed on a bounded row panel of
the same workload.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

FP64_MFMA_PEAK_TFLOPS = 78.6  # MI355X published dense FP64 matrix peak
HBM_PEAK_TBS = 8.0            # MI355X published HBM3E bandwidth


def profiled_traffic(wname, level, variant):
    """HBM bytes per fused-kernel launch (FETCH_SIZE + WRITE_SIZE, scaled by a plain copy kernel) from the committed
    counter summary of this exact workload; None if there is none.  The counters need the profiler, so they are
    collected in separate runs of this script under rocprofv3 --pmc and written down in profiles/."""
    import re

    path = os.path.join(ROOT, "profiles", f"fused_kernel_{wname}_level{level}_{variant}.md")
    try:
        m = re.search(r"^hbm_traffic_bytes_per_launch\s*=\s*([0-9.eE+]+)", open(path).read(), re.M)
    except OSError:
        return None
    return float(m.group(1)) if m else None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--size", type=int, default=16384, help="m = n = k of the square contraction")
    ap.add_argument("--workload", default="", help="another benchmark configuration instead of the square one: cfg1, cfg3, cfg4a, cfg4b, cfg5")
    ap.add_argument("--level", type=int, default=1)
    ap.add_argument("--variant", default="abc")
    ap.add_argument("--modes", default="0abc,1abc,1ab,1naive,1hybrid,2abc,2ab,2naive,2hybrid", help="other modes to time (level+variant)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calib-copy", action="store_true",
                    help="also launch one plain element-wise copy of 512 MiB (for scaling the profiler's HBM byte counters)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        sys.exit("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1")

    import numpy as np
    import torch

    import paper_1704_03092_amd as tc
    import workloads

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    tc.load_library()  # no fallback: fails if the HIP library is missing
    torch.cuda.set_device(0)
    N = args.size
    if args.workload:
        cfg = workloads.configs()[args.workload]
        wname = args.workload
        wtext = f"{cfg.name} contraction {cfg.idxC}-{cfg.idxA}-{cfg.idxB}, lengths {cfg.lengths}, {cfg.kind}, alpha={cfg.alpha:g} beta={cfg.beta:g}, generalized column-major"
    else:
        cfg = workloads.gemm(N)
        wname = f"cfg2_{N}"
        wtext = f"cfg2 square contraction ij-ik-kj, m=n=k={N}, uniform[-1,1), alpha=1 beta=1, column-major"
    m, n, k = cfg.mnk()
    flops = 2.0 * m * n * k
    A, B, C = cfg.tensors()
    dA = torch.from_numpy(A.data).to("cuda")
    dB = torch.from_numpy(B.data).to("cuda")
    dC0 = torch.from_numpy(C.data).to("cuda")
    dC = dC0.clone()
    st = torch.cuda.current_stream()
    ws_cache = {}

    def workspace(nbytes):
        if nbytes == 0:
            return None
        if nbytes not in ws_cache:
            ws_cache.clear()
            ws_cache[nbytes] = torch.empty(nbytes // 8, dtype=torch.float64, device="cuda")
        return ws_cache[nbytes]

    def one_step(level, variant, alpha=cfg.alpha, beta=cfg.beta):
        plan = tc.tc_plan(A, B, C, level, variant, st)
        ws = workspace(tc.tc_plan_workspace_bytes(plan))
        tc.tc_contract(plan, alpha, dA, dB, beta, dC, ws, st)
        info = tc.tc_plan_info(plan)
        tc.tc_destroy(plan)
        return info

    def time_mode(level, variant, steps, warmup):
        """(wall ms per step incl. plan, event ms per tc_contract, plan info)"""
        dC.copy_(dC0)
        for _ in range(warmup):
            info = one_step(level, variant)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            info = one_step(level, variant)
        torch.cuda.synchronize()
        wall_ms = (time.perf_counter() - t0) * 1e3 / steps
        # kernel time alone: HIP events on the launch stream around tc_contract of a prepared plan
        plan = tc.tc_plan(A, B, C, level, variant, st)
        ws = workspace(tc.tc_plan_workspace_bytes(plan))
        evs = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(steps)]
        for e0, e1 in evs:
            e0.record(st)
            tc.tc_contract(plan, cfg.alpha, dA, dB, cfg.beta, dC, ws, st)
            e1.record(st)
        torch.cuda.synchronize()
        ev_ms = sum(e0.elapsed_time(e1) for e0, e1 in evs) / steps
        # time of every launch alone: an event after every launch (tc_contract_launch_times), averaged over the same steps
        launches = tc.tc_plan_launches(plan)
        per = [0.0] * len(launches)
        for _ in range(steps):
            for i, ms in enumerate(tc.tc_contract_launch_times(plan, cfg.alpha, dA, dB, cfg.beta, dC, ws, st)):
                per[i] += ms / steps
        tc.tc_destroy(plan)
        fused = [(L, ms) for L, ms in zip(launches, per) if L["kind"] == 0]
        fam = {}
        for L, ms in fused:
            f = fam.setdefault(f"{L['terms_a']}x{L['terms_b']}", {"launches": 0, "ms": 0.0, "flops": 0.0})
            f["launches"] += 1
            f["ms"] += ms
            f["flops"] += 2.0 * L["n_products"] * L["rows"] * L["cols"] * L["depth"]
        kern = {"fused_ms": sum(ms for _, ms in fused), "elementwise_ms": sum(ms for L, ms in zip(launches, per) if L["kind"] != 0),
                "fused_launches": len(fused), "elementwise_launches": len(launches) - len(fused), "families": fam,
                "fused_flops": sum(f["flops"] for f in fam.values())}
        return wall_ms, ev_ms, info, kern

    if args.calib_copy:  # reads 2^26 doubles and writes 2^26 doubles, nothing else
        cx = torch.rand(1 << 26, dtype=torch.float64, device="cuda")
        cy = torch.empty_like(cx)
        torch.mul(cx, 1.0, out=cy)
        torch.cuda.synchronize()
        del cx, cy

    # ---- the machine's ceiling first: what the matrix cores sustain with nothing else going on (same instruction as the
    #      kernels; about 50 ms of work, which also brings the GPU out of its idle clocks before anything is timed) ----
    mfma_only_4x4 = tc.tc_bench_mfma_peak(0, st)  # v_mfma_f64_4x4x4_4b_f64
    mfma_only = tc.tc_bench_mfma_peak(1, st)      # v_mfma_f64_16x16x4_f64, the fused kernel's instruction

    # ---- headline mode ----
    wall_ms, ev_ms, info, kern = time_mode(args.level, args.variant, args.steps, args.warmup)
    value = flops / (wall_ms * 1e-3) * 1e-9

    # ---- parity of the timed configuration on sampled rows (the oracle computes them one by one) ----
    import oracle

    rng = np.random.default_rng(7)
    g = 1 << info["level"]
    rows = sorted(set([0, m - 1] + [b * info["mb"] + d for b in range(g) for d in (-1, 0, 1) if 0 <= b * info["mb"] + d < m]
                      + list(rng.integers(0, m, size=24))))
    rows = np.array(rows, dtype=np.int64)
    dC.copy_(dC0)
    one_step(args.level, args.variant)
    torch.cuda.synchronize()
    orders = (list(info["I"]), list(info["J"]), list(info["P"]))  # the matrix view the plan chose
    view = oracle.matrix_view(A, B, C, orders=orders)
    drows = torch.from_numpy(view["rsC"][rows]).to("cuda")
    dcols = torch.from_numpy(view["csC"]).to("cuda")
    got = dC[drows[:, None] + dcols[None, :]].cpu().numpy()
    ref = oracle.contract_rows(A, B, C, rows, cfg.alpha, cfg.beta, view=view)
    normA_rows = oracle.fro(A.data[view["rsA"][rows][:, None] + view["csA"][None, :]])
    parity = oracle.error_metric(got, ref, normA_rows, oracle.tensor_norm(B))

    # ---- roofline of the fused kernel (gather + operand sums + MFMA + update): executed flops / its own launch durations ----
    # (block extents are rounded up to multiples of 16, so the executed flops are what the launches really multiply)
    executed = kern["fused_flops"]
    achieved = executed / (kern["fused_ms"] * 1e-3) * 1e-12
    nC = 2.0 if cfg.beta != 0.0 else 1.0
    compulsory_bytes = 8.0 * (m * k + k * n + nC * m * n)  # every element of A and B read once, C read (beta != 0) and written
    hbm_tbs = compulsory_bytes / (ev_ms * 1e-3) * 1e-12
    mfma_frac, hbm_frac = achieved / FP64_MFMA_PEAK_TFLOPS, hbm_tbs / HBM_PEAK_TBS
    families = {name: {"launches": f["launches"], "avg_launch_ms": round(f["ms"] / f["launches"], 4),
                       "achieved": round(f["flops"] / (f["ms"] * 1e-3) * 1e-12, 2),
                       "frac": round(f["flops"] / (f["ms"] * 1e-3) * 1e-12 / FP64_MFMA_PEAK_TFLOPS, 4)} for name, f in sorted(kern["families"].items())}
    if mfma_frac >= hbm_frac:
        roofline = {"bound": "mfma", "achieved": round(achieved, 2), "peak": FP64_MFMA_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": round(mfma_frac, 4)}
    else:
        roofline = {"bound": "hbm", "achieved": round(hbm_tbs * 1e3, 1), "peak": HBM_PEAK_TBS * 1e3, "unit": "GB/s", "frac": round(hbm_frac, 4)}
    roofline.update({"traffic": profiled_traffic(wname, info["level"], "abc" if info["level"] == 0 else args.variant),
                     "kernel": "fused_kernel", "launches_per_contract": kern["fused_launches"],
                     "flops_per_launch": executed / max(kern["fused_launches"], 1),
                     "avg_launch_ms": round(kern["fused_ms"] / max(kern["fused_launches"], 1), 4),
                     "other_kernels_ms_per_contract": round(kern["elementwise_ms"], 3),
                     "families": families,
                     "mfma_tflops": round(achieved, 2), "mfma_frac": round(mfma_frac, 4),
                     "measured_mfma_only_tflops": round(mfma_only, 2), "frac_measured_mfma_peak": round(achieved / mfma_only, 4),
                     "measured_mfma_only_tflops_4x4x4": round(mfma_only_4x4, 2),
                     "compulsory_hbm_gbs": round(hbm_tbs * 1e3, 1), "hbm_frac": round(hbm_frac, 4)})

    # ---- the other modes ----
    modes = {}
    for md in [x for x in args.modes.split(",") if x]:
        lv, var = int(md[0]), md[1:]
        w, e, inf, kn = time_mode(lv, var, max(2, args.steps // 2 + 1), 1)
        modes[md] = {"ms_per_step": round(w, 3), "contract_ms": round(e, 3), "eff_gflops": round(flops / w * 1e-6, 1),
                     "frac_peak_eff": round(flops / w * 1e-9 / FP64_MFMA_PEAK_TFLOPS, 4), "launches": inf["n_launches"],
                     # executed TFLOP/s of the fused kernel per family (blocks in the sums of A x B) and the other kernels' time
                     "fused_tflops_by_family": {name: round(f["flops"] / (f["ms"] * 1e-3) * 1e-12, 2) for name, f in sorted(kn["families"].items())},
                     "elementwise_ms": round(kn["elementwise_ms"], 3)}

    # ---- CPU oracle on a bounded row panel of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        t0 = time.perf_counter()
        oracle.contract_rows(A, B, C, np.arange(256, dtype=np.int64), cfg.alpha, cfg.beta)
        probe = time.perf_counter() - t0
        nrows = int(min(m, 8192, max(256, 256 * 12.0 / max(probe, 1e-3))))  # about 12 s of CPU work
        nrows -= nrows % 32
        t0 = time.perf_counter()
        oracle.contract_rows(A, B, C, np.arange(nrows, dtype=np.int64), cfg.alpha, cfg.beta)
        dt = time.perf_counter() - t0
        cpu = {"value": round(2.0 * nrows * n * k / dt * 1e-9, 2), "unit": "GFLOPS", "cores": oracle.num_threads(), "kind": "oracle",
               "sample": f"rows 0..{nrows - 1} of the {m}x{n}x{k} contraction (all n and k), tiled classical loop nest, {dt:.1f} s"}

    out = {
        "metric": "effective fp64 GFLOPS (2mnk/t)", "value": round(value, 1), "unit": "GFLOPS", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 3), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f64", "data": "synthetic",
        "config": {"workload": wtext,
                   "level": info["level"], "variant": args.variant, "step": "tc_plan + tc_contract + tc_destroy",
                   "contract_ms": round(ev_ms, 3), "frac_fp64_mfma_peak_effective": round(value * 1e-3 / FP64_MFMA_PEAK_TFLOPS, 4),
                   "parity_sampled_rows": float(f"{parity:.3e}"), "parity_rows": int(len(rows)),
                   "speedup_vs_classical": round(value / modes["0abc"]["eff_gflops"], 4) if "0abc" in modes else None,
                   "modes": modes},
        "roofline": roofline, "cpu_baseline": cpu,
    }
    print(json.dumps(out))


if __name__ == "__main__":
    main()
