"""Regression grid over the synthetic shape families of the paper's experiments (Sec. 6: square, rank-k with
m = n fixed, fixed k with m = n growing), every level and variant, on one GPU:

    python -m paper_1704_03092_amd.sweep [--family square|rankk|fixedk|all] [--reps 3]

Prints one CSV line per (shape, mode): measured milliseconds of tc_contract (median), effective TFLOP/s, the
performance model's prediction for that plan, and whether the model's automatic choice (TC_LEVEL_AUTO /
TC_VARIANT_AUTO) is that mode; then per shape the measured loss of the automatic choice against the fastest mode.
Inputs are uniform[-1,1) from torch's generator (timing only; parity is the tests' business)."""
import argparse
import sys

MODES = [(0, "abc"), (1, "abc"), (1, "ab"), (1, "naive"), (2, "abc"), (2, "ab"), (2, "naive"), (1, "hybrid"), (2, "hybrid")]

FAMILIES = {
    "square": [(n, n, n) for n in (1024, 2048, 4096, 6144, 8192, 12288, 16384)],
    "rankk": [(16384, 16384, k) for k in (256, 512, 1024, 2048, 4096)],
    "fixedk": [(n, n, 1024) for n in (2048, 4096, 8192, 12288)],
}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--family", default="all")
    ap.add_argument("--reps", type=int, default=3)
    args = ap.parse_args()
    import torch

    import paper_1704_03092_amd as tc

    assert torch.cuda.is_available(), "the sweep needs a GPU"
    tc.load_library()
    st = torch.cuda.current_stream()
    shapes = []
    for fam in (FAMILIES if args.family == "all" else [args.family]):
        shapes += [(fam,) + s for s in FAMILIES[fam]]
    print("family,m,n,k,level,variant,ms,tflops_eff,model_ms,auto")
    losses = []
    for fam, m, n, k in shapes:
        dA = torch.rand(m * k, dtype=torch.float64, device="cuda") * 2 - 1
        dB = torch.rand(k * n, dtype=torch.float64, device="cuda") * 2 - 1
        dC = torch.zeros(m * n, dtype=torch.float64, device="cuda")
        desc = (("ik", (m, k), (1, m)), ("kj", (k, n), (1, k)), ("ij", (m, n), (1, m)))
        auto = tc.tc_plan(*desc, tc.TC_LEVEL_AUTO, "auto", st)
        ai = tc.tc_plan_info(auto)
        tc.tc_destroy(auto)
        rows = {}
        for level, variant in MODES:
            plan = tc.tc_plan(*desc, level, variant, st)
            nb = tc.tc_plan_workspace_bytes(plan)
            ws = torch.empty(max(nb // 8, 1), dtype=torch.float64, device="cuda") if nb else None
            pred = tc.tc_plan_predict(plan)["total"] * 1e3
            for _ in range(2):
                tc.tc_contract(plan, 1.0, dA, dB, 1.0, dC, ws, st)
            ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.reps)]
            for e0, e1 in ev:
                e0.record(st)
                tc.tc_contract(plan, 1.0, dA, dB, 1.0, dC, ws, st)
                e1.record(st)
            torch.cuda.synchronize()
            tc.tc_destroy(plan)
            del ws
            ms = sorted(e0.elapsed_time(e1) for e0, e1 in ev)[len(ev) // 2]
            is_auto = int(ai["level"] == level and ai["variant"] == tc.VARIANTS[variant])
            rows[(level, variant)] = (ms, is_auto)
            print(f"{fam},{m},{n},{k},{level},{variant},{ms:.3f},{2.0 * m * n * k / ms * 1e-9:.2f},{pred:.3f},{is_auto}", flush=True)
        best = min(v[0] for v in rows.values())
        chosen = [v[0] for v in rows.values() if v[1]][0]
        losses.append((fam, m, n, k, chosen / best - 1.0))
        del dA, dB, dC
    print("# measured loss of the automatic choice against the fastest mode")
    for fam, m, n, k, loss in losses:
        print(f"# {fam} {m}x{n}x{k}: {100 * loss:.1f} %")
    print(f"# worst {100 * max(l[-1] for l in losses):.1f} %, mean {100 * sum(l[-1] for l in losses) / len(losses):.1f} %")


if __name__ == "__main__":
    sys.exit(main())
