"""Regression grid over the shape families of the paper's experiments (Sec. 6.1), every level and variant, on one GPU:

    python -m paper_1704_03092_amd.sweep [--family square|rankk|fixedk|ladder|tensor|all] [--reduced] [--reps 3]
    python -m paper_1704_03092_amd.sweep --fit [--reduced]

Families: square (m = n = k), rank-k (m = n fixed, k growing), fixed-k (k fixed, m = n growing), ladder (the
shape-dependence experiment: C[abij] += A[abef] B[efij] with N_a : N_i from 1 to 5 at roughly the flops of 16000^3),
tensor (seeded 2-D ... 6-D tensors: each bundle split into one to three dimensions, the index strings, hence the
storage orders, shuffled).  Inputs come from the seeded generators in workloads/.

The grid prints one CSV line per (shape, mode): measured milliseconds of tc_contract (median), effective TFLOP/s, the
performance model's prediction for that plan, and whether the model's automatic choice (TC_LEVEL_AUTO /
TC_VARIANT_AUTO) is that mode; then per shape the measured loss of the automatic choice against the fastest mode, and
per family the first shape at which one level and two levels of Strassen beat the classical algorithm.

--fit times every launch of a set of plans (tc_contract_launch_times), fits the parameters of the library's model
(tc_model_params_t) to them by non-negative least squares on relative residuals, and prints them as the initialiser
of the defaults in csrc/tc_host.cpp."""
import argparse
import random
import sys

MODES = [(0, "abc"), (1, "abc"), (1, "ab"), (1, "naive"), (2, "abc"), (2, "ab"), (2, "naive"), (1, "hybrid"), (2, "hybrid")]
FAMILIES = ("square", "rankk", "fixedk", "ladder", "tensor")
# (N_a, N_i) of the ladder family by ratio: 2 N_a^4 N_i^2 stays near 2 * 16000^3 flops
LADDER = {1: (128, 128), 2: (160, 80), 3: (180, 60), 4: (192, 48), 5: (220, 44)}


def _plain(m, n, k):
    import workloads

    return workloads.Contraction(f"gemm_{m}x{n}x{k}", "ij", "ik", "kj", {"i": m, "j": n, "k": k}, seed=170403092 + m + 3 * n + 7 * k)


def _split(rng, total, parts):
    """total as a product of `parts` factors (the last takes what is left; factors from a fixed list)."""
    out, rem = [], total
    for p in range(parts):
        if p == parts - 1:
            out.append(max(1, rem))
            break
        f = rng.choice([f for f in (2, 3, 4, 6, 8, 12, 16) if rem % f == 0 and rem // f >= 8] or [1])
        out.append(f)
        rem //= f
    rng.shuffle(out)
    return out


def _tensor_cases(reduced):
    import workloads

    rng = random.Random(170403092)
    sizes = [768, 1536, 2304] if reduced else [1536, 3072, 4608, 6144]
    out = []
    for t in range(4 if reduced else 10):
        labels = list("abcdefghi")
        rng.shuffle(labels)
        nI, nJ, nP = rng.randint(1, 3), rng.randint(1, 3), rng.randint(1, 3)
        while nI + nP > 6 or nP + nJ > 6 or nI + nJ > 6 or max(nI + nP, nP + nJ, nI + nJ) < 2:
            nI, nJ, nP = rng.randint(1, 3), rng.randint(1, 3), rng.randint(1, 3)
        I, J, P = labels[:nI], labels[nI:nI + nJ], labels[nI + nJ:nI + nJ + nP]
        lengths = {}
        for group in (I, J, P):
            for c, f in zip(group, _split(rng, rng.choice(sizes), len(group))):
                lengths[c] = f
        idx = []
        for s in (I + P, P + J, I + J):
            s = list(s)
            rng.shuffle(s)
            idx.append("".join(s))
        out.append(workloads.Contraction(f"tensor{t}_{idx[2]}-{idx[0]}-{idx[1]}", idx[2], idx[0], idx[1], lengths, seed=170403092 + 100 + t))
    return out


def cases(family, reduced=False):
    """The contractions of one family (workloads.Contraction), in the order of the sweep."""
    import workloads

    if family == "square":
        return [_plain(n, n, n) for n in ((1024, 2048, 4096, 6144) if reduced else (1024, 2048, 4096, 6144, 8192, 12288, 16384))]
    if family == "rankk":
        N = 8192 if reduced else 16384
        return [_plain(N, N, k) for k in ((256, 1024, 4096) if reduced else (256, 512, 1024, 2048, 4096, 8192))]
    if family == "fixedk":
        return [_plain(n, n, 1024) for n in ((2048, 6144) if reduced else (2048, 4096, 8192, 12288, 16384))]
    if family == "ladder":
        out = []
        for r, (na, ni) in LADDER.items():
            if reduced:
                if r not in (1, 4):
                    continue
                na, ni = na // 2, ni // 2
            out.append(workloads.Contraction(f"ladder_{r}to1_Na{na}_Ni{ni}", "abij", "abef", "efij",
                                             {"a": na, "b": na, "e": na, "f": na, "i": ni, "j": ni}, seed=170403092 + 50 + r))
        return out
    if family == "tensor":
        return _tensor_cases(reduced)
    raise ValueError(family)


class _Device:
    """The operands of one contraction on the GPU and a workspace that grows as needed."""

    def __init__(self, cfg):
        import torch

        A, B, C = cfg.tensors()
        self.A, self.B, self.C = A, B, C
        self.dA, self.dB, self.dC = (torch.from_numpy(t.data).to("cuda") for t in (A, B, C))
        self.ws = None
        self.st = torch.cuda.current_stream()

    def workspace(self, nbytes):
        import torch

        if nbytes and (self.ws is None or self.ws.numel() * 8 < nbytes):
            self.ws = None
            self.ws = torch.empty(nbytes // 8, dtype=torch.float64, device="cuda")
        return self.ws if nbytes else None


def _warm(plan, dev, ws, seconds=0.03):
    """At least two contractions and `seconds` of them: short shapes would otherwise be timed at idle clocks."""
    import time

    import torch

    import paper_1704_03092_amd as tc

    t0, n = time.perf_counter(), 0
    while n < 2 or time.perf_counter() - t0 < seconds:
        tc.tc_contract(plan, 1.0, dev.dA, dev.dB, 1.0, dev.dC, ws, dev.st)
        torch.cuda.synchronize()
        n += 1


def measure(cfg, reps=3, modes=MODES):
    """{(level, variant): (measured ms, modelled ms)} of one contraction and the mode the library picks by itself."""
    import torch

    import paper_1704_03092_amd as tc

    dev = _Device(cfg)
    auto = tc.tc_plan(dev.A, dev.B, dev.C, tc.TC_LEVEL_AUTO, "auto", dev.st)
    ai = tc.tc_plan_info(auto)
    tc.tc_destroy(auto)
    names = {v: k for k, v in tc.VARIANTS.items() if k != "auto"}
    rows = {}
    for level, variant in modes:
        plan = tc.tc_plan(dev.A, dev.B, dev.C, level, variant, dev.st)
        if tc.tc_plan_info(plan)["level"] != level:  # the shape is too small for this level
            tc.tc_destroy(plan)
            continue
        ws = dev.workspace(tc.tc_plan_workspace_bytes(plan))
        pred = tc.tc_plan_predict(plan)["total"] * 1e3
        _warm(plan, dev, ws)
        ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(reps)]
        for e0, e1 in ev:
            e0.record(dev.st)
            tc.tc_contract(plan, 1.0, dev.dA, dev.dB, 1.0, dev.dC, ws, dev.st)
            e1.record(dev.st)
        torch.cuda.synchronize()
        tc.tc_destroy(plan)
        rows[(level, variant)] = (sorted(e0.elapsed_time(e1) for e0, e1 in ev)[len(ev) // 2], pred)
    return rows, ((ai["level"], names[ai["variant"]]) if ai["level"] > 0 else (0, "abc"))  # no variants without Strassen


def auto_loss(rows, auto):
    """Measured time of the library's own choice over the fastest measured mode, minus one."""
    return rows[auto][0] / min(v[0] for v in rows.values()) - 1.0


def run_grid(families, reduced, reps, out=sys.stdout):
    print("family,case,m,n,k,level,variant,ms,tflops_eff,model_ms,auto", file=out)
    losses, cross = [], {}
    for fam in families:
        for cfg in cases(fam, reduced):
            m, n, k = cfg.mnk()
            rows, auto = measure(cfg, reps)
            for (level, variant), (ms, pred) in rows.items():
                print(f"{fam},{cfg.name},{m},{n},{k},{level},{variant},{ms:.4f},{2.0 * m * n * k / ms * 1e-9:.2f},{pred:.4f},{int((level, variant) == auto)}",
                      file=out, flush=True)
            losses.append((fam, cfg.name, auto_loss(rows, auto)))
            best = {L: min(v[0] for (lv, _), v in rows.items() if lv == L) for L in (0, 1, 2) if any(lv == L for lv, _ in rows)}
            for L in (1, 2):
                if L in best and best[L] < best[0]:
                    cross.setdefault((fam, L), cfg.name)
    print("# measured loss of the automatic choice against the fastest mode", file=out)
    for fam, name, loss in losses:
        print(f"# {fam} {name}: {100 * loss:.1f} %", file=out)
    if losses:
        print(f"# worst {100 * max(l[-1] for l in losses):.1f} %, mean {100 * sum(l[-1] for l in losses) / len(losses):.1f} %", file=out)
    print("# first shape of each family (in sweep order) at which Strassen beats the classical algorithm", file=out)
    for fam in families:
        print(f"# {fam}: one level from {cross.get((fam, 1), 'none')}, two levels from {cross.get((fam, 2), 'none')}", file=out)
    return losses


# ---- the fit of the model's parameters ----

def launch_samples(cfg, reps=5):
    """Measured time and the model's inputs of every launch of a set of plans of one contraction."""
    import paper_1704_03092_amd as tc

    dev = _Device(cfg)
    out = []
    for level, variant, kw in ((0, "abc", {"tile_n": 128}), (0, "abc", {"tile_n": 64}), (1, "abc", {"tile_n": 128}), (2, "abc", {"tile_n": 128}),
                               (1, "hybrid", {"tile_n": 128}), (1, "hybrid", {"tile_n": 64}), (1, "ab", {"tile_n": 128})):
        plan = tc.tc_plan(dev.A, dev.B, dev.C, level, variant, dev.st, tail_split=-1, **kw)
        if tc.tc_plan_info(plan)["level"] != level:
            tc.tc_destroy(plan)
            continue
        ws = dev.workspace(tc.tc_plan_workspace_bytes(plan))
        _warm(plan, dev, ws)
        times = [tc.tc_contract_launch_times(plan, 1.0, dev.dA, dev.dB, 1.0, dev.dC, ws, dev.st) for _ in range(reps)]
        info = tc.tc_plan_launches(plan)
        tc.tc_destroy(plan)
        for i, L in enumerate(info):
            if L["kind"] == 0 and L["terms_a"] == 0:
                continue  # the family that counts terms at run time is not modelled apart
            out.append(dict(L, ms=sorted(t[i] for t in times)[reps // 2], case=cfg.name, plan_level=level, plan_variant=variant))
    return out


def fit(samples, defaults):
    """Non-negative least squares on relative residuals (launches shorter than 50 us count less).  Unknowns: 1 / rho for
    the tiles gathered by stride and for those gathered through the tables, each for 1, 2 and 4 terms in 128 x 128
    tiles and for 128 x 64 tiles; t_tile, t_tile_small, 1 / rho_b, lambda_ab / rho_b, t_launch (the fixed part of a
    kernel's duration; the gap between two launches is not seen); then rho_gather from the launches with element-wise
    gathers."""
    import numpy as np
    from scipy.optimize import nnls

    peak, bw, units = defaults["peak_flops"], defaults["bandwidth"], defaults["units"]
    NU = 13  # 0..3 by stride (1, 2, 4 terms, small), 4..7 through tables, 8 t_tile, 9 t_tile_small, 10 1/rho_b, 11 lambda/rho_b, 12 t_launch

    def row(L):
        r = np.zeros(NU)
        r[12] = 1.0
        if L["kind"] == 0:
            wgs = 128 // L["tile_n"]
            rounds = -(-L["tiles"] // (units * wgs))
            flops = rounds * units * 2.0 * 128 * 128 * L["depth"] / peak
            cls = 3 if L["tile_n"] == 64 else {1: 0, 2: 1, 4: 2}[max(L["terms_a"], L["terms_b"])]
            free = L["tiles_table_free"] / L["tiles"] if L["tail_tiles"] == 0 else 0.0
            r[cls], r[4 + cls] = flops * free, flops * (1.0 - free)
            r[9 if L["tile_n"] == 64 else 8] = rounds
            r[11] = 8.0 * L["tiles"] * L["depth"] * (128 * L["terms_a"] + L["tile_n"] * L["terms_b"]) / bw
        r[10] = 8.0 * L["moved_elems"] / bw
        return r

    pairs = [L for L in samples if L["kind"] == 1 or (L["pairs_a"] and L["pairs_b"])]
    w = np.array([L["ms"] / (L["ms"] + 0.05) for L in pairs])
    M = np.array([row(L) / (L["ms"] * 1e-3) for L in pairs])
    # first everything but the 128 x 64 geometry, then its two parameters with the others held, on the classical
    # plans alone (each of them was also measured in 128 x 128 tiles: the choice between the two shapes is what these
    # parameters are for)
    small = np.array([L["kind"] == 0 and L["tile_n"] == 64 for L in pairs])
    direct = np.array([L["kind"] == 0 and L["tile_n"] == 64 and L.get("plan_level", 0) == 0 for L in pairs])
    own = [3, 7, 9]
    rest = [c for c in range(NU) if c not in own]
    x = np.zeros(NU)
    x[rest], _ = nnls(M[~small][:, rest] * w[~small, None], w[~small])
    if direct.any():
        target = 1.0 - M[direct][:, rest] @ x[rest]
        x[own], _ = nnls(M[direct][:, own] * w[direct, None], target * w[direct])
    rel = M @ x - 1.0
    p = dict(defaults)
    inv = lambda v, d: 1.0 / v if v > 0 else d
    p["rho_a"] = [inv(x[i], defaults["rho_a"][i]) for i in range(3)]
    p["rho_table"] = [inv(x[4 + i], defaults["rho_table"][i]) for i in range(3)]
    p["rho_small"] = inv(x[3], p["rho_a"][0] * defaults["rho_small"]) / p["rho_a"][0]
    p["rho_small_table"] = inv(x[7], p["rho_table"][0] * defaults["rho_small_table"]) / p["rho_table"][0]
    p["t_tile"], p["t_tile_small"] = float(x[8]), float(x[9])
    p["rho_b"] = inv(x[10], defaults["rho_b"])
    p["lambda_ab"] = float(x[11] * p["rho_b"])
    p["t_launch"] = float(x[12])
    # element-wise gathers: what is left of the measured time after the other terms, against the arithmetic term
    ratios = []
    for L in samples:
        if L["kind"] == 0 and not (L["pairs_a"] and L["pairs_b"]) and L["ms"] >= 0.05:
            r = row(L)
            arith = float(r[:8] @ x[:8])
            rest = L["ms"] * 1e-3 - float(r[8:] @ x[8:])
            if arith > 0 and rest > 0:
                ratios.append(arith / rest)
    if ratios:
        p["rho_gather"] = float(np.median(ratios))
    return p, rel


def run_fit(families, reduced, out=sys.stdout, save=None, load=None):
    import json

    import numpy as np

    import paper_1704_03092_amd as tc

    defaults = tc.tc_model_defaults()
    samples = []
    if load:
        samples = json.load(open(load))
    else:
        for fam in families:
            for cfg in cases(fam, reduced):
                s = launch_samples(cfg)
                samples += s
                print(f"# {cfg.name}: {len(s)} launches", file=out, flush=True)
    if save:
        json.dump(samples, open(save, "w"))
    p, rel = fit(samples, defaults)
    print(f"# {len(samples)} launches; relative residuals of the fit: rms {100 * float(np.sqrt(np.mean(rel ** 2))):.1f} %, worst {100 * float(np.max(np.abs(rel))):.1f} %", file=out)
    print("const tc_model_params_t kDefaultModel = {", file=out)
    print(f"    {p['peak_flops']:.4g},", file=out)
    print("    {" + ", ".join(f"{v:.3f}" for v in p["rho_a"]) + "},", file=out)
    print(f"    {p['bandwidth']:.4g},\n    {p['rho_b']:.3f},\n    {p['t_launch']:.3g},\n    {p['t_tile']:.3g},\n    {p['units']}, {{0, 0, 0}},", file=out)
    print(f"    {p['rho_small']:.3f},\n    {p['t_tile_small']:.3g},\n    {p['rho_gather']:.3f},\n    {p['lambda_ab']:.4f},", file=out)
    print("    {" + ", ".join(f"{v:.3f}" for v in p["rho_table"]) + "},", file=out)
    print(f"    {p['rho_small_table']:.3f}}};", file=out)
    return p


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--family", default="all")
    ap.add_argument("--reps", type=int, default=3)
    ap.add_argument("--reduced", action="store_true", help="a grid of smaller shapes that finishes in about a minute")
    ap.add_argument("--fit", action="store_true", help="fit the model's parameters to per-launch times instead of running the grid")
    ap.add_argument("--save-samples", default="", help="with --fit: write the measured launches to this JSON file")
    ap.add_argument("--samples", default="", help="with --fit: fit to the launches of this JSON file instead of measuring (needs no GPU)")
    args = ap.parse_args()
    families = FAMILIES if args.family == "all" else tuple(args.family.split(","))
    if args.fit and args.samples:
        import paper_1704_03092_amd as tc

        tc.load_library()
        run_fit(families, args.reduced, load=args.samples)
        return 0
    import torch  # (before the library: both bring a HIP runtime, torch's must be the one in the process)

    import paper_1704_03092_amd as tc

    assert torch.cuda.is_available(), "the sweep needs a GPU"
    tc.load_library()
    if args.fit:
        run_fit(families, args.reduced, save=args.save_samples or None)
    else:
        run_grid(families, args.reduced, args.reps)


if __name__ == "__main__":
    sys.exit(main())
