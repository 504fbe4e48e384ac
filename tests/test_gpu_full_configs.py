"""GPU parity at the full sizes of the five benchmark configurations, in the launch configuration bench.py times.

Every configuration, the three largest included (cfg2 at 16384, cfg3, cfg5), is compared element by element with the
full classical oracle (the tiled loop nest over the whole of C; 10 to 25 s each on the GPU machine's host cores).

Tolerance: ||C - C_ref||_F / (||A||_F ||B||_F) <= 1e-13 (level 0 and 1), 1e-12 (level 2)."""
import time

import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu

TOL = {0: 1e-13, 1: 1e-13, 2: 1e-12}


@pytest.fixture(scope="module")
def gpu():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1704_03092_amd as tc

    tc.load_library()
    return tc


def _modes(cfg, extra=()):
    return [(l, v, {}) for (l, v) in cfg.modes] + list(extra)


def _run_modes(tc, cfg, extra=()):
    import torch

    t0 = time.time()
    A, B, C = cfg.tensors()
    m, n, k = cfg.mnk()
    print(f"[{cfg.name}] m={m} n={n} k={k} inputs generated in {time.time() - t0:.1f}s", flush=True)
    dA, dB, dC0 = (torch.from_numpy(T.data).to("cuda") for T in (A, B, C))
    st = torch.cuda.current_stream()
    nA, nB = oracle.tensor_norm(A), oracle.tensor_norm(B)
    full_ref = None
    for level, variant, kw in _modes(cfg, extra):
        plan = tc.tc_plan(A, B, C, level, variant, st, **kw)
        info = tc.tc_plan_info(plan)
        orders = (list(info["I"]), list(info["J"]), list(info["P"]))
        nbytes = tc.tc_plan_workspace_bytes(plan)
        ws = torch.full((max(nbytes // 8, 1),), float("nan"), dtype=torch.float64, device="cuda") if nbytes else None
        dC = dC0.clone()
        level = info["level"]
        variant = f"{variant}{kw if kw else ''}"
        print(f"[{cfg.name}] level {level} {variant}: launching ({info['n_launches']} launches)", flush=True)
        tc.tc_contract(plan, cfg.alpha, dA, dB, cfg.beta, dC, ws, st)  # warm-up + result
        torch.cuda.synchronize()
        got_flat = dC.cpu().numpy()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record(st)
        tc.tc_contract(plan, cfg.alpha, dA, dB, cfg.beta, dC, ws, st)
        e1.record(st)
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        tc.tc_destroy(plan)
        del dC, ws
        Cg = workloads.Tensor(C.idx, C.lens, C.strides, got_flat)
        if full_ref is None:
            t0 = time.time()
            full_ref = C.copy()
            oracle.contract_matrix(A, B, full_ref, cfg.alpha, cfg.beta, orders=orders)
            print(f"[{cfg.name}] full oracle in {time.time() - t0:.1f}s", flush=True)
        err = oracle.error_metric(Cg.view(), full_ref.view(), nA, nB)
        print(f"[{cfg.name}] level {level} {variant}: {ms:.3f} ms = {cfg.flops() / ms * 1e-9:.2f} TFLOP/s effective; err {err:.2e}",
              flush=True)
        assert err <= TOL[level], (cfg.name, level, variant, err)


def test_cfg1(gpu):
    _run_modes(gpu, workloads.configs()["cfg1"])


@pytest.mark.parametrize("N", [4096, 10001, 8192, 16384])
def test_cfg2_full_oracle(gpu, N):
    _run_modes(gpu, workloads.configs()[f"cfg2_{N}"])


def test_cfg3(gpu):
    _run_modes(gpu, workloads.configs()["cfg3"])


def test_cfg4a(gpu):
    # 72 tiles of 128 x 128 on 256 compute units: also with the contracted bundle cut into chunks, and with everything automatic
    _run_modes(gpu, workloads.configs()["cfg4a"],
               extra=[(0, "abc", {"split_k": 2}), (0, "abc", {"split_k": -1}), (-1, "auto", {"split_k": -1})])


def test_cfg4b(gpu):
    _run_modes(gpu, workloads.configs()["cfg4b"])


def test_cfg5(gpu):
    _run_modes(gpu, workloads.configs()["cfg5"])
