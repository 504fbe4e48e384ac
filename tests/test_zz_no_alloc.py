"""tc_contract_static (the entry point for callers that cannot allocate) against tc_contract with an explicit
workspace: same kernels, so the results must agree bit for bit; and both against the CPU oracle.  Two calls in a
row on the GPU's one static buffer, the second on a smaller problem, then the size limit."""
import numpy as np
import pytest

import oracle
import workloads

pytestmark = pytest.mark.gpu


def _case(tc, torch, lengths, level, variant, seed, **kw):
    c = workloads.Contraction("g", "ij", "ik", "kj", lengths, seed=seed)
    A, B, C = c.tensors()
    st = torch.cuda.current_stream()
    dA, dB = (torch.from_numpy(T.data).to("cuda") for T in (A, B))
    plan = tc.tc_plan(A, B, C, level, variant, st, **kw)
    nbytes = tc.tc_plan_workspace_bytes(plan)
    assert 0 < nbytes <= tc.TC_STATIC_WORKSPACE_BYTES, nbytes  # the case must use the scratch buffer
    print(f"static workspace case {lengths} level={level} {variant} {kw}: workspace {nbytes} bytes", flush=True)
    ws = torch.full((nbytes // 8,), float("nan"), dtype=torch.float64, device="cuda")
    dC1 = torch.from_numpy(C.data).to("cuda")
    dC2 = dC1.clone()
    tc.tc_contract(plan, 1.25, dA, dB, 0.5, dC1, ws, st)
    tc.tc_contract_static(plan, 1.25, dA, dB, 0.5, dC2, st)
    torch.cuda.synchronize()
    tc.tc_destroy(plan)
    assert torch.equal(dC1, dC2)
    ref = C.copy()
    oracle.contract_matrix(A, B, ref, 1.25, 0.5)
    got = np.lib.stride_tricks.as_strided(dC2.cpu().numpy(), shape=C.lens, strides=tuple(8 * s for s in C.strides))
    err = oracle.error_metric(got, ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B))
    assert err <= (1e-12 if level == 2 else 1e-13), err


def test_static_workspace_two_calls_then_the_limit():
    import torch

    import paper_1704_03092_amd as tc

    assert torch.cuda.is_available()
    tc.load_library()
    # AB keeps each product M in the workspace; a forced tail split adds the chunks of every tile
    _case(tc, torch, {"i": 1100, "j": 900, "k": 1408}, 1, "ab", 3, tail_split=3)
    _case(tc, torch, {"i": 300, "j": 275, "k": 190}, 2, "naive", 4)  # smaller: the buffer still holds the first call's data
    _case(tc, torch, {"i": 672, "j": 608, "k": 704}, 1, "hybrid", 5)
    # a plan whose workspace does not fit is refused before anything is enqueued
    big = workloads.Contraction("g", "ij", "ik", "kj", {"i": 6000, "j": 6000, "k": 256}, seed=1)
    A, B, C = big.tensors()
    st = torch.cuda.current_stream()
    plan = tc.tc_plan(A, B, C, 1, "ab", st)
    assert tc.tc_plan_workspace_bytes(plan) > tc.TC_STATIC_WORKSPACE_BYTES
    dA, dB, dC = (torch.from_numpy(T.data).to("cuda") for T in (A, B, C))
    before = dC.clone()
    with pytest.raises(tc.TcError) as e:
        tc.tc_contract_static(plan, 1.0, dA, dB, 1.0, dC, st)
    assert e.value.status == -12 and "TC_STATIC_WORKSPACE_BYTES" in tc.tc_strerror(-12)
    torch.cuda.synchronize()
    assert torch.equal(dC, before)
    tc.tc_destroy(plan)
    # no workspace needed: the call works without touching the buffer
    small = workloads.Contraction("g", "ij", "ik", "kj", {"i": 256, "j": 256, "k": 64}, seed=2)
    A, B, C = small.tensors()
    plan = tc.tc_plan(A, B, C, 0, "abc", st, tail_split=-1)
    assert tc.tc_plan_workspace_bytes(plan) == 0
    dA, dB, dC1 = (torch.from_numpy(T.data).to("cuda") for T in (A, B, C))
    dC2 = dC1.clone()
    tc.tc_contract(plan, 1.0, dA, dB, 1.0, dC1, None, st)
    tc.tc_contract_static(plan, 1.0, dA, dB, 1.0, dC2, st)
    torch.cuda.synchronize()
    tc.tc_destroy(plan)
    assert torch.equal(dC1, dC2)
