"""Helpers for the GPU parity tests: move seeded tensors to the device, run the HIP library through its C ABI,
bring the result back."""
import numpy as np

import paper_1704_03092_amd as tc


def to_dev(T):
    import torch

    return torch.from_numpy(T.data).to("cuda")


def run_gpu(A, B, C, alpha=1.0, beta=1.0, level=0, variant="abc", dev=None, poison_ws=True, **plan_kw):
    """Returns (flat numpy copy of C's storage after the contraction, plan info)."""
    import torch

    dA, dB, dC = dev if dev is not None else (to_dev(A), to_dev(B), to_dev(C))
    if dev is not None:
        dC = dC.clone()
    st = torch.cuda.current_stream()
    plan = tc.tc_plan(A, B, C, level, variant, st, **plan_kw)
    try:
        info = tc.tc_plan_info(plan)
        nbytes = tc.tc_plan_workspace_bytes(plan)
        ws = None
        if nbytes:
            ws = torch.full((nbytes // 8,), float("nan") if poison_ws else 0.0, dtype=torch.float64, device="cuda")
        tc.tc_contract(plan, alpha, dA, dB, beta, dC, ws, st)
        torch.cuda.synchronize()
    finally:
        tc.tc_destroy(plan)
    return dC.cpu().numpy(), info


def logical(T, flat):
    """Logical N-d view of flat storage laid out like tensor T."""
    return np.lib.stride_tricks.as_strided(flat, shape=T.lens, strides=tuple(8 * s for s in T.strides))
