"""ctypes binding of libstrassen_tc.so.

Only marshals arguments: tensors are described by (labels, lengths, strides) and passed as device pointers
(``torch`` tensors on the GPU, or raw integers).  There is no CPU fallback: if the shared library is missing
or no GPU is present the calls fail with an error.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
_ROOT = os.path.dirname(_HERE)
_LIB = os.path.join(_HERE, "libstrassen_tc.so")
_lib = None

VARIANTS = {"naive": 0, "ab": 1, "abc": 2, "hybrid": 3, "auto": -1}
TC_LEVEL_AUTO = -1
TC_VARIANT_AUTO = -1
TC_MAX_NDIM = 16

HIPCC_FLAGS = ["-O3", "--offload-arch=gfx950", "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-std=c++17", "-shared",
               "-fPIC"]


def lib_path() -> str:
    return _LIB


def build(verbose: bool = False) -> str:
    """Compile the HIP library for gfx950 with hipcc (cross-compiles without a GPU); translation units in parallel."""
    from concurrent.futures import ThreadPoolExecutor

    names = ["tc_host.cpp", "tc_device.hip", "tc_fused_11.hip", "tc_fused_12.hip", "tc_fused_21.hip", "tc_fused_22.hip", "tc_fused_14.hip", "tc_fused_41.hip", "tc_fused_24.hip", "tc_fused_42.hip", "tc_fused_44.hip", "tc_fused_any.hip", "tc_small_11.hip"]
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    objdir = os.path.join(_HERE, "csrc", "_build")
    os.makedirs(objdir, exist_ok=True)
    flags = [f for f in HIPCC_FLAGS if f != "-shared"]

    def compile_one(name):
        obj = os.path.join(objdir, name + ".o")
        cmd = [hipcc] + flags + ["-I" + os.path.join(_ROOT, "include"), "-c", "-o", obj, os.path.join(_HERE, "csrc", name)]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        out = "\n".join(l for l in res.stdout.splitlines() if "packed-fp32-ops" not in l)
        if res.returncode != 0:
            raise RuntimeError(f"hipcc failed on {name}:\n" + out)
        return obj, out

    with ThreadPoolExecutor(max_workers=min(len(names), int(os.environ.get("MAX_JOBS", "8")))) as ex:
        results = list(ex.map(compile_one, names))
    link = [hipcc, "--offload-arch=gfx950", "-shared", "-fPIC", "-o", _LIB] + [o for o, _ in results]
    res = subprocess.run(link, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    if res.returncode != 0:
        raise RuntimeError("hipcc link failed:\n" + res.stdout)
    if verbose:
        for _, out in results:
            if out.strip():
                print(out)
    global _lib
    _lib = None
    return _LIB


class tc_tensor_desc_t(ctypes.Structure):
    _fields_ = [("ndim", ctypes.c_int), ("len", ctypes.POINTER(ctypes.c_int64)), ("stride", ctypes.POINTER(ctypes.c_int64)),
                ("idx", ctypes.c_char_p)]


class tc_options_t(ctypes.Structure):
    _fields_ = [("bs_block", ctypes.c_int), ("host_only", ctypes.c_int), ("no_merge", ctypes.c_int), ("split_k", ctypes.c_int),
                ("tail_split", ctypes.c_int), ("tile_n", ctypes.c_int), ("no_peel", ctypes.c_int), ("no_repack", ctypes.c_int)]


class tc_launch_info_t(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int), ("n_products", ctypes.c_int), ("max_terms", ctypes.c_int), ("tail_tiles", ctypes.c_int),
                ("tail_chunks", ctypes.c_int), ("terms_a", ctypes.c_int), ("terms_b", ctypes.c_int), ("tile_n", ctypes.c_int), ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("depth", ctypes.c_int64), ("tiles", ctypes.c_int64), ("tail_kc", ctypes.c_int64), ("tiles_table_free", ctypes.c_int64),
                ("moved_elems", ctypes.c_double), ("pairs_a", ctypes.c_int), ("pairs_b", ctypes.c_int)]


class tc_plan_info_t(ctypes.Structure):
    _fields_ = [("m", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64), ("level_requested", ctypes.c_int),
                ("level", ctypes.c_int), ("variant", ctypes.c_int), ("n_products", ctypes.c_int), ("n_launches", ctypes.c_int),
                ("bs_block", ctypes.c_int), ("a_mode", ctypes.c_int), ("b_mode", ctypes.c_int), ("mb", ctypes.c_int64),
                ("nb", ctypes.c_int64), ("kb", ctypes.c_int64), ("I", ctypes.c_char * (TC_MAX_NDIM + 1)),
                ("J", ctypes.c_char * (TC_MAX_NDIM + 1)), ("P", ctypes.c_char * (TC_MAX_NDIM + 1)), ("m_peel", ctypes.c_int64),
                ("n_peel", ctypes.c_int64)]


class tc_product_t(ctypes.Structure):
    _fields_ = [("n_a", ctypes.c_int), ("n_b", ctypes.c_int), ("n_c", ctypes.c_int)] + \
               [(f"{o}_{w}", ctypes.c_int * 4) for o in "abc" for w in ("row", "col", "sign")] + \
               [("c_first", ctypes.c_int * 4), ("launch", ctypes.c_int)]


class tc_model_params_t(ctypes.Structure):
    _fields_ = [("peak_flops", ctypes.c_double), ("rho_a", ctypes.c_double * 3), ("bandwidth", ctypes.c_double), ("rho_b", ctypes.c_double),
                ("t_launch", ctypes.c_double), ("t_tile", ctypes.c_double), ("units", ctypes.c_int), ("reserved", ctypes.c_int * 3),
                ("rho_small", ctypes.c_double), ("t_tile_small", ctypes.c_double), ("rho_gather", ctypes.c_double), ("lambda_ab", ctypes.c_double),
                ("rho_table", ctypes.c_double * 3), ("rho_small_table", ctypes.c_double)]


class tc_model_time_t(ctypes.Structure):
    _fields_ = [("total", ctypes.c_double), ("arith", ctypes.c_double), ("c_update", ctypes.c_double), ("temporaries", ctypes.c_double),
                ("launch", ctypes.c_double), ("operands", ctypes.c_double)]


class tc_launch_times_t(ctypes.Structure):
    _fields_ = [("fused_ms", ctypes.c_double), ("elementwise_ms", ctypes.c_double), ("fused_launches", ctypes.c_int),
                ("elementwise_launches", ctypes.c_int)]


class TcError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: {tc_strerror(status)} ({status})")
        self.status = status


def load_library():
    """Load libstrassen_tc.so; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB):
            raise RuntimeError(f"{_LIB} is missing: run `python -c 'import __graft_entry__ as g; g.build()'` first")
        lib = ctypes.CDLL(_LIB)
        vp, ci, dbl = ctypes.c_void_p, ctypes.c_int, ctypes.c_double
        dp = ctypes.POINTER(tc_tensor_desc_t)
        lib.tc_plan.restype = ci
        lib.tc_plan.argtypes = [ctypes.POINTER(vp), dp, dp, dp, ci, ci, vp]
        lib.tc_plan_ex.restype = ci
        lib.tc_plan_ex.argtypes = [ctypes.POINTER(vp), dp, dp, dp, ci, ci, ctypes.POINTER(tc_options_t), vp]
        lib.tc_plan_workspace_bytes.restype = ctypes.c_size_t
        lib.tc_plan_workspace_bytes.argtypes = [vp]
        lib.tc_contract.restype = ci
        lib.tc_contract.argtypes = [vp, dbl, vp, vp, dbl, vp, vp, vp]
        lib.tc_contract_static.restype = ci
        lib.tc_contract_static.argtypes = [vp, dbl, vp, vp, dbl, vp, vp]
        lib.tc_contract_launch_times.restype = ci
        lib.tc_contract_launch_times.argtypes = [vp, dbl, vp, vp, dbl, vp, vp, vp, ctypes.POINTER(ctypes.c_double), ci]
        lib.tc_bench_mfma_peak.restype = ci
        lib.tc_bench_mfma_peak.argtypes = [ci, vp, ctypes.POINTER(ctypes.c_double)]
        lib.tc_contract_timed.restype = ci
        lib.tc_contract_timed.argtypes = [vp, dbl, vp, vp, dbl, vp, vp, vp, ctypes.POINTER(tc_launch_times_t)]
        lib.tc_destroy.restype = ci
        lib.tc_destroy.argtypes = [vp]
        lib.tc_strerror.restype = ctypes.c_char_p
        lib.tc_strerror.argtypes = [ci]
        lib.tc_plan_info.restype = ci
        lib.tc_plan_info.argtypes = [vp, ctypes.POINTER(tc_plan_info_t)]
        lib.tc_plan_schedule.restype = ci
        lib.tc_plan_schedule.argtypes = [vp, ci, ctypes.POINTER(tc_product_t)]
        lib.tc_plan_launch.restype = ci
        lib.tc_plan_launch.argtypes = [vp, ci, ctypes.POINTER(tc_launch_info_t)]
        lib.tc_model_defaults.restype = ci
        lib.tc_model_defaults.argtypes = [ctypes.POINTER(tc_model_params_t)]
        lib.tc_plan_predict.restype = ci
        lib.tc_plan_predict.argtypes = [vp, ctypes.POINTER(tc_model_params_t), ctypes.POINTER(tc_model_time_t)]
        lib.tc_plan_vector.restype = ctypes.c_int64
        lib.tc_plan_vector.argtypes = [vp, ci, vp, ctypes.c_int64]
        _lib = lib
    return _lib


def tc_strerror(status: int) -> str:
    return load_library().tc_strerror(int(status)).decode()


def _desc(idx: str, lens: Sequence[int], strides: Sequence[int]):
    n = len(idx)
    if len(lens) != n or len(strides) != n:
        raise ValueError("labels, lengths and strides must have the same number of entries")
    L = (ctypes.c_int64 * max(n, 1))(*[int(x) for x in lens])
    S = (ctypes.c_int64 * max(n, 1))(*[int(x) for x in strides])
    d = tc_tensor_desc_t(n, L, S, idx.encode())
    d._keep = (L, S)
    return d


def _ptr(x) -> Optional[int]:
    if x is None:
        return None
    if isinstance(x, int):
        return x
    return int(x.data_ptr())  # torch tensor


def _stream(stream) -> Optional[int]:
    if stream is None:
        return None
    if isinstance(stream, int):
        return stream or None
    return int(stream.cuda_stream) or None  # torch.cuda.Stream


class Plan:
    """Owner of a tc_plan_t*."""

    def __init__(self, handle: int):
        self.handle = handle

    def __del__(self):
        try:
            tc_destroy(self)
        except Exception:
            pass


def tc_plan(A, B, C, level: int = 0, variant="abc", stream=None, bs_block: int = 0, host_only: bool = False,
            no_merge: bool = False, split_k: int = 0, tail_split: int = 0, tile_n: int = 0, no_peel: bool = False, no_repack: bool = False) -> Plan:
    """A, B, C: (labels, lengths, strides) triples or objects with .idx/.lens/.strides.
    tail_split: 0 = automatic, -1 = never, 2..16 = forced chunk count; tile_n: 0 = automatic, 64 or 128 (see tc_options_t)."""
    lib = load_library()
    ds = []
    for T in (A, B, C):
        if hasattr(T, "idx"):
            ds.append(_desc(T.idx, T.lens, T.strides))
        else:
            ds.append(_desc(*T))
    v = VARIANTS[variant] if isinstance(variant, str) else int(variant)
    out = ctypes.c_void_p()
    opts = tc_options_t(int(bs_block), int(bool(host_only)), int(bool(no_merge)), int(split_k), int(tail_split), int(tile_n),
                        int(bool(no_peel)), int(bool(no_repack)))
    rc = lib.tc_plan_ex(ctypes.byref(out), ctypes.byref(ds[0]), ctypes.byref(ds[1]), ctypes.byref(ds[2]), int(level), v,
                        ctypes.byref(opts), _stream(stream))
    if rc != 0:
        raise TcError(rc, "tc_plan")
    return Plan(out.value)


def tc_plan_workspace_bytes(plan: Plan) -> int:
    return int(load_library().tc_plan_workspace_bytes(plan.handle))


def tc_contract(plan: Plan, alpha: float, A, B, beta: float, C, workspace=None, stream=None) -> None:
    rc = load_library().tc_contract(plan.handle, float(alpha), _ptr(A), _ptr(B), float(beta), _ptr(C), _ptr(workspace), _stream(stream))
    if rc != 0:
        raise TcError(rc, "tc_contract")


TC_STATIC_WORKSPACE_BYTES = 32 << 20


def tc_contract_static(plan: Plan, alpha: float, A, B, beta: float, C, stream=None) -> None:
    """tc_contract with the library's static per-GPU workspace (no allocation; plans up to TC_STATIC_WORKSPACE_BYTES)."""
    rc = load_library().tc_contract_static(plan.handle, float(alpha), _ptr(A), _ptr(B), float(beta), _ptr(C), _stream(stream))
    if rc != 0:
        raise TcError(rc, "tc_contract_static")


def tc_contract_launch_times(plan: Plan, alpha: float, A, B, beta: float, C, workspace=None, stream=None) -> list:
    """tc_contract with a HIP event after every launch; blocks; returns the milliseconds of each launch (tc_plan_launches order)."""
    n = tc_plan_info(plan)["n_launches"]
    buf = (ctypes.c_double * max(n, 1))()
    rc = load_library().tc_contract_launch_times(plan.handle, float(alpha), _ptr(A), _ptr(B), float(beta), _ptr(C), _ptr(workspace),
                                                 _stream(stream), buf, max(n, 1))
    if rc < 0:
        raise TcError(rc, "tc_contract_launch_times")
    return [buf[i] for i in range(rc)]


def tc_bench_mfma_peak(instruction: int = 0, stream=None) -> float:
    """TFLOP/s of an MFMA-only kernel (0: v_mfma_f64_4x4x4_4b_f64, 1: v_mfma_f64_16x16x4_f64)."""
    out = ctypes.c_double()
    rc = load_library().tc_bench_mfma_peak(int(instruction), _stream(stream), ctypes.byref(out))
    if rc != 0:
        raise TcError(rc, "tc_bench_mfma_peak")
    return out.value


def tc_contract_timed(plan: Plan, alpha: float, A, B, beta: float, C, workspace=None, stream=None) -> dict:
    """tc_contract with per-launch HIP events; blocks; returns the time per kind of kernel."""
    out = tc_launch_times_t()
    rc = load_library().tc_contract_timed(plan.handle, float(alpha), _ptr(A), _ptr(B), float(beta), _ptr(C), _ptr(workspace), _stream(stream),
                                          ctypes.byref(out))
    if rc != 0:
        raise TcError(rc, "tc_contract_timed")
    return {k: getattr(out, k) for k, _ in tc_launch_times_t._fields_}


def tc_destroy(plan: Plan) -> None:
    if plan.handle:
        load_library().tc_destroy(plan.handle)
        plan.handle = None


def tc_plan_info(plan: Plan) -> dict:
    info = tc_plan_info_t()
    rc = load_library().tc_plan_info(plan.handle, ctypes.byref(info))
    if rc != 0:
        raise TcError(rc, "tc_plan_info")
    d = {k: getattr(info, k) for k, _ in tc_plan_info_t._fields_}
    for k in "IJP":
        d[k] = d[k].decode()
    return d


def tc_model_defaults() -> dict:
    mp = tc_model_params_t()
    rc = load_library().tc_model_defaults(ctypes.byref(mp))
    if rc != 0:
        raise TcError(rc, "tc_model_defaults")
    return {"peak_flops": mp.peak_flops, "rho_a": list(mp.rho_a), "bandwidth": mp.bandwidth, "rho_b": mp.rho_b, "t_launch": mp.t_launch,
            "t_tile": mp.t_tile, "units": mp.units, "rho_small": mp.rho_small, "t_tile_small": mp.t_tile_small,
            "rho_gather": mp.rho_gather, "lambda_ab": mp.lambda_ab, "rho_table": list(mp.rho_table), "rho_small_table": mp.rho_small_table}


def tc_plan_predict(plan: Plan, params: Optional[dict] = None) -> dict:
    """Modelled seconds of one tc_contract (beta != 0); params as returned by tc_model_defaults (None: the defaults)."""
    mp = None
    if params is not None:
        mp = tc_model_params_t(params["peak_flops"], (ctypes.c_double * 3)(*params["rho_a"]), params["bandwidth"], params["rho_b"],
                               params["t_launch"], params["t_tile"], int(params["units"]), (ctypes.c_int * 3)(),
                               params["rho_small"], params["t_tile_small"], params["rho_gather"], params["lambda_ab"],
                               (ctypes.c_double * 3)(*params["rho_table"]), params["rho_small_table"])
    out = tc_model_time_t()
    rc = load_library().tc_plan_predict(plan.handle, ctypes.byref(mp) if mp is not None else None, ctypes.byref(out))
    if rc != 0:
        raise TcError(rc, "tc_plan_predict")
    return {k: getattr(out, k) for k, _ in tc_model_time_t._fields_}


def tc_plan_launches(plan: Plan) -> list:
    """Every launch of the schedule (tc_plan_launch) as a dict."""
    lib = load_library()
    out = []
    for i in range(tc_plan_info(plan)["n_launches"]):
        L = tc_launch_info_t()
        rc = lib.tc_plan_launch(plan.handle, i, ctypes.byref(L))
        if rc != 0:
            raise TcError(rc, "tc_plan_launch")
        out.append({k: getattr(L, k) for k, _ in tc_launch_info_t._fields_ if k != "reserved"})
    return out


def tc_plan_schedule(plan: Plan) -> list:
    lib = load_library()
    n = tc_plan_info(plan)["n_products"]
    out = []
    for i in range(n):
        p = tc_product_t()
        rc = lib.tc_plan_schedule(plan.handle, i, ctypes.byref(p))
        if rc != 0:
            raise TcError(rc, "tc_plan_schedule")
        e = {"launch": p.launch}
        for o, cnt in (("a", p.n_a), ("b", p.n_b), ("c", p.n_c)):
            e[o] = [(getattr(p, f"{o}_row")[t], getattr(p, f"{o}_col")[t], getattr(p, f"{o}_sign")[t]) for t in range(cnt)]
        e["c_first"] = [p.c_first[t] for t in range(p.n_c)]
        out.append(e)
    return out


def tc_plan_vector(plan: Plan, which: int):
    """Planner output `which` (0..5 scatter vectors, 6..11 block scatter vectors) as a numpy int64 array."""
    import numpy as np

    lib = load_library()
    n = lib.tc_plan_vector(plan.handle, int(which), None, 0)
    if n < 0:
        raise TcError(int(n), "tc_plan_vector")
    out = np.zeros(max(int(n), 1), dtype=np.int64)
    rc = lib.tc_plan_vector(plan.handle, int(which), out.ctypes.data, int(n))
    if rc < 0:
        raise TcError(int(rc), "tc_plan_vector")
    return out[:int(n)]


def contract(A_desc, B_desc, C_desc, A, B, C, alpha=1.0, beta=1.0, level=0, variant="abc", stream=None):
    """Convenience: plan, allocate the workspace with torch, contract, destroy.  A, B, C are torch CUDA tensors (flat storage)."""
    import torch

    plan = tc_plan(A_desc, B_desc, C_desc, level, variant, stream)
    try:
        nbytes = tc_plan_workspace_bytes(plan)
        ws = torch.empty(max(nbytes // 8, 1), dtype=torch.float64, device=C.device) if nbytes else None
        tc_contract(plan, alpha, A, B, beta, C, ws, stream if stream is not None else torch.cuda.current_stream())
    finally:
        tc_destroy(plan)
    return C
