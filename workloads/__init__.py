"""Seeded synthetic workloads: tensor data generators, layouts and the benchmark
contraction shapes.

This package is the only code shared by the CPU oracle's tests and the GPU
path's tests/bench.  It describes inputs (labels, lengths, strides, values) and
contains none of the contraction or Strassen arithmetic.

Data values come from a counter-based generator keyed on (seed, tensor id,
logical column-major element index); the C implementation in ``gen.c`` is used
when it has been built (``workloads.build()``), else an equivalent numpy one.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field
from typing import Dict, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libworkloads.so")
_lib = None

KIND_UNIFORM, KIND_NORMAL, KIND_SMALLINT = 0, 1, 2
_KINDS = {"uniform": KIND_UNIFORM, "normal": KIND_NORMAL, "smallint": KIND_SMALLINT}


def build(force: bool = True) -> str:
    """Compile gen.c into libworkloads.so (gcc, OpenMP)."""
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src, "-lm"])
    global _lib
    _lib = None
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None and os.path.exists(_LIB_PATH):
        lib = ctypes.CDLL(_LIB_PATH)
        lib.wl_fill.restype = ctypes.c_int
        lib.wl_fill.argtypes = [ctypes.c_void_p, ctypes.c_int64, ctypes.c_int64, ctypes.c_uint64, ctypes.c_uint64, ctypes.c_int]
        _lib = lib
    return _lib


_G1 = np.uint64(0x9E3779B97F4A7C15)
_G2 = np.uint64(0xD1B54A32D192ED03)


def _mix64(x: np.ndarray) -> np.ndarray:
    x = x ^ (x >> np.uint64(30))
    x = x * np.uint64(0xBF58476D1CE4E5B9)
    x = x ^ (x >> np.uint64(27))
    x = x * np.uint64(0x94D049BB133111EB)
    x = x ^ (x >> np.uint64(31))
    return x


def _fill_numpy(first: int, count: int, seed: int, tid: int, kind: int) -> np.ndarray:
    with np.errstate(over="ignore"):
        key = np.uint64(seed) ^ (np.uint64(tid) * _G2)
        c = np.arange(first, first + count, dtype=np.uint64)
        two53 = 1.0 / 9007199254740992.0
        if kind == KIND_UNIFORM:
            x = _mix64(key + (c + np.uint64(1)) * _G1)
            return 2.0 * ((x >> np.uint64(11)).astype(np.float64) * two53) - 1.0
        if kind == KIND_NORMAL:
            x1 = _mix64(key + (np.uint64(2) * c + np.uint64(1)) * _G1)
            x2 = _mix64(key + (np.uint64(2) * c + np.uint64(2)) * _G1)
            u1 = ((x1 >> np.uint64(11)).astype(np.float64) + 1.0) * two53
            u2 = (x2 >> np.uint64(11)).astype(np.float64) * two53
            return np.sqrt(-2.0 * np.log(u1)) * np.cos(6.283185307179586476925286766559 * u2)
        if kind == KIND_SMALLINT:
            x = _mix64(key + (c + np.uint64(1)) * _G1)
            return ((x >> np.uint64(11)) % np.uint64(9)).astype(np.float64) - 4.0
    raise ValueError("unknown kind")


def fill(count: int, seed: int, tid: int, kind="uniform", first: int = 0, use_c: Optional[bool] = None) -> np.ndarray:
    """``count`` fp64 values for logical elements first..first+count-1 of tensor ``tid``."""
    k = _KINDS[kind] if isinstance(kind, str) else int(kind)
    lib = _load() if use_c in (None, True) else None
    if use_c is True and lib is None:
        raise RuntimeError("libworkloads.so is not built")
    if lib is None:
        return _fill_numpy(first, count, seed, tid, k)
    out = np.empty(count, dtype=np.float64)
    rc = lib.wl_fill(out.ctypes.data, first, count, seed, tid, k)
    if rc != 0:
        raise RuntimeError("wl_fill failed")
    return out


# ----------------------------------------------------------------------------
# layouts
# ----------------------------------------------------------------------------

def strides_for_order(lens: Sequence[int], order: Sequence[int], pad: int = 0) -> Tuple[int, ...]:
    """Strides (in elements) when dimension order[0] is stored fastest, order[1] next, ...;
    ``pad`` extra elements are inserted after the fastest dimension."""
    strides = [0] * len(lens)
    s = 1
    for n, d in enumerate(order):
        strides[d] = s
        s *= max(int(lens[d]), 1)
        if n == 0:
            s += pad
    return tuple(strides)


def col_major(lens: Sequence[int]) -> Tuple[int, ...]:
    return strides_for_order(lens, list(range(len(lens))))


def row_major(lens: Sequence[int]) -> Tuple[int, ...]:
    return strides_for_order(lens, list(range(len(lens) - 1, -1, -1)))


def storage_size(lens: Sequence[int], strides: Sequence[int]) -> int:
    if any(int(n) == 0 for n in lens):
        return 1
    return 1 + sum((int(n) - 1) * int(s) for n, s in zip(lens, strides))


@dataclass
class Tensor:
    """A strided fp64 tensor: flat storage + labels + lengths + strides (in elements)."""
    idx: str
    lens: Tuple[int, ...]
    strides: Tuple[int, ...]
    data: np.ndarray  # 1-D float64 storage

    def view(self) -> np.ndarray:
        """Logical N-d view (no copy) of the strided storage."""
        return np.lib.stride_tricks.as_strided(self.data, shape=self.lens, strides=tuple(8 * s for s in self.strides))

    def copy(self) -> "Tensor":
        return Tensor(self.idx, self.lens, self.strides, self.data.copy())

    def relabel(self, mapping: Dict[str, str]) -> "Tensor":
        return Tensor("".join(mapping.get(c, c) for c in self.idx), self.lens, self.strides, self.data)


def from_dense(idx: str, dense: np.ndarray, strides: Optional[Sequence[int]] = None, fillvalue: float = 0.0) -> Tensor:
    """Store a logical dense array with the given strides (default: generalized column-major)."""
    lens = tuple(int(n) for n in dense.shape)
    if strides is None:
        strides = col_major(lens)
    strides = tuple(int(s) for s in strides)
    data = np.full(storage_size(lens, strides), fillvalue, dtype=np.float64)
    t = Tensor(idx, lens, strides, data)
    if dense.size:
        t.view()[...] = dense
    return t


def make_tensor(idx: str, lengths: Dict[str, int], seed: int, tid: int, kind="uniform",
                strides: Optional[Sequence[int]] = None) -> Tensor:
    """Seeded tensor: element with logical column-major linear index e gets draw e."""
    lens = tuple(int(lengths[c]) for c in idx)
    count = int(np.prod(lens, dtype=np.int64)) if lens else 1
    flat = fill(count, seed, tid, kind)
    if strides is None or tuple(strides) == col_major(lens):
        return Tensor(idx, lens, col_major(lens), flat)
    return from_dense(idx, flat.reshape(lens, order="F"), strides)


# ----------------------------------------------------------------------------
# the benchmark contractions (synthetic stand-ins shaped like the paper's workloads)
# ----------------------------------------------------------------------------

@dataclass
class Contraction:
    name: str
    idxC: str
    idxA: str
    idxB: str
    lengths: Dict[str, int]
    alpha: float = 1.0
    beta: float = 1.0
    kind: str = "uniform"
    seed: int = 170403092
    note: str = ""
    modes: Tuple[Tuple[int, str], ...] = field(default_factory=tuple)  # (level, variant)

    def bundles(self):
        I = [c for c in self.idxA if c in self.idxC]
        J = [c for c in self.idxB if c in self.idxC]
        P = [c for c in self.idxA if c in self.idxB]
        return I, J, P

    def mnk(self) -> Tuple[int, int, int]:
        I, J, P = self.bundles()
        prod = lambda L: int(np.prod([self.lengths[c] for c in L], dtype=np.int64)) if L else 1
        return prod(I), prod(J), prod(P)

    def flops(self) -> float:
        m, n, k = self.mnk()
        return 2.0 * m * n * k

    def tensors(self, kind: Optional[str] = None, layout: str = "col"):
        """(A, B, C) seeded tensors; tensor ids A=0, B=1, C=2."""
        kd = kind or self.kind
        out = []
        for tid, idx in enumerate((self.idxA, self.idxB, self.idxC)):
            lens = [self.lengths[c] for c in idx]
            st = col_major(lens) if layout == "col" else row_major(lens)
            out.append(make_tensor(idx, self.lengths, self.seed, tid, kd, st))
        return tuple(out)


_ALL9 = tuple((l, v) for l in (1, 2) for v in ("naive", "ab", "abc"))


def gemm(N: int, seed_off: int = 0, **kw) -> Contraction:
    return Contraction(f"gemm{N}", "ij", "ik", "kj", {"i": N, "j": N, "k": N}, 1.0, 1.0, "uniform",
                       170403092 + 2 + seed_off, "square GEMM, paper's synthetic square family", ((0, "abc"),) + _ALL9 + ((1, "hybrid"), (2, "hybrid")), **kw)


def configs() -> Dict[str, Contraction]:
    """The five benchmark configurations (C-A-B index strings, generalized column-major)."""
    c = {}
    c["cfg1"] = Contraction("cfg1", "abcd", "aebf", "dfce", {x: 16 for x in "abcdef"}, 1.0, 0.0, "uniform", 170403092 + 1,
                            "4-D CCSD-style index string, all lengths 16", ((0, "abc"), (1, "abc")))
    for N in (4096, 8192, 16384, 10001):
        c[f"cfg2_{N}"] = gemm(N)
    c["cfg3"] = Contraction("cfg3", "abij", "abef", "efij", {"a": 192, "b": 192, "e": 192, "f": 192, "i": 48, "j": 48},
                            1.0, 1.0, "normal", 170403092 + 3, "CCSD particle-particle ladder shape",
                            ((0, "abc"), (1, "abc"), (1, "hybrid"), (2, "abc"), (2, "hybrid")))
    c["cfg4a"] = Contraction("cfg4a", "abc", "daec", "ebd", {"a": 96, "b": 96, "c": 96, "d": 64, "e": 64}, 1.0, 1.0, "uniform",
                             170403092 + 4, "permuted strides, conflicting order in the contracted bundle",
                             ((0, "abc"), (1, "abc"), (1, "ab"), (2, "abc")))
    c["cfg4b"] = Contraction("cfg4b", "abcd", "aeb", "ecd", {"a": 128, "b": 128, "c": 128, "d": 128, "e": 256}, 1.0, 1.0, "uniform",
                             170403092 + 5, "rank-k shape", ((0, "abc"), (1, "abc"), (1, "ab"), (2, "abc")))
    c["cfg5"] = Contraction("cfg5", "abcdef", "agbch", "hdgef", {**{x: 24 for x in "abcdef"}, "g": 96, "h": 96}, 1.0, 1.0, "uniform",
                            170403092 + 6, "6-D contraction",
                            ((0, "abc"), (1, "ab"), (1, "abc"), (1, "hybrid"), (2, "ab"), (2, "abc"), (2, "hybrid")))
    return c


def scaled(cfg: Contraction, lengths: Dict[str, int], name: Optional[str] = None) -> Contraction:
    """Same index strings and distribution at other lengths (reduced-size parity cases)."""
    L = dict(cfg.lengths)
    L.update(lengths)
    return Contraction(name or (cfg.name + "_small"), cfg.idxC, cfg.idxA, cfg.idxB, L, cfg.alpha, cfg.beta, cfg.kind, cfg.seed,
                       cfg.note, cfg.modes)
