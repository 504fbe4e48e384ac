"""CPU oracle for fp64 tensor contraction and its Strassen evaluation.

TEST INFRASTRUCTURE, NOT THE PRODUCT.  Only ``tests/``, ``__graft_entry__.smoke()``
and ``bench.py``'s ``cpu_baseline`` leg may import this package.  It shares no code
with the HIP library (``paper_1704_03092_amd``) and never calls it.

What is here, and the passage of the paper each part follows:

* ``classify`` / ``scatter_vector`` / ``block_scatter`` / ``matrix_view`` -- index
  bundles I, J, P and the (block) scatter vectors of the matrix view
  (Sec. 2.3, "Tensor Contraction" and "Block Scatter Matrix View", the scatter-matrix location formula).
* ``contract_literal`` -- the definition of tensor contraction, loop nest in C
  (Sec. 2.3, displayed definition; locations by the general stride layout).
* ``contract_matrix`` / ``contract_rows`` -- the same sum on the matrix view, tiled
  and OpenMP-parallel in C; used at sizes the literal loop nest cannot reach.
* ``STRASSEN_U/V/W`` and ``strassen_tables`` -- the seven products M_0..M_6 displayed in Sec. 2.2
  as coefficient triples, and their L-level extension read as the Kronecker
  product of the one-level triples (Sec. 3 says only that the scheme "can be
  extended to multiple levels"; the 2-level operation counts 49/95/95/144 in the
  performance-model table are what this reading reproduces).
* ``strassen_recursive`` -- Strassen on the matrix view with explicit temporaries
  (the Naive formulation of Sec. 4.1), recursion depth L, classical product at the
  leaves, dynamic peeling for odd sizes (Sec. 3, last paragraph).
* ``strassen_flat`` -- the same result from the flattened 7^L-product schedule of
  the general primitive displayed in Sec. 3; rows/columns beyond the matrix are
  treated as zeros (the zero-padding option of Sec. 3, last paragraph).
* ``error_metric`` -- ||C - C_ref||_F / (||A||_F ||B||_F).
* ``freivalds`` -- randomized estimate of ||C - C_ref||_F over the whole of C.

Every function is pinned by tests/test_oracle_*.py against something other than
itself (numpy einsum/matmul, brute force in pure Python, the paper's worked
layout example, Brent's equations, exact integer arithmetic, invariants).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "liboracle.so")
_lib = None

_I64P = ctypes.POINTER(ctypes.c_int64)


def build(force: bool = True) -> str:
    """Compile tc_oracle.c into liboracle.so (gcc -O3, OpenMP, no fast-math, no FMA contraction: every operation rounds once)."""
    src = os.path.join(_HERE, "tc_oracle.c")
    if force or not os.path.exists(_LIB_PATH) or os.path.getmtime(_LIB_PATH) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O3", "-march=x86-64-v3", "-ffp-contract=off", "-fopenmp", "-shared", "-fPIC", "-o", _LIB_PATH, src])
    global _lib
    _lib = None
    return _LIB_PATH


def _load():
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            build()
        lib = ctypes.CDLL(_LIB_PATH)
        vp, i64, dbl, ci = ctypes.c_void_p, ctypes.c_int64, ctypes.c_double, ctypes.c_int
        lib.orc_contract_literal.restype = ci
        lib.orc_contract_literal.argtypes = [ci, vp, vp, ctypes.c_char_p, vp] * 3 + [dbl, dbl]
        lib.orc_scatter.restype = ci
        lib.orc_scatter.argtypes = [ci, vp, vp, vp]
        lib.orc_block_scatter.restype = ci
        lib.orc_block_scatter.argtypes = [vp, i64, i64, vp]
        lib.orc_contract_rows.restype = ci
        lib.orc_contract_rows.argtypes = [vp] * 10 + [i64, i64, i64, dbl, dbl, vp]
        lib.orc_matvec.restype = ci
        lib.orc_matvec.argtypes = [vp, vp, vp, i64, i64, vp, vp]
        lib.orc_num_threads.restype = ci
        lib.orc_num_threads.argtypes = []
        _lib = lib
    return _lib


def num_threads() -> int:
    """Threads the tiled oracle runs on."""
    return int(_load().orc_num_threads())


def _i64(a) -> np.ndarray:
    return np.ascontiguousarray(np.asarray(a, dtype=np.int64))


def _ptr(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data


# ----------------------------------------------------------------------------
# bundles, scatter vectors, matrix view
# ----------------------------------------------------------------------------

def classify(idxA: str, idxB: str, idxC: str) -> Tuple[List[str], List[str], List[str]]:
    """Free bundles I (A and C), J (B and C) and contracted bundle P (A and B)."""
    for s in (idxA, idxB, idxC):
        if len(set(s)) != len(s):
            raise ValueError("label repeated inside a tensor")
    for c in set(idxA + idxB + idxC):
        if (c in idxA) + (c in idxB) + (c in idxC) != 2:
            raise ValueError(f"label {c!r} must occur in exactly two tensors")
    I = [c for c in idxA if c in idxC]
    J = [c for c in idxB if c in idxC]
    P = [c for c in idxA if c in idxB]
    return I, J, P


def scatter_vector(lens: Sequence[int], strides: Sequence[int]) -> np.ndarray:
    """scat[i] = sum_k i_k * s_k where i = sum_k i_k * prod_{l<k} N_l (first index of the bundle fastest)."""
    lens_a, str_a = _i64(lens), _i64(strides)
    total = int(np.prod(lens_a, dtype=np.int64)) if len(lens_a) else 1
    out = np.zeros(total, dtype=np.int64)
    rc = _load().orc_scatter(len(lens_a), _ptr(lens_a), _ptr(str_a), _ptr(out))
    if rc != 0:
        raise RuntimeError(f"orc_scatter failed: {rc}")
    return out


def block_scatter(scat: np.ndarray, blk: int) -> np.ndarray:
    """Stride of each block of ``blk`` consecutive scatter entries, 0 where the block is not regularly strided."""
    scat = _i64(scat)
    out = np.zeros((len(scat) + blk - 1) // blk, dtype=np.int64)
    rc = _load().orc_block_scatter(_ptr(scat), len(scat), blk, _ptr(out))
    if rc != 0:
        raise RuntimeError(f"orc_block_scatter failed: {rc}")
    return out


def default_orders(A, B, C) -> Tuple[List[str], List[str], List[str]]:
    """Order inside each bundle: I and J by ascending stride in C, P by ascending stride in A."""
    I, J, P = classify(A.idx, B.idx, C.idx)
    sC = dict(zip(C.idx, C.strides))
    sA = dict(zip(A.idx, A.strides))
    return sorted(I, key=lambda c: sC[c]), sorted(J, key=lambda c: sC[c]), sorted(P, key=lambda c: sA[c])


def matrix_view(A, B, C, orders=None) -> Dict[str, np.ndarray]:
    """The six scatter vectors: I -> rscat_A, rscat_C; J -> cscat_B, cscat_C; P -> cscat_A, rscat_B."""
    I, J, P = orders if orders is not None else default_orders(A, B, C)
    cI, cJ, cP = classify(A.idx, B.idx, C.idx)
    if sorted(I) != sorted(cI) or sorted(J) != sorted(cJ) or sorted(P) != sorted(cP):
        raise ValueError("orders do not match the bundles")
    for c in set(A.idx + B.idx + C.idx):
        ls = [t.lens[t.idx.index(c)] for t in (A, B, C) if c in t.idx]
        if ls[0] != ls[1]:
            raise ValueError(f"label {c!r} has different lengths")

    def sv(T, bundle):
        return scatter_vector([T.lens[T.idx.index(c)] for c in bundle], [T.strides[T.idx.index(c)] for c in bundle])

    return {"rsA": sv(A, I), "csA": sv(A, P), "rsB": sv(B, P), "csB": sv(B, J), "rsC": sv(C, I), "csC": sv(C, J),
            "I": I, "J": J, "P": P}


# ----------------------------------------------------------------------------
# classical contraction
# ----------------------------------------------------------------------------

def contract_literal(A, B, C, alpha: float = 1.0, beta: float = 1.0) -> None:
    """C := alpha * sum_P A*B + beta*C, in place, by the literal loop nest (small sizes only)."""
    lib = _load()
    args = []
    keep = []
    for T in (A, B, C):
        L, S = _i64(T.lens), _i64(T.strides)
        keep += [L, S]
        if T.data.dtype != np.float64 or not T.data.flags["C_CONTIGUOUS"]:
            raise ValueError("tensor storage must be contiguous float64")
        args += [len(T.lens), _ptr(L), _ptr(S), T.idx.encode(), T.data.ctypes.data]
    rc = lib.orc_contract_literal(*args, float(alpha), float(beta))
    if rc != 0:
        raise ValueError(f"orc_contract_literal failed: {rc}")


def contract_rows(A, B, C, rows: Optional[np.ndarray], alpha: float = 1.0, beta: float = 1.0, orders=None, view=None) -> np.ndarray:
    """Reference values of the given rows of the matrix view of C (all rows if None): dense (nrows, n) array."""
    v = view if view is not None else matrix_view(A, B, C, orders)
    m, n, k = len(v["rsA"]), len(v["csB"]), len(v["csA"])
    rows_a = None if rows is None else _i64(rows)
    nrows = m if rows_a is None else len(rows_a)
    out = np.zeros((nrows, n), dtype=np.float64)
    rc = _load().orc_contract_rows(A.data.ctypes.data, B.data.ctypes.data, C.data.ctypes.data,
                                   _ptr(v["rsA"]), _ptr(v["csA"]), _ptr(v["rsB"]), _ptr(v["csB"]), _ptr(v["rsC"]), _ptr(v["csC"]),
                                   _ptr(rows_a), nrows, n, k, float(alpha), float(beta), _ptr(out))
    if rc != 0:
        raise RuntimeError(f"orc_contract_rows failed: {rc}")
    return out


def contract_matrix(A, B, C, alpha: float = 1.0, beta: float = 1.0, orders=None) -> None:
    """C := alpha*A*B + beta*C in place through the matrix view (tiled, OpenMP)."""
    v = matrix_view(A, B, C, orders)
    out = contract_rows(A, B, C, None, alpha, beta, view=v)
    if out.size:
        C.data[v["rsC"][:, None] + v["csC"][None, :]] = out


def gather_matrix(T, rs: np.ndarray, cs: np.ndarray) -> np.ndarray:
    """Dense copy of the matrix view: M[i, j] = T[rs[i] + cs[j]]."""
    return T.data[rs[:, None] + cs[None, :]]


# ----------------------------------------------------------------------------
# Strassen
# ----------------------------------------------------------------------------

# Quadrants X0 X1 / X2 X3.  Row r: M_r = (sum_q U[r,q] A_q)(sum_q V[r,q] B_q);  C_q += W[r,q] M_r.
STRASSEN_U = np.array([[1, 0, 0, 1], [0, 0, 1, 1], [1, 0, 0, 0], [0, 0, 0, 1], [1, 1, 0, 0], [-1, 0, 1, 0], [0, 1, 0, -1]])
STRASSEN_V = np.array([[1, 0, 0, 1], [1, 0, 0, 0], [0, 1, 0, -1], [-1, 0, 1, 0], [0, 0, 0, 1], [1, 1, 0, 0], [0, 0, 1, 1]])
STRASSEN_W = np.array([[1, 0, 0, 1], [0, 0, 1, -1], [0, 1, 0, 1], [1, 0, 1, 0], [-1, 1, 0, 0], [0, 0, 0, 1], [1, 0, 0, 0]])


def _block_of(quads: Sequence[int]) -> Tuple[int, int]:
    """(block row, block col) in the 2^L x 2^L grid of a path of quadrant numbers, outermost first."""
    r = c = 0
    for q in quads:
        r = 2 * r + (q >> 1)
        c = 2 * c + (q & 1)
    return r, c


def strassen_tables(level: int):
    """Coefficients of the 7^L products over the 2^L x 2^L block grid.

    Returns (U, V, W), each of shape (7^L, 2^L, 2^L): product r uses sum_{bi,bk} U[r,bi,bk] A[bi,bk],
    sum V[r,bk,bj] B[bk,bj] and updates C[bi,bj] += W[r,bi,bj] * M_r.
    """
    g = 1 << level
    out = []
    for T in (STRASSEN_U, STRASSEN_V, STRASSEN_W):
        tab = np.zeros((7 ** level, g, g), dtype=np.int64)
        for r in range(7 ** level):
            digits = [(r // 7 ** (level - 1 - d)) % 7 for d in range(level)]
            for qcode in range(4 ** level):
                quads = [(qcode // 4 ** (level - 1 - d)) % 4 for d in range(level)]
                coef = 1
                for d in range(level):
                    coef *= int(T[digits[d], quads[d]])
                if coef:
                    br, bc = _block_of(quads)
                    tab[r, br, bc] = coef
        out.append(tab)
    return tuple(out)


def strassen_recursive(A: np.ndarray, B: np.ndarray, level: int) -> np.ndarray:
    """A @ B on dense matrices by L levels of Strassen with temporaries, dynamic peeling for odd sizes."""
    m, k = A.shape
    n = B.shape[1]
    if level == 0 or min(m, n, k) < 2:
        return A @ B
    m2, n2, k2 = m - m % 2, n - n % 2, k - k % 2
    mh, nh, kh = m2 // 2, n2 // 2, k2 // 2
    Aq = [A[:mh, :kh], A[:mh, kh:k2], A[mh:m2, :kh], A[mh:m2, kh:k2]]
    Bq = [B[:kh, :nh], B[:kh, nh:n2], B[kh:k2, :nh], B[kh:k2, nh:n2]]
    C = np.zeros((m, n), dtype=np.float64)
    Cq = [C[:mh, :nh], C[:mh, nh:n2], C[mh:m2, :nh], C[mh:m2, nh:n2]]
    for r in range(7):
        X = np.zeros((mh, kh))
        Y = np.zeros((kh, nh))
        for q in range(4):
            if STRASSEN_U[r, q]:
                X = X + STRASSEN_U[r, q] * Aq[q]
            if STRASSEN_V[r, q]:
                Y = Y + STRASSEN_V[r, q] * Bq[q]
        M = strassen_recursive(X, Y, level - 1)
        for q in range(4):
            if STRASSEN_W[r, q]:
                Cq[q] += STRASSEN_W[r, q] * M
    # peeled fringes, classical
    if k2 < k:
        C[:m2, :n2] += A[:m2, k2:] @ B[k2:, :n2]
    if n2 < n:
        C[:m2, n2:] = A[:m2, :] @ B[:, n2:]
    if m2 < m:
        C[m2:, :] = A[m2:, :] @ B
    return C


def strassen_flat(A: np.ndarray, B: np.ndarray, level: int) -> np.ndarray:
    """A @ B by the flattened schedule of 7^L products; sizes are padded with zeros to a multiple of 2^L."""
    m, k = A.shape
    n = B.shape[1]
    g = 1 << level
    mb, nb, kb = -(-m // g), -(-n // g), -(-k // g)
    Ap = np.zeros((mb * g, kb * g))
    Bp = np.zeros((kb * g, nb * g))
    Ap[:m, :k] = A
    Bp[:k, :n] = B
    Cp = np.zeros((mb * g, nb * g))
    U, V, W = strassen_tables(level)
    for r in range(7 ** level):
        X = np.zeros((mb, kb))
        Y = np.zeros((kb, nb))
        for bi in range(g):
            for bk in range(g):
                if U[r, bi, bk]:
                    X = X + U[r, bi, bk] * Ap[bi * mb:(bi + 1) * mb, bk * kb:(bk + 1) * kb]
        for bk in range(g):
            for bj in range(g):
                if V[r, bk, bj]:
                    Y = Y + V[r, bk, bj] * Bp[bk * kb:(bk + 1) * kb, bj * nb:(bj + 1) * nb]
        M = X @ Y
        for bi in range(g):
            for bj in range(g):
                if W[r, bi, bj]:
                    Cp[bi * mb:(bi + 1) * mb, bj * nb:(bj + 1) * nb] += W[r, bi, bj] * M
    return Cp[:m, :n]


def contract_strassen(A, B, C, level: int, alpha: float = 1.0, beta: float = 1.0, orders=None, flat: bool = False) -> None:
    """C := alpha*A*B + beta*C in place, the product evaluated by L-level Strassen on the matrix view."""
    v = matrix_view(A, B, C, orders)
    Am = gather_matrix(A, v["rsA"], v["csA"])
    Bm = gather_matrix(B, v["rsB"], v["csB"])
    M = strassen_flat(Am, Bm, level) if flat else strassen_recursive(Am, Bm, level)
    loc = v["rsC"][:, None] + v["csC"][None, :]
    if M.size:
        C.data[loc] = alpha * M if beta == 0.0 else alpha * M + beta * C.data[loc]


# ----------------------------------------------------------------------------
# error measures
# ----------------------------------------------------------------------------

def fro(x: np.ndarray) -> float:
    """Frobenius norm accumulated in extended precision over chunks."""
    x = np.asarray(x, dtype=np.float64).ravel()
    tot = np.longdouble(0)
    for s in range(0, x.size, 1 << 22):
        c = x[s:s + (1 << 22)].astype(np.longdouble)
        tot += np.dot(c, c)
    return float(np.sqrt(tot))


def error_metric(Cval: np.ndarray, Cref: np.ndarray, normA: float, normB: float) -> float:
    """||C - C_ref||_F / (||A||_F * ||B||_F)."""
    d = np.asarray(Cval, dtype=np.float64) - np.asarray(Cref, dtype=np.float64)
    den = normA * normB
    num = fro(d)
    if den == 0.0:
        return 0.0 if num == 0.0 else float("inf")
    return num / den


def tensor_norm(T) -> float:
    return fro(T.view())


def _matvec(T, rs, cs, x) -> np.ndarray:
    """y = M x for the matrix view M[i, j] = T[rs[i] + cs[j]]."""
    lib = _load()
    x = np.ascontiguousarray(x, dtype=np.float64)
    m, n = len(rs), len(cs)
    y = np.zeros(m, dtype=np.float64)
    lib.orc_matvec(T.data.ctypes.data, _ptr(rs), _ptr(cs), m, n, x.ctypes.data, y.ctypes.data)
    return y


def freivalds(Cnew, A, B, C0, alpha: float, beta: float, trials: int = 8, seed: int = 0, orders=None, view=None) -> float:
    """Estimate ||C_new - (alpha*A*B + beta*C0)||_F from ``trials`` random +-1 vectors x over the J bundle:
    E ||(C_new - C_ref) x||^2 = ||C_new - C_ref||_F^2.  C0 may be None when beta == 0."""
    v = view if view is not None else matrix_view(A, B, Cnew, orders)
    rng = np.random.default_rng(seed)
    n = len(v["csB"])
    acc = 0.0
    for _ in range(trials):
        x = rng.integers(0, 2, size=n).astype(np.float64) * 2.0 - 1.0
        r = _matvec(Cnew, v["rsC"], v["csC"], x)
        bx = _matvec(B, v["rsB"], v["csB"], x)
        r -= alpha * _matvec(A, v["rsA"], v["csA"], bx)
        if beta != 0.0:
            r -= beta * _matvec(C0, v["rsC"], v["csC"], x)
        acc += float(np.dot(r, r))
    return float(np.sqrt(acc / trials))
