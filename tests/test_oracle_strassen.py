"""Pins for the Strassen part of the CPU oracle: Brent's equations, the operation counts the paper prints,
exact integer arithmetic, and agreement with the classical oracle and with numpy's matmul."""
import random

import numpy as np
import pytest

import oracle
import workloads
from oracle import STRASSEN_U, STRASSEN_V, STRASSEN_W


def _brent_ok(U, V, W, g):
    """sum_r U[r,(i,p)] V[r,(p',j)] W[r,(i',j')] == [p==p'][i==i'][j==j'] for all block indices."""
    R = U.shape[0]
    T = np.einsum("rab,rcd,ref->abcdef", U, V, W)
    want = np.zeros((g,) * 6, dtype=np.int64)
    for i in range(g):
        for p in range(g):
            for j in range(g):
                want[i, p, p, j, i, j] = 1
    return np.array_equal(T, want)


def test_one_level_table_satisfies_brent_equations():
    U, V, W = oracle.strassen_tables(1)
    assert U.shape == (7, 2, 2)
    assert _brent_ok(U, V, W, 2)
    # flat (quadrant-numbered) tables are the same object in another shape
    assert np.array_equal(U.reshape(7, 4), STRASSEN_U)
    assert np.array_equal(V.reshape(7, 4), STRASSEN_V)
    assert np.array_equal(W.reshape(7, 4), STRASSEN_W)


def test_brent_check_is_sensitive_to_single_mistakes():
    U, V, W = oracle.strassen_tables(1)
    for T in (U, V, W):
        for r in range(7):
            for a in range(2):
                for b in range(2):
                    for newval in (-1, 0, 1):
                        if newval == T[r, a, b]:
                            continue
                        old = T[r, a, b]
                        T[r, a, b] = newval
                        assert not _brent_ok(U, V, W, 2)
                        T[r, a, b] = old
    assert _brent_ok(U, V, W, 2)


def test_operation_counts_match_the_performance_model_table():
    """Non-zeros 12/12/12 => 5, 5 additions and 12 C updates (one level); 144 each => 95, 95, 144 (two levels); 7 and 49 products."""
    U, V, W = oracle.strassen_tables(1)
    assert (np.count_nonzero(U), np.count_nonzero(V), np.count_nonzero(W)) == (12, 12, 12)
    assert np.count_nonzero(U) - 7 == 5 and np.count_nonzero(V) - 7 == 5
    U2, V2, W2 = oracle.strassen_tables(2)
    assert U2.shape == (49, 4, 4)
    assert (np.count_nonzero(U2), np.count_nonzero(V2), np.count_nonzero(W2)) == (144, 144, 144)
    assert np.count_nonzero(U2) - 49 == 95 and np.count_nonzero(V2) - 49 == 95
    # each product touches 1, 2 or 4 blocks per operand
    for T in (U2, V2, W2):
        assert set(np.count_nonzero(T.reshape(49, -1), axis=1)) <= {1, 2, 4}


def test_two_level_tables_satisfy_brent_equations():
    U, V, W = oracle.strassen_tables(2)
    assert _brent_ok(U, V, W, 4)


def test_seven_products_written_out():
    """The seven products of Sec. 2.2 typed out product by product on random quadrants reproduces the blocked product."""
    rng = np.random.default_rng(0)
    A = [rng.integers(-3, 4, (3, 4)).astype(float) for _ in range(4)]
    B = [rng.integers(-3, 4, (4, 5)).astype(float) for _ in range(4)]
    M0 = (A[0] + A[3]) @ (B[0] + B[3])
    M1 = (A[2] + A[3]) @ B[0]
    M2 = A[0] @ (B[1] - B[3])
    M3 = A[3] @ (B[2] - B[0])
    M4 = (A[0] + A[1]) @ B[3]
    M5 = (A[2] - A[0]) @ (B[0] + B[1])
    M6 = (A[1] - A[3]) @ (B[2] + B[3])
    C0, C1, C2, C3 = M0 + M3 - M4 + M6, M2 + M4, M1 + M3, M0 - M1 + M2 + M5
    Afull = np.block([[A[0], A[1]], [A[2], A[3]]])
    Bfull = np.block([[B[0], B[1]], [B[2], B[3]]])
    want = Afull @ Bfull
    assert np.array_equal(np.block([[C0, C1], [C2, C3]]), want)
    assert np.array_equal(oracle.strassen_recursive(Afull, Bfull, 1), want)
    assert np.array_equal(oracle.strassen_flat(Afull, Bfull, 1), want)


@pytest.mark.parametrize("level", [1, 2])
def test_exact_on_small_integers_all_shapes(level):
    rng = np.random.default_rng(level)
    shapes = [(8, 8, 8), (7, 5, 9), (1, 1, 1), (2, 3, 1), (13, 16, 11), (4, 1, 4), (33, 18, 27), (3, 3, 3)]
    for (m, n, k) in shapes:
        A = rng.integers(-4, 5, (m, k)).astype(float)
        B = rng.integers(-4, 5, (k, n)).astype(float)
        want = A @ B
        assert np.array_equal(oracle.strassen_recursive(A, B, level), want)
        assert np.array_equal(oracle.strassen_flat(A, B, level), want)


@pytest.mark.parametrize("level", [1, 2])
def test_tensor_strassen_matches_classical_oracle(level):
    rng = random.Random(40 + level)
    from test_oracle_pins import _random_case

    for trial in range(12):
        A, B, C = _random_case(rng, maxlen=6)
        ref = C.copy()
        oracle.contract_literal(A, B, ref, 0.75, -1.25)
        nA, nB = oracle.tensor_norm(A), oracle.tensor_norm(B)
        for flat in (False, True):
            got = C.copy()
            oracle.contract_strassen(A, B, got, level, 0.75, -1.25, flat=flat)
            err = oracle.error_metric(got.view(), ref.view(), nA, nB)
            assert err <= 1e-15, (trial, flat, err)
    # integers: exact, including beta = 0 on NaN-filled C
    A, B, C = _random_case(rng, maxlen=6, kind="smallint")
    ref = C.copy()
    oracle.contract_literal(A, B, ref, 2.0, 0.0)
    C.data[:] = np.nan
    oracle.contract_strassen(A, B, C, level, 2.0, 0.0)
    assert np.array_equal(C.view(), ref.view())


def test_strassen_error_stays_within_a_small_factor_of_classical():
    """Normwise error of 1- and 2-level Strassen on a 4-D contraction, relative to ||A|| ||B||, is far below 1e-13."""
    cfg = workloads.scaled(workloads.configs()["cfg1"], {x: 6 for x in "abcdef"})
    A, B, C0 = cfg.tensors()
    ref = C0.copy()
    oracle.contract_matrix(A, B, ref, 1.0, 0.0)
    nA, nB = oracle.tensor_norm(A), oracle.tensor_norm(B)
    want = np.einsum("aebf,dfce->abcd", A.view(), B.view())
    assert oracle.error_metric(ref.view(), want, nA, nB) < 1e-16
    for level in (1, 2):
        got = C0.copy()
        oracle.contract_strassen(A, B, got, level, 1.0, 0.0)
        assert oracle.error_metric(got.view(), ref.view(), nA, nB) < 5e-16
