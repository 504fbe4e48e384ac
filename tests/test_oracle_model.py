"""Pins of the performance-model oracle (oracle/model.py) against what the paper and the mathematics fix.

* the coefficient table of Sec. 5 against counts derived from the Strassen tables (pinned by Brent's equations in
  test_oracle_strassen.py): products, additions per operand, destination updates, and the traffic coefficients that
  are such counts; the three two-level entries that are not (194, 194, 293) are asserted as printed;
* level 0 against the closed form of the classical column of the middle table;
* the arithmetic term's 7/8 ratio per level;
* the shape claims of Sec. 5 / Sec. 6 that the authors read off the model, evaluated with their machine's parameters
  (Sec. 6: 28.32 GFLOPS, 59.7 GB/s, m_C = 96, n_C = 4096, k_C = 256).
"""
import math

import numpy as np
import pytest

import oracle
from oracle import model as M


def _counts(level):
    U, V, W = oracle.strassen_tables(level)
    U, V, W = np.array(U), np.array(V), np.array(W)
    nnz = lambda T: int(np.count_nonzero(T))
    adds = lambda T: int(sum(np.count_nonzero(r) - 1 for r in T))
    return len(U), nnz(U), nnz(V), nnz(W), adds(U), adds(V)


@pytest.mark.parametrize("level", [1, 2])
def test_coefficients_follow_from_the_strassen_tables(level):
    R, nU, nV, nW, aU, aV = _counts(level)
    for v in M.VARIANTS:
        w = M.coefficients(level, v)
        assert w["a_mul"] == R == 7 ** level
        assert (w["a_A"], w["a_B"], w["a_C"]) == (aU, aV, nW)  # 5, 5, 12 and 95, 95, 144
    abc, ab, naive = (M.coefficients(level, v) for v in ("abc", "ab", "naive"))
    assert abc["m_Cx"] == nW and ab["m_Cx"] == R and naive["m_Cx"] == R  # every product updates its destinations / its M
    assert naive["m_Ax"] == R and naive["m_Bx"] == R                    # one dense temporary per product and operand
    assert ab["m_C+"] == naive["m_C+"] == 3 * nW and abc["m_C+"] == 0     # M read, C read and written, per destination
    if level == 1:
        assert abc["m_Ax"] == ab["m_Ax"] == nU == 12 and abc["m_Bx"] == ab["m_Bx"] == nV == 12
        assert naive["m_A+"] == nU + R == 19 and naive["m_B+"] == nV + R == 19  # blocks read + temporaries written
    else:
        # as printed; the Kronecker counts would give 144 and 144 + 49 = 193
        assert abc["m_Ax"] == ab["m_Ax"] == abc["m_Bx"] == ab["m_Bx"] == 194 and nU == nV == 144
        assert naive["m_A+"] == naive["m_B+"] == 293


def test_level0_closed_form():
    p = M.PaperParams(28.32, 59.7, lam=0.8)
    for m, n, k in ((500, 700, 900), (4096, 5000, 256), (96, 4097, 257)):
        want = p.tau_a * 2 * m * n * k + p.tau_b * (m * k * math.ceil(n / p.n_c) + n * k + 2 * p.lam * m * n * math.ceil(k / p.k_c))
        for v in M.VARIANTS:
            assert M.paper_time(m, n, k, 0, v, p) == pytest.approx(want, rel=1e-14)
    assert M.effective_gflops(10, 20, 30, 2.0) == pytest.approx(2 * 10 * 20 * 30 / 2.0 * 1e-9)
    assert p.tau_a == pytest.approx(1 / (0.95 * 28.32e9)) and p.tau_b == pytest.approx(8 / (0.7 * 59.7e9))


def test_multiplication_term_shrinks_by_seven_eighths_per_level():
    p = M.PaperParams(100.0, 50.0)
    t0 = M.paper_terms(4096, 2048, 1024, 0, "abc", p)["a_mul"]
    for level in (1, 2):
        for v in M.VARIANTS:
            assert M.paper_terms(4096, 2048, 1024, level, v, p)["a_mul"] == pytest.approx(t0 * (7 / 8) ** level, rel=1e-14)


@pytest.mark.parametrize("lam", [0.55, 0.75, 1.0])
def test_shape_claims_read_off_the_model(lam):
    p = M.PaperParams(28.32, 59.7, lam=lam)
    gf = lambda m, n, k, L, v: M.effective_gflops(m, n, k, M.paper_time(m, n, k, L, v, p))
    # square: one-level ABC overtakes the classical routine at about 2 k_C ~ 500; Naive is the slowest one-level variant there
    assert gf(512, 512, 512, 1, "abc") > gf(512, 512, 512, 0, "abc")
    assert gf(512, 512, 512, 1, "abc") > gf(512, 512, 512, 1, "ab") > gf(512, 512, 512, 1, "naive")
    # rank-k (m = n ~ 14400): small k favours ABC, large k favours AB, and two-level AB ends up on top
    m = n = 14400
    assert gf(m, n, 512, 1, "abc") > gf(m, n, 512, 1, "ab") and gf(m, n, 512, 2, "abc") > gf(m, n, 512, 2, "ab")
    assert gf(m, n, 8192, 1, "ab") > gf(m, n, 8192, 1, "abc") and gf(m, n, 8192, 2, "ab") > gf(m, n, 8192, 2, "abc")
    best = max(((L, v) for L in (0, 1, 2) for v in M.VARIANTS), key=lambda lv: gf(m, n, 8192, *lv))
    assert best == (2, "ab")
    # k = 2^L k_C: ABC is the best variant of its level
    for L in (1, 2):
        k = 2 ** L * p.k_c
        assert gf(m, n, k, L, "abc") > max(gf(m, n, k, L, "ab"), gf(m, n, k, L, "naive"))
