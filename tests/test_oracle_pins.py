"""Pins for the classical CPU oracle: every check compares it with something that is not the oracle
(the paper's printed example, numpy's einsum/matmul, pure-Python brute force, closed forms, invariants)."""
import itertools
import os
import random

import numpy as np
import pytest

import oracle
import workloads
from workloads import Tensor, col_major, from_dense, row_major, strides_for_order

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _parse_golden():
    d = {}
    with open(os.path.join(GOLDEN, "paper_layout_example.txt")) as f:
        for line in f:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            k, *rest = line.split()
            d[k] = rest
    return d


# --------------------------------------------------------------------------------------
# layout: the worked example of Sec. 2.3 / Fig. 2
# --------------------------------------------------------------------------------------

def test_paper_layout_example():
    g = _parse_golden()
    L = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in g["lengths"]}
    sC = {kv.split("=")[0]: int(kv.split("=")[1]) for kv in g["strides_C"]}
    lensC = [L[c] for c in "abc"]
    assert dict(zip("abc", col_major(lensC))) == sC  # generalized column-major strides 1, 4, 32
    A = Tensor("dca", tuple(L[c] for c in "dca"), col_major([L[c] for c in "dca"]), np.zeros(64))
    B = Tensor("db", tuple(L[c] for c in "db"), col_major([L[c] for c in "db"]), np.zeros(64))
    C = Tensor("abc", tuple(lensC), col_major(lensC), np.zeros(64))
    I, J, P = oracle.classify(A.idx, B.idx, C.idx)
    assert sorted(I) == ["a", "c"] and J == ["b"] and P == ["d"]
    v = oracle.matrix_view(A, B, C, orders=(["a", "c"], ["b"], ["d"]))
    i, val = map(int, g["rscat_C_entry"])
    assert v["rsC"][i] == val
    j, val = map(int, g["cscat_C_entry"])
    assert v["csC"][j] == val
    # LOC(C_{2,3,1}) = LOC(C_{6,3}) = 34 + 12
    assert 2 * sC["a"] + 3 * sC["b"] + 1 * sC["c"] == int(g["loc_C_2_3_1"][0]) == v["rsC"][6] + v["csC"][3]
    # rscat_C;i = a + 32c with i = a + 4c
    for a in range(4):
        for c in range(2):
            assert v["rsC"][a + 4 * c] == a + 32 * c
    blk = int(g["block"][0])
    assert list(oracle.block_scatter(v["rsC"], blk)) == list(map(int, g["rbs_C"]))
    assert list(oracle.block_scatter(v["csC"], blk)) == list(map(int, g["cbs_C"]))


def test_scatter_vector_is_the_stride_layout():
    """rscat_i + cscat_j equals the general-stride location of the element (the scatter-matrix location formula against the general-stride one, Sec. 2.3)."""
    rng = random.Random(5)
    for _ in range(30):
        nd = rng.randint(1, 5)
        lens = [rng.randint(1, 4) for _ in range(nd)]
        order = list(range(nd))
        rng.shuffle(order)
        strides = strides_for_order(lens, order, pad=rng.randint(0, 3))
        split = rng.randint(0, nd)
        dims = list(range(nd))
        rng.shuffle(dims)
        rdims, cdims = dims[:split], dims[split:]
        rs = oracle.scatter_vector([lens[d] for d in rdims], [strides[d] for d in rdims])
        cs = oracle.scatter_vector([lens[d] for d in cdims], [strides[d] for d in cdims])
        for multi in itertools.product(*[range(n) for n in lens]):
            loc = sum(t * s for t, s in zip(multi, strides))
            i = 0
            w = 1
            for d in rdims:
                i += multi[d] * w
                w *= lens[d]
            j = 0
            w = 1
            for d in cdims:
                j += multi[d] * w
                w *= lens[d]
            assert rs[i] + cs[j] == loc


def test_block_scatter_rules():
    s = np.array([0, 1, 2, 3, 32, 33, 34, 35, 64, 70])
    assert list(oracle.block_scatter(s, 4)) == [1, 1, 6]
    assert list(oracle.block_scatter(s, 8)) == [0, 6]
    assert list(oracle.block_scatter(s, 3)) == [1, 0, 0, 1]  # last block has one entry -> regular by convention
    assert list(oracle.block_scatter(np.array([5, 5, 5, 5]), 2)) == [0, 0]  # zero stride is not a regular stride
    assert list(oracle.block_scatter(np.array([], dtype=np.int64), 4)) == []


# --------------------------------------------------------------------------------------
# the contraction itself
# --------------------------------------------------------------------------------------

def _random_case(rng, maxlen=5, kind="uniform", max_bundle=2):
    labels = list("abcdefghijkl")
    rng.shuffle(labels)
    nI, nJ, nP = rng.randint(0, max_bundle), rng.randint(0, max_bundle), rng.randint(0, max_bundle)
    I, J, P = labels[:nI], labels[nI:nI + nJ], labels[nI + nJ:nI + nJ + nP]
    lengths = {c: rng.randint(1, maxlen) for c in I + J + P}
    idxA, idxB, idxC = I + P, P + J, I + J
    for s in (idxA, idxB, idxC):
        rng.shuffle(s)
    tens = []
    for tid, idx in enumerate((idxA, idxB, idxC)):
        lens = [lengths[c] for c in idx]
        order = list(range(len(idx)))
        rng.shuffle(order)
        st = strides_for_order(lens, order, pad=rng.randint(0, 2))
        tens.append(workloads.make_tensor("".join(idx), lengths, rng.randint(0, 10 ** 6), tid, kind, st))
    return tens


def _einsum(A, B, C, alpha, beta):
    spec = f"{A.idx},{B.idx}->{C.idx}"
    return alpha * np.einsum(spec, A.view(), B.view()) + beta * C.view()


def test_literal_matches_einsum_on_random_contractions():
    rng = random.Random(11)
    for _ in range(120):
        A, B, C = _random_case(rng)
        alpha, beta = rng.choice([1.0, -0.5, 2.25]), rng.choice([0.0, 1.0, -1.5])
        want = _einsum(A, B, C, alpha, beta)
        oracle.contract_literal(A, B, C, alpha, beta)
        scale = max(1.0, np.abs(want).max()) if want.size else 1.0
        assert np.abs(C.view() - want).max() <= 1e-13 * scale if want.size else True


def test_literal_matches_pure_python_brute_force():
    """C_abc += A_dca * B_db (the paper's example contraction) by plain Python loops."""
    L = {"a": 3, "b": 4, "c": 2, "d": 5}
    A = workloads.make_tensor("dca", L, 3, 0, "smallint")
    B = workloads.make_tensor("db", L, 3, 1, "smallint")
    C = workloads.make_tensor("abc", L, 3, 2, "smallint")
    want = C.view().copy()
    Av, Bv = A.view(), B.view()
    for a in range(3):
        for b in range(4):
            for c in range(2):
                s = 0.0
                for d in range(5):
                    s += Av[d, c, a] * Bv[d, b]
                want[a, b, c] = 2.0 * s + 3.0 * want[a, b, c]
    oracle.contract_literal(A, B, C, 2.0, 3.0)
    assert np.array_equal(C.view(), want)  # small integers: exact


def test_matrix_special_case_is_textbook_gemm():
    rng = np.random.default_rng(2)
    for (m, n, k) in [(7, 5, 9), (1, 1, 1), (16, 3, 2), (33, 65, 17)]:
        a, b, c = rng.standard_normal((m, k)), rng.standard_normal((k, n)), rng.standard_normal((m, n))
        for sa, sb, sc in [(col_major, col_major, col_major), (row_major, col_major, row_major)]:
            A, B, C = from_dense("ik", a, sa(a.shape)), from_dense("kj", b, sb(b.shape)), from_dense("ij", c, sc(c.shape))
            C2 = C.copy()
            oracle.contract_literal(A, B, C, 1.5, -0.5)
            oracle.contract_matrix(A, B, C2, 1.5, -0.5)
            want = 1.5 * (a @ b) - 0.5 * c
            assert np.allclose(C.view(), want, rtol=0, atol=1e-13 * k)
            assert np.allclose(C2.view(), want, rtol=0, atol=1e-13 * k)


def test_tiled_matrix_form_equals_literal_bit_for_bit():
    """Same summation order over P (first contracted label of A fastest) => identical floating-point results."""
    rng = random.Random(23)
    for _ in range(25):
        A, B, C = _random_case(rng, maxlen=7)
        I, J, P = oracle.classify(A.idx, B.idx, C.idx)  # P in A's order, as the literal loop nest sums
        C2 = C.copy()
        oracle.contract_literal(A, B, C, 1.25, 0.75)
        oracle.contract_matrix(A, B, C2, 1.25, 0.75, orders=(I, J, P))
        assert np.array_equal(C.data, C2.data)
    # a case larger than the tile sizes in every direction (tiles: 4 x 8 register tile, 64 columns, 256 rows, 1024 deep)
    L = {"i": 300, "j": 70, "k": 1100}
    A = workloads.make_tensor("ik", L, 9, 0)
    B = workloads.make_tensor("kj", L, 9, 1)
    C = workloads.make_tensor("ij", L, 9, 2)
    C2 = C.copy()
    oracle.contract_literal(A, B, C, 1.0, 1.0)
    oracle.contract_matrix(A, B, C2, 1.0, 1.0)
    assert np.array_equal(C.data, C2.data)
    want = A.view() @ B.view() + workloads.make_tensor("ij", L, 9, 2).view()
    assert np.abs(C.view() - want).max() < 1e-11


def test_contract_rows_is_a_row_subset():
    L = {"a": 6, "b": 5, "c": 4, "d": 3, "e": 7}
    A = workloads.make_tensor("dae", L, 1, 0)
    B = workloads.make_tensor("ebd", L, 1, 1)
    C = workloads.make_tensor("ab", L, 1, 2)
    v = oracle.matrix_view(A, B, C)
    full = oracle.contract_rows(A, B, C, None, 0.5, 2.0, view=v)
    rows = np.array([5, 0, 3, 3])
    part = oracle.contract_rows(A, B, C, rows, 0.5, 2.0, view=v)
    assert np.array_equal(part, full[rows])
    want = 0.5 * np.einsum("dae,ebd->ab", A.view(), B.view()) + 2.0 * C.view()
    assert v["I"] == ["a"] and v["J"] == ["b"]  # so the (m, n) result is indexed [a, b]
    assert np.allclose(full, want, atol=1e-13)


def test_linearity_in_alpha_and_beta():
    rng = random.Random(3)
    A, B, C0 = _random_case(rng, maxlen=6)

    def run(alpha, beta):
        C = C0.copy()
        oracle.contract_literal(A, B, C, alpha, beta)
        return C.view().copy()

    ab = run(1.0, 0.0)
    assert np.allclose(run(2.5, 0.0), 2.5 * ab, rtol=1e-14, atol=1e-14)
    assert np.allclose(run(0.75, 0.0) + run(0.5, 0.0), run(1.25, 0.0), rtol=1e-13, atol=1e-13)
    assert np.allclose(run(1.0, -2.0), ab - 2.0 * C0.view(), rtol=1e-13, atol=1e-13)
    assert np.allclose(run(0.0, 3.0), 3.0 * C0.view(), rtol=1e-15, atol=0)


def test_beta_zero_does_not_read_C():
    rng = random.Random(4)
    A, B, C = _random_case(rng, maxlen=4)
    C.data[:] = np.nan
    C2 = C.copy()
    oracle.contract_literal(A, B, C, 1.0, 0.0)
    oracle.contract_matrix(A, B, C2, 1.0, 0.0)
    assert np.all(np.isfinite(C.view()))
    assert np.all(np.isfinite(C2.view()))


def test_invariance_under_relabelling_and_storage_permutation():
    rng = random.Random(8)
    for _ in range(10):
        A, B, C = _random_case(rng, maxlen=5)
        ref = C.copy()
        oracle.contract_literal(A, B, ref, 1.0, 1.0)
        # consistent relabelling: identical storage afterwards
        labels = sorted(set(A.idx + B.idx + C.idx))
        new = list("mnopqrstuvwx")[:len(labels)]
        rng.shuffle(new)
        mp = dict(zip(labels, new))
        C2 = C.copy().relabel(mp)
        oracle.contract_literal(A.relabel(mp), B.relabel(mp), C2, 1.0, 1.0)
        assert np.array_equal(C2.data, ref.data)
        # permute the dimensions of every tensor and re-store them with new strides: same logical result
        out = []
        for T in (A, B, C):
            perm = list(range(len(T.idx)))
            rng.shuffle(perm)
            dense = np.transpose(T.view(), perm) if perm else T.view()
            order = list(range(len(perm)))
            rng.shuffle(order)
            st = strides_for_order(dense.shape, order, pad=rng.randint(0, 2))
            out.append(from_dense("".join(T.idx[p] for p in perm), np.array(dense), st))
        A3, B3, C3 = out
        oracle.contract_literal(A3, B3, C3, 1.0, 1.0)
        inv = [C3.idx.index(c) for c in C.idx]
        got = np.transpose(C3.view(), inv) if inv else C3.view()
        assert np.allclose(got, ref.view(), rtol=1e-13, atol=1e-13)


def test_flop_count_closed_form():
    cfgs = workloads.configs()
    assert cfgs["cfg1"].mnk() == (256, 256, 256)
    assert cfgs["cfg3"].mnk() == (36864, 2304, 36864)
    assert cfgs["cfg4a"].mnk() == (9216, 96, 4096)
    assert cfgs["cfg4b"].mnk() == (16384, 16384, 256)
    assert cfgs["cfg5"].mnk() == (13824, 13824, 9216)
    assert cfgs["cfg5"].flops() == 2.0 * 13824 * 13824 * 9216


def test_classical_rounding_error_bound():
    """|C_hat - C| <= k u |A||B| elementwise (textbook bound), checked against exact rational arithmetic on a small case."""
    from fractions import Fraction

    L = {"i": 6, "j": 5, "k": 40}
    A = workloads.make_tensor("ik", L, 77, 0)
    B = workloads.make_tensor("kj", L, 77, 1)
    C = from_dense("ij", np.zeros((6, 5)))
    oracle.contract_literal(A, B, C, 1.0, 0.0)
    Av, Bv = A.view(), B.view()
    u = 2.0 ** -53
    for i in range(6):
        for j in range(5):
            exact = sum(Fraction(Av[i, p]) * Fraction(Bv[p, j]) for p in range(40))
            bound = 40 * u * float(sum(abs(Fraction(Av[i, p]) * Fraction(Bv[p, j])) for p in range(40)))
            assert abs(float(Fraction(C.view()[i, j]) - exact)) <= bound


def test_error_metric_and_freivalds_detect_a_planted_error():
    L = {"a": 12, "b": 9, "c": 10, "d": 8, "e": 6}
    A = workloads.make_tensor("adbe", L, 5, 0)
    B = workloads.make_tensor("edc", L, 5, 1)
    C0 = workloads.make_tensor("cab", L, 5, 2)
    C = C0.copy()
    oracle.contract_literal(A, B, C, 1.5, 0.5)
    nA, nB = oracle.tensor_norm(A), oracle.tensor_norm(B)
    assert oracle.error_metric(C.view(), C.view(), nA, nB) == 0.0
    est0 = oracle.freivalds(C, A, B, C0, 1.5, 0.5, trials=8, seed=1)
    assert est0 / (nA * nB) < 1e-15
    bad = C.copy()
    bad.view()[3, 7, 2] += 0.25
    bad.view()[1, 1, 1] -= 0.5
    planted = np.sqrt(0.25 ** 2 + 0.5 ** 2)
    assert abs(oracle.error_metric(bad.view(), C.view(), nA, nB) * nA * nB - planted) < 1e-12
    est = oracle.freivalds(bad, A, B, C0, 1.5, 0.5, trials=8, seed=1)
    assert abs(est - planted) < 1e-9  # errors in distinct rows: every +-1 vector sees them exactly


def test_literal_rejects_malformed_label_sets():
    z = np.zeros(16)
    mk = lambda idx: Tensor(idx, tuple(2 for _ in idx), col_major([2] * len(idx)), z.copy())
    with pytest.raises(ValueError):
        oracle.contract_literal(mk("ij"), mk("jk"), mk("ijk"))  # j in all three
    with pytest.raises(ValueError):
        oracle.contract_literal(mk("ii"), mk("ik"), mk("k"))  # repeated label
    with pytest.raises(ValueError):
        oracle.contract_literal(mk("ij"), mk("jk"), mk("il"))  # k, l in one tensor only
    bad = Tensor("jk", (3, 2), (1, 3), np.zeros(6))
    with pytest.raises(ValueError):
        oracle.contract_literal(mk("ij"), bad, mk("ik"))  # length mismatch on j
