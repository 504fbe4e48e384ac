"""CPU-only checks of the C ABI: the library loads, exports every declared symbol, rejects malformed problems,
and its host-side schedule (inspected through host-only plans) satisfies Brent's equations."""
import ctypes
import os
import re

import numpy as np
import pytest

import paper_1704_03092_amd as tc
import workloads

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module", autouse=True)
def _lib():
    if not os.path.exists(tc.lib_path()):
        tc.build()
    tc.load_library()


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "strassen_tc.h")).read()
    names = set(re.findall(r"\b(tc_[a-z_]+)\s*\(", hdr))
    assert {"tc_plan", "tc_contract", "tc_destroy", "tc_plan_workspace_bytes", "tc_strerror"} <= names
    lib = ctypes.CDLL(tc.lib_path())
    for n in names:
        assert hasattr(lib, n), n


def _plan(A, B, C, level=0, variant="abc", **kw):
    kw.setdefault("tail_split", -1)  # the schedules below are those of the paper; the tail split has tests of its own
    kw.setdefault("tile_n", 128)     # and so has the choice of the tile shape
    return tc.tc_plan(A, B, C, level, variant, host_only=True, **kw)


def test_error_paths():
    ok = (("ik", (4, 5), (1, 4)), ("kj", (5, 6), (1, 5)), ("ij", (4, 6), (1, 4)))
    tc.tc_destroy(_plan(*ok))
    cases = [
        ((("ik", (4, 5), (1, 4)), ("kj", (5, 6), (1, 5)), ("ijk", (4, 6, 5), (1, 4, 24))), -3),  # k in all three
        ((("ii", (4, 4), (1, 4)), ("ij", (4, 6), (1, 4)), ("j", (6,), (1,))), -3),  # repeated label
        ((("ik", (4, 5), (1, 4)), ("kj", (5, 6), (1, 5)), ("il", (4, 6), (1, 4))), -3),  # j, l in one tensor only
        ((("ik", (4, 5), (1, 4)), ("kj", (7, 6), (1, 7)), ("ij", (4, 6), (1, 4))), -4),  # k has two lengths
        ((("ik", (4, -5), (1, 4)), ("kj", (-5, 6), (1, 5)), ("ij", (4, 6), (1, 4))), -4),  # negative length
        ((("ik", (4, 5), (1, -4)), ("kj", (5, 6), (1, 5)), ("ij", (4, 6), (1, 4))), -5),  # negative stride
        ((("ik", (4, 5), (0, 4)), ("kj", (5, 6), (1, 5)), ("ij", (4, 6), (1, 4))), -5),  # zero stride, len > 1
        ((("ik", (4, 5), (1, 4)), ("kj", (5, 6), (1, 5)), ("ij", (4, 6), (1, 3))), -5),  # C overlaps itself
    ]
    for (A, B, C), status in cases:
        with pytest.raises(tc.TcError) as e:
            _plan(A, B, C)
        assert e.value.status == status, (A, B, C)
    with pytest.raises(tc.TcError) as e:
        _plan(*ok, level=3)
    assert e.value.status == -6
    with pytest.raises(tc.TcError) as e:
        _plan(*ok, variant=7)
    assert e.value.status == -7
    many = "abcdefghijklmnopq"  # 17 labels > TC_MAX_NDIM
    with pytest.raises(tc.TcError) as e:
        _plan((many, (1,) * 17, (1,) * 17), ("", (), ()), (many, (1,) * 17, (1,) * 17))
    assert e.value.status == -2
    # a host-only plan cannot run
    p = _plan(*ok)
    with pytest.raises(tc.TcError) as e:
        tc.tc_contract(p, 1.0, 8, 8, 1.0, 8)
    assert e.value.status == -10
    assert "host-only" in tc.tc_strerror(-10)


def test_interleaved_layouts_of_C_are_decided_exactly():
    """C's elements must be pairwise distinct.  Nested layouts pass a cheap sufficient test; interleaved ones are listed
    and sorted: lengths (2, 3) with strides (3, 2) give the locations 0, 3, 2, 5, 4, 7 (legal), strides (2, 1) give
    0, 2, 1, 3, 2, 4 (location 2 twice)."""
    A, B = ("ik", (2, 5), (1, 2)), ("kj", (5, 3), (1, 5))
    tc.tc_destroy(_plan(A, B, ("ij", (2, 3), (3, 2))))
    with pytest.raises(tc.TcError) as e:
        _plan(A, B, ("ij", (2, 3), (2, 1)))
    assert e.value.status == -5
    # three dimensions, interleaved and legal: offsets i + 2 j with j < 2 cover 0..3, the last dimension steps over them
    tc.tc_destroy(_plan(("ik", (2, 5), (1, 2)), ("kjl", (5, 2, 3), (1, 5, 10)), ("ijl", (2, 2, 3), (1, 2, 4))))
    # an interleaved layout too large to list is refused, a nested one of the same size is not
    big = 1 << 23  # rows at odd locations 3 + 2 j, columns at even ones: legal, but 2^24 elements are not listed
    A, B = ("ik", (2, 2), (1, 2)), ("kj", (2, big), (1, 2))
    tc.tc_destroy(_plan(A, B, ("ij", (2, big), (1, 2))))
    tc.tc_destroy(_plan(A, ("kj", (2, 1 << 20), (1, 2)), ("ij", (2, 1 << 20), (3, 2))))
    with pytest.raises(tc.TcError) as e:
        _plan(A, B, ("ij", (2, big), (3, 2)))
    assert e.value.status == -5


def test_plan_info_bundles_and_modes():
    # the paper's example contraction C_abc += A_dca * B_db, generalized column-major
    L = dict(a=4, b=8, c=2, d=8)
    cm = lambda idx: (idx, tuple(L[x] for x in idx), tuple(int(np.prod([L[y] for y in idx[:i]])) for i in range(len(idx))))
    p = _plan(cm("dca"), cm("db"), cm("abc"), bs_block=4)
    info = tc.tc_plan_info(p)
    assert (info["m"], info["n"], info["k"]) == (8, 8, 8)
    assert sorted(info["I"]) == ["a", "c"] and info["J"] == "b" and info["P"] == "d"
    assert info["bs_block"] == 4 and info["n_products"] == 1 and info["level"] == 0
    assert info["a_mode"] == 1 and info["b_mode"] == 1  # d is the stride-1 index of both A and B
    # level is lowered while a bundle is shorter than 2^level
    p2 = _plan(("ik", (1, 64), (1, 1)), ("kj", (64, 64), (1, 64)), ("ij", (1, 64), (1, 1)), level=2)
    assert tc.tc_plan_info(p2)["level"] == 0
    p3 = _plan(("ik", (3, 64), (1, 3)), ("kj", (64, 64), (1, 64)), ("ij", (3, 64), (1, 3)), level=2)
    assert tc.tc_plan_info(p3)["level"] == 1
    assert tc.tc_plan_info(p3)["level_requested"] == 2


@pytest.mark.parametrize("level", [1, 2])
@pytest.mark.parametrize("variant", ["abc", "ab", "naive", "hybrid"])
def test_schedule_satisfies_brent_equations(level, variant):
    """The library's own product schedule, read back through the ABI, multiplies block matrices correctly."""
    N = 64
    g = 1 << level
    p = _plan(("ik", (N, N), (1, N)), ("kj", (N, N), (1, N)), ("ij", (N, N), (1, N)), level=level, variant=variant)
    info = tc.tc_plan_info(p)
    assert info["level"] == level and info["n_products"] == 7 ** level
    sched = tc.tc_plan_schedule(p)
    T = np.zeros((g,) * 6, dtype=np.int64)
    seen = set()
    for e in sched:
        for (ai, ak, sa) in e["a"]:
            for (bk, bj, sb) in e["b"]:
                for (ci, cj, sc) in e["c"]:
                    T[ai, ak, bk, bj, ci, cj] += sa * sb * sc
        for (ci, cj, _), first in zip(e["c"], e["c_first"]):
            assert bool(first) == ((ci, cj) not in seen)
            seen.add((ci, cj))
    want = np.zeros_like(T)
    for i in range(g):
        for k in range(g):
            for j in range(g):
                want[i, k, k, j, i, j] = 1
    assert np.array_equal(T, want)
    assert len(seen) == g * g  # every block of C is written, each takes beta exactly once
    na = sum(len(e["a"]) for e in sched)
    nb = sum(len(e["b"]) for e in sched)
    nc = sum(len(e["c"]) for e in sched)
    assert (na, nb, nc) == ((12, 12, 12) if level == 1 else (144, 144, 144))
    # products sharing a launch write disjoint blocks
    by_launch = {}
    for e in sched:
        blocks = by_launch.setdefault(e["launch"], set())
        for (ci, cj, _) in e["c"]:
            assert (ci, cj) not in blocks
            blocks.add((ci, cj))
    ws = tc.tc_plan_workspace_bytes(p)
    blk = info["mb"] * info["nb"], info["mb"] * info["kb"], info["kb"] * info["nb"]
    hybrid_ws = 8 * (4 if level == 2 else 1) * (blk[1] + blk[2])  # one first-level block of A and of B
    assert ws == {"abc": 0, "ab": 8 * blk[0], "naive": 8 * sum(blk), "hybrid": hybrid_ws}[variant]
    if variant == "hybrid":
        # 5 + 5 stored operand sums; per first-level product one launch, or the four launches of one-level ABC
        assert info["n_launches"] == 10 + 7 * (4 if level == 2 else 1)
    if variant == "abc":
        assert info["n_launches"] == (4 if level == 1 else len(by_launch))
        assert info["n_launches"] < 7 ** level


def test_schedule_prunes_blocks_in_the_padding():
    """Block extents (Sec. 3, last paragraph: zero padding): even where the operands read a bundle as one constant-stride
    run, multiples of the 16-entry blocks of the block scatter vectors elsewhere; blocks wholly in the padding are
    pruned from the schedule."""
    # m = 20 as rows a + 4 b of an A whose b stride (8) leaves gaps: read through the block scatter vector, extent 16
    # at level 2 => block rows 2 and 3 are empty
    p = _plan(("abk", (4, 5, 64), (1, 8, 40)), ("kj", (64, 64), (1, 64)), ("abj", (4, 5, 64), (1, 4, 20)), level=2)
    info = tc.tc_plan_info(p)
    assert (info["m"], info["mb"]) == (20, 16)
    for e in tc.tc_plan_schedule(p):
        assert all(r < 2 for (r, _, _) in e["a"]) and all(r < 2 for (r, _, _) in e["c"])
        assert e["a"] and e["b"] and e["c"]
    tc.tc_destroy(p)
    # plain matrices: m = 20 => 6, 6, 6, 2 rows, nothing pruned; m = 9 => extent 4, block row 3 is empty
    p = _plan(("ik", (20, 64), (1, 20)), ("kj", (64, 64), (1, 64)), ("ij", (20, 64), (1, 20)), level=2)
    assert tc.tc_plan_info(p)["mb"] == 6 and len(tc.tc_plan_schedule(p)) == 49
    tc.tc_destroy(p)
    p = _plan(("ik", (9, 64), (1, 9)), ("kj", (64, 64), (1, 64)), ("ij", (9, 64), (1, 9)), level=2)
    assert tc.tc_plan_info(p)["mb"] == 4
    for e in tc.tc_plan_schedule(p):
        assert all(r < 3 for (r, _, _) in e["a"]) and all(r < 3 for (r, _, _) in e["c"])
    tc.tc_destroy(p)
    # equal blocks wherever the length allows: 16200 = 2 * 8100 = 4 * 4050 (zero padding; with peeling the row and
    # column blocks are whole tiles: 63 and 31 of them)
    for level, want, tiles in ((1, 8100, 63), (2, 4050, 31)):
        p = _plan(*_gemm_desc(16200, 16200, 16200), level=level, no_peel=True)
        info = tc.tc_plan_info(p)
        assert (info["mb"], info["nb"], info["kb"]) == (want, want, want)
        tc.tc_destroy(p)
        p = _plan(*_gemm_desc(16200, 16200, 16200), level=level)
        info = tc.tc_plan_info(p)
        assert (info["mb"], info["nb"], info["kb"]) == (128 * tiles, 128 * tiles, want)
        tc.tc_destroy(p)


def test_empty_bundles():
    p = _plan(("ik", (0, 5), (1, 1)), ("kj", (5, 6), (1, 5)), ("ij", (0, 6), (1, 1)))
    assert tc.tc_plan_info(p)["n_launches"] == 0
    p = _plan(("ik", (4, 0), (1, 4)), ("kj", (0, 6), (1, 1)), ("ij", (4, 6), (1, 4)), level=1)
    assert tc.tc_plan_info(p)["n_launches"] == 1  # C := beta * C
    p = _plan(("", (), ()), ("", (), ()), ("", (), ()))  # scalar times scalar
    info = tc.tc_plan_info(p)
    assert (info["m"], info["n"], info["k"]) == (1, 1, 1)


def _gemm_desc(m, n, k):
    return ("ik", (m, k), (1, m)), ("kj", (k, n), (1, k)), ("ij", (m, n), (1, m))


# Model parameters in powers of two, so that the totals below can be worked out by hand: a wave of 16 tiles of
# 128 x 128 with 512 contracted entries is 16 * 2 * 128 * 128 * 512 = 2^28 flops; rho_a * peak = 2^28, 2^27, 2^26
# flop/s for one-, two- and four-block sums; rho_b * bandwidth = 2^24 byte/s.
_HAND = dict(peak_flops=2.0 ** 29, rho_a=[0.5, 0.25, 0.125], bandwidth=2.0 ** 25, rho_b=0.5, t_launch=0.125, t_tile=0.25, units=16,
             rho_small=0.5, t_tile_small=0.125, rho_gather=0.5, lambda_ab=0.0, rho_table=[0.5, 0.25, 0.125], rho_small_table=0.25)


@pytest.mark.parametrize("shape,level,variant,opts,want", [
    # one launch of 64 tiles = 4 waves of 1 s + 0.25 s; C read and written: 2 * 2^20 elements * 8 B = 2^24 B = 1 s
    ((1024, 1024, 512), 0, "abc", dict(tile_n=128), dict(arith=5.0, c_update=1.0, temporaries=0.0, launch=0.125)),
    # 128 x 64 tiles: 128 tiles, 32 at a time = 4 waves; the same 2^28 flops per wave at half the rate = 2 s + 0.125 s
    ((1024, 1024, 512), 0, "abc", dict(tile_n=64), dict(arith=8.5, c_update=1.0, temporaries=0.0, launch=0.125)),
    # 72 tiles, all of them tail for the 256 units the plan is made for; cut in 2 chunks of 256 entries = 144 pieces =
    # 9 waves of 16 at 0.5 s + 0.25 s; the pieces written and read back: 2 * 144 * 128 * 128 * 8 B = 2.25 * 2^24 B;
    # a second launch; C: 2 * 1152 * 1024 * 8 B = 1.125 * 2^24 B
    ((1152, 1024, 512), 0, "abc", dict(tile_n=128, tail_split=2), dict(arith=6.75, c_update=1.125, temporaries=2.25, launch=0.25)),
    # one level, sums and updates in the kernel: 7 products of 64 tiles in 4 launches (64 + 3 * 128 tiles = 28 waves),
    # each launch with a two-block sum: 2 s + 0.25 s per wave; 12 destination blocks read and written
    ((2048, 2048, 1024), 1, "abc", dict(tile_n=128), dict(arith=63.0, c_update=12.0, temporaries=0.0, launch=0.5)),
    # AB: 7 launches of 4 waves at 2.25 s; each product written once to M (2^23 B = 0.5 s); 7 passes that read M and
    # read and write the 12 destination blocks: (7 + 2 * 12) * 2^23 B = 15.5 s; 14 launches
    ((2048, 2048, 1024), 1, "ab", dict(tile_n=128), dict(arith=63.0, c_update=3.5, temporaries=15.5, launch=1.75)),
    # Naive: operand sums stored first: per product (blocks + 1) * 2^19 elements on each side, 12 + 7 blocks-plus-one
    # per side = 38 * 2^22 B = 9.5 s; then single-block products: 28 waves of 1.25 s; M and the C passes as for AB
    ((2048, 2048, 1024), 1, "naive", dict(tile_n=128), dict(arith=35.0, c_update=3.5, temporaries=25.0, launch=3.5)),
    # operand reads with weight 1/4: each of the 64 tiles reads a 128 x 512 panel of A and a 512 x 128 panel of B:
    # 64 * 512 * 256 * 8 B = 2^26 B = 4 s, a quarter of it counted
    ((1024, 1024, 512), 0, "abc", dict(tile_n=128, lambda_ab=0.25), dict(arith=5.0, c_update=1.0, temporaries=0.0, launch=0.125, operands=1.0)),
    # the same in 128 x 64 tiles: 128 tiles read 128 + 64 columns and rows of depth 512: 128 * 512 * 192 * 8 B = 6 s
    ((1024, 1024, 512), 0, "abc", dict(tile_n=64, lambda_ab=0.25), dict(arith=8.5, c_update=1.0, temporaries=0.0, launch=0.125, operands=1.5)),
    # two-block sums: the seven products have 12 + 12 summed blocks; per tile and block a 128 x 512 panel:
    # 64 * 24 * 128 * 512 * 8 B = 48 * 2^24 B = 48 s, a quarter counted
    ((2048, 2048, 1024), 1, "abc", dict(tile_n=128, lambda_ab=0.25), dict(arith=63.0, c_update=12.0, temporaries=0.0, launch=0.5, operands=12.0)),
    # A without a stride-one index (stored with stride 2 along its rows): gathered element by element, half the rate:
    # 4 waves of 2 s + 0.25 s
    ((1024, 1024, 512), 0, "abc", dict(tile_n=128, stride_a=2), dict(arith=9.0, c_update=1.0, temporaries=0.0, launch=0.125)),
    # 1000 rows: the 8 tiles of the last tile row are ragged and go through the scatter tables at half the rate of the
    # 56 others: 1 / rho = (7/8) / 0.5 + (1/8) / 0.25 = 2.25, a wave takes 2.25 * 2^28 / 2^29 s + 0.25 s; C: 2 * 1000 * 1024 * 8 B
    ((1000, 1024, 512), 0, "abc", dict(tile_n=128, rho_table=[0.25, 0.25, 0.25]), dict(arith=5.5, c_update=0.9765625, temporaries=0.0, launch=0.125)),
    # the same in 128 x 64 tiles: 112 tiles by stride at 0.5 * 0.5, the 16 ragged ones through the tables at 0.25 * 0.25:
    # 1 / rho = (7/8) / 0.25 + (1/8) / 0.0625 = 5.5; 4 waves of 32 tiles, each 5.5 * 2^28 / 2^29 s + 0.125 s
    ((1000, 1024, 512), 0, "abc", dict(tile_n=64, rho_table=[0.25, 0.25, 0.25]), dict(arith=11.5, c_update=0.9765625, temporaries=0.0, launch=0.125)),
])
def test_model_prediction_hand_computed(shape, level, variant, opts, want):
    """Sec. 5 eq. (2)-(4): the modelled time is the sum of the arithmetic term, the destination updates, the operand
    reads, the temporaries and the launches; whole tiles run in whole waves.  Expected values worked out by hand (see
    the parameters above)."""
    opts = dict(opts)
    params = dict(tc.tc_model_defaults(), **_HAND)
    params["lambda_ab"] = opts.pop("lambda_ab", 0.0)
    params["rho_table"] = opts.pop("rho_table", params["rho_table"])
    sa = opts.pop("stride_a", 1)
    A, B, C = _gemm_desc(*shape)
    A = (A[0], A[1], (sa, sa * shape[0]))
    plan = _plan(A, B, C, level=level, variant=variant, **opts)
    assert all(L["pairs_a"] == (sa == 1) and L["pairs_b"] == 1 for L in tc.tc_plan_launches(plan) if L["kind"] == 0)
    got = tc.tc_plan_predict(plan, params)
    tc.tc_destroy(plan)
    want = dict({"operands": 0.0}, **want)
    for key, value in want.items():
        assert got[key] == pytest.approx(value, rel=1e-12, abs=1e-15), (key, got)
    assert got["total"] == pytest.approx(sum(want.values()), rel=1e-12)


def test_model_reduces_to_the_printed_model_for_whole_waves():
    """With every launch a whole number of waves, no fixed costs and one efficiency for every kernel family, the
    library's arithmetic and destination-update terms are T_a^x and T_m^{Cx} of the model as printed (Sec. 5 eq. (2)-(4),
    one-level ABC with k_C equal to the block's contracted extent).  Its operand term with weight 1 is the printed
    T_m^{Ax} with n_C = 128 (every tile of 128 columns reads its panel of A) plus the printed T_m^{Bx} once per tile
    row (the printed model packs B once; here every tile of 128 rows reads its panel of B)."""
    import oracle
    from oracle import model as M

    m = n = 128 * 16  # 2 x 2 blocks of 8 x 8 tiles = one wave of 64 each
    k = 4096
    params = dict(tc.tc_model_defaults(), peak_flops=50e12, rho_a=[0.9, 0.9, 0.9], rho_table=[0.9, 0.9, 0.9], bandwidth=4e12, rho_b=0.5, t_launch=0.0,
                  t_tile=0.0, units=64, lambda_ab=1.0)
    plan = _plan(*_gemm_desc(m, n, k), level=1, variant="abc", tile_n=128)
    got = tc.tc_plan_predict(plan, params)
    tc.tc_destroy(plan)
    p = M.PaperParams(50e3, 4e3, rho_a=0.9, rho_b=0.5, lam=1.0, k_c=k, n_c=128)
    t = M.paper_terms(m, n, k, 1, "abc", p)
    assert got["arith"] == pytest.approx(t["a_mul"], rel=1e-13)
    assert got["c_update"] == pytest.approx(t["m_Cx"], rel=1e-13)
    assert got["operands"] == pytest.approx(t["m_Ax"] + t["m_Bx"] * (m // 2 // 128), rel=1e-13)
    assert got["total"] == pytest.approx(t["a_mul"] + t["m_Cx"] + got["operands"], rel=1e-13)


def test_automatic_choice_is_the_argmin_of_the_model():
    for shape in [(16384, 16384, 16384), (4096, 4096, 4096), (512, 512, 512), (16384, 16384, 256), (9216, 96, 4096), (36864, 2304, 36864)]:
        desc = _gemm_desc(*shape)
        times = {}
        for level in (0, 1, 2):
            for variant in ("abc", "ab", "naive") + (("hybrid",) if level >= 1 else ()):
                plan = _plan(*desc, level=level, variant=variant)
                if tc.tc_plan_info(plan)["level"] == level:
                    times[(level, tc.VARIANTS[variant])] = tc.tc_plan_predict(plan)["total"]
                tc.tc_destroy(plan)
        auto = _plan(*desc, level=tc.TC_LEVEL_AUTO, variant="auto")
        info = tc.tc_plan_info(auto)
        assert times[(info["level"], info["variant"])] == min(times.values()), (shape, info["level"], info["variant"], times)
        tc.tc_destroy(auto)
        # one of the two fixed by the caller
        auto = _plan(*desc, level=tc.TC_LEVEL_AUTO, variant="ab")
        info = tc.tc_plan_info(auto)
        assert info["variant"] == 1 and times[(info["level"], 1)] == min(t for (L, v), t in times.items() if v == 1)
        tc.tc_destroy(auto)
        auto = _plan(*desc, level=1, variant="auto")
        info = tc.tc_plan_info(auto)
        assert info["level"] == 1 and times[(1, info["variant"])] == min(t for (L, v), t in times.items() if L == 1)
        tc.tc_destroy(auto)
    with pytest.raises(tc.TcError) as e:
        _plan(*_gemm_desc(8, 8, 8), level=5, variant="auto")
    assert e.value.status == -6


def test_launch_info_counts_tiles_gathered_by_stride():
    """Sec. 4.1 "Packing": a tile is gathered by stride iff every block scatter entry of its rows and columns is
    non-zero in every summed block (here also: the contracted bundle is one run, no missing row or column in the tile,
    at least four k-steps without zero padding, pairs of entries contiguous).  tc_plan_launch reports how many tiles
    of each launch that is."""
    def launches(A, B, C, level=0, variant="abc", **kw):
        p = _plan(A, B, C, level=level, variant=variant, **kw)
        out = [(L["tiles"], L["tiles_table_free"]) for L in tc.tc_plan_launches(p) if L["kind"] == 0]
        tc.tc_destroy(p)
        return out

    cm = lambda idx, L: (idx, tuple(L[x] for x in idx), tuple(int(np.prod([L[y] for y in idx[:i]])) for i in range(len(idx))))
    # the rank-k configuration: A[a e b] has rows a + 128 b (a is exactly one tile of rows: every tile regular, the
    # bundle as a whole not one run), B and C are plain matrices
    L = dict(a=128, b=128, c=128, d=128, e=256)
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L)) == [(16384, 16384)]
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L), level=1) == [(4096, 4096), (8192, 8192), (8192, 8192), (8192, 8192)]
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L), bs_block=8) == [(16384, 0)]  # the kernel reads blocks of 16 only
    # lengths 24 next to 128: rows a + 24 b cross a run of 24 in every tile; with a = 192 two tiles of three are regular
    L = dict(a=24, b=32, c=128, d=2, e=64)
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L)) == [(12, 0)]
    L = dict(a=192, b=4, c=128, d=2, e=64)  # rows 0..767: tiles [0,128) ok, [128,256) crosses 192, [256,384) ok, [384,512) ok, [512,640) crosses 576, [640,768) ok
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L)) == [(12, 8)]
    # plain matrices: whole tiles only (10001 = 78 * 128 + 17); a padded last k-step goes through the tables after
    # the whole ones, of which there must be four (32-deep k-steps: 500 = 15 whole ones + 20, 100 = 3 + 4)
    g = lambda n, k: (("ik", (n, k), (1, n)), ("kj", (k, n), (1, k)), ("ij", (n, n), (1, n)))
    assert launches(*g(1024, 512)) == [(64, 64)]
    assert launches(*g(1000, 512)) == [(64, 49)]
    assert launches(*g(1024, 500)) == [(64, 64)]
    assert launches(*g(1024, 100)) == [(64, 0)]
    assert launches(*g(10001, 10001)) == [(6241, 78 * 78)]
    # element-by-element gathers (odd leading extent next to another dimension): never by stride
    L = dict(a=127, b=4, c=128, d=2, e=64)
    assert launches(cm("aeb", L), cm("ecd", L), cm("abcd", L)) == [(8, 0)]


def test_split_k_schedule():
    desc = _gemm_desc(9216, 96, 4096)
    plain = _plan(*desc)
    assert tc.tc_plan_workspace_bytes(plain) == 0 and tc.tc_plan_info(plain)["n_launches"] == 1
    t1 = tc.tc_plan_predict(plain)["total"]
    tc.tc_destroy(plain)
    times = {1: t1}
    for s in (2, 3, 4):
        plan = _plan(*desc, split_k=s)
        info = tc.tc_plan_info(plan)
        assert info["n_products"] == s and info["n_launches"] == 2 and info["level"] == 0
        assert tc.tc_plan_workspace_bytes(plan) == s * 9216 * 96 * 8
        times[s] = tc.tc_plan_predict(plan)["total"]
        tc.tc_destroy(plan)
    auto = _plan(*desc, split_k=-1)
    info = tc.tc_plan_info(auto)
    assert times[info["n_products"]] == min(times.values()) and info["n_products"] > 1  # 72 tiles on 256 units: splitting pays
    tc.tc_destroy(auto)
    # chunks shorter than 64 entries are not made; Strassen levels ignore the option; out-of-range values are refused
    short = _plan(*_gemm_desc(256, 256, 90), split_k=4)
    assert tc.tc_plan_info(short)["n_products"] == 1 and tc.tc_plan_workspace_bytes(short) == 0
    tc.tc_destroy(short)
    lvl1 = _plan(*desc, level=1, variant="abc", split_k=4)
    assert tc.tc_plan_info(lvl1)["n_products"] == 7 and tc.tc_plan_workspace_bytes(lvl1) == 0
    tc.tc_destroy(lvl1)
    with pytest.raises(tc.TcError) as e:
        _plan(*desc, split_k=5)
    assert e.value.status == -10
    # a large square problem has tiles enough: the model keeps it whole
    big = _plan(*_gemm_desc(8192, 8192, 8192), split_k=-1)
    assert tc.tc_plan_info(big)["n_products"] == 1
    tc.tc_destroy(big)


@pytest.mark.parametrize("tile_n", [128, 64])
@pytest.mark.parametrize("shape,level,variant", [((36864, 2304, 36864), 1, "abc"), ((36864, 2304, 36864), 1, "hybrid"),
                                                  ((10001, 10001, 10001), 1, "abc"), ((9216, 96, 4096), 0, "abc"),
                                                  ((13824, 13824, 9216), 2, "hybrid"), ((16384, 16384, 16384), 1, "abc"),
                                                  ((256, 256, 256), 0, "abc"), ((3000, 2000, 700), 1, "ab")])
def test_tail_split_is_the_argmin_of_the_model(shape, level, variant, tile_n):
    """Every launch: the tail is what is left after whole rounds of the units (one 128 x 128 or two 128 x 64 tiles per
    unit); the automatic chunk count is no slower, by the library's own model, than no split and than every forced
    count 2..16 (chunks of a multiple of 64 entries; at most 1024 chunks); the workspace holds the largest launch's chunks."""
    units = tc.tc_model_defaults()["units"]
    desc = _gemm_desc(*shape)
    plain = _plan(*desc, level=level, variant=variant, tile_n=tile_n)
    plan = _plan(*desc, level=level, variant=variant, tail_split=0, tile_n=tile_n)
    L0, L1 = tc.tc_plan_launches(plain), tc.tc_plan_launches(plan)
    assert len(L0) == len(L1)
    most = 0
    for a, b in zip(L0, L1):
        same = lambda L: {k: v for k, v in L.items() if not k.startswith("tail") and k != "tiles_table_free"}  # (chunks have their own depth)
        assert same(a) == same(b)
        assert a["tail_tiles"] == 0
        if b["kind"] == 1 or b["tail_tiles"] == 0:
            assert b["tail_tiles"] == 0
            continue
        assert b["tail_tiles"] == b["tiles"] % (units * (128 // b["tile_n"]))
        assert b["tail_kc"] % 64 == 0 and 2 <= b["tail_chunks"] <= 16 and b["tail_tiles"] * b["tail_chunks"] <= 1024
        assert (b["tail_chunks"] - 1) * b["tail_kc"] < b["depth"] <= b["tail_chunks"] * b["tail_kc"]
        most = max(most, b["tail_tiles"] * b["tail_chunks"] * 128 * b["tile_n"])
    best = tc.tc_plan_predict(plan)["total"]
    others = [tc.tc_plan_predict(plain)["total"]]
    for forced in range(2, 17):
        alt = _plan(*desc, level=level, variant=variant, tail_split=forced, tile_n=tile_n)
        others.append(tc.tc_plan_predict(alt)["total"])
        tc.tc_destroy(alt)
    assert best <= min(others) * (1 + 1e-12), (best, others)
    if len([L for L in L1 if L["kind"] == 0]) == 1:  # one multiplying launch: the automatic choice is one of the forced ones
        assert any(best == pytest.approx(o, rel=1e-12) for o in others)
    assert tc.tc_plan_workspace_bytes(plan) == tc.tc_plan_workspace_bytes(plain) + most * 8
    tc.tc_destroy(plain)
    tc.tc_destroy(plan)


def test_tail_split_shapes():
    # the ladder contraction: 1296 tiles per product = 5 rounds of 256 units and 16 tiles, which 16 chunks each fill a round
    plan = _plan(*_gemm_desc(36864, 2304, 36864), level=1, variant="hybrid", tail_split=0)
    fused = [L for L in tc.tc_plan_launches(plan) if L["kind"] == 0]
    assert len(fused) == 7 and all(L["tiles"] == 1296 and L["tail_tiles"] == 16 and L["tail_chunks"] == 16 for L in fused)
    tc.tc_destroy(plan)
    # whole rounds: nothing to split, no workspace
    plan = _plan(*_gemm_desc(16384, 16384, 16384), tail_split=0)
    assert tc.tc_plan_launches(plan)[0]["tail_tiles"] == 0 and tc.tc_plan_workspace_bytes(plan) == 0
    tc.tc_destroy(plan)
    # with the automatic tail split, split_k = -1 leaves the job to it
    plan = _plan(*_gemm_desc(9216, 96, 4096), split_k=-1, tail_split=0)
    info = tc.tc_plan_info(plan)
    assert info["n_products"] == 1 and info["n_launches"] == 1 and tc.tc_plan_launches(plan)[0]["tail_tiles"] == 72
    tc.tc_destroy(plan)
    with pytest.raises(tc.TcError) as e:
        _plan(*_gemm_desc(64, 64, 64), tail_split=17)
    assert e.value.status == -10
    # forced: chunks of a multiple of 64 entries
    plan = _plan(*_gemm_desc(300, 200, 500), tail_split=3)
    L = tc.tc_plan_launches(plan)[0]
    assert (L["tiles"], L["tail_tiles"], L["tail_chunks"], L["tail_kc"]) == (6, 6, 3, 192)
    assert tc.tc_plan_workspace_bytes(plan) == 18 * 128 * 128 * 8
    tc.tc_destroy(plan)
    plan = _plan(*_gemm_desc(300, 200, 100), tail_split=4)  # 128-entry chunks would leave a single one: chunks of 64
    L = tc.tc_plan_launches(plan)[0]
    assert (L["tail_tiles"], L["tail_chunks"], L["tail_kc"]) == (6, 2, 64)
    tc.tc_destroy(plan)


def test_sweep_families_plan_on_the_host():
    """The regression grid's case generators (Sec. 6.1 families): seeded, reproducible, and every case plans in every
    mode; the ladder family keeps 2 N_a^4 N_i^2 within a factor 1.5 of 2 * 16000^3 flops over the ratios 1 ... 5."""
    from paper_1704_03092_amd import sweep

    for reduced in (True, False):
        for fam in sweep.FAMILIES:
            a, b = sweep.cases(fam, reduced), sweep.cases(fam, reduced)
            assert [c.name for c in a] == [c.name for c in b] and [c.lengths for c in a] == [c.lengths for c in b] and a
            for c in a:
                desc = []
                for idx in (c.idxA, c.idxB, c.idxC):
                    lens = [c.lengths[x] for x in idx]
                    st, acc = [], 1
                    for n in lens:
                        st.append(acc)
                        acc *= n
                    desc.append((idx, tuple(lens), tuple(st)))
                assert 2 <= max(len(d[0]) for d in desc) <= 6
                for level, variant in ((0, "abc"), (1, "abc"), (2, "hybrid"), (tc.TC_LEVEL_AUTO, "auto")):
                    plan = tc.tc_plan(*desc, level, variant, host_only=True)
                    info = tc.tc_plan_info(plan)
                    assert (info["m"], info["n"], info["k"]) == c.mnk()
                    tc.tc_destroy(plan)
    ratios = {}
    for c in sweep.cases("ladder"):
        na, ni = c.lengths["a"], c.lengths["i"]
        ratios[round(na / ni)] = c.flops() / (2.0 * 16000.0 ** 3)
    assert sorted(ratios) == [1, 2, 3, 4, 5] and all(1 / 1.5 <= v <= 1.5 for v in ratios.values()), ratios


def test_dynamic_peeling_of_rows_and_columns():
    """Sec. 3, last paragraph (dynamic peeling): the Strassen grid covers a leading part of the row
    and column bundles, classical edge products the rest: rows [m - m_peel, m) over all columns, then the leading
    rows over columns [n - n_peel, n).  Long bundles are cut at whole tiles per block (at most a tenth left over),
    others at whole block units if they are no whole number of equal blocks; the contracted bundle and short bundles
    are completed with zeros; no_peel turns peeling off."""
    # 10001 = 39 * 256 + 17 = 19 * 512 + 273
    for level, block, peel in ((1, 4992, 17), (2, 2432, 273)):
        p = _plan(*_gemm_desc(10001, 10001, 10001), level=level)
        info = tc.tc_plan_info(p)
        assert (info["m_peel"], info["n_peel"], info["mb"], info["nb"]) == (peel, peel, block, block)
        assert info["kb"] == 2 * ((10001 + 2 ** (level + 1) - 1) // 2 ** (level + 1))  # zero padding: even, >= k / 2^level
        fused = [L for L in tc.tc_plan_launches(p) if L["kind"] == 0]
        assert [(L["rows"], L["cols"], L["depth"], L["terms_a"], L["terms_b"]) for L in fused[-2:]] == \
            [(peel, 10001, 10001, 1, 1), (10001 - peel, peel, 10001, 1, 1)]
        assert all((L["rows"], L["cols"]) == (block, block) and L["tiles_table_free"] == L["tiles"] for L in fused[:-2])
        assert len(tc.tc_plan_schedule(p)) == 7 ** level  # the schedule lists the Strassen products only
        tc.tc_destroy(p)
        q = _plan(*_gemm_desc(10001, 10001, 10001), level=level, no_peel=True)
        info = tc.tc_plan_info(q)
        assert (info["m_peel"], info["n_peel"]) == (0, 0) and info["mb"] == 2 * ((10001 + 2 ** (level + 1) - 1) // 2 ** (level + 1))
        tc.tc_destroy(q)
        for variant in ("ab", "naive", "hybrid"):  # whole tiles per block: every variant
            q = _plan(*_gemm_desc(10001, 10001, 10001), level=level, variant=variant)
            info = tc.tc_plan_info(q)
            assert (info["m_peel"], info["n_peel"], info["mb"]) == (peel, peel, block)
            tc.tc_destroy(q)
    # 16200 = 63 * 256 + 72 (equal blocks of 8100 would have ragged last tiles); 2000 = 7 * 256 + 208 is more than a
    # tenth: cut at block units, and 2000 is two equal blocks already; 2001 leaves one row
    for shape, level, want in (((16200, 16384, 16200), 1, (72, 0)), ((2000, 2001, 657), 1, (0, 1)), ((16384, 8192, 100), 2, (0, 0)),
                               ((10001, 10001, 10001), 0, (0, 0)), ((501, 300, 657), 2, (0, 0))):
        p = _plan(*_gemm_desc(*shape), level=level)
        info = tc.tc_plan_info(p)
        assert (info["m_peel"], info["n_peel"]) == want, shape
        tc.tc_destroy(p)
    # block units are peeled only where blocks are summed inside the multiplying kernel (ABC, AB): single-block products
    # have no blocks of different length to reconcile
    for variant, want in (("ab", (0, 1)), ("naive", (0, 0)), ("hybrid", (0, 0))):
        p = _plan(*_gemm_desc(2000, 2001, 657), level=1, variant=variant)
        info = tc.tc_plan_info(p)
        assert (info["m_peel"], info["n_peel"]) == want, variant
        tc.tc_destroy(p)
    # a row bundle read through the block scatter vector: blocks are multiples of 16, so up to 31 rows are peeled at one level
    p = _plan(("abk", (24, 50, 64), (1, 32, 1600)), ("kj", (64, 700), (1, 64)), ("abj", (24, 50, 700), (1, 24, 1200)), level=1)
    info = tc.tc_plan_info(p)
    assert (info["m"], info["mb"], info["m_peel"], info["n_peel"]) == (1200, 592, 16, 0)
    tc.tc_destroy(p)


def test_operand_with_scattered_gathers_is_repacked():
    """Both A and B have their unit-stride index in the contracted bundle; the bundle follows A, so consecutive contracted
    entries of B lie megabytes apart: B is copied into a dense temporary first (one element-wise pass), and the
    product reads the temporary pair-wise.  no_repack keeps the gather from the caller's tensor."""
    lengths = {"e": 2, "d": 256, "a": 256, "f": 12, "g": 16, "h": 16}
    descs = []
    for idx in ("fgehd", "hgaf", "ead"):
        lens = [lengths[c] for c in idx]
        descs.append((idx, tuple(lens), tuple(workloads.col_major(lens))))
    m, n, k = 2 * 256, 256, 12 * 16 * 16
    for level, variant in ((0, "abc"), (1, "abc"), (1, "ab")):
        plan = tc.tc_plan(*descs, level, variant, None, host_only=True)
        L = tc.tc_plan_launches(plan)
        assert L[0]["kind"] == 1 and (L[0]["rows"], L[0]["cols"]) == (k, n)  # the copy of B
        fused = [l for l in L if l["kind"] == 0]
        assert fused and all(l["pairs_a"] == 1 and l["pairs_b"] == 1 for l in fused)
        plain = tc.tc_plan(*descs, level, variant, None, host_only=True, no_repack=True)
        Lp = tc.tc_plan_launches(plain)
        assert len(Lp) == len(L) - 1 and all(l["pairs_b"] == 0 for l in Lp if l["kind"] == 0)
        assert tc.tc_plan_workspace_bytes(plan) == tc.tc_plan_workspace_bytes(plain) + 8 * k * n
    # too few row tiles to pay for the copy; the stored-sum schedules keep their own temporaries
    small = dict(lengths, d=64)
    descs_small = []
    for idx in ("fgehd", "hgaf", "ead"):
        lens = [small[c] for c in idx]
        descs_small.append((idx, tuple(lens), tuple(workloads.col_major(lens))))
    assert all(l["kind"] == 0 for l in tc.tc_plan_launches(tc.tc_plan(*descs_small, 0, "abc", None, host_only=True)))
    hyb = tc.tc_plan_launches(tc.tc_plan(*descs, 1, "hybrid", None, host_only=True))
    assert not (hyb[0]["kind"] == 1 and (hyb[0]["rows"], hyb[0]["cols"]) == (k, n))
