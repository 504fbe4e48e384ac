"""GPU parity: the HIP library (through its C ABI) against the classical CPU oracle, element by element,
on seeded inputs.  Tolerance: ||C - C_ref||_F / (||A||_F ||B||_F) <= 1e-13 (level 0 and 1), 1e-12 (level 2);
small-integer inputs must agree bit for bit."""
import random

import numpy as np
import pytest

import oracle
import workloads
from workloads import from_dense, strides_for_order

pytestmark = pytest.mark.gpu

TOL = {0: 1e-13, 1: 1e-13, 2: 1e-12}
MODES = [(0, "abc"), (1, "abc"), (1, "ab"), (1, "naive"), (1, "hybrid"), (2, "abc"), (2, "ab"), (2, "naive"), (2, "hybrid")]


@pytest.fixture(scope="module")
def gpu():
    import torch

    assert torch.cuda.is_available(), "these tests need the GPU"
    import paper_1704_03092_amd as tc

    tc.load_library()
    from gpu_util import run_gpu, logical

    return run_gpu, logical


def _check(gpu, A, B, C, alpha, beta, level, variant, exact=False, **kw):
    run_gpu, logical = gpu
    ref = C.copy()
    oracle.contract_matrix(A, B, ref, alpha, beta)
    print(f"case idx={C.idx}-{A.idx}-{B.idx} lens={C.lens}/{A.lens}/{B.lens} level={level} variant={variant} a={alpha} b={beta}", flush=True)
    got_flat, info = run_gpu(A, B, C, alpha, beta, level, variant, **kw)
    got = logical(C, got_flat)
    # storage outside the tensor (padding between strides) must be untouched
    mask = np.ones(C.data.shape, dtype=bool)
    mask[(oracle.matrix_view(A, B, C)["rsC"][:, None] + oracle.matrix_view(A, B, C)["csC"][None, :]).ravel()] = False
    assert np.array_equal(got_flat[mask], C.data[mask], equal_nan=True)
    if exact:
        assert np.array_equal(got, ref.view()), (level, variant)
    else:
        err = oracle.error_metric(got, ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B))
        assert err <= TOL[info["level"]], (level, variant, err)
    return info


@pytest.mark.parametrize("level,variant", MODES)
def test_small_gemm_all_modes(gpu, level, variant):
    # spans several 128x128 tiles with ragged edges in every direction, odd sizes
    for (m, n, k) in [(300, 275, 190), (129, 130, 33), (1, 1, 1), (5, 3, 2), (257, 64, 512)]:
        c = workloads.Contraction("g", "ij", "ik", "kj", {"i": m, "j": n, "k": k}, seed=m * 7 + n)
        A, B, C = c.tensors()
        _check(gpu, A, B, C, 1.0, 1.0, level, variant)
        Ai, Bi, Ci = c.tensors(kind="smallint")
        _check(gpu, Ai, Bi, Ci, 2.0, -1.0, level, variant, exact=True)


@pytest.mark.parametrize("level,variant", MODES)
def test_alpha_beta_and_nan_poisoned_C(gpu, level, variant):
    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 200, "j": 150, "k": 100}, seed=5)
    A, B, C = c.tensors()
    _check(gpu, A, B, C, -0.75, 0.5, level, variant)
    C.data[:] = np.nan
    run_gpu, logical = gpu
    got_flat, _ = run_gpu(A, B, C, 1.5, 0.0, level, variant)
    ref = from_dense("ij", np.zeros((200, 150)))
    oracle.contract_matrix(A, B, ref, 1.5, 0.0)
    err = oracle.error_metric(logical(C, got_flat), ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B))
    assert err <= TOL[level]


def _random_case(rng, kind="uniform"):
    labels = list("abcdefghijkl")
    rng.shuffle(labels)
    nI, nJ, nP = rng.randint(0, 3), rng.randint(0, 3), rng.randint(0, 3)
    I, J, P = labels[:nI], labels[nI:nI + nJ], labels[nI + nJ:nI + nJ + nP]
    lengths = {c: rng.choice([1, 2, 3, 5, 7, 12, 17]) for c in I + J + P}
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


def _random_midsize_case(rng, kind):
    """Up to three dimensions per bundle whose lengths multiply to a few hundred .. a couple of thousand; random
    storage order and padding for every tensor."""
    labels = list("abcdefghijkl")
    rng.shuffle(labels)
    nI, nJ, nP = rng.randint(1, 3), rng.randint(1, 3), rng.randint(1, 3)
    I, J, P = labels[:nI], labels[nI:nI + nJ], labels[nI + nJ:nI + nJ + nP]
    lengths = {}
    for group, target in ((I, rng.choice([130, 300, 700, 1100])), (J, rng.choice([130, 300, 700, 1100])), (P, rng.choice([200, 900, 1700]))):
        rem = target
        for n, c in enumerate(group):
            f = rem if n == len(group) - 1 else min(rng.choice([2, 3, 4, 5, 7, 8, 12, 16, 17, 24]), rem)
            lengths[c] = max(1, f)
            rem = max(1, rem // max(1, f))
    idxA, idxB, idxC = I + P, P + J, I + J
    for s in (idxA, idxB, idxC):
        rng.shuffle(s)
    tens = []
    for tid, idx in enumerate((idxA, idxB, idxC)):
        lens = [lengths[c] for c in idx]
        order = list(range(len(idx)))
        rng.shuffle(order)
        tens.append(workloads.make_tensor("".join(idx), lengths, rng.randint(0, 10 ** 6), tid, kind, strides_for_order(lens, order, pad=rng.randint(0, 2))))
    return tens


def test_random_midsize_contractions_every_mode(gpu):
    rng = random.Random(1704)
    modes = [(l, v, {}) for (l, v) in MODES] + [(0, "abc", {"split_k": 3}), (-1, "auto", {"split_k": -1}), (1, "hybrid", {})]
    for trial in range(66):
        kind = "smallint" if trial % 2 else "uniform"
        A, B, C = _random_midsize_case(rng, kind)
        level, variant, kw = modes[trial % len(modes)]
        _check(gpu, A, B, C, rng.choice([1.0, -2.0]), rng.choice([0.0, 1.0, 3.0]), level, variant, exact=bool(trial % 2), **kw)


def test_random_contractions_random_layouts(gpu):
    rng = random.Random(2024)
    for trial in range(40):
        A, B, C = _random_case(rng, "smallint" if trial % 2 else "uniform")
        level, variant = MODES[trial % len(MODES)]
        _check(gpu, A, B, C, rng.choice([1.0, -2.0]), rng.choice([0.0, 1.0, 3.0]), level, variant, exact=bool(trial % 2))


@pytest.mark.parametrize("idxA,idxB", [("ik", "kj"), ("ki", "kj"), ("ik", "jk"), ("ki", "jk")])
def test_midsize_every_kernel_family(gpu, idxA, idxB):
    """Sizes at which the padding-free loops of the fused kernel run (several full 128 x 128 tiles and k-steps per
    Strassen block at level 2) next to ragged tiles, for the four combinations of gather direction; at levels 1 and 2
    the products cover every exact (terms of A, terms of B) kernel family.  Once with even extents (pair-wise
    gathers, 16-byte aligned), once with an odd leading dimension (pairs only 8-byte aligned), once with odd extents."""
    for (m, n, k), pad, kind in (((672, 608, 704), 0, "uniform"), ((672, 608, 704), 1, "smallint"), ((645, 583, 657), 0, "uniform")):
        lengths = {"i": m, "j": n, "k": k}
        tens = []
        for tid, idx in enumerate((idxA, idxB, "ij")):
            lens = [lengths[c] for c in idx]
            st = strides_for_order(lens, list(range(len(idx))), pad=pad)
            tens.append(workloads.make_tensor(idx, lengths, 77 + tid, tid, kind, st))
        A, B, C = tens
        for level, variant in ((0, "abc"), (1, "abc"), (2, "abc"), (1, "naive"), (2, "ab"), (1, "hybrid"), (2, "hybrid")):
            _check(gpu, A, B, C, 1.0, 1.0, level, variant, exact=(kind == "smallint"))


def test_general_strides_two_levels_one_product_per_launch(gpu):
    """A 6-D contraction whose A has an odd fastest dimension (gathered element by element) and whose B is gathered
    pair-wise along the contracted bundle; block extents 272 x 32 x 432 at two levels, so that every launch has three
    ragged tiles and the last contracted block is shorter than the others.  Run with one product per launch, with
    the tail cut into chunks of 64 contracted entries, and through the AB temporaries: small integers, bit for bit."""
    L = {"d": 12, "g": 18, "j": 106, "h": 16, "k": 5, "i": 3, "b": 5, "f": 8}
    A = workloads.make_tensor("dgjhk", L, 41, 0, "smallint", (183168, 10176, 96, 6, 1))
    B = workloads.make_tensor("ibhjf", L, 42, 1, "smallint", (17, 51, 1, 255, 27030))
    C = workloads.make_tensor("gdbifk", L, 43, 2, "smallint", (10080, 35, 7, 420, 1260, 1))
    for level, variant, kw in ((2, "abc", {}), (2, "abc", {"tail_split": -1, "no_merge": True}), (2, "ab", {"tail_split": -1}),
                               (2, "abc", {"tail_split": 5}), (1, "abc", {"tail_split": -1, "no_merge": True}), (2, "hybrid", {})):
        for rep in range(2):
            _check(gpu, A, B, C, -2.0, 0.0, level, variant, exact=True, **kw)


def test_tiles_gathered_by_stride_next_to_tiles_through_the_tables(gpu):
    """Contractions whose row bundle is no single constant-stride run: the kernel reads the block scatter vectors and
    gathers a tile by stride where all its 16-entry blocks are regular and join up (Sec. 4.1 "Packing"), through the
    scatter tables elsewhere, within one launch.  Lengths 128 (every tile regular), 192 (two tiles of three), 24 and 48
    (none); small integers, bit for bit; the launch info reports the split."""
    import torch

    import paper_1704_03092_amd as tc

    cases = [  # lengths, padding after the fastest dimension of A, gap between B's slices, tiles gathered by stride at level 0 (of how many)
        (dict(a=128, b=4, c=128, d=2, e=64), 0, 0, (8, 8)),
        (dict(a=128, b=4, c=128, d=2, e=64), 6, 0, (8, 8)),
        (dict(a=192, b=4, c=128, d=2, e=64), 0, 0, (8, 12)),
        (dict(a=192, b=4, c=192, d=2, e=128), 0, 0, (12, 18)),  # rows: four of six tiles regular; B is one run as a whole
        (dict(a=192, b=4, c=192, d=2, e=128), 0, 5, (8, 18)),   # B's slices d apart from each other: two of three column tiles regular
        (dict(a=24, b=16, c=48, d=8, e=64), 0, 0, (0, 9)),
        (dict(a=128, b=5, c=128, d=3, e=96), 0, 0, (0, 15)),     # k = 96 is no even number of 32-deep steps: zero padding in every tile
    ]
    st = torch.cuda.current_stream()
    for L, pad, gap, (free, total) in cases:
        lensA = [L[x] for x in "aeb"]
        A = workloads.make_tensor("aeb", L, 61, 0, "smallint", strides_for_order(lensA, [0, 1, 2], pad=pad))
        B = workloads.make_tensor("ecd", L, 62, 1, "smallint", (1, L["e"], L["e"] * (L["c"] + gap)))
        C = workloads.make_tensor("abcd", L, 63, 2, "smallint")
        plan = tc.tc_plan(A, B, C, 0, "abc", st, tail_split=-1, tile_n=128)
        fused = [x for x in tc.tc_plan_launches(plan) if x["kind"] == 0]
        tc.tc_destroy(plan)
        assert [(x["tiles_table_free"], x["tiles"]) for x in fused] == [(free, total)], (L, pad, gap)
        for level, variant, kw in ((0, "abc", {"tile_n": 128}), (0, "abc", {"tile_n": 64}), (0, "abc", {"tail_split": 2}), (1, "abc", {}), (2, "abc", {}),
                                   (1, "hybrid", {}), (1, "ab", {})):
            _check(gpu, A, B, C, 2.0, -1.0, level, variant, exact=True, **kw)


def test_automatic_level_and_variant(gpu):
    """TC_LEVEL_AUTO / TC_VARIANT_AUTO: whatever the model picks, the result is the contraction."""
    import paper_1704_03092_amd as tc

    for lengths in ({"i": 300, "j": 260, "k": 90}, {"i": 1500, "j": 1400, "k": 1300}):
        c = workloads.Contraction("g", "ij", "ik", "kj", lengths, seed=9)
        A, B, C = c.tensors()
        info = _check(gpu, A, B, C, 1.0, 1.0, tc.TC_LEVEL_AUTO, "auto")
        assert info["level"] in (0, 1, 2) and info["variant"] in (0, 1, 2) and info["level_requested"] == info["level"]


def test_split_k(gpu):
    """Level 0 with the contracted bundle cut into chunks (temporaries + one summing pass), also through general strides."""
    cfg = workloads.scaled(workloads.configs()["cfg4a"], {"a": 13, "b": 21, "c": 12, "d": 37, "e": 19})  # k = 703
    for kind in ("uniform", "smallint"):
        A, B, C = cfg.tensors(kind=kind)
        for split in (2, 3, 4, -1):
            info = _check(gpu, A, B, C, 1.5, -0.5, 0, "abc", exact=(kind == "smallint"), split_k=split)
            assert split == -1 or info["n_products"] == split
    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 300, "j": 96, "k": 1000}, seed=3)
    A, B, C = c.tensors()
    C.data[:] = np.nan  # beta = 0 must not read C
    run_gpu, logical = gpu
    got_flat, info = run_gpu(A, B, C, 2.0, 0.0, 0, "abc", split_k=4)
    ref = from_dense("ij", np.zeros((300, 96)))
    oracle.contract_matrix(A, B, ref, 2.0, 0.0)
    assert info["n_products"] == 4
    assert oracle.error_metric(logical(C, got_flat), ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B)) <= TOL[0]


@pytest.mark.parametrize("idxA,idxB,idxC", [("ik", "kj", "ij"), ("ki", "jk", "ji"), ("ki", "kj", "ij"), ("ik", "jk", "ji")])
def test_tail_split_every_mode(gpu, idxA, idxB, idxC):
    """Forced tail split: every tile of these launches is a tail tile (fewer tiles than compute units), cut into 2, 3
    or 5 chunks along the contracted bundle; the chunks are added by the second kernel.  Gather directions and the
    destination's contiguous direction in all combinations, ragged tiles, Strassen padding, every variant; small
    integers must agree bit for bit (the chunk sums are exact there)."""
    import paper_1704_03092_amd as tc

    for (m, n, k), pad, kind in (((672, 608, 1408), 0, "uniform"), ((645, 583, 1111), 1, "smallint")):
        lengths = {"i": m, "j": n, "k": k}
        tens = []
        for tid, idx in enumerate((idxA, idxB, idxC)):
            lens = [lengths[c] for c in idx]
            tens.append(workloads.make_tensor(idx, lengths, 31 + tid, tid, kind, strides_for_order(lens, list(range(len(idx))), pad=pad)))
        A, B, C = tens
        for (level, variant), chunks in zip(MODES, (2, 3, 5, 2, 3, 5, 2, 3, 5)):
            _check(gpu, A, B, C, 1.5, 0.5, level, variant, exact=(kind == "smallint"), tail_split=chunks)
    # the plan really splits: every tile, in as many chunks as asked for
    st = __import__("torch").cuda.current_stream()
    plan = tc.tc_plan(A, B, C, 1, "abc", st, tail_split=3)
    fused = [L for L in tc.tc_plan_launches(plan) if L["kind"] == 0]
    assert fused and all(L["tail_tiles"] == L["tiles"] and L["tail_chunks"] == 3 for L in fused)
    tc.tc_destroy(plan)


def test_tail_split_whole_and_split_tiles_together(gpu):
    """More tiles than compute units: whole tiles and chunks of tail tiles in one launch (300 = 256 + 44 tiles at
    level 0; the Strassen products have 80 tiles each), the automatic choice next to forced ones, general strides,
    beta = 0 on a NaN-filled C."""
    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 2500, "j": 1850, "k": 900}, seed=21)
    A, B, C = c.tensors()
    for level, variant, chunks in ((0, "abc", 2), (0, "abc", 4), (0, "abc", 0), (1, "abc", 3), (1, "hybrid", 2), (2, "abc", 2), (1, "ab", 0)):
        _check(gpu, A, B, C, -1.0, 2.0, level, variant, tail_split=chunks)
    Ai, Bi, Ci = c.tensors(kind="smallint")
    _check(gpu, Ai, Bi, Ci, 2.0, -1.0, 0, "abc", exact=True, tail_split=3)
    C.data[:] = np.nan
    run_gpu, logical = gpu
    got_flat, _ = run_gpu(A, B, C, 1.5, 0.0, 0, "abc", tail_split=3)
    ref = from_dense("ij", np.zeros((2500, 1850)))
    oracle.contract_matrix(A, B, ref, 1.5, 0.0)
    assert oracle.error_metric(logical(C, got_flat), ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B)) <= TOL[0]
    cfg = workloads.scaled(workloads.configs()["cfg4a"], {"a": 40, "b": 21, "c": 38, "d": 37, "e": 19})  # m = 1520, n = 21, k = 703
    A, B, C = cfg.tensors()
    for chunks in (2, 4, 11):
        _check(gpu, A, B, C, 1.0, 1.0, 0, "abc", tail_split=chunks)
    rng = random.Random(99)
    for trial in range(12):
        kind = "smallint" if trial % 2 else "uniform"
        A, B, C = _random_midsize_case(rng, kind)
        level, variant = MODES[trial % len(MODES)]
        _check(gpu, A, B, C, rng.choice([1.0, -2.0]), rng.choice([0.0, 1.0, 3.0]), level, variant, exact=bool(trial % 2), tail_split=rng.choice([2, 3, 7]))


@pytest.mark.parametrize("tile_n", [64, 128])
def test_both_tile_shapes_of_single_block_products(gpu, tile_n):
    """Products with single-block operand sums (level 0, Naive, the stored-sum variant at one level) run in 128 x 128
    or in 128 x 64 tiles.  Both shapes forced in turn: ragged GEMMs in the four gather directions and both
    destination orders, padded leading dimensions, random general-stride contractions, forced and automatic tail
    splits with whole and split tiles in one launch, the tiles gathered by stride next to those through the tables,
    beta = 0 over NaN.  Launches with multi-block sums keep 128 columns."""
    import paper_1704_03092_amd as tc

    run_gpu, logical = gpu
    for idxA, idxB, idxC in (("ik", "kj", "ij"), ("ki", "jk", "ji"), ("ki", "kj", "ij"), ("ik", "jk", "ji")):
        for (m, n, k), pad, kind in (((672, 608, 704), 0, "uniform"), ((645, 583, 657), 1, "smallint"), ((130, 65, 48), 0, "smallint"),
                                     ((128, 64, 32), 0, "smallint"), ((1, 1, 1), 0, "uniform")):
            lengths = {"i": m, "j": n, "k": k}
            tens = []
            for tid, idx in enumerate((idxA, idxB, idxC)):
                lens = [lengths[c] for c in idx]
                tens.append(workloads.make_tensor(idx, lengths, 11 + tid, tid, kind, strides_for_order(lens, list(range(len(idx))), pad=pad)))
            A, B, C = tens
            for level, variant, kw in ((0, "abc", {}), (0, "abc", {"tail_split": 3}), (1, "naive", {}), (1, "hybrid", {"tail_split": 2}), (2, "naive", {}),
                                       (1, "abc", {})):
                _check(gpu, A, B, C, 1.5, 0.5, level, variant, exact=(kind == "smallint"), tile_n=tile_n, **kw)
    # what the plan reports
    st = __import__("torch").cuda.current_stream()
    for level, variant in ((0, "abc"), (1, "hybrid"), (1, "abc")):
        plan = tc.tc_plan(A, B, C, level, variant, st, tile_n=tile_n)
        for L in tc.tc_plan_launches(plan):
            if L["kind"] == 0:
                assert L["tile_n"] == (tile_n if (L["terms_a"], L["terms_b"]) == (1, 1) else 128), L
        tc.tc_destroy(plan)
    # more tiles than one round: whole and split tiles in one launch; beta = 0 on a NaN-filled C
    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 2500, "j": 1850, "k": 900}, seed=21)
    A, B, C = c.tensors()
    for level, variant, chunks in ((0, "abc", 2), (0, "abc", 0), (0, "abc", -1), (1, "hybrid", 3), (1, "naive", 0)):
        _check(gpu, A, B, C, -1.0, 2.0, level, variant, tail_split=chunks, tile_n=tile_n)
    Ai, Bi, Ci = c.tensors(kind="smallint")
    _check(gpu, Ai, Bi, Ci, 2.0, -1.0, 0, "abc", exact=True, tail_split=3, tile_n=tile_n)
    C.data[:] = np.nan
    got_flat, _ = run_gpu(A, B, C, 1.5, 0.0, 0, "abc", tail_split=3, tile_n=tile_n)
    ref = from_dense("ij", np.zeros((2500, 1850)))
    oracle.contract_matrix(A, B, ref, 1.5, 0.0)
    assert oracle.error_metric(logical(C, got_flat), ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B)) <= TOL[0]
    # general strides
    rng = random.Random(640 + tile_n)
    for trial in range(24):
        kind = "smallint" if trial % 2 else "uniform"
        A, B, C = _random_midsize_case(rng, kind)
        level, variant = ((0, "abc"), (1, "naive"), (1, "hybrid"), (2, "hybrid"))[trial % 4]
        _check(gpu, A, B, C, rng.choice([1.0, -2.0]), rng.choice([0.0, 1.0, 3.0]), level, variant, exact=bool(trial % 2),
               tail_split=rng.choice([0, 0, 2, 5]), tile_n=tile_n)
    # tiles gathered by stride (rows a + 128 b: every tile of A regular) and the rank-k shape at reduced extents
    L = dict(a=128, b=3, c=64, d=5, e=96)
    cm = lambda idx: strides_for_order([L[x] for x in idx], list(range(len(idx))), pad=0)
    A = workloads.make_tensor("aeb", L, 3, 0, "smallint", cm("aeb"))
    B = workloads.make_tensor("ecd", L, 3, 1, "smallint", cm("ecd"))
    C = workloads.make_tensor("abcd", L, 3, 2, "smallint", cm("abcd"))
    plan = tc.tc_plan(A, B, C, 0, "abc", st, tail_split=-1, tile_n=tile_n)
    (launch,) = [x for x in tc.tc_plan_launches(plan) if x["kind"] == 0]
    tc.tc_destroy(plan)
    # 384 x 320 x 96: with 64 columns every tile is whole and 96 is a whole, even number of its k-steps of 16
    assert (launch["tiles"], launch["tiles_table_free"]) == ((15, 15) if tile_n == 64 else (9, 0))
    for kw in ({}, {"tail_split": 3}):
        _check(gpu, A, B, C, 1.0, 1.0, 0, "abc", exact=True, tile_n=tile_n, **kw)


@pytest.mark.parametrize("no_peel", [False, True])
def test_sizes_that_the_block_grid_does_not_divide(gpu, no_peel):
    """Sec. 3, last paragraph: dynamic peeling (classical edge products for the rows and columns beyond the largest
    whole number of equal blocks) and zero padding (no_peel) give the classical result; odd extents in every bundle,
    every variant, both levels, general strides, beta = 0 over NaN in the peeled part."""
    import paper_1704_03092_amd as tc

    run_gpu, logical = gpu
    st = __import__("torch").cuda.current_stream()
    for (m, n, k), kind in (((645, 583, 657), "smallint"), ((1031, 517, 300), "uniform"), ((519, 1290, 129), "smallint")):
        c = workloads.Contraction("g", "ij", "ik", "kj", {"i": m, "j": n, "k": k}, seed=m + n)
        A, B, C = c.tensors(kind=kind)
        for level, variant in MODES[1:]:
            _check(gpu, A, B, C, 1.5, 0.5, level, variant, exact=(kind == "smallint"), no_peel=no_peel)
        plan = tc.tc_plan(A, B, C, 1, "abc", st, no_peel=no_peel)
        info = tc.tc_plan_info(plan)
        tc.tc_destroy(plan)
        assert (info["m_peel"] > 0 or info["n_peel"] > 0) == (not no_peel)
        C.data[:] = np.nan
        got_flat, _ = run_gpu(A, B, C, 2.0, 0.0, 2, "abc", no_peel=no_peel)
        ref = from_dense("ij", np.zeros((m, n)))
        oracle.contract_matrix(A, B, ref, 2.0, 0.0)
        assert oracle.error_metric(logical(C, got_flat), ref.view(), oracle.tensor_norm(A), oracle.tensor_norm(B)) <= TOL[2]
    # tensor-shaped: rows a + 24 b (read through the block scatter vector: blocks in multiples of 16, 16 rows peeled)
    L = dict(a=24, b=50, c=30, d=23, e=40, f=9)
    A = workloads.make_tensor("aebf", L, 7, 0, "smallint")
    B = workloads.make_tensor("fdec", L, 7, 1, "smallint")
    C = workloads.make_tensor("abcd", L, 7, 2, "smallint")
    for level, variant in ((1, "abc"), (1, "hybrid"), (2, "abc"), (1, "ab")):
        _check(gpu, A, B, C, 1.0, 1.0, level, variant, exact=True, no_peel=no_peel)


@pytest.mark.parametrize("no_repack", [False, True])
def test_operand_repacked_into_a_dense_temporary(gpu, no_repack):
    # A and B both have their unit-stride index in the contracted bundle, which follows A: B's gathers are scattered
    # and B is copied into a dense temporary first (unless told not to).  Small integers: bit for bit.
    c = workloads.Contraction("hostile", "ead", "fgehd", "hgaf", {"e": 2, "d": 260, "a": 200, "f": 8, "g": 16, "h": 16}, seed=77)
    run_gpu, logical = gpu
    for level, variant in [(0, "abc"), (1, "abc"), (1, "ab"), (2, "abc")]:
        A, B, C = c.tensors(kind="smallint")
        info = _check(gpu, A, B, C, 2.0, -1.0, level, variant, exact=True, no_repack=no_repack)
        A, B, C = c.tensors()
        _check(gpu, A, B, C, 0.5, 1.0, level, variant, no_repack=no_repack)
    import paper_1704_03092_amd as tc

    A, B, C = c.tensors()
    plan = tc.tc_plan(A, B, C, 0, "abc", None, host_only=True, no_repack=no_repack)
    kinds = [l["kind"] for l in tc.tc_plan_launches(plan)]
    assert kinds == ([0] if no_repack else [1, 0])


def test_operand_without_a_unit_stride_is_repacked(gpu):
    # A is every 16th element of a larger array along both of its indices (no unit-stride index at all: each gathered
    # element has a memory line of its own) and is read by 5 column tiles: copied into a dense temporary first.  B has
    # the same layout but is read by 2 row tiles only and stays where it is.
    L = {"i": 200, "k": 150, "j": 600}
    run_gpu, logical = gpu
    import paper_1704_03092_amd as tc

    for kind, exact in (("smallint", True), ("uniform", False)):
        A = workloads.make_tensor("ik", L, 5, 0, kind, (16, 16 * 200 + 48))
        B = workloads.make_tensor("kj", L, 6, 1, kind, (16, 16 * 150))
        C = workloads.make_tensor("ij", L, 7, 2, kind)
        for level, variant in [(0, "abc"), (1, "abc"), (1, "ab")]:
            _check(gpu, A, B, C, -1.0, 2.0, level, variant, exact=exact)
            _check(gpu, A, B, C, -1.0, 2.0, level, variant, exact=exact, no_repack=True)
    launches = tc.tc_plan_launches(tc.tc_plan(A, B, C, 0, "abc", None, host_only=True))
    assert [(l["kind"], l["rows"], l["cols"]) for l in launches[:1]] == [(1, 200, 150)] and len(launches) == 2
    assert launches[1]["pairs_a"] == 1 and launches[1]["pairs_b"] == 0


def test_column_stride_beyond_the_table_free_limit(gpu):
    """Plain matrices whose column stride is 2^20 + 8 elements: the table-free gather (strides below 2^20 only) must
    step aside for the gather through the scatter tables; full tiles, several k-steps, every family at level 1."""
    ld = (1 << 20) + 8
    m, n, k = 256, 160, 128
    A = workloads.make_tensor("ik", {"i": m, "k": k}, 5, 0, "smallint", (1, ld))
    B = workloads.make_tensor("kj", {"k": k, "j": n}, 5, 1, "smallint", (1, k))
    C = workloads.make_tensor("ij", {"i": m, "j": n}, 5, 2, "smallint", (1, m))
    for level, variant in ((0, "abc"), (1, "abc"), (1, "hybrid")):
        _check(gpu, A, B, C, 1.0, 1.0, level, variant, exact=True)


def test_results_are_reproducible(gpu):
    """No floating-point atomics anywhere: the same plan gives the same bits on every call, also with the tail of a
    launch cut into chunks and with the contracted bundle split."""
    import torch

    import paper_1704_03092_amd as tc
    from gpu_util import to_dev

    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 2500, "j": 1850, "k": 900}, seed=33)
    A, B, C = c.tensors()
    st = torch.cuda.current_stream()
    dA, dB = to_dev(A), to_dev(B)
    for level, variant, kw in ((0, "abc", {"tail_split": 4}), (1, "abc", {}), (1, "hybrid", {"tail_split": 3}), (2, "ab", {}), (0, "abc", {"split_k": 3})):
        plan = tc.tc_plan(A, B, C, level, variant, st, **kw)
        ws = torch.empty(max(tc.tc_plan_workspace_bytes(plan) // 8, 1), dtype=torch.float64, device="cuda")
        outs = []
        for _ in range(3):
            dC = to_dev(C)
            ws.fill_(float("nan"))
            tc.tc_contract(plan, 1.25, dA, dB, 0.5, dC, ws, st)
            torch.cuda.synchronize()
            outs.append(dC)
        tc.tc_destroy(plan)
        assert torch.equal(outs[0], outs[1]) and torch.equal(outs[0], outs[2]), (level, variant, kw)


def test_contract_timed_matches_contract(gpu):
    """tc_contract_timed enqueues the same launches: identical bits, and it counts the launches per kind."""
    import torch

    import paper_1704_03092_amd as tc
    from gpu_util import to_dev

    c = workloads.Contraction("g", "ij", "ik", "kj", {"i": 512, "j": 384, "k": 260}, seed=11)  # (whole tiles per block: no rows or columns to peel)
    A, B, C = c.tensors()
    st = torch.cuda.current_stream()
    for level, variant, fused, other in ((0, "abc", 1, 0), (1, "abc", 4, 0), (1, "hybrid", 7, 10), (1, "naive", 7, 21)):
        plan = tc.tc_plan(A, B, C, level, variant, st)
        nbytes = tc.tc_plan_workspace_bytes(plan)
        ws = torch.zeros(max(nbytes // 8, 1), dtype=torch.float64, device="cuda")
        dA, dB, dC1, dC2 = to_dev(A), to_dev(B), to_dev(C), to_dev(C)
        tc.tc_contract(plan, 1.25, dA, dB, 0.5, dC1, ws, st)
        times = tc.tc_contract_timed(plan, 1.25, dA, dB, 0.5, dC2, ws, st)
        torch.cuda.synchronize()
        tc.tc_destroy(plan)
        assert torch.equal(dC1, dC2)
        assert (times["fused_launches"], times["elementwise_launches"]) == (fused, other)
        assert times["fused_ms"] > 0 and times["elementwise_ms"] >= 0


def test_benchmark_index_strings_reduced_sizes(gpu):
    cfgs = workloads.configs()
    small = {
        "cfg1": {x: 5 for x in "abcdef"},
        "cfg3": {"a": 12, "b": 11, "e": 13, "f": 9, "i": 6, "j": 7},
        "cfg4a": {"a": 13, "b": 21, "c": 12, "d": 17, "e": 9},
        "cfg4b": {"a": 18, "b": 9, "c": 11, "d": 14, "e": 40},
        "cfg5": {"a": 6, "b": 5, "c": 7, "d": 4, "e": 6, "f": 5, "g": 11, "h": 9},
    }
    for name, L in small.items():
        cfg = workloads.scaled(cfgs[name], L)
        for level, variant in [(0, "abc"), (1, "abc"), (1, "ab"), (2, "abc"), (2, "naive"), (2, "hybrid")]:
            for layout in ("col", "row"):
                A, B, C = cfg.tensors(layout=layout)
                _check(gpu, A, B, C, cfg.alpha, cfg.beta, level, variant)


def test_planner_vectors_match_oracle_and_paper_example(gpu):
    import torch
    import paper_1704_03092_amd as tc

    # the paper's example, block size 4
    L = dict(a=4, b=8, c=2, d=8)
    A = workloads.make_tensor("dca", L, 1, 0)
    B = workloads.make_tensor("db", L, 1, 1)
    C = workloads.make_tensor("abc", L, 1, 2)
    p = tc.tc_plan(A, B, C, 0, "abc", torch.cuda.current_stream(), bs_block=4)
    info = tc.tc_plan_info(p)
    assert info["I"] == "ac" and info["J"] == "b" and info["P"] == "d"
    rsC, csC = tc.tc_plan_vector(p, 4), tc.tc_plan_vector(p, 5)
    assert rsC[6] == 34 and csC[3] == 12  # LOC(C_{2,3,1}) = 34 + 12
    assert list(rsC) == [0, 1, 2, 3, 32, 33, 34, 35]
    assert list(tc.tc_plan_vector(p, 10)) == [1, 1] and list(tc.tc_plan_vector(p, 11)) == [4, 4]  # rbs_C, cbs_C
    tc.tc_destroy(p)
    # random tensors: all twelve vectors equal the oracle's, using the bundle orders the plan chose
    rng = random.Random(77)
    for _ in range(10):
        A, B, C = _random_case(rng)
        bs = rng.choice([1, 3, 4, 16])
        p = tc.tc_plan(A, B, C, 0, "abc", torch.cuda.current_stream(), bs_block=bs)
        info = tc.tc_plan_info(p)
        v = oracle.matrix_view(A, B, C, orders=(list(info["I"]), list(info["J"]), list(info["P"])))
        for which, key in enumerate(["rsA", "csA", "rsB", "csB", "rsC", "csC"]):
            got = tc.tc_plan_vector(p, which)
            assert np.array_equal(got, v[key]), key
            assert np.array_equal(tc.tc_plan_vector(p, 6 + which), oracle.block_scatter(v[key], bs)), key
        tc.tc_destroy(p)


def test_degenerate_shapes(gpu):
    run_gpu, logical = gpu
    # empty contracted bundle: outer product; empty free bundles: dot product; k = 0: C := beta C; m = 0: no-op
    A = workloads.make_tensor("i", {"i": 37}, 1, 0)
    B = workloads.make_tensor("j", {"j": 41}, 1, 1)
    C = workloads.make_tensor("ij", {"i": 37, "j": 41}, 1, 2)
    _check(gpu, A, B, C, 2.0, 1.0, 0, "abc")
    _check(gpu, A, B, C, 2.0, 1.0, 1, "ab")
    A = workloads.make_tensor("k", {"k": 1000}, 2, 0)
    B = workloads.make_tensor("k", {"k": 1000}, 2, 1)
    C = workloads.make_tensor("", {}, 2, 2)
    _check(gpu, A, B, C, 1.0, 0.5, 0, "abc")
    _check(gpu, A, B, C, 1.0, 0.5, 2, "abc")
    A = workloads.make_tensor("ik", {"i": 9, "k": 0}, 3, 0)
    B = workloads.make_tensor("kj", {"j": 8, "k": 0}, 3, 1)
    C = workloads.make_tensor("ij", {"i": 9, "j": 8}, 3, 2)
    got, _ = run_gpu(A, B, C, 1.0, -2.0, 1, "abc")
    assert np.array_equal(got, -2.0 * C.data)
    got, _ = run_gpu(A, B, C, 1.0, 0.0, 0, "abc")
    assert np.array_equal(got, np.zeros_like(C.data))
    A = workloads.make_tensor("ik", {"i": 0, "k": 5}, 3, 0)
    B = workloads.make_tensor("kj", {"j": 8, "k": 5}, 3, 1)
    C = workloads.make_tensor("ij", {"i": 0, "j": 8}, 3, 2)
    got, info = run_gpu(A, B, C, 1.0, 1.0, 1, "naive")
    assert info["n_launches"] == 0
