"""Pins of the oracle planner against what the paper and the mathematics fix.

None of these re-types the oracle's loop nest: they count coverage of the
(i, k, j) iteration space by brute force, compare with closed forms and with
textbook block algorithms, and show that plausible mistakes are caught.
"""
import os

import numpy as np
import pytest

import workloads
from oracle import planner
from oracle.planner import DistMatrix, PlanError, Task
from oracle import execute as oexec
from tests import helpers
from tests.helpers import dist

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _plan(prob):
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    return planner.plan(A, B, C, prob["nranks"]), A, B, C


# --- brute force: exactly-once coverage, shares, extents, ownership, count ----

@pytest.mark.parametrize("seed", range(120))
def test_random_small_problems_cover_iteration_space_once(seed):
    prob = helpers.random_problem(seed)
    tasks, A, B, C = _plan(prob)
    helpers.check_task_list(tasks, A, B, C, prob["nranks"])


@pytest.mark.parametrize("seed", range(1000, 1040))
def test_random_small_problems_with_empty_tiles(seed):
    prob = helpers.random_problem(seed, allow_empty=True)
    tasks, A, B, C = _plan(prob)
    helpers.check_task_list(tasks, A, B, C, prob["nranks"])


def test_all_replication_combinations_p8():
    """Section 4.2: any combination of replication factors of A, B and C works
    unchanged.  All 4^3 divisor triples of p = 8 on misaligned 1-D/2-D grids."""
    p, M, K, N = 8, 12, 16, 10
    for cA in helpers.divisors(p):
        for cB in helpers.divisors(p):
            for cC in helpers.divisors(p):
                A = DistMatrix(M, K, (0, 5, 12), (0, 7, 16), 1, 1, cA)
                B = DistMatrix(K, N, (0, 3, 9, 16), (0, 10), 1, 1, cB)
                C = DistMatrix(M, N, (0, 4, 12), (0, 6, 10), 1, 1, cC)
                tasks = planner.plan(A, B, C, p)
                helpers.check_task_list(tasks, A, B, C, p)


# --- textbook special cases -----------------------------------------------------

@pytest.mark.parametrize("g", [1, 2, 3, 4])
def test_aligned_2d_grid_is_summa_block_products(g):
    """Aligned g x g grids, no replication (the 'traditional' case of Section
    5.2): the ops are the g^3 block products A(i,l) B(l,j) of SUMMA / Cannon
    (Section 2.1), g of them on the rank that owns C(i,j), l ascending."""
    n = 6 * g
    cuts = tuple(range(0, n + 1, 6))
    X = DistMatrix(n, n, cuts, cuts, g, g, 1)
    tasks = planner.plan(X, X, X, g * g)
    assert len(tasks) == g ** 3
    want = []
    for i in range(g):
        for j in range(g):
            for l in range(g):
                want.append(Task(i * g + j, 0, i, l, 0, l, j, 0, i, j,
                                 6 * i, 6 * i + 6, 6 * l, 6 * l + 6, 6 * j, 6 * j + 6))
    assert tasks == want


def test_inner_product_1d():
    """A row-block, B column-block, C 2-D (inner-product style, Section 2.2):
    C(i,j) = A(i,:) B(:,j), one op per C tile spanning all of k."""
    p, n = 4, 8
    A = DistMatrix(n, n, (0, 4, 8), (0, 8), 2, 1, 1)
    B = DistMatrix(n, n, (0, 8), (0, 4, 8), 1, 2, 1)
    C = DistMatrix(n, n, (0, 4, 8), (0, 4, 8), 2, 2, 1)
    tasks = planner.plan(A, B, C, p)
    assert tasks == [Task(2 * i + j, 0, i, 0, 0, 0, j, 0, i, j, 4 * i, 4 * i + 4, 0, 8, 4 * j, 4 * j + 4)
                     for i in range(2) for j in range(2)]


def test_outer_product_1d_replicated_c():
    """A column-block, B row-block, C replicated on every rank (outer-product /
    Megatron-style second MLP matmul, Section 2.2): rank r computes the partial
    product A(:, r-th k block) B(r-th k block, :) into its own copy of C."""
    p, n = 4, 8
    A = DistMatrix(n, n, (0, 8), (0, 2, 4, 6, 8), 1, 4, 1)
    B = DistMatrix(n, n, (0, 2, 4, 6, 8), (0, 8), 4, 1, 1)
    C = DistMatrix(n, n, (0, 8), (0, 8), 1, 1, p)
    tasks = planner.plan(A, B, C, p)
    assert tasks == [Task(r, 0, 0, r, 0, r, 0, r, 0, 0, 0, 8, 2 * r, 2 * r + 2, 0, 8) for r in range(p)]


# --- values the paper prints ------------------------------------------------------

def test_replication_example_p12():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "replication_p12.txt")) if not l.startswith("#")]
    for r in rows:
        p, c = int(r[0]), int(r[1])
        D = DistMatrix(24, 24, (0, 24), (0, 24), 1, 1, c)
        if r[2] == "rejected":
            with pytest.raises(PlanError) as e:
                D.validate(p)
            assert e.value.kind == "EREPL"
        else:
            D.validate(p)
            copies, per = int(r[2]), int(r[3])
            assert D.ranks_per_replica(p) == per
            assert sorted({D.replica_of(rank, p) for rank in range(p)}) == list(range(copies))
            for rep in range(copies):
                assert sum(D.replica_of(rank, p) == rep for rank in range(p)) == per


def test_benchmark_config_counts():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "task_counts.txt")) if not l.startswith("#")]
    assert [r[0] for r in rows] == list(workloads.CONFIG_NAMES)
    for name, ntasks, ngroups in rows:
        cfg = workloads.config(name)
        tasks, A, B, C = _plan(cfg)
        order, offsets = planner.reorder(tasks)
        assert len(tasks) == int(ntasks)
        assert len(offsets) - 1 == int(ngroups)
        helpers.check_reorder(tasks, order, offsets, C)


@pytest.mark.parametrize("name,dims", [("cfg1", (16, 16, 16)), ("cfg2", (32, 24, 32)), ("cfg3", (16, 8, 32)),
                                       ("cfg4", (24, 24, 24)), ("cfg5", (45, 50, 40))])
def test_benchmark_families_small(name, dims):
    """The five partitioning families at sizes the 3-D counter can hold."""
    cfg = workloads.scaled_config(name, *dims)
    tasks, A, B, C = _plan(cfg)
    helpers.check_task_list(tasks, A, B, C, cfg["nranks"])


def test_cfg4_replica_shares():
    """2.5D: replica r of C works on k in [4096 r, 4096 (r+1))."""
    cfg = workloads.config("cfg4")
    tasks, A, B, C = _plan(cfg)
    for t in tasks:
        assert t.c_rep == t.rank // 16 and 4096 * t.c_rep <= t.k0 < t.k1 <= 4096 * (t.c_rep + 1)
        assert (t.m1 - t.m0, t.k1 - t.k0, t.n1 - t.n0) == (2048, 2048, 2048)
    assert sum((t.m1 - t.m0) * (t.k1 - t.k0) * (t.n1 - t.n0) for t in tasks) == 8192 ** 3


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_full_size_configs_volume_and_disjointness(name):
    """At full size the 3-D counter does not fit; check instead that the boxes'
    volume is M K N and that boxes are pairwise disjoint (which together mean
    exactly-once coverage)."""
    cfg = workloads.config(name)
    tasks, A, B, C = _plan(cfg)
    assert sum((t.m1 - t.m0) * (t.k1 - t.k0) * (t.n1 - t.n0) for t in tasks) == cfg["M"] * cfg["K"] * cfg["N"]
    for a in range(len(tasks)):
        for b in range(a + 1, len(tasks)):
            s, t = tasks[a], tasks[b]
            apart = (s.m1 <= t.m0 or t.m1 <= s.m0 or s.k1 <= t.k0 or t.k1 <= s.k0
                     or s.n1 <= t.n0 or t.n1 <= s.n0)
            assert apart, f"tasks {a} and {b} overlap"


# --- primitives of Table 1 ------------------------------------------------------

def test_tile_bounds_and_overlapping_tiles_bruteforce():
    rng = np.random.default_rng(7)
    for _ in range(50):
        rows, cols = int(rng.integers(1, 20)), int(rng.integers(1, 20))
        d = helpers.random_matrix_desc(rng, rows, cols, 4)
        D = dist(d)
        owner_of = -np.ones((rows, cols), dtype=np.int64)
        gr, gc = D.grid_shape()
        for ti in range(gr):
            for tj in range(gc):
                (r0, r1), (c0, c1) = D.tile_bounds((ti, tj))
                assert (owner_of[r0:r1, c0:c1] == -1).all()
                owner_of[r0:r1, c0:c1] = ti * gc + tj
        assert (owner_of >= 0).all()          # tiles partition the matrix
        r0, r1 = sorted(int(x) for x in rng.integers(0, rows + 1, size=2))
        c0, c1 = sorted(int(x) for x in rng.integers(0, cols + 1, size=2))
        got = D.overlapping_tiles(((r0, r1), (c0, c1)))
        want = sorted({(int(v) // gc, int(v) % gc) for v in np.unique(owner_of[r0:r1, c0:c1])})
        assert got == want


def test_block_cyclic_ownership():
    """ScaLAPACK convention (Section 2.1): tile (ti, tj) goes to process
    (ti mod P_r, tj mod P_c) of a row-major P_r x P_c grid."""
    D = DistMatrix(8, 8, tuple(range(9)), tuple(range(9)), 2, 3, 2)
    p = 12
    assert D.owner((0, 0), 0, p) == 0 and D.owner((0, 4), 0, p) == 1 and D.owner((3, 5), 0, p) == 5
    assert D.owner((3, 5), 1, p) == 6 + 5
    counts = np.zeros(p, dtype=int)
    for ti in range(8):
        for tj in range(8):
            counts[D.owner((ti, tj), 1, p)] += 1
    assert counts[:6].sum() == 0 and counts[6:].sum() == 64


# --- error paths -----------------------------------------------------------------

def test_rejections():
    ok = DistMatrix(8, 8, (0, 8), (0, 8), 1, 1, 1)
    with pytest.raises(PlanError) as e:
        planner.plan(DistMatrix(8, 6, (0, 8), (0, 6), 1, 1, 1), ok, ok, 2)
    assert e.value.kind == "ESHAPE"
    with pytest.raises(PlanError) as e:
        planner.plan(DistMatrix(8, 8, (0, 8), (0, 8), 1, 1, 3), ok, ok, 4)
    assert e.value.kind == "EREPL"
    with pytest.raises(PlanError) as e:
        planner.plan(DistMatrix(8, 8, (0, 8), (0, 8), 2, 2, 2), ok, ok, 4)   # 4 procs per replica, only 2 ranks
    assert e.value.kind == "EREPL"
    for bad in [(0, 5, 3, 8), (1, 8), (0, 7)]:
        with pytest.raises(PlanError) as e:
            planner.plan(DistMatrix(8, 8, bad, (0, 8), 1, 1, 1), ok, ok, 1)
        assert e.value.kind == "EINVAL"


# --- planted mistakes must be caught ------------------------------------------------

def _misaligned():
    A = DistMatrix(12, 16, (0, 5, 12), (0, 7, 16), 2, 2, 1)
    B = DistMatrix(16, 10, (0, 3, 9, 16), (0, 4, 10), 3, 1, 1)
    C = DistMatrix(12, 10, (0, 4, 12), (0, 6, 10), 2, 2, 2)
    return A, B, C, 8


def test_checker_catches_mutated_lists():
    A, B, C, p = _misaligned()
    tasks = planner.plan(A, B, C, p)
    helpers.check_task_list(tasks, A, B, C, p)
    mutants = [
        tasks[:-1],                                                 # dropped op
        tasks + [tasks[0]],                                         # duplicated op
        [tasks[0]._replace(k1=tasks[0].k1 - 1)] + tasks[1:],        # off-by-one bound
        [tasks[0]._replace(a_tj=tasks[0].a_tj ^ 1)] + tasks[1:],    # wrong A tile
        [tasks[0]._replace(rank=(tasks[0].rank + 1) % p)] + tasks[1:],  # wrong owner
        [t._replace(m0=t.n0, m1=t.n1, n0=t.m0, n1=t.m1) for t in tasks],  # transposed output
    ]
    for bad in mutants:
        with pytest.raises(AssertionError):
            helpers.check_task_list(bad, A, B, C, p)


def test_literal_listing_subscript_breaks_coverage(monkeypatch):
    """Algorithm 1 as printed searches B with the A tile's *row* range.  Planting
    that reading in the oracle (tile_bounds of A returns its row range twice, so
    the B search and the k bound both use it) must fail the coverage pin."""
    A, B, C, p = _misaligned()
    real = DistMatrix.tile_bounds

    def planted(self, idx):
        b = real(self, idx)
        return (b[0], b[0]) if self is A else b

    monkeypatch.setattr(DistMatrix, "tile_bounds", planted)
    tasks = planner.plan(A, B, C, p)
    monkeypatch.setattr(DistMatrix, "tile_bounds", real)
    with pytest.raises(AssertionError):
        helpers.check_task_list(tasks, A, B, C, p)


def test_wrong_share_rule_is_caught(monkeypatch):
    """A replica that searches all of k (ignoring Section 4.1's 1/c rule) does
    the whole product c times over."""
    A, B, C, p = _misaligned()
    monkeypatch.setattr(planner, "replica_share", lambda r, K, c: (0, K))
    tasks = planner.plan(A, B, C, p)
    with pytest.raises(AssertionError):
        helpers.check_task_list(tasks, A, B, C, p)


# --- Stationary B and Stationary A (Algorithm 2 and its mirror image) --------------------

@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("seed", range(60))
def test_stationary_b_and_a_cover_iteration_space_once(seed, mode):
    prob = helpers.random_problem(seed + 300, allow_empty=(seed % 3 == 0))
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    tasks = planner.plan(A, B, C, prob["nranks"], stationary=mode)
    helpers.check_task_list(tasks, A, B, C, prob["nranks"], stationary=mode)


@pytest.mark.parametrize("mode", ["B", "A"])
def test_stationary_b_and_a_all_replication_combinations_p8(mode):
    p, M, K, N = 8, 12, 16, 10
    for cA in helpers.divisors(p):
        for cB in helpers.divisors(p):
            for cC in helpers.divisors(p):
                A = DistMatrix(M, K, (0, 5, 12), (0, 7, 16), 1, 1, cA)
                B = DistMatrix(K, N, (0, 3, 9, 16), (0, 10), 1, 1, cB)
                C = DistMatrix(M, N, (0, 4, 12), (0, 6, 10), 1, 1, cC)
                tasks = planner.plan(A, B, C, p, stationary=mode)
                helpers.check_task_list(tasks, A, B, C, p, stationary=mode)


@pytest.mark.parametrize("seed", range(40))
def test_three_modes_multiply_the_same_boxes_without_replication(seed):
    """Without replication the set of (m, k, n) boxes is the common refinement of the
    three grids whichever matrix stays in place (Section 4.1: only the process that
    performs an op changes); the Stationary-C list is pinned by brute force above."""
    prob = helpers.random_problem(seed + 700)
    for X in "ABC":
        prob[X] = dict(prob[X], replication=1)
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    boxes = {}
    for mode in "CBA":
        tasks = planner.plan(A, B, C, prob["nranks"], stationary=mode)
        boxes[mode] = sorted((t.a_ti, t.a_tj, t.b_ti, t.b_tj, t.c_ti, t.c_tj, t.m0, t.m1, t.k0, t.k1, t.n0, t.n1)
                             for t in tasks)
    assert boxes["C"] == boxes["B"] == boxes["A"]


def test_stationary_b_by_hand():
    """M = 4, K = 6, N = 4; B in two row blocks (k 0:3 and 3:6) on two ranks; A whole,
    C in two row blocks.  Rank q multiplies A(:, its k block) by its B tile into both
    C tiles: two ops per rank, worked out by hand."""
    A = DistMatrix(4, 6, (0, 4), (0, 6), 1, 1, 1)
    B = DistMatrix(6, 4, (0, 3, 6), (0, 4), 2, 1, 1)
    C = DistMatrix(4, 4, (0, 2, 4), (0, 4), 2, 1, 1)
    tasks = planner.plan(A, B, C, 2, stationary="B")
    want = [Task(0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 2, 0, 3, 0, 4),
            Task(0, 0, 0, 0, 0, 0, 0, 0, 1, 0, 2, 4, 0, 3, 0, 4),
            Task(1, 0, 0, 0, 0, 1, 0, 0, 0, 0, 0, 2, 3, 6, 0, 4),
            Task(1, 0, 0, 0, 0, 1, 0, 0, 1, 0, 2, 4, 3, 6, 0, 4)]
    assert tasks == want


def test_stationary_a_by_hand_replicated():
    """A whole and replicated twice over two ranks: replica r takes the columns
    [2r, 2r + 2) of N = 4 (the dimension A does not index).  B and C are whole and
    not replicated, so both ranks address replica 0 of them."""
    A = DistMatrix(3, 5, (0, 3), (0, 5), 1, 1, 2)
    B = DistMatrix(5, 4, (0, 5), (0, 4), 1, 1, 1)
    C = DistMatrix(3, 4, (0, 3), (0, 4), 1, 1, 1)
    tasks = planner.plan(A, B, C, 2, stationary="A")
    want = [Task(0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 0, 3, 0, 5, 0, 2),
            Task(1, 1, 0, 0, 0, 0, 0, 0, 0, 0, 0, 3, 0, 5, 2, 4)]
    assert tasks == want


@pytest.mark.parametrize("mode", ["B", "A"])
def test_wrong_split_dimension_is_caught(monkeypatch, mode):
    """Replicas of a stationary B (A) that split the inner dimension's extent instead
    of M's (N's) are caught: planted by making every share the full range."""
    A = DistMatrix(12, 16, (0, 5, 12), (0, 7, 16), 2, 2, 2)
    B = DistMatrix(16, 10, (0, 3, 9, 16), (0, 4, 10), 3, 1, 2)
    C = DistMatrix(12, 10, (0, 4, 12), (0, 6, 10), 2, 2, 1)
    good = planner.plan(A, B, C, 8, stationary=mode)
    helpers.check_task_list(good, A, B, C, 8, stationary=mode)
    monkeypatch.setattr(planner, "replica_share", lambda r, L, c: (0, L))
    bad = planner.plan(A, B, C, 8, stationary=mode)
    with pytest.raises(AssertionError):
        helpers.check_task_list(bad, A, B, C, 8, stationary=mode)


@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("seed", range(20))
def test_executing_stationary_b_and_a_lists_gives_the_product(seed, mode):
    prob = helpers.random_problem(seed + 900)
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    tasks = planner.plan(A, B, C, prob["nranks"], stationary=mode)
    rng = np.random.default_rng(seed + 99)
    Ag = rng.standard_normal((prob["M"], prob["K"]))
    Bg = rng.standard_normal((prob["K"], prob["N"]))
    c_tiles = oexec.execute_tasks(tasks, A, B, C, oexec.split_tiles(Ag, A), oexec.split_tiles(Bg, B))
    got = oexec.reduce_and_gather(c_tiles, C)
    np.testing.assert_allclose(got, Ag @ Bg, rtol=0, atol=1e-12 * prob["K"])
    order, offsets = planner.reorder(tasks)
    helpers.check_reorder(tasks, order, offsets, C)


# --- iteration offset (Section 4.2) -----------------------------------------------------------

@pytest.mark.parametrize("g", [2, 3, 4, 5])
def test_iteration_offset_staggers_a_process_row_and_column(g):
    """What the offset is for: on an aligned g x g grid without it, at step s every process of
    process row i fetches the same tile A(i, s) and every process of column j the same B(s, j);
    with it, process (i, j) starts at l = (i + j) mod g, so at any step the g processes of a row
    ask for g different tiles of A and those of a column for g different tiles of B (the skew of
    Cannon's algorithm)."""
    n = 6 * g
    cuts = tuple(range(0, n + 1, 6))
    X = DistMatrix(n, n, cuts, cuts, g, g, 1)
    plain = planner.plan(X, X, X, g * g)
    skew = planner.plan(X, X, X, g * g, iteration_offset=True)
    per_rank = lambda tasks: [[t for t in tasks if t.rank == r] for r in range(g * g)]
    for step in range(g):
        for i in range(g):
            row = [per_rank(plain)[i * g + j][step] for j in range(g)]
            assert len({(t.a_ti, t.a_tj) for t in row}) == 1
            row = [per_rank(skew)[i * g + j][step] for j in range(g)]
            assert len({(t.a_ti, t.a_tj) for t in row}) == g
        for j in range(g):
            col = [per_rank(skew)[i * g + j][step] for i in range(g)]
            assert len({(t.b_ti, t.b_tj) for t in col}) == g
    for r in range(g * g):
        i, j = divmod(r, g)
        assert [t.a_tj for t in per_rank(skew)[r]] == [(i + j + s) % g for s in range(g)]


@pytest.mark.parametrize("mode", ["C", "B", "A"])
@pytest.mark.parametrize("seed", range(30))
def test_iteration_offset_is_a_rotation_per_stationary_tile(seed, mode):
    prob = helpers.random_problem(seed + 1300)
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    p = prob["nranks"]
    plain = planner.plan(A, B, C, p, stationary=mode)
    skew = planner.plan(A, B, C, p, stationary=mode, iteration_offset=True)
    helpers.check_task_list(skew, A, B, C, p, stationary=mode)
    assert sorted(plain) == sorted(skew) and [t.rank for t in plain] == [t.rank for t in skew]
    runs = {}
    for lst, which in ((plain, 0), (skew, 1)):
        for t in lst:
            runs.setdefault((t.rank, planner.stationary_tile(t, mode)), ([], []))[which].append(t)
    for (rank, (ti, tj)), (a, b) in runs.items():
        k = (ti + tj) % len(a)
        assert b == a[k:] + a[:k]
    # the grouped order does not depend on it: same groups, same K-segments
    o1, g1 = planner.reorder(plain)
    o2, g2 = planner.reorder(skew)
    assert g1 == g2 and [plain[i] for i in o1] == [skew[i] for i in o2]


@pytest.mark.parametrize("name", workloads.MLP_NAMES)
def test_mlp_workloads_counts_and_pins(name):
    """Section 5.2's MLP shapes over 8 ranks: task counts of the four partitionings
    (closed forms: column block 8 products of full A; inner product 8 x 8 block pairs;
    outer product 8 rank-(K/8) updates, one per C replica; 2-D 2 x 4 x lcm-refined k)."""
    cfg = workloads.config(name)
    small = workloads.scaled_config(name, 16, 24, 32)
    A, B, C = dist(small["A"]), dist(small["B"]), dist(small["C"])
    helpers.check_task_list(planner.plan(A, B, C, 8), A, B, C, 8)
    A, B, C = dist(cfg["A"]), dist(cfg["B"]), dist(cfg["C"])
    tasks = planner.plan(A, B, C, 8)
    part = name.split("-")[1]
    assert len(tasks) == dict(column=8, inner=64, outer=8, **{"2d": 32})[part]
    assert sum((t.m1 - t.m0) * (t.k1 - t.k0) * (t.n1 - t.n0) for t in tasks) == cfg["M"] * cfg["K"] * cfg["N"]
    if part == "outer":
        assert sorted(t.c_rep for t in tasks) == list(range(8))
        assert all(t.k1 - t.k0 == cfg["K"] // 8 for t in tasks)


# --- grouping -----------------------------------------------------------------------

@pytest.mark.parametrize("seed", range(40))
def test_reorder_valid_and_equal_to_dictionary_grouping(seed):
    prob = helpers.random_problem(seed)
    tasks, A, B, C = _plan(prob)
    order, offsets = planner.reorder(tasks)
    helpers.check_reorder(tasks, order, offsets, C)
    # independent statement: bucket by output sub-tile, buckets in key order, k ascending
    buckets = {}
    for idx, t in enumerate(tasks):
        buckets.setdefault((t.c_rep, t.c_ti, t.c_tj, t.m0, t.n0), []).append(idx)
    flat, offs = [], [0]
    for key in sorted(buckets):
        flat += sorted(buckets[key], key=lambda i: tasks[i].k0)
        offs.append(len(flat))
    assert flat == order and offs == offsets
    # every group's K-segments tile its replica's share of k
    for g in range(len(offsets) - 1):
        members = [tasks[t] for t in order[offsets[g]:offsets[g + 1]]]
        r = members[0].c_rep
        share = ((r * A.cols) // C.replication, ((r + 1) * A.cols) // C.replication)
        assert members[0].k0 == share[0] and members[-1].k1 == share[1]
        assert all(a.k1 == b.k0 for a, b in zip(members, members[1:]))


# --- the plan's meaning: executing it gives A B ----------------------------------------

@pytest.mark.parametrize("seed", range(30))
def test_executing_the_task_list_gives_the_product(seed):
    prob = helpers.random_problem(seed)
    tasks, A, B, C = _plan(prob)
    rng = np.random.default_rng(seed + 99)
    Ag = rng.standard_normal((prob["M"], prob["K"]))
    Bg = rng.standard_normal((prob["K"], prob["N"]))
    c_tiles = oexec.execute_tasks(tasks, A, B, C, oexec.split_tiles(Ag, A), oexec.split_tiles(Bg, B))
    got = oexec.reduce_and_gather(c_tiles, C)
    np.testing.assert_allclose(got, Ag @ Bg, rtol=0, atol=1e-12 * prob["K"])


@pytest.mark.parametrize("origin", [0, 1])
def test_reduce_then_broadcast_leaves_the_product_in_every_replica(origin):
    A = DistMatrix(12, 16, (0, 5, 12), (0, 7, 16), 2, 2, 1)
    B = DistMatrix(16, 10, (0, 3, 9, 16), (0, 4, 10), 3, 1, 1)
    C = DistMatrix(12, 10, (0, 4, 12), (0, 6, 10), 2, 2, 2)
    rng = np.random.default_rng(5)
    Ag, Bg = rng.standard_normal((12, 16)), rng.standard_normal((16, 10))
    tasks = planner.plan(A, B, C, 8)
    c_tiles = oexec.execute_tasks(tasks, A, B, C, oexec.split_tiles(Ag, A), oexec.split_tiles(Bg, B))
    oexec.reduce_and_gather(c_tiles, C, origin)
    oexec.broadcast_replica(c_tiles, C, origin)
    for rep in range(2):
        for (ti, tj) in [(0, 0), (0, 1), (1, 0), (1, 1)]:
            (r0, r1), (c0, c1) = C.tile_bounds((ti, tj))
            np.testing.assert_allclose(c_tiles[(rep, ti, tj)], (Ag @ Bg)[r0:r1, c0:c1], rtol=0, atol=1e-12)
