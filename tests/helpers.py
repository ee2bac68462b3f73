"""Shared test helpers: random partitioned problems and the brute-force checkers
that pin a task list to the mathematics (they look only at the task records, so
they serve the oracle's list and the library's list alike)."""
from __future__ import annotations

import numpy as np

from oracle.planner import DistMatrix


def divisors(p):
    return [c for c in range(1, p + 1) if p % c == 0]


def random_cuts(rng, dim, nblocks, allow_empty=False):
    """nblocks+1 cut points spanning [0, dim]."""
    if nblocks == 1:
        return (0, dim)
    if allow_empty:
        inner = np.sort(rng.integers(0, dim + 1, size=nblocks - 1))
    else:
        inner = np.sort(rng.choice(np.arange(1, dim), size=nblocks - 1, replace=False))
    return (0,) + tuple(int(x) for x in inner) + (dim,)


def random_matrix_desc(rng, rows, cols, p, allow_empty=False):
    """Random tile grid, random (possibly smaller => block-cyclic) process grid,
    random replication factor among the divisors of p that leave room for it."""
    gr = int(rng.integers(1, min(rows, 5) + 1))
    gc = int(rng.integers(1, min(cols, 5) + 1))
    c = int(rng.choice(divisors(p)))
    per = p // c
    # process grid: at most the tile grid, at most `per` ranks
    choices = [(a, b) for a in range(1, gr + 1) for b in range(1, gc + 1) if a * b <= per]
    pr, pc = choices[int(rng.integers(0, len(choices)))]
    return dict(rows=rows, cols=cols,
                row_cuts=random_cuts(rng, rows, gr, allow_empty),
                col_cuts=random_cuts(rng, cols, gc, allow_empty),
                proc_rows=pr, proc_cols=pc, replication=c)


def random_problem(seed, max_dim=24, allow_empty=False):
    rng = np.random.default_rng(seed)
    p = int(rng.choice([1, 2, 3, 4, 6, 8, 12]))
    M, K, N = (int(x) for x in rng.integers(2, max_dim + 1, size=3))
    return dict(M=M, K=K, N=N, nranks=p,
                A=random_matrix_desc(rng, M, K, p, allow_empty),
                B=random_matrix_desc(rng, K, N, p, allow_empty),
                C=random_matrix_desc(rng, M, N, p, allow_empty))


def dist(d) -> DistMatrix:
    return DistMatrix(**d)


def merged_intervals(lo, hi, *cut_lists):
    """Number of non-empty intervals of the merged cut set inside [lo, hi)."""
    pts = {lo, hi}
    for cuts in cut_lists:
        pts.update(c for c in cuts if lo < c < hi)
    return len(pts) - 1 if hi > lo else 0


# -- checkers on task records (fields by name; works for any namedtuple-like) --

def coverage_counter(tasks, M, K, N, c_rep=None, rep_field="c_rep"):
    """3-D counter over the (i, k, j) iteration space, +1 for every task box
    (optionally only the tasks whose ``rep_field`` equals ``c_rep``)."""
    cnt = np.zeros((M, K, N), dtype=np.int32)
    for t in tasks:
        if c_rep is not None and getattr(t, rep_field) != c_rep:
            continue
        cnt[t.m0:t.m1, t.k0:t.k1, t.n0:t.n1] += 1
    return cnt


def check_task_list(tasks, A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, stationary: str = "C"):
    """Everything the paper and the mathematics fix about a task list generated
    with the given stationary matrix; raises AssertionError naming the first
    violated property."""
    M, K, N = A.rows, A.cols, B.cols
    S = dict(A=A, B=B, C=C)[stationary]
    cS = S.replication
    # the dimension the replicas of the stationary matrix split: the one it does not index
    axis = dict(C=1, B=0, A=2)[stationary]
    L = (M, K, N)[axis]
    rep_field = stationary.lower() + "_rep"
    # (1) the boxes tile the iteration space exactly once (Sections 2.1, 4.1)
    cnt = coverage_counter(tasks, M, K, N)
    assert cnt.min(initial=1) == 1 and cnt.max(initial=1) == 1, "iteration space not covered exactly once"
    # (2) each replica of the stationary matrix covers exactly its 1/c share of that dimension
    for r in range(cS):
        lo, hi = (r * L) // cS, ((r + 1) * L) // cS
        cr = np.moveaxis(coverage_counter(tasks, M, K, N, c_rep=r, rep_field=rep_field), axis, 0)
        assert (cr[lo:hi] == 1).all(), f"replica {r} misses part of its share"
        assert cr[:lo].sum() == 0 and cr[hi:].sum() == 0, f"replica {r} works outside its share"
    for t in tasks:
        # (3) non-empty boxes, each slice inside its tile
        assert t.m0 < t.m1 and t.k0 < t.k1 and t.n0 < t.n1, "empty task"
        (ar, ac) = A.tile_bounds((t.a_ti, t.a_tj))
        (br, bc) = B.tile_bounds((t.b_ti, t.b_tj))
        (cr_, cc) = C.tile_bounds((t.c_ti, t.c_tj))
        assert ar[0] <= t.m0 and t.m1 <= ar[1] and ac[0] <= t.k0 and t.k1 <= ac[1], "A slice leaves its tile"
        assert br[0] <= t.k0 and t.k1 <= br[1] and bc[0] <= t.n0 and t.n1 <= bc[1], "B slice leaves its tile"
        assert cr_[0] <= t.m0 and t.m1 <= cr_[1] and cc[0] <= t.n0 and t.n1 <= cc[1], "C slice leaves its tile"
        # (4) the stationary tile belongs to the rank; everything comes from (goes to) its local replicas
        s_idx = dict(A=(t.a_ti, t.a_tj), B=(t.b_ti, t.b_tj), C=(t.c_ti, t.c_tj))[stationary]
        assert S.owner(s_idx, getattr(t, rep_field), p) == t.rank, "task on a rank that does not own the stationary tile"
        assert t.c_rep == C.replica_of(t.rank, p)
        assert t.a_rep == A.replica_of(t.rank, p) and t.b_rep == B.replica_of(t.rank, p), "not the local replica"
    # (5) closed-form count: product of the merged-cut interval counts, per replica share
    cuts = [(A.row_cuts, C.row_cuts), (A.col_cuts, B.row_cuts), (B.col_cuts, C.col_cuts)]
    dims = (M, K, N)
    want = 0
    for r in range(cS):
        lo, hi = (r * L) // cS, ((r + 1) * L) // cS
        n = 1
        for ax in range(3):
            n *= merged_intervals(lo, hi, *cuts[ax]) if ax == axis else merged_intervals(0, dims[ax], *cuts[ax])
        want += n
    assert len(tasks) == want, f"{len(tasks)} tasks, closed form says {want}"


def check_reorder(tasks, order, offsets, C: DistMatrix):
    """Validity of a grouping: permutation, sorted keys, one output sub-tile per
    group with disjoint ascending K-segments, groups pairwise disjoint."""
    n = len(tasks)
    assert sorted(order) == list(range(n)), "order is not a permutation"
    keys = [(tasks[t].c_rep, tasks[t].c_ti, tasks[t].c_tj, tasks[t].m0, tasks[t].n0, tasks[t].k0) for t in order]
    assert keys == sorted(keys), "keys not ascending"
    assert offsets[0] == 0 and offsets[-1] == n and all(a < b for a, b in zip(offsets, offsets[1:])) or n == 0
    seen = set()
    K = None
    for g in range(len(offsets) - 1):
        members = [tasks[t] for t in order[offsets[g]:offsets[g + 1]]]
        head = members[0]
        box = (head.c_rep, head.c_ti, head.c_tj, head.m0, head.m1, head.n0, head.n1)
        assert box not in seen
        seen.add(box)
        for a, b in zip(members, members[1:]):
            assert (b.c_rep, b.c_ti, b.c_tj, b.m0, b.m1, b.n0, b.n1) == box[:3] + (a.m0, a.m1, a.n0, a.n1)
            assert a.k1 <= b.k0, "K-segments overlap or descend"
    # output boxes of different groups in one replica never overlap
    if n:
        M = max(t.m1 for t in tasks)
        N = max(t.n1 for t in tasks)
        for r in range(C.replication):
            hit = np.zeros((M, N), dtype=np.int32)
            for (rep, _, _, m0, m1, n0, n1) in seen:
                if rep == r:
                    hit[m0:m1, n0:n1] += 1
            assert hit.max(initial=0) <= 1, "two groups write the same C element"
