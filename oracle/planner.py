"""Oracle planner: distributed-matrix descriptor + op generation (Stationary C, B, A).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python, integer
arithmetic only, no blocking or shortcuts: ``overlapping_tiles`` scans every
tile of the grid, op generation is the loop nest of Algorithm 1.

What follows the paper, and where:

* ``DistMatrix``                 -- Section 3: shape + partition (tile grid and
  process grid, ScaLAPACK convention, Section 2.1) + replication factor c, with
  c replicas each laid out over p/c processes.
* ``grid_shape / tile_bounds / overlapping_tiles`` -- Table 1.
* ``gen_ops_stationary_c``       -- Algorithm 1, with the change Section 4.1
  asks for when the stationary matrix is replicated: replica r searches only
  its 1/c share of the inner dimension and every k-bound is clipped to it.
* ``gen_ops_stationary_b``       -- Algorithm 2; ``gen_ops_stationary_a`` is its mirror
  image (Section 4.1 calls it analogous and omits it).
* ``reorder``                    -- not in the paper: the plain definition
  (a stable sort) of the grouping by output sub-tile that the GPU path uses.

Readings where the paper is silent or at odds with itself (each one is listed
again in the design notes):

* rank -> replica: contiguous blocks, ``replica = rank // (p/c)``.
* tile -> owner inside a replica: row-major process grid, block-cyclic,
  ``local = (ti % proc_rows) * proc_cols + (tj % proc_cols)``.
* replica r's share of the inner dimension: the contiguous element range
  ``[floor(r K / c), floor((r+1) K / c))``, independent of tile cuts.
* Algorithm 1 searches B with the *column* range of the A tile (the k axis);
  the listing's subscript 0 there is dimensionally wrong (B's rows are k, which
  are A's columns) and the prose of Section 4.1 pairs A(rows, 0:k) with
  B(0:k, cols).  ``tests/test_oracle_planner.py`` shows that the literal
  subscript breaks the exactly-once coverage of the iteration space.
* ``bound(x, y)`` is half-open interval intersection; an empty result means no
  op is emitted.
* ``overlapping_tiles`` returns tiles in ascending (tile row, tile column).
* the global list is the concatenation of the per-process lists by ascending
  rank.  The iteration offset of Section 4.2 is applied on request only: the ops
  of the stationary tile (i, j) are rotated to start at position (i + j) modulo
  their number ("add the two indices of the stationary tile"); tiles with one op
  are unchanged.
* Algorithm 2 names the op's B tile and C tile with identifiers it never
  defines; they are read as the stationary tile (k, j) and the C tile of the
  innermost loop.
* Section 4.1 states the 1/c rule for a replicated stationary C only (its
  replicas split the inner dimension).  For a replicated stationary B the
  replicas split M, for a replicated stationary A they split N: in each case the
  one dimension the stationary matrix does not index, in contiguous element
  ranges ``[floor(r L / c), floor((r+1) L / c))``.  The test of this reading is
  that every point of the iteration space is still covered exactly once.
* with Stationary B or A an op's product goes to the C tile in the process'
  local replica of C (Section 3: a primitive without replica index addresses the
  local replica); regions of a C replica that receive nothing hold zero, so that
  the replica sum is the product.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import List, NamedTuple, Sequence, Tuple

Interval = Tuple[int, int]          # half-open [lo, hi)
Slice2D = Tuple[Interval, Interval]  # (row interval, column interval)


class PlanError(ValueError):
    """Descriptor rejected.  ``kind`` is one of 'EINVAL', 'ESHAPE', 'EREPL'."""

    def __init__(self, kind: str, msg: str):
        super().__init__(f"{kind}: {msg}")
        self.kind = kind


def bound(x: Interval, y: Interval) -> Interval:
    """Algorithm 1, ``bound(x, y)``: intersection of two half-open intervals."""
    return (max(x[0], y[0]), min(x[1], y[1]))


def is_empty(iv: Interval) -> bool:
    return iv[0] >= iv[1]


@dataclass(frozen=True)
class DistMatrix:
    """Section 3: matrix shape, partition object, replication factor.

    The partition is an explicit tile grid (cut points per axis; a uniform tile
    shape is the special case ``cuts[i] = min(i * t, dim)``) and a process grid
    ``proc_rows x proc_cols`` onto which tiles are dealt block-cyclically
    (Section 2.1, ScaLAPACK convention).
    """

    rows: int
    cols: int
    row_cuts: Tuple[int, ...]
    col_cuts: Tuple[int, ...]
    proc_rows: int
    proc_cols: int
    replication: int = 1

    # -- Table 1 ---------------------------------------------------------
    def grid_shape(self) -> Tuple[int, int]:
        return (len(self.row_cuts) - 1, len(self.col_cuts) - 1)

    def tile_bounds(self, idx: Tuple[int, int]) -> Slice2D:
        ti, tj = idx
        return ((self.row_cuts[ti], self.row_cuts[ti + 1]),
                (self.col_cuts[tj], self.col_cuts[tj + 1]))

    def overlapping_tiles(self, slc: Slice2D, replica_idx: int = 0) -> List[Tuple[int, int]]:
        """All tiles whose bounds intersect ``slc``; full scan, row-major order.

        Every replica has the same tile grid, so ``replica_idx`` does not change
        the answer; it is kept because the primitive takes it (Table 1).
        """
        out = []
        gr, gc = self.grid_shape()
        for ti in range(gr):
            for tj in range(gc):
                tb = self.tile_bounds((ti, tj))
                if not is_empty(bound(tb[0], slc[0])) and not is_empty(bound(tb[1], slc[1])):
                    out.append((ti, tj))
        return out

    # -- replication and ownership (Section 3) ---------------------------
    def ranks_per_replica(self, p: int) -> int:
        return p // self.replication

    def replica_of(self, rank: int, p: int) -> int:
        return rank // self.ranks_per_replica(p)

    def owner(self, idx: Tuple[int, int], replica: int, p: int) -> int:
        ti, tj = idx
        local = (ti % self.proc_rows) * self.proc_cols + (tj % self.proc_cols)
        return replica * self.ranks_per_replica(p) + local

    # -- validation -------------------------------------------------------
    def validate(self, p: int) -> None:
        for name, cuts, dim in (("row", self.row_cuts, self.rows), ("col", self.col_cuts, self.cols)):
            if len(cuts) < 2:
                raise PlanError("EINVAL", f"{name} grid needs at least one tile")
            if cuts[0] != 0 or cuts[-1] != dim:
                raise PlanError("EINVAL", f"{name} cuts must span [0, {dim}]")
            for a, b in zip(cuts, cuts[1:]):
                if b < a:
                    raise PlanError("EINVAL", f"{name} cuts must be non-decreasing")
        if self.rows < 0 or self.cols < 0:
            raise PlanError("EINVAL", "negative shape")
        if self.proc_rows < 1 or self.proc_cols < 1:
            raise PlanError("EINVAL", "process grid must be at least 1x1")
        c = self.replication
        if c < 1 or p % c != 0:
            # Section 2.1: p / c must be an integer.
            raise PlanError("EREPL", f"replication {c} does not divide {p} ranks")
        if self.proc_rows * self.proc_cols > p // c:
            raise PlanError("EREPL", "process grid larger than the ranks of one replica")


class Task(NamedTuple):
    """One op of Algorithm 1: three tile ids and the global box it multiplies.

    The A slice is rows [m0,m1) x cols [k0,k1), the B slice rows [k0,k1) x cols
    [n0,n1), the C slice rows [m0,m1) x cols [n0,n1), all in global indices
    (local offsets are global minus the tile's lower bound, footnote of
    Section 4.1).
    """

    rank: int
    a_rep: int
    a_ti: int
    a_tj: int
    b_rep: int
    b_ti: int
    b_tj: int
    c_rep: int
    c_ti: int
    c_tj: int
    m0: int
    m1: int
    k0: int
    k1: int
    n0: int
    n1: int


def validate_problem(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int) -> None:
    if p < 1:
        raise PlanError("EINVAL", "need at least one rank")
    for X in (A, B, C):
        X.validate(p)
    if A.cols != B.rows or A.rows != C.rows or B.cols != C.cols:
        raise PlanError("ESHAPE", "shapes do not form C[m,n] = A[m,k] B[k,n]")


def k_share(replica: int, K: int, c: int) -> Interval:
    """Section 4.1: replica r of a c-fold replicated stationary matrix works on
    1/c of the inner dimension (of M or N when B or A is the stationary matrix)."""
    return ((replica * K) // c, ((replica + 1) * K) // c)


def gen_ops_stationary_c(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, rank: int) -> List[Task]:
    """Algorithm 1 for one process, plus the replication rule of Section 4.1."""
    ops: List[Task] = []
    K = A.cols
    c_rep = C.replica_of(rank, p)
    a_rep = A.replica_of(rank, p)   # "its local replica" (Sections 3, 4.2)
    b_rep = B.replica_of(rank, p)
    share = k_share(c_rep, K, C.replication)
    gr, gc = C.grid_shape()
    for i in range(gr):
        for j in range(gc):
            if C.owner((i, j), c_rep, p) != rank:
                continue
            c_bounds = C.tile_bounds((i, j))
            # tiles of A(rows of my C tile, my share of 0:k)
            a_tiles = A.overlapping_tiles((c_bounds[0], share), a_rep)
            for a_idx in a_tiles:
                a_bounds = A.tile_bounds(a_idx)
                # tiles of B(the k range of this A tile, columns of my C tile)
                b_tiles = B.overlapping_tiles((bound(a_bounds[1], share), c_bounds[1]), b_rep)
                for b_idx in b_tiles:
                    b_bounds = B.tile_bounds(b_idx)
                    m_bound = bound(c_bounds[0], a_bounds[0])
                    k_bound = bound(bound(a_bounds[1], b_bounds[0]), share)
                    n_bound = bound(b_bounds[1], c_bounds[1])
                    if is_empty(m_bound) or is_empty(k_bound) or is_empty(n_bound):
                        continue
                    ops.append(Task(rank, a_rep, a_idx[0], a_idx[1],
                                    b_rep, b_idx[0], b_idx[1],
                                    c_rep, i, j,
                                    m_bound[0], m_bound[1],
                                    k_bound[0], k_bound[1],
                                    n_bound[0], n_bound[1]))
    return ops


def gen_ops_stationary_b(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, rank: int) -> List[Task]:
    """Algorithm 2 for one process: its tiles of B stay in place.

    A replicated B splits M between its replicas (see the module docstring)."""
    ops: List[Task] = []
    M = A.rows
    b_rep = B.replica_of(rank, p)
    a_rep = A.replica_of(rank, p)
    c_rep = C.replica_of(rank, p)
    share = k_share(b_rep, M, B.replication)         # this replica's rows of A and C
    gr, gc = B.grid_shape()
    for k in range(gr):
        for j in range(gc):
            if B.owner((k, j), b_rep, p) != rank:
                continue
            b_bounds = B.tile_bounds((k, j))
            # tiles of A(my share of the rows, the k range of my B tile)
            a_tiles = A.overlapping_tiles((share, b_bounds[0]), a_rep)
            for a_idx in a_tiles:
                a_bounds = A.tile_bounds(a_idx)
                # tiles of C this product updates: rows of the A tile, columns of my B tile
                c_tiles = C.overlapping_tiles((bound(a_bounds[0], share), b_bounds[1]), c_rep)
                for c_idx in c_tiles:
                    c_bounds = C.tile_bounds(c_idx)
                    m_bound = bound(bound(c_bounds[0], a_bounds[0]), share)
                    k_bound = bound(a_bounds[1], b_bounds[0])
                    n_bound = bound(b_bounds[1], c_bounds[1])
                    if is_empty(m_bound) or is_empty(k_bound) or is_empty(n_bound):
                        continue
                    ops.append(Task(rank, a_rep, a_idx[0], a_idx[1],
                                    b_rep, k, j,
                                    c_rep, c_idx[0], c_idx[1],
                                    m_bound[0], m_bound[1],
                                    k_bound[0], k_bound[1],
                                    n_bound[0], n_bound[1]))
    return ops


def gen_ops_stationary_a(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, rank: int) -> List[Task]:
    """The mirror image of Algorithm 2: the process' tiles of A stay in place.

    A replicated A splits N between its replicas (see the module docstring)."""
    ops: List[Task] = []
    N = B.cols
    a_rep = A.replica_of(rank, p)
    b_rep = B.replica_of(rank, p)
    c_rep = C.replica_of(rank, p)
    share = k_share(a_rep, N, A.replication)         # this replica's columns of B and C
    gr, gc = A.grid_shape()
    for i in range(gr):
        for l in range(gc):
            if A.owner((i, l), a_rep, p) != rank:
                continue
            a_bounds = A.tile_bounds((i, l))
            # tiles of B(the k range of my A tile, my share of the columns)
            b_tiles = B.overlapping_tiles((a_bounds[1], share), b_rep)
            for b_idx in b_tiles:
                b_bounds = B.tile_bounds(b_idx)
                # tiles of C this product updates: rows of my A tile, columns of the B tile
                c_tiles = C.overlapping_tiles((a_bounds[0], bound(b_bounds[1], share)), c_rep)
                for c_idx in c_tiles:
                    c_bounds = C.tile_bounds(c_idx)
                    m_bound = bound(c_bounds[0], a_bounds[0])
                    k_bound = bound(a_bounds[1], b_bounds[0])
                    n_bound = bound(bound(b_bounds[1], c_bounds[1]), share)
                    if is_empty(m_bound) or is_empty(k_bound) or is_empty(n_bound):
                        continue
                    ops.append(Task(rank, a_rep, i, l,
                                    b_rep, b_idx[0], b_idx[1],
                                    c_rep, c_idx[0], c_idx[1],
                                    m_bound[0], m_bound[1],
                                    k_bound[0], k_bound[1],
                                    n_bound[0], n_bound[1]))
    return ops


_GENERATORS = {"C": gen_ops_stationary_c, "B": gen_ops_stationary_b, "A": gen_ops_stationary_a}


def stationary_tile(t: Task, stationary: str) -> Tuple[int, int]:
    return {"A": (t.a_ti, t.a_tj), "B": (t.b_ti, t.b_tj), "C": (t.c_ti, t.c_tj)}[stationary]


def apply_iteration_offset(ops: Sequence[Task], stationary: str) -> List[Task]:
    """Section 4.2, iteration offset, on one process' list: the ops of each
    stationary tile (a contiguous run of the list) start (i + j) positions
    later in their own cyclic order, i and j being the tile's grid indices."""
    out: List[Task] = []
    pos = 0
    while pos < len(ops):
        tile = stationary_tile(ops[pos], stationary)
        end = pos
        while end < len(ops) and stationary_tile(ops[end], stationary) == tile:
            end += 1
        run = list(ops[pos:end])
        shift = (tile[0] + tile[1]) % len(run)
        out.extend(run[shift:] + run[:shift])
        pos = end
    return out


def plan(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, stationary: str = "C",
         iteration_offset: bool = False) -> List[Task]:
    """Task list of the whole job: every rank's ops, ranks in ascending order.

    ``stationary`` names the data movement strategy of Section 4: the matrix
    whose tiles stay in place and decide which process performs an op."""
    validate_problem(A, B, C, p)
    gen = _GENERATORS[stationary]
    tasks: List[Task] = []
    for rank in range(p):
        ops = gen(A, B, C, p, rank)
        if iteration_offset:
            ops = apply_iteration_offset(ops, stationary)
        tasks.extend(ops)
    return tasks


def reorder(tasks: Sequence[Task]) -> Tuple[List[int], List[int]]:
    """Grouping by output sub-tile, as a definition.

    Returns ``(order, group_offsets)``: ``order`` is the stable sort of task
    indices by (c_rep, c_ti, c_tj, m0, n0, k0); a new group starts whenever
    (c_rep, c_ti, c_tj, m0, n0) changes, and ``group_offsets`` (length
    groups+1) indexes into ``order``.
    """
    order = sorted(range(len(tasks)),
                   key=lambda t: (tasks[t].c_rep, tasks[t].c_ti, tasks[t].c_tj,
                                  tasks[t].m0, tasks[t].n0, tasks[t].k0))
    offsets = []
    prev = None
    for pos, t in enumerate(order):
        key = (tasks[t].c_rep, tasks[t].c_ti, tasks[t].c_tj, tasks[t].m0, tasks[t].n0)
        if key != prev:
            offsets.append(pos)
            prev = key
    offsets.append(len(order))
    return order, offsets
