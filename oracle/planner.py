"""Oracle planner: distributed-matrix descriptor + op generation (Stationary C, B, A).

TEST INFRASTRUCTURE ONLY (see the package docstring).  Plain Python, integer
arithmetic only, no blocking or shortcuts: ``overlapping_tiles`` scans every
tile of the grid, op generation narrows a box of the (m, k, n) index space tile by tile.

What follows the paper, and where:

* ``DistMatrix``                 -- Section 3: shape + partition (tile grid and
  process grid, ScaLAPACK convention, Section 2.1) + replication factor c, with
  c replicas each laid out over p/c processes.
* ``grid_shape / tile_bounds / overlapping_tiles`` -- Table 1.
* ``ops_of_rank``                -- what Algorithm 1 (Stationary C), Algorithm 2
  (Stationary B) and its mirror image (Stationary A; Section 4.1 calls it
  analogous and omits it) compute for one process, with the change Section 4.1
  asks for when the stationary matrix is replicated: replica r searches only
  its 1/c share of the dimension that matrix does not index, and every bound on
  that axis is clipped to the share.
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


def replica_share(replica: int, extent: int, c: int) -> Interval:
    """Section 4.1: replica r of a c-fold replicated stationary matrix works on
    1/c of the dimension that matrix does not index (the inner dimension when C
    stays in place; M for B, N for A): elements [floor(r L / c), floor((r+1) L / c))."""
    return ((replica * extent) // c, ((replica + 1) * extent) // c)


# A product C = A B runs over the index space (m, k, n).  Each matrix sees two of the three axes
# (rows, columns); the third is the one its replicas share out between them.
_AXES = {"A": ("m", "k"), "B": ("k", "n"), "C": ("m", "n")}
# Whichever matrix stays in place, the other two are searched in the order A before B before C
# (Algorithm 1: A tiles, then B tiles; Algorithm 2: A tiles, then C tiles; its mirror image for a
# stationary A: B tiles, then C tiles).
_SEARCHED = {"C": ("A", "B"), "B": ("A", "C"), "A": ("B", "C")}

Box = dict   # axis name -> half-open interval


def _view(box: Box, name: str) -> Slice2D:
    """The 2-D slice of matrix ``name`` that the box touches."""
    r, c = _AXES[name]
    return (box[r], box[c])


def _narrow(box: Box, name: str, tile: Slice2D) -> Box:
    """The part of the box inside a tile of matrix ``name`` (``bound`` on the two axes it sees)."""
    r, c = _AXES[name]
    out = dict(box)
    out[r] = bound(box[r], tile[0])
    out[c] = bound(box[c], tile[1])
    return out


def ops_of_rank(A: DistMatrix, B: DistMatrix, C: DistMatrix, p: int, rank: int, stationary: str = "C") -> List[Task]:
    """The ops one process performs (Algorithm 1 for ``stationary == "C"``, Algorithm 2 for "B",
    its mirror image for "A"), with the replication rule of Section 4.1.

    Slicing, stated on boxes of the (m, k, n) index space: the process starts from the whole
    space, cut down to its replica's share of the axis the stationary matrix does not see.  Each
    stationary tile it owns narrows that box on the tile's two axes; every tile of the first
    searched matrix that meets the box narrows it further; every tile of the second searched
    matrix that meets what is left narrows it to the box of one op.  The tiles of the searched
    matrices are taken from the process' local replicas (Section 3)."""
    mats = {"A": A, "B": B, "C": C}
    rep = {name: X.replica_of(rank, p) for name, X in mats.items()}
    S = mats[stationary]
    whole: Box = {"m": (0, A.rows), "k": (0, A.cols), "n": (0, B.cols)}
    (shared_axis,) = set(whole) - set(_AXES[stationary])
    whole[shared_axis] = replica_share(rep[stationary], whole[shared_axis][1], S.replication)
    first, second = _SEARCHED[stationary]
    out: List[Task] = []
    rows, cols = S.grid_shape()
    for ti in range(rows):
        for tj in range(cols):
            if S.owner((ti, tj), rep[stationary], p) != rank:
                continue
            mine = _narrow(whole, stationary, S.tile_bounds((ti, tj)))
            for t1 in mats[first].overlapping_tiles(_view(mine, first), rep[first]):
                with_first = _narrow(mine, first, mats[first].tile_bounds(t1))
                for t2 in mats[second].overlapping_tiles(_view(with_first, second), rep[second]):
                    op = _narrow(with_first, second, mats[second].tile_bounds(t2))
                    if is_empty(op["m"]) or is_empty(op["k"]) or is_empty(op["n"]):
                        continue
                    tile = {stationary: (ti, tj), first: t1, second: t2}
                    out.append(Task(rank,
                                    rep["A"], tile["A"][0], tile["A"][1],
                                    rep["B"], tile["B"][0], tile["B"][1],
                                    rep["C"], tile["C"][0], tile["C"][1],
                                    op["m"][0], op["m"][1], op["k"][0], op["k"][1], op["n"][0], op["n"][1]))
    return out


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
    tasks: List[Task] = []
    for rank in range(p):
        ops = ops_of_rank(A, B, C, p, rank, stationary)
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
