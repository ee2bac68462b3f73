"""Oracle direct execution of a task list -- TEST INFRASTRUCTURE ONLY.

Section 4.2 ("direct execution"): every op names one tile of A, B and C and the
slices of them to multiply; the result is added to the C tile.  Here every
virtual rank's tiles are plain numpy arrays, a "get" is a view, the local
multiply is fp64 ``numpy.matmul`` (a library primitive used as one step), and
ops run in list order.  When C is replicated each replica holds the partial sum
over its share of the inner dimension and ``reduce_replicas`` adds them
(Section 4.2, last paragraph).
"""
from __future__ import annotations

from typing import Dict, Sequence, Tuple

import numpy as np

from .planner import DistMatrix, Task

TileKey = Tuple[int, int, int]  # (replica, tile row, tile col)


def split_tiles(X: np.ndarray, D: DistMatrix) -> Dict[TileKey, np.ndarray]:
    """Tiles of every replica of a global matrix, by ``tile_bounds`` (Table 1).
    Replicas of an input hold the same data (Section 3)."""
    tiles = {}
    gr, gc = D.grid_shape()
    for rep in range(D.replication):
        for ti in range(gr):
            for tj in range(gc):
                (r0, r1), (c0, c1) = D.tile_bounds((ti, tj))
                tiles[(rep, ti, tj)] = np.array(X[r0:r1, c0:c1], dtype=np.float64)
    return tiles


def execute_tasks(tasks: Sequence[Task], A: DistMatrix, B: DistMatrix, C: DistMatrix,
                  a_tiles: Dict[TileKey, np.ndarray], b_tiles: Dict[TileKey, np.ndarray]
                  ) -> Dict[TileKey, np.ndarray]:
    """Run the ops in order; returns fp64 C tiles (partials when C is replicated)."""
    c_tiles: Dict[TileKey, np.ndarray] = {}
    gr, gc = C.grid_shape()
    for rep in range(C.replication):
        for ti in range(gr):
            for tj in range(gc):
                (r0, r1), (c0, c1) = C.tile_bounds((ti, tj))
                c_tiles[(rep, ti, tj)] = np.zeros((r1 - r0, c1 - c0), dtype=np.float64)
    for t in tasks:
        (ar0, _), (ac0, _) = A.tile_bounds((t.a_ti, t.a_tj))
        (br0, _), (bc0, _) = B.tile_bounds((t.b_ti, t.b_tj))
        (cr0, _), (cc0, _) = C.tile_bounds((t.c_ti, t.c_tj))
        a = a_tiles[(t.a_rep, t.a_ti, t.a_tj)][t.m0 - ar0:t.m1 - ar0, t.k0 - ac0:t.k1 - ac0]
        b = b_tiles[(t.b_rep, t.b_ti, t.b_tj)][t.k0 - br0:t.k1 - br0, t.n0 - bc0:t.n1 - bc0]
        c = c_tiles[(t.c_rep, t.c_ti, t.c_tj)]
        c[t.m0 - cr0:t.m1 - cr0, t.n0 - cc0:t.n1 - cc0] += a @ b
    return c_tiles


def reduce_and_gather(c_tiles: Dict[TileKey, np.ndarray], C: DistMatrix, origin: int = 0) -> np.ndarray:
    """Sum the replicas of every tile in ascending replica order (into the
    origin replica) and assemble the global matrix from the origin's tiles."""
    out = np.zeros((C.rows, C.cols), dtype=np.float64)
    gr, gc = C.grid_shape()
    for ti in range(gr):
        for tj in range(gc):
            s = c_tiles[(0, ti, tj)].copy()
            for rep in range(1, C.replication):
                s = s + c_tiles[(rep, ti, tj)]
            c_tiles[(origin, ti, tj)] = s
            (r0, r1), (c0, c1) = C.tile_bounds((ti, tj))
            out[r0:r1, c0:c1] = s
    return out


def broadcast_replica(c_tiles: Dict[TileKey, np.ndarray], C: DistMatrix, origin: int = 0) -> None:
    """Table 1, broadcast_replica: every other replica's tiles become copies of the
    origin replica's tiles (in place, in the dictionary of tiles)."""
    gr, gc = C.grid_shape()
    for ti in range(gr):
        for tj in range(gc):
            for rep in range(C.replication):
                if rep != origin:
                    c_tiles[(rep, ti, tj)] = c_tiles[(origin, ti, tj)].copy()
