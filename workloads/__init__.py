"""Seeded synthetic workloads: partition descriptors and operand values.

This module serves both the GPU path's tests/bench and the CPU oracle, so it
holds no arithmetic of the method itself: only (a) descriptor *data* -- shapes,
tile-grid cut points, process grids, replication factors -- for the partitioning
families the paper evaluates (1-D inner/outer product, 2-D, misaligned,
replicated; Sections 2.1, 2.2 and 5.2), and (b) seeded random operand values
(the paper initialises all matrices randomly, artifact appendix).  Everything
is a plain dict / numpy array; each side converts to its own types.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

# ---------------------------------------------------------------------------
# bf16 helpers (storage format only: the upper half of an IEEE fp32)


def bf16_round(x: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rnd = ((u >> np.uint32(16)) & np.uint32(1)) + np.uint32(0x7FFF)
    return ((u + rnd) >> np.uint32(16)).astype(np.uint16)


def bf16_to_f32(bits: np.ndarray) -> np.ndarray:
    """bf16 bit patterns (uint16) -> the float32 values they denote (exact)."""
    return (bits.astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------------------
# cut points


def uniform_cuts(dim: int, nblocks: int) -> List[int]:
    """One tile shape t = ceil(dim / nblocks) along an axis; only the last tile
    may be ragged (the ScaLAPACK-style partition of Section 2.1)."""
    t = -(-dim // nblocks) if nblocks else 0
    return [min(i * t, dim) for i in range(nblocks + 1)]


def jittered_cuts(dim: int, nblocks: int, seed: int) -> List[int]:
    """Uneven blocks: cut_i = round(i dim / n) + U{-w..w}, w = floor(dim/(4n))."""
    rng = np.random.default_rng(seed)
    w = dim // (4 * nblocks)
    jit = rng.integers(-w, w + 1, size=max(nblocks - 1, 0))
    cuts = [0] + [int(round(i * dim / nblocks)) + int(jit[i - 1]) for i in range(1, nblocks)] + [dim]
    return cuts


def desc(rows: int, cols: int, row_cuts, col_cuts, proc_rows: int, proc_cols: int,
         replication: int = 1) -> Dict:
    return dict(rows=int(rows), cols=int(cols),
                row_cuts=tuple(int(c) for c in row_cuts), col_cuts=tuple(int(c) for c in col_cuts),
                proc_rows=int(proc_rows), proc_cols=int(proc_cols), replication=int(replication))


def block_desc(rows: int, cols: int, grid_rows: int, grid_cols: int, replication: int = 1,
               proc_rows: int = None, proc_cols: int = None) -> Dict:
    """Uniform grid_rows x grid_cols blocks on a process grid of the same shape
    (row block: grid_cols = 1, column block: grid_rows = 1)."""
    return desc(rows, cols, uniform_cuts(rows, grid_rows), uniform_cuts(cols, grid_cols),
                proc_rows or grid_rows, proc_cols or grid_cols, replication)


# ---------------------------------------------------------------------------
# the five benchmark configurations


def _cfg1() -> Dict:
    M = K = N = 256
    return dict(name="cfg1", M=M, K=K, N=N, dtype="f32", nranks=4,
                A=block_desc(M, K, 4, 1), B=block_desc(K, N, 2, 2), C=block_desc(M, N, 2, 2),
                dist=("normal", 1.0), seeds=(1001, 1002),
                what="A 1D row-block x4, B 2x2, C 2x2, no replication")


def _cfg2() -> Dict:
    M = K = N = 4096
    return dict(name="cfg2", M=M, K=K, N=N, dtype="bf16", nranks=8,
                A=block_desc(M, K, 8, 1), B=block_desc(K, N, 1, 8), C=block_desc(M, N, 4, 2),
                dist=("normal", 1.0 / 64.0), seeds=(2001, 2002),
                what="A row-block x8, B column-block x8, C 4x2 (misaligned boundaries)")


def _cfg3() -> Dict:
    M, K, N = 16384, 8192, 28672
    return dict(name="cfg3", M=M, K=K, N=N, dtype="bf16", nranks=8,
                A=block_desc(M, K, 1, 1, replication=8), B=block_desc(K, N, 1, 8),
                C=block_desc(M, N, 1, 8),
                dist=("normal", 0.02), seeds=(3001, 3002),
                what="tensor-parallel shape: A replicated x8, B and C column-block x8")


def _cfg4() -> Dict:
    M = K = N = 8192
    return dict(name="cfg4", M=M, K=K, N=N, dtype="bf16", nranks=32,
                A=block_desc(M, K, 4, 4, replication=2), B=block_desc(K, N, 4, 4, replication=2),
                C=block_desc(M, N, 4, 4, replication=2),
                dist=("normal", 1.0 / np.sqrt(8192.0)), seeds=(4001, 4002),
                what="2.5D: A, B, C 4x4 blocks, replication 2 over 32 ranks, replica sum")


def _cfg5() -> Dict:
    M, K, N = 12289, 9973, 11003
    A = desc(M, K, jittered_cuts(M, 3, 5011), jittered_cuts(K, 5, 5012), 3, 5)
    B = desc(K, N, jittered_cuts(K, 7, 5013), [0, N], 7, 1)
    C = desc(M, N, jittered_cuts(M, 5, 5014), jittered_cuts(N, 3, 5015), 5, 3)
    return dict(name="cfg5", M=M, K=K, N=N, dtype="bf16", nranks=15, A=A, B=B, C=C,
                dist=("uniform", 1.0), seeds=(5001, 5002),
                what="ragged: A 3x5 uneven, B 7 uneven row blocks, C 5x3 uneven")


# ---------------------------------------------------------------------------
# the MLP-shaped products of Section 5.2 (GPT-like MLP layer, hidden size 12K):
# MLP-1 expands m x 12K to m x 48K, MLP-2 shrinks m x 48K back to m x 12K, over 8
# ranks, in the partitionings that section compares.  m (the batch) is 8192 here.

MLP_BATCH = 8192
MLP_PARTITIONINGS = ("column", "inner", "outer", "2d")


def _mlp(layer: int, part: str) -> Dict:
    M = MLP_BATCH
    K, N = (12288, 49152) if layer == 1 else (49152, 12288)
    p = 8
    if part == "column":      # B and C in column blocks, A on every rank (tensor-parallel linear layer)
        A, B, C = block_desc(M, K, 1, 1, replication=p), block_desc(K, N, 1, p), block_desc(M, N, 1, p)
        what = "column block: A replicated x8, B and C column-block x8"
    elif part == "inner":     # row block times column block
        A, B, C = block_desc(M, K, p, 1), block_desc(K, N, 1, p), block_desc(M, N, 4, 2)
        what = "inner product: A row-block x8, B column-block x8, C 4x2"
    elif part == "outer":     # column block times row block, every rank a partial C, then the replica sum
        A, B, C = block_desc(M, K, 1, p), block_desc(K, N, p, 1), block_desc(M, N, 1, 1, replication=p)
        what = "outer product: A column-block x8, B row-block x8, C replicated x8, replica sum"
    elif part == "2d":
        A, B, C = block_desc(M, K, 2, 4), block_desc(K, N, 2, 4), block_desc(M, N, 2, 4)
        what = "2D: A, B, C in 2x4 blocks"
    else:
        raise KeyError(part)
    return dict(name=f"mlp{layer}-{part}", M=M, K=K, N=N, dtype="bf16", nranks=p, A=A, B=B, C=C,
                dist=("normal", 0.02), seeds=(6000 + 10 * layer, 6001 + 10 * layer),
                what=f"MLP-{layer} ({what})")


# ---------------------------------------------------------------------------
# ScaLAPACK-style block-cyclic layouts (Section 2.1): one tile shape nb x nb per matrix,
# the tile grid much larger than the process grid, tiles dealt to the ranks cyclically.

BLOCK_CYCLIC_NB = (512, 256, 128)


def block_cyclic_desc(rows: int, cols: int, nb_rows: int, nb_cols: int, proc_rows: int, proc_cols: int,
                      replication: int = 1) -> Dict:
    """Tiles of nb_rows x nb_cols (the last row / column of tiles may be ragged) on a
    proc_rows x proc_cols process grid."""
    rc = [min(i * nb_rows, rows) for i in range(-(-rows // nb_rows) + 1)]
    cc = [min(j * nb_cols, cols) for j in range(-(-cols // nb_cols) + 1)]
    return desc(rows, cols, rc, cc, proc_rows, proc_cols, replication)


def _block_cyclic(nb: int, M: int = 8192, K: int = 8192, N: int = 8192) -> Dict:
    p, pr, pc = 8, 2, 4
    return dict(name=f"bc{nb}", M=M, K=K, N=N, dtype="bf16", nranks=p,
                A=block_cyclic_desc(M, K, nb, nb, pr, pc), B=block_cyclic_desc(K, N, nb, nb, pr, pc),
                C=block_cyclic_desc(M, N, nb, nb, pr, pc),
                dist=("normal", 1.0 / np.sqrt(float(K))), seeds=(7000 + nb, 7001 + nb),
                what=f"block-cyclic: A, B, C in {nb} x {nb} tiles dealt to a 2x4 process grid")


_BUILDERS = dict(cfg1=_cfg1, cfg2=_cfg2, cfg3=_cfg3, cfg4=_cfg4, cfg5=_cfg5)
CONFIG_NAMES = tuple(_BUILDERS)
BLOCK_CYCLIC_NAMES = tuple(f"bc{nb}" for nb in BLOCK_CYCLIC_NB)
BLOCK_CYCLIC_FINE_NAMES = ("bc64", "bc32")      # 2.1 M and 16.8 M ops: for the benchmark, not for the CPU tests
MLP_NAMES = tuple(f"mlp{layer}-{part}" for layer in (1, 2) for part in MLP_PARTITIONINGS)


def config(name: str) -> Dict:
    if name in _BUILDERS:
        return _BUILDERS[name]()
    if name in MLP_NAMES:
        layer, part = name.split("-")
        return _mlp(int(layer[3:]), part)
    if name in BLOCK_CYCLIC_NAMES or name in BLOCK_CYCLIC_FINE_NAMES:
        return _block_cyclic(int(name[2:]))
    raise KeyError(name)


def scaled_config(name: str, M: int, K: int, N: int) -> Dict:
    """Same partitioning family as ``name`` at another size (for quick tests):
    uniform grids are rebuilt for the new shape, jittered ones re-drawn."""
    if name in BLOCK_CYCLIC_NAMES:
        return dict(_block_cyclic(int(name[2:]), M, K, N), name=f"{name}@{M}x{K}x{N}")
    base = config(name)
    out = dict(base, M=M, K=K, N=N, name=f"{name}@{M}x{K}x{N}")
    dims = dict(A=(M, K), B=(K, N), C=(M, N))
    seeds = dict(A=(5011, 5012), B=(5013, 5016), C=(5014, 5015))
    for X in "ABC":
        d = base[X]
        gr, gc = len(d["row_cuts"]) - 1, len(d["col_cuts"]) - 1
        r, c = dims[X]
        if name == "cfg5":
            rc = jittered_cuts(r, gr, seeds[X][0]) if gr > 1 else [0, r]
            cc = jittered_cuts(c, gc, seeds[X][1]) if gc > 1 else [0, c]
        else:
            rc, cc = uniform_cuts(r, gr), uniform_cuts(c, gc)
        out[X] = desc(r, c, rc, cc, d["proc_rows"], d["proc_cols"], d["replication"])
    return out


# ---------------------------------------------------------------------------
# operand values


def make_matrix(rows: int, cols: int, dist: Tuple[str, float], seed: int) -> np.ndarray:
    """Seeded float32 matrix: ('normal', sigma) or ('uniform', half_width)."""
    rng = np.random.default_rng(seed)
    kind, scale = dist
    if kind == "normal":
        x = rng.standard_normal(size=(rows, cols), dtype=np.float32)
        x *= np.float32(scale)
    elif kind == "uniform":
        x = rng.random(size=(rows, cols), dtype=np.float32)
        x *= np.float32(2.0 * scale)
        x -= np.float32(scale)
    else:
        raise ValueError(kind)
    return x


def make_operands(cfg: Dict) -> Tuple[np.ndarray, np.ndarray]:
    """Global A (M x K) and B (K x N) in the config's storage type: float32, or
    uint16 bf16 bit patterns (values drawn in fp32, rounded to nearest even)."""
    A = make_matrix(cfg["M"], cfg["K"], cfg["dist"], cfg["seeds"][0])
    B = make_matrix(cfg["K"], cfg["N"], cfg["dist"], cfg["seeds"][1])
    if cfg["dtype"] == "bf16":
        return bf16_round(A), bf16_round(B)
    return A, B


def flops(cfg: Dict) -> float:
    return 2.0 * cfg["M"] * cfg["K"] * cfg["N"]
