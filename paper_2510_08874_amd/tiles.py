"""Tile buffers on the GPU: every (replica, tile) of a distributed matrix is its
own torch allocation, as every virtual rank's tile is its own HBM buffer.
Allocation, host<->device copies and slicing by cut points only."""
from __future__ import annotations

from typing import Dict, List, Optional, Tuple

import numpy as np
import torch


def _round_up(x: int, m: int) -> int:
    return ((x + m - 1) // m) * m


class TileSet:
    """All tiles of all replicas of one matrix, in the table order of the ABI:
    ``rep * (grid_rows * grid_cols) + ti * grid_cols + tj``."""

    def __init__(self, desc: Dict, torch_dtype, device="cuda", ld_multiple: int = 1, fill: Optional[float] = None):
        self.desc = desc
        self.dtype = torch_dtype
        rc, cc = desc["row_cuts"], desc["col_cuts"]
        self.gr, self.gc = len(rc) - 1, len(cc) - 1
        self.tensors: List[Optional[torch.Tensor]] = []
        self.ld: List[int] = []
        for rep in range(desc["replication"]):
            for ti in range(self.gr):
                for tj in range(self.gc):
                    h, w = rc[ti + 1] - rc[ti], cc[tj + 1] - cc[tj]
                    ld = max(_round_up(w, ld_multiple), 1)
                    self.ld.append(ld)
                    if h == 0 or w == 0:
                        self.tensors.append(None)
                        continue
                    t = torch.empty((h, ld), dtype=torch_dtype, device=device)
                    if fill is not None:
                        t.fill_(fill)
                    self.tensors.append(t)

    def index(self, rep: int, ti: int, tj: int) -> int:
        return rep * self.gr * self.gc + ti * self.gc + tj

    def bounds(self, ti: int, tj: int) -> Tuple[int, int, int, int]:
        rc, cc = self.desc["row_cuts"], self.desc["col_cuts"]
        return rc[ti], rc[ti + 1], cc[tj], cc[tj + 1]

    def scatter(self, X: np.ndarray) -> None:
        """Copy a global host matrix into every replica's tiles.  ``X`` is
        float32, or uint16 bf16 bit patterns when the tiles are bfloat16."""
        if self.dtype == torch.bfloat16:
            host = torch.from_numpy(X.view(np.int16)).view(torch.bfloat16)
        else:
            host = torch.from_numpy(X)
        for ti in range(self.gr):
            for tj in range(self.gc):
                r0, r1, c0, c1 = self.bounds(ti, tj)
                if r1 == r0 or c1 == c0:
                    continue
                dev = host[r0:r1, c0:c1].contiguous().to(self.tensors[self.index(0, ti, tj)].device)
                for rep in range(self.desc["replication"]):
                    self.tensors[self.index(rep, ti, tj)][:, :c1 - c0].copy_(dev)

    def gather(self, rep: int = 0) -> np.ndarray:
        """Global host matrix assembled from one replica's tiles (float32)."""
        out = np.zeros((self.desc["rows"], self.desc["cols"]), dtype=np.float32)
        for ti in range(self.gr):
            for tj in range(self.gc):
                r0, r1, c0, c1 = self.bounds(ti, tj)
                if r1 == r0 or c1 == c0:
                    continue
                out[r0:r1, c0:c1] = self.tensors[self.index(rep, ti, tj)][:, :c1 - c0].float().cpu().numpy()
        return out

    def gather_rows(self, rows: np.ndarray, rep: int = 0) -> np.ndarray:
        """Selected global rows (all columns) from one replica's tiles."""
        rows = np.asarray(rows)
        out = np.zeros((len(rows), self.desc["cols"]), dtype=np.float32)
        rc = self.desc["row_cuts"]
        for ti in range(self.gr):
            sel = np.nonzero((rows >= rc[ti]) & (rows < rc[ti + 1]))[0]
            if len(sel) == 0:
                continue
            local = torch.as_tensor(rows[sel] - rc[ti], device="cpu")
            for tj in range(self.gc):
                r0, r1, c0, c1 = self.bounds(ti, tj)
                if c1 == c0:
                    continue
                t = self.tensors[self.index(rep, ti, tj)]
                out[sel, c0:c1] = t[local.to(t.device), :c1 - c0].float().cpu().numpy()
        return out

    def nbytes(self) -> int:
        return sum(t.numel() * t.element_size() for t in self.tensors if t is not None)


class DeviceProblem:
    """One partitioned product resident on the GPU: the plan, the three tile
    sets and the marshalled argument arrays of ``dmm_execute``."""

    def __init__(self, cfg: Dict, A_host: Optional[np.ndarray] = None, B_host: Optional[np.ndarray] = None,
                 ld_multiple: int = 1, c_fill: Optional[float] = None, device="cuda", c_dtype: str = "f32"):
        from . import binding
        self.cfg = cfg
        self.binding = binding
        self.dtype_code = binding.DMM_BF16 if cfg["dtype"] == "bf16" else binding.DMM_F32
        tdt = torch.bfloat16 if cfg["dtype"] == "bf16" else torch.float32
        self.plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"],
                                 binding.STATIONARY_FLAGS[cfg.get("stationary", "C")] |
                                 (binding.DMM_ITERATION_OFFSET if cfg.get("iteration_offset") else 0) |
                                 (binding.DMM_MERGE_ALWAYS if cfg.get("merge_always") else 0))
        self.A = TileSet(cfg["A"], tdt, device, ld_multiple)
        self.B = TileSet(cfg["B"], tdt, device, ld_multiple)
        # C tiles are fp32, or bf16 when asked for (DMM_C_BF16 then goes with every execute)
        self.c_flags = binding.DMM_C_BF16 if c_dtype == "bf16" else 0
        self.C = TileSet(cfg["C"], torch.bfloat16 if c_dtype == "bf16" else torch.float32, device, ld_multiple,
                         fill=c_fill)
        if A_host is not None:
            self.A.scatter(A_host)
        if B_host is not None:
            self.B.scatter(B_host)
        self.args = self.plan.marshal(self.A.tensors, self.A.ld, self.B.tensors, self.B.ld,
                                      self.C.tensors, self.C.ld)

    def execute(self, flags: int = 0, stream: Optional[int] = None) -> None:
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.plan.execute_marshalled(self.dtype_code, self.args, flags | self.c_flags, stream)

    def reduce(self, origin: int = 0, stream: Optional[int] = None) -> None:
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.plan.reduce_replicas(self.C.tensors, self.C.ld, origin, stream)

    def broadcast(self, origin: int = 0, stream: Optional[int] = None) -> None:
        if stream is None:
            stream = torch.cuda.current_stream().cuda_stream
        self.plan.broadcast_replica(self.C.tensors, self.C.ld, origin, stream)

    def c_global(self, rep: int = 0) -> np.ndarray:
        torch.cuda.synchronize()
        return self.C.gather(rep)

    def close(self) -> None:
        torch.cuda.synchronize()
        self.plan.destroy()
