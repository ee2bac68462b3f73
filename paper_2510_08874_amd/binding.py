"""ctypes binding of ``include/dmm.h``: same names, argument marshalling only.

Every step of the path (planning, grouping, the grouped GEMM, the replica sum)
runs inside ``libdmm.so``; this module converts Python descriptors and torch /
integer device pointers into the C structures and back.  There is no fallback:
if the library is missing, importing a function from here raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Dict, List, Optional, Sequence

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdmm.so")

DMM_OK, DMM_EINVAL, DMM_ESHAPE, DMM_EREPL, DMM_ENOMEM, DMM_EHIP, DMM_ELD, DMM_ELIMIT = 0, -1, -2, -3, -4, -5, -6, -7
DMM_BF16, DMM_F32 = 1, 2
DMM_STATIONARY_B = 0x1        # dmm_plan flags (bits 0 .. 7)
DMM_STATIONARY_A = 0x2
DMM_ITERATION_OFFSET = 0x4
DMM_MERGE_ALWAYS = 0x8
DMM_NO_REDUCE = 0x100         # dmm_execute flags (bits 8 .. 15)
DMM_TIMING = 0x200
DMM_C_BF16 = 0x400
DMM_NO_MERGE = 0x800
DMM_SEPARATE_REDUCE = 0x1000
DMM_STATIC_SCRATCH_BYTES = 1 << 20
STATIONARY_FLAGS = {"C": 0, "B": DMM_STATIONARY_B, "A": DMM_STATIONARY_A}
STATUS_NAMES = {0: "OK", -1: "EINVAL", -2: "ESHAPE", -3: "EREPL", -4: "ENOMEM", -5: "EHIP", -6: "ELD", -7: "ELIMIT"}


class dmm_matrix_desc(C.Structure):
    _fields_ = [("rows", C.c_int64), ("cols", C.c_int64),
                ("grid_rows", C.c_int32), ("grid_cols", C.c_int32),
                ("row_cuts", C.POINTER(C.c_int64)), ("col_cuts", C.POINTER(C.c_int64)),
                ("proc_rows", C.c_int32), ("proc_cols", C.c_int32),
                ("replication", C.c_int32)]


class dmm_task(C.Structure):
    _fields_ = [("rank", C.c_int32),
                ("a_rep", C.c_int32), ("a_ti", C.c_int32), ("a_tj", C.c_int32),
                ("b_rep", C.c_int32), ("b_ti", C.c_int32), ("b_tj", C.c_int32),
                ("c_rep", C.c_int32), ("c_ti", C.c_int32), ("c_tj", C.c_int32),
                ("m0", C.c_int64), ("m1", C.c_int64), ("k0", C.c_int64), ("k1", C.c_int64),
                ("n0", C.c_int64), ("n1", C.c_int64)]

    def astuple(self):
        return tuple(int(getattr(self, f)) for f, _ in self._fields_)


class dmm_work_item(C.Structure):
    _fields_ = [("group", C.c_int64), ("m0", C.c_int64), ("n0", C.c_int64),
                ("m_ext", C.c_int32), ("n_ext", C.c_int32),
                ("c_rep", C.c_int32), ("c_ti", C.c_int32), ("c_tj", C.c_int32),
                ("reserved", C.c_int32)]


class dmm_merged_item(C.Structure):
    _fields_ = [("m0", C.c_int64), ("n0", C.c_int64), ("m_ext", C.c_int32), ("n_ext", C.c_int32),
                ("c_rep", C.c_int32), ("row_pieces", C.c_int32), ("col_pieces", C.c_int32),
                ("reserved", C.c_int32)]


class dmm_execute_report(C.Structure):
    _fields_ = [("ran_merged", C.c_int32), ("ran_k_split", C.c_int32), ("ran_fused", C.c_int32), ("table_reused", C.c_int32)]


class DmmError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        self.kind = STATUS_NAMES.get(status, str(status))
        msg = lib().dmm_strerror(status).decode()
        if status == DMM_EHIP:
            msg += f" (hipError_t {lib().dmm_last_hip_error()})"
        super().__init__(f"{where}: {self.kind}: {msg}")


_lib = None


def lib() -> C.CDLL:
    """The loaded library.  Raises if it has not been built (no fallback)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2510_08874_amd.build` "
                              "(there is no CPU or PyTorch fallback)")
        L = C.CDLL(LIB_PATH)
        P = C.c_void_p
        L.dmm_plan.restype = C.c_int
        L.dmm_plan.argtypes = [C.POINTER(dmm_matrix_desc)] * 3 + [C.c_int32, C.c_uint32, C.POINTER(P)]
        L.dmm_plan_num_tasks.restype = C.c_int64
        L.dmm_plan_num_tasks.argtypes = [P]
        L.dmm_plan_tasks.restype = C.POINTER(dmm_task)
        L.dmm_plan_tasks.argtypes = [P]
        L.dmm_plan_order.restype = C.POINTER(C.c_int64)
        L.dmm_plan_order.argtypes = [P]
        L.dmm_plan_num_groups.restype = C.c_int64
        L.dmm_plan_num_groups.argtypes = [P]
        L.dmm_plan_group_offsets.restype = C.POINTER(C.c_int64)
        L.dmm_plan_group_offsets.argtypes = [P]
        L.dmm_plan_num_items.restype = C.c_int64
        L.dmm_plan_num_items.argtypes = [P]
        L.dmm_plan_items.restype = C.POINTER(dmm_work_item)
        L.dmm_plan_items.argtypes = [P]
        L.dmm_plan_num_merged_items.restype = C.c_int64
        L.dmm_plan_num_merged_items.argtypes = [P]
        L.dmm_plan_merged_items.restype = C.POINTER(dmm_merged_item)
        L.dmm_plan_merged_items.argtypes = [P]
        L.dmm_plan_last_execute.restype = C.c_int
        L.dmm_plan_last_execute.argtypes = [P, C.POINTER(dmm_execute_report)]
        L.dmm_plan_macro_tile.restype = C.c_int32
        L.dmm_plan_macro_tile.argtypes = [P]
        L.dmm_execute.restype = C.c_int
        L.dmm_execute.argtypes = [P, C.c_int, P, P, P, P, P, P, C.c_uint32, P]
        L.dmm_reduce_replicas.restype = C.c_int
        L.dmm_reduce_replicas.argtypes = [P, P, P, C.c_int32, P]
        L.dmm_broadcast_replica.restype = C.c_int
        L.dmm_broadcast_replica.argtypes = [P, P, P, C.c_int32, P]
        L.dmm_reduce_replicas_static.restype = C.c_int
        L.dmm_reduce_replicas_static.argtypes = [P, P, P, C.c_int32, P]
        L.dmm_plan_elapsed_ms.restype = C.c_int
        L.dmm_plan_elapsed_ms.argtypes = [P, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        L.dmm_plan_gemm_launch_ms.restype = C.c_int
        L.dmm_plan_gemm_launch_ms.argtypes = [P, C.POINTER(C.c_float), C.POINTER(C.c_double)]
        L.dmm_plan_destroy.restype = None
        L.dmm_plan_destroy.argtypes = [P]
        L.dmm_strerror.restype = C.c_char_p
        L.dmm_strerror.argtypes = [C.c_int]
        L.dmm_last_hip_error.restype = C.c_int
        L.dmm_version.restype = C.c_int
        L.dmm_measure_mfma_rate.restype = C.c_int
        L.dmm_measure_mfma_rate.argtypes = [C.c_float, C.c_int, C.POINTER(C.c_float), C.POINTER(C.c_float)]
        _lib = L
    return _lib


EXPORTS = ("dmm_plan", "dmm_plan_num_tasks", "dmm_plan_tasks", "dmm_plan_order", "dmm_plan_num_groups",
           "dmm_plan_group_offsets", "dmm_plan_num_items", "dmm_plan_items", "dmm_plan_macro_tile",
           "dmm_plan_num_merged_items", "dmm_plan_merged_items", "dmm_plan_last_execute",
           "dmm_reduce_replicas_static",
           "dmm_execute", "dmm_reduce_replicas", "dmm_broadcast_replica", "dmm_plan_elapsed_ms", "dmm_plan_gemm_launch_ms", "dmm_plan_destroy", "dmm_strerror",
           "dmm_last_hip_error", "dmm_version", "dmm_measure_mfma_rate")


def _desc(d: Dict, keep: List) -> dmm_matrix_desc:
    rc = (C.c_int64 * len(d["row_cuts"]))(*d["row_cuts"])
    cc = (C.c_int64 * len(d["col_cuts"]))(*d["col_cuts"])
    keep += [rc, cc]
    return dmm_matrix_desc(d["rows"], d["cols"], len(d["row_cuts"]) - 1, len(d["col_cuts"]) - 1,
                           C.cast(rc, C.POINTER(C.c_int64)), C.cast(cc, C.POINTER(C.c_int64)),
                           d["proc_rows"], d["proc_cols"], d["replication"])


def _ptr(x) -> int:
    """Device address of a torch tensor, or an int address, or None."""
    if x is None:
        return 0
    if isinstance(x, int):
        return x
    return int(x.data_ptr())


def _table(entries: Sequence, ctype):
    return (ctype * max(len(entries), 1))(*entries)


class Plan:
    """Owns a ``dmm_plan_t``.  Descriptors are dicts with the fields of
    ``dmm_matrix_desc`` (rows, cols, row_cuts, col_cuts, proc_rows, proc_cols,
    replication)."""

    def __init__(self, A: Dict, B: Dict, Cd: Dict, nranks: int, flags: int = 0):
        keep: List = []
        a, b, c = _desc(A, keep), _desc(B, keep), _desc(Cd, keep)
        handle = C.c_void_p()
        rc = lib().dmm_plan(C.byref(a), C.byref(b), C.byref(c), nranks, flags, C.byref(handle))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_plan")
        self._h = handle
        self.A, self.B, self.C, self.nranks = A, B, Cd, nranks

    # -- accessors ---------------------------------------------------------
    @property
    def handle(self):
        return self._h

    def num_tasks(self) -> int:
        return int(lib().dmm_plan_num_tasks(self._h))

    def tasks(self) -> List[tuple]:
        p = lib().dmm_plan_tasks(self._h)
        return [p[i].astuple() for i in range(self.num_tasks())]

    def order(self) -> List[int]:
        p = lib().dmm_plan_order(self._h)
        return [int(p[i]) for i in range(self.num_tasks())]

    def num_groups(self) -> int:
        return int(lib().dmm_plan_num_groups(self._h))

    def group_offsets(self) -> List[int]:
        p = lib().dmm_plan_group_offsets(self._h)
        return [int(p[i]) for i in range(self.num_groups() + 1)]

    def num_items(self) -> int:
        return int(lib().dmm_plan_num_items(self._h))

    def items(self) -> List[Dict]:
        p = lib().dmm_plan_items(self._h)
        return [{f: int(getattr(p[i], f)) for f, _ in dmm_work_item._fields_ if f != "reserved"}
                for i in range(self.num_items())]

    def num_merged_items(self) -> int:
        return int(lib().dmm_plan_num_merged_items(self._h))

    def merged_items(self) -> List[Dict]:
        p = lib().dmm_plan_merged_items(self._h)
        return [{f: int(getattr(p[i], f)) for f, _ in dmm_merged_item._fields_ if f != "reserved"}
                for i in range(self.num_merged_items())]

    def last_execute(self) -> "dmm_execute_report":
        """What the last execute on this plan did (dmm_plan_last_execute)."""
        rep = dmm_execute_report()
        rc = lib().dmm_plan_last_execute(self._h, C.byref(rep))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_plan_last_execute")
        return rep

    def ran_merged(self) -> bool:
        return bool(self.last_execute().ran_merged)

    def table_reused(self) -> bool:
        """The last execute launched from the work tables the call before it had left on the device."""
        return bool(self.last_execute().table_reused)

    def ran_fused(self) -> int:
        """0: the last execute did not sum C's replicas in the GEMM; 1: it did, in one launch; 2: in two."""
        return int(self.last_execute().ran_fused)

    def ran_k_split(self) -> bool:
        return bool(self.last_execute().ran_k_split)

    def macro_tile(self) -> int:
        return int(lib().dmm_plan_macro_tile(self._h))

    # -- device calls --------------------------------------------------------
    def execute(self, dtype: int, a_tiles: Sequence, a_ld: Sequence[int], b_tiles: Sequence,
                b_ld: Sequence[int], c_tiles: Sequence, c_ld: Sequence[int], flags: int = 0,
                stream: Optional[int] = None) -> None:
        """``dmm_execute``.  Tile tables are sequences of torch tensors / int
        device addresses / None in table order; ``stream`` is a hipStream_t as int."""
        args = self.marshal(a_tiles, a_ld, b_tiles, b_ld, c_tiles, c_ld)
        self.execute_marshalled(dtype, args, flags, stream)

    def marshal(self, a_tiles, a_ld, b_tiles, b_ld, c_tiles, c_ld):
        """The six C arrays of ``dmm_execute`` (reusable across calls)."""
        return (_table([_ptr(t) for t in a_tiles], C.c_void_p), _table(list(a_ld), C.c_int64),
                _table([_ptr(t) for t in b_tiles], C.c_void_p), _table(list(b_ld), C.c_int64),
                _table([_ptr(t) for t in c_tiles], C.c_void_p), _table(list(c_ld), C.c_int64))

    def execute_marshalled(self, dtype: int, args, flags: int = 0, stream: Optional[int] = None) -> None:
        rc = lib().dmm_execute(self._h, dtype, *args, flags, C.c_void_p(stream or 0))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_execute")

    def reduce_replicas(self, c_tiles: Sequence, c_ld: Sequence[int], origin: int = 0,
                        stream: Optional[int] = None) -> None:
        ct = _table([_ptr(t) for t in c_tiles], C.c_void_p)
        cl = _table(list(c_ld), C.c_int64)
        rc = lib().dmm_reduce_replicas(self._h, ct, cl, origin, C.c_void_p(stream or 0))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_reduce_replicas")

    def reduce_replicas_static(self, c_tiles: Sequence, c_ld: Sequence[int], origin: int = 0,
                               stream: Optional[int] = None) -> None:
        ct = _table([_ptr(t) for t in c_tiles], C.c_void_p)
        cl = _table(list(c_ld), C.c_int64)
        rc = lib().dmm_reduce_replicas_static(self._h, ct, cl, origin, C.c_void_p(stream or 0))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_reduce_replicas_static")

    def broadcast_replica(self, c_tiles: Sequence, c_ld: Sequence[int], origin: int = 0,
                          stream: Optional[int] = None) -> None:
        ct = _table([_ptr(t) for t in c_tiles], C.c_void_p)
        cl = _table(list(c_ld), C.c_int64)
        rc = lib().dmm_broadcast_replica(self._h, ct, cl, origin, C.c_void_p(stream or 0))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_broadcast_replica")

    def elapsed_ms(self):
        """(gemm_ms, reduce_ms) of the last execute with DMM_TIMING; -1 = not timed."""
        g, r = C.c_float(-1.0), C.c_float(-1.0)
        rc = lib().dmm_plan_elapsed_ms(self._h, C.byref(g), C.byref(r))
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_plan_elapsed_ms")
        return float(g.value), float(r.value)

    def gemm_launch_ms(self):
        """((ms, flops) of the launch over replicas 1.., (ms, flops) of the launch over replica 0) of the last
        execute with DMM_TIMING that fused the replica sum; ms = -1 where there is nothing to report."""
        ms, fl = (C.c_float * 2)(), (C.c_double * 2)()
        rc = lib().dmm_plan_gemm_launch_ms(self._h, ms, fl)
        if rc != DMM_OK:
            raise DmmError(rc, "dmm_plan_gemm_launch_ms")
        return (float(ms[0]), float(fl[0])), (float(ms[1]), float(fl[1]))

    def destroy(self) -> None:
        if getattr(self, "_h", None):
            lib().dmm_plan_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.destroy()
        except Exception:
            pass


def dmm_plan(A: Dict, B: Dict, Cd: Dict, nranks: int, flags: int = 0) -> Plan:
    return Plan(A, B, Cd, nranks, flags)


def dmm_execute(plan: Plan, dtype: int, a_tiles, a_ld, b_tiles, b_ld, c_tiles, c_ld, flags: int = 0,
                stream: Optional[int] = None) -> None:
    plan.execute(dtype, a_tiles, a_ld, b_tiles, b_ld, c_tiles, c_ld, flags, stream)


def dmm_reduce_replicas(plan: Plan, c_tiles, c_ld, origin: int = 0, stream: Optional[int] = None) -> None:
    plan.reduce_replicas(c_tiles, c_ld, origin, stream)


def dmm_reduce_replicas_static(plan: Plan, c_tiles, c_ld, origin: int = 0, stream: Optional[int] = None) -> None:
    plan.reduce_replicas_static(c_tiles, c_ld, origin, stream)


def dmm_plan_destroy(plan: Plan) -> None:
    plan.destroy()


def dmm_strerror(status: int) -> str:
    return lib().dmm_strerror(status).decode()


def dmm_version() -> int:
    return int(lib().dmm_version())


def dmm_measure_mfma_rate(milliseconds: float, random_operands: bool = True):
    """(TFLOP/s, shader MHz) of a register-only MFMA loop on the current device."""
    tf, mhz = C.c_float(0.0), C.c_float(0.0)
    rc = lib().dmm_measure_mfma_rate(C.c_float(milliseconds), 1 if random_operands else 0, C.byref(tf), C.byref(mhz))
    if rc != DMM_OK:
        raise DmmError(rc, "dmm_measure_mfma_rate")
    return float(tf.value), float(mhz.value)
