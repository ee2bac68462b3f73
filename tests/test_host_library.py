"""CPU-side tests of the library: it loads, exports the whole ABI, and its
planner / grouping agree bit for bit with the oracle (no GPU, no compute call)."""
import ctypes
import os
import re

import numpy as np
import pytest

import workloads
from oracle import planner as oplanner
from tests import helpers
from tests.helpers import dist

binding = pytest.importorskip("paper_2510_08874_amd.binding")

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _both(prob, mode="C"):
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    want = oplanner.plan(A, B, C, prob["nranks"], stationary=mode)
    plan = binding.Plan(prob["A"], prob["B"], prob["C"], prob["nranks"], binding.STATIONARY_FLAGS[mode])
    return plan, want, (A, B, C)


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "dmm.h")).read()
    declared = set(re.findall(r"\b(dmm_[a-z_]+)\s*\(", header))
    declared -= {"dmm_plan_t"}
    assert declared == set(binding.EXPORTS)
    L = ctypes.CDLL(binding.LIB_PATH)
    for name in declared:
        assert hasattr(L, name), name
    assert binding.dmm_version() >= 1
    assert "replication" in binding.dmm_strerror(binding.DMM_EREPL)


@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_benchmark_configs_bit_exact(name):
    cfg = workloads.config(name)
    plan, want, (A, B, C) = _both(cfg)
    assert plan.tasks() == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    plan.destroy()


@pytest.mark.parametrize("seed", range(150))
def test_random_problems_bit_exact(seed):
    prob = helpers.random_problem(seed, allow_empty=(seed % 3 == 0))
    plan, want, (A, B, C) = _both(prob)
    got = plan.tasks()
    assert got == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    # and the library's own list satisfies the mathematical pins directly
    helpers.check_task_list([oplanner.Task(*t) for t in got], A, B, C, prob["nranks"])


@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("name", workloads.CONFIG_NAMES)
def test_benchmark_configs_bit_exact_stationary_b_and_a(name, mode):
    cfg = workloads.config(name)
    plan, want, (A, B, C) = _both(cfg, mode)
    assert plan.tasks() == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    plan.destroy()


@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("seed", range(100))
def test_random_problems_bit_exact_stationary_b_and_a(seed, mode):
    prob = helpers.random_problem(seed + 2000, allow_empty=(seed % 3 == 0))
    plan, want, (A, B, C) = _both(prob, mode)
    got = plan.tasks()
    assert got == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    helpers.check_task_list([oplanner.Task(*t) for t in got], A, B, C, prob["nranks"], stationary=mode)
    plan.destroy()


@pytest.mark.parametrize("mode", ["C", "B", "A"])
@pytest.mark.parametrize("seed", range(40))
def test_iteration_offset_bit_exact(seed, mode):
    prob = helpers.random_problem(seed + 3000, allow_empty=(seed % 4 == 0))
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    want = oplanner.plan(A, B, C, prob["nranks"], stationary=mode, iteration_offset=True)
    plan = binding.Plan(prob["A"], prob["B"], prob["C"], prob["nranks"],
                        binding.STATIONARY_FLAGS[mode] | binding.DMM_ITERATION_OFFSET)
    assert plan.tasks() == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    # the work items do not depend on the flag
    plain = binding.Plan(prob["A"], prob["B"], prob["C"], prob["nranks"], binding.STATIONARY_FLAGS[mode])
    assert plan.items() == plain.items()
    plan.destroy()
    plain.destroy()


def test_stationary_flags_exclusive():
    ok = dict(rows=8, cols=8, row_cuts=(0, 8), col_cuts=(0, 8), proc_rows=1, proc_cols=1, replication=1)
    for flags in (3, 7, 11, 16, 32):
        with pytest.raises(binding.DmmError) as e:
            binding.Plan(ok, ok, ok, 1, flags)
        assert e.value.kind == "EINVAL"


@pytest.mark.parametrize("mode", ["C", "B", "A"])
@pytest.mark.parametrize("seed", range(40))
def test_work_items_tile_every_replica_of_c_once(seed, mode):
    prob = helpers.random_problem(seed, max_dim=40, allow_empty=(seed % 2 == 0))
    plan, want, (A, B, C) = _both(prob, mode)
    T = plan.macro_tile()
    hit = np.zeros((C.replication, prob["M"], prob["N"]), dtype=np.int32)
    groups = plan.group_offsets()
    order = plan.order()
    for it in plan.items():
        assert 1 <= it["m_ext"] <= T and 1 <= it["n_ext"] <= T
        (r0, r1), (c0, c1) = C.tile_bounds((it["c_ti"], it["c_tj"]))
        assert r0 <= it["m0"] and it["m0"] + it["m_ext"] <= r1 and c0 <= it["n0"] and it["n0"] + it["n_ext"] <= c1
        hit[it["c_rep"], it["m0"]:it["m0"] + it["m_ext"], it["n0"]:it["n0"] + it["n_ext"]] += 1
        if it["group"] >= 0:
            head = want[order[groups[it["group"]]]]
            assert (head.c_rep, head.c_ti, head.c_tj) == (it["c_rep"], it["c_ti"], it["c_tj"])
            assert head.m0 <= it["m0"] and it["m0"] + it["m_ext"] <= head.m1
            assert head.n0 <= it["n0"] and it["n0"] + it["n_ext"] <= head.n1
        else:
            r = it["c_rep"]
            if mode == "C":
                assert (r * prob["K"]) // C.replication == ((r + 1) * prob["K"]) // C.replication
            # a zero-fill item lies where no task writes in that replica
            for t in want:
                if t.c_rep == r:
                    assert (t.m1 <= it["m0"] or it["m0"] + it["m_ext"] <= t.m0 or
                            t.n1 <= it["n0"] or it["n0"] + it["n_ext"] <= t.n0)
    assert (hit == 1).all()


def test_large_config_items():
    cfg = workloads.config("cfg4")
    plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"])
    items = plan.items()
    assert len(items) == 2 * (8192 // 256) ** 2
    cfg = workloads.config("cfg5")
    plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"])
    area = sum(it["m_ext"] * it["n_ext"] for it in plan.items())
    assert area == cfg["M"] * cfg["N"]


def test_error_codes_match_the_oracle():
    ok = dict(rows=8, cols=8, row_cuts=(0, 8), col_cuts=(0, 8), proc_rows=1, proc_cols=1, replication=1)
    cases = [
        (dict(ok, cols=6, col_cuts=(0, 6)), ok, ok, 2),
        (dict(ok, replication=3), ok, ok, 4),
        (dict(ok, proc_rows=2, proc_cols=2, replication=2), ok, ok, 4),
        (dict(ok, row_cuts=(0, 5, 3, 8)), ok, ok, 1),
        (dict(ok, row_cuts=(1, 8)), ok, ok, 1),
        (dict(ok, row_cuts=(0, 7)), ok, ok, 1),
        (ok, ok, dict(ok, replication=5), 12),
    ]
    for A, B, Cd, p in cases:
        with pytest.raises(oplanner.PlanError) as want:
            oplanner.plan(dist(A), dist(B), dist(Cd), p)
        with pytest.raises(binding.DmmError) as got:
            binding.Plan(A, B, Cd, p)
        assert got.value.kind == want.value.kind


def test_null_arguments_rejected():
    L = binding.lib()
    assert L.dmm_plan(None, None, None, 1, 0, None) == binding.DMM_EINVAL
    assert L.dmm_plan_num_tasks(None) == 0
    assert L.dmm_execute(None, 1, None, None, None, None, None, None, 0, None) == binding.DMM_EINVAL
    assert L.dmm_reduce_replicas(None, None, None, 0, None) == binding.DMM_EINVAL
    assert L.dmm_reduce_replicas_static(None, None, None, 0, None) == binding.DMM_EINVAL
    assert L.dmm_plan_last_execute(None, None) == binding.DMM_EINVAL
    rep = binding.dmm_execute_report(7, 7, 7, 7)
    assert L.dmm_plan_last_execute(None, rep) == binding.DMM_OK
    assert (rep.ran_merged, rep.ran_k_split, rep.ran_fused, rep.table_reused) == (0, 0, 0, 0)
    assert L.dmm_plan_gemm_launch_ms(None, None, None) == binding.DMM_EINVAL
    ok = dict(rows=8, cols=8, row_cuts=(0, 8), col_cuts=(0, 8), proc_rows=1, proc_cols=1, replication=1)
    fresh = binding.Plan(ok, ok, ok, 1)
    assert fresh.gemm_launch_ms() == ((-1.0, 0.0), (-1.0, 0.0))      # nothing ran: nothing to report, no device call
    fresh.destroy()
    L.dmm_plan_destroy(None)


def test_plan_and_execute_flags_share_no_bit():
    """A flag handed to the wrong call is rejected instead of being taken for another one."""
    plan_flags = binding.DMM_STATIONARY_B | binding.DMM_STATIONARY_A | binding.DMM_ITERATION_OFFSET | binding.DMM_MERGE_ALWAYS
    exec_flags = [binding.DMM_NO_REDUCE, binding.DMM_TIMING, binding.DMM_C_BF16, binding.DMM_NO_MERGE, binding.DMM_SEPARATE_REDUCE]
    ok = dict(rows=8, cols=8, row_cuts=(0, 8), col_cuts=(0, 8), proc_rows=1, proc_cols=1, replication=1)
    for f in exec_flags:
        assert f & plan_flags == 0
        with pytest.raises(binding.DmmError) as e:
            binding.Plan(ok, ok, ok, 1, f)
        assert e.value.kind == "EINVAL"
    header = open(os.path.join(ROOT, "include", "dmm.h")).read()
    for name in ("DMM_STATIONARY_B", "DMM_STATIONARY_A", "DMM_ITERATION_OFFSET", "DMM_MERGE_ALWAYS", "DMM_NO_REDUCE",
                 "DMM_TIMING", "DMM_C_BF16", "DMM_NO_MERGE", "DMM_SEPARATE_REDUCE"):
        value = int(re.search(r"#define %s (0x[0-9a-fA-F]+)u" % name, header).group(1), 16)
        assert value == getattr(binding, name), name


# ---- block-cyclic layouts: tile grid much larger than the process grid (Section 2.1) ----------

@pytest.mark.parametrize("mode", ["C", "B", "A"])
@pytest.mark.parametrize("dims,nb", [((768, 512, 640), 64), ((700, 333, 517), 96)])
def test_block_cyclic_bit_exact(dims, nb, mode):
    """Up to 12 x 12 tiles dealt to a 2 x 4 process grid, ragged last tiles in the second case:
    every rank owns many scattered tiles, and the list, its grouped order and the group offsets
    still equal the oracle's."""
    cfg = workloads._block_cyclic(nb, *dims)
    plan, want, (A, B, C) = _both(cfg, mode)
    got = plan.tasks()
    assert got == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    owners = {t[0] for t in got}
    assert owners == set(range(8))
    plan.destroy()


@pytest.mark.parametrize("name", workloads.BLOCK_CYCLIC_NAMES)
def test_block_cyclic_full_size_counts(name):
    """At the benchmark size (up to 64^3 = 262144 ops) the properties that hold at any size:
    g^3 ops, g^2 groups of g ascending K-segments each, every op a full nb^3 box, every rank g^3 / 8 ops."""
    cfg = workloads.config(name)
    nb = int(name[2:])
    g = 8192 // nb
    plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"])
    assert plan.num_tasks() == g ** 3 and plan.num_groups() == g * g
    n = plan.num_tasks()
    T = np.ctypeslib.as_array(ctypes.cast(binding.lib().dmm_plan_tasks(plan.handle), ctypes.POINTER(ctypes.c_int32)),
                              shape=(n, ctypes.sizeof(binding.dmm_task) // 4))
    ranks = T[:, 0]
    assert (np.bincount(ranks, minlength=8) == g ** 3 // 8).all()
    box = T[:, 10:].copy().view(np.int64)                     # m0 m1 k0 k1 n0 n1
    assert ((box[:, 1] - box[:, 0] == nb) & (box[:, 3] - box[:, 2] == nb) & (box[:, 5] - box[:, 4] == nb)).all()
    order = np.ctypeslib.as_array(binding.lib().dmm_plan_order(plan.handle), shape=(n,))
    off = np.ctypeslib.as_array(binding.lib().dmm_plan_group_offsets(plan.handle), shape=(g * g + 1,))
    assert (np.diff(off) == g).all() and sorted(order.tolist()) == list(range(n))
    k0 = box[order, 2].reshape(g * g, g)
    assert (k0 == np.arange(g) * nb).all()                  # every group walks k = 0, nb, 2 nb, ...
    mn = box[order][:, [0, 4]].reshape(g * g, g, 2)
    assert (mn == mn[:, :1, :]).all()                         # one output sub-tile per group
    # owner of C tile (i, j) on the 2 x 4 process grid
    ti, tj = mn[:, 0, 0] // nb, mn[:, 0, 1] // nb
    assert (ranks[order].reshape(g * g, g) == ((ti % 2) * 4 + tj % 4)[:, None]).all()
    plan.destroy()


def test_grouping_falls_back_when_output_sub_tiles_outnumber_ops():
    """Eight C replicas but a single k value: seven replicas get no op at all, so a dense numbering of
    (replica, row interval, column interval) is much larger than the op list and the library takes
    its comparison sort; the result still equals the oracle's."""
    M, K, N, p = 70, 1, 66, 8
    cuts_m, cuts_n = tuple(range(0, M + 1, 2)), tuple(range(0, N + 1, 2))
    prob = dict(nranks=p,
                A=dict(rows=M, cols=K, row_cuts=cuts_m, col_cuts=(0, K), proc_rows=1, proc_cols=1, replication=8),
                B=dict(rows=K, cols=N, row_cuts=(0, K), col_cuts=cuts_n, proc_rows=1, proc_cols=1, replication=8),
                C=dict(rows=M, cols=N, row_cuts=(0, M), col_cuts=(0, N), proc_rows=1, proc_cols=1, replication=8))
    plan, want, _ = _both(prob)
    assert len(want) == 35 * 33
    assert plan.tasks() == [tuple(t) for t in want]
    order, offsets = oplanner.reorder(want)
    assert plan.order() == order and plan.group_offsets() == offsets
    plan.destroy()


# ---- merged macro-tiles ----------------------------------------------------------------------

def _check_merged(plan, prob):
    """What has to hold for the alternative work list, from the descriptors alone."""
    A, B, C = dist(prob["A"]), dist(prob["B"]), dist(prob["C"])
    items = plan.merged_items()
    T = plan.macro_tile()
    assert len(items) * 10 <= plan.num_items() * 9 or (plan.num_tasks() >= 4096 and plan.num_tasks() >= 16 * plan.num_items()), \
        "merged list kept although it saves neither a tenth of the macro-tiles nor a long op list"
    mc = sorted(set(A.row_cuts) | set(C.row_cuts))
    nc = sorted(set(B.col_cuts) | set(C.col_cuts))
    hit = np.zeros((C.replication, A.rows, B.cols), dtype=np.int32)
    for it in items:
        assert 1 <= it["m_ext"] <= T and 1 <= it["n_ext"] <= T
        m0, m1, n0, n1 = it["m0"], it["m0"] + it["m_ext"], it["n0"], it["n0"] + it["n_ext"]
        hit[it["c_rep"], m0:m1, n0:n1] += 1
        inner_m = [c for c in mc if m0 < c < m1]
        inner_n = [c for c in nc if n0 < c < n1]
        assert it["row_pieces"] == len(inner_m) + 1 <= 8 and it["col_pieces"] == len(inner_n) + 1 <= 8
        assert all((c - n0) % 8 == 0 for c in inner_n), "a column piece starts inside a 16-byte chunk"
    assert (hit == 1).all(), "merged macro-tiles do not tile every C replica exactly once"


@pytest.mark.parametrize("seed", range(60))
def test_merged_items_tile_every_replica_of_c_once(seed):
    prob = helpers.random_problem(seed + 7000, max_dim=600, allow_empty=(seed % 4 == 0))
    plan = binding.Plan(prob["A"], prob["B"], prob["C"], prob["nranks"])
    cA, cB, cC = (prob[x]["replication"] for x in "ABC")
    K = prob["K"]
    for mode in ("B", "A"):
        other = binding.Plan(prob["A"], prob["B"], prob["C"], prob["nranks"], binding.STATIONARY_FLAGS[mode])
        if cA == cB == cC == 1:
            assert other.merged_items() == plan.merged_items()
        else:
            assert other.num_merged_items() == 0
        other.destroy()
    eligible = all((r * K) // cC < ((r + 1) * K) // cC for r in range(cC))      # no replica of C with an empty share of K
    if not eligible:
        assert plan.num_merged_items() == 0
    if plan.num_merged_items():
        _check_merged(plan, prob)
    plan.destroy()


def test_merged_items_of_named_workloads():
    want = dict(bc128=1024, bc256=1024, bc512=0, cfg1=1, cfg2=0, cfg3=0, cfg4=0, cfg5=0)
    for name, n in want.items():
        cfg = workloads.config(name)
        plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"])
        assert plan.num_merged_items() == n, name
        if n and cfg["M"] <= 1024:
            _check_merged(plan, cfg)
        plan.destroy()
    # 96 x 96 tiles: 256 = 2 x 96 + 64, so macro-tiles meet three or four tiles per axis and start inside tiles
    cfg = workloads._block_cyclic(96, 700, 333, 517)
    plan = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"])
    assert plan.num_merged_items() == 3 * 3 and plan.num_items() == 8 * 6
    _check_merged(plan, cfg)
    # many short segments: full macro-tiles (to be run in windows of segments), not small ones
    long_k = workloads._block_cyclic(24, 300, 4100, 300)
    lp = binding.Plan(long_k["A"], long_k["B"], long_k["C"], long_k["nranks"])
    assert [(it["m_ext"], it["row_pieces"]) for it in lp.merged_items() if it["n0"] == 0 and it["m0"] in (0, 192)] == [(192, 8), (108, 5)]
    _check_merged(lp, long_k)
    lp.destroy()
    # Stationary B / A plans: the same list while nothing is replicated, none otherwise
    for mode in ("B", "A"):
        other = binding.Plan(cfg["A"], cfg["B"], cfg["C"], cfg["nranks"], binding.STATIONARY_FLAGS[mode])
        assert other.merged_items() == plan.merged_items()
        rep = dict(cfg["A"], replication=2)
        assert binding.Plan(rep, cfg["B"], cfg["C"], 16, binding.STATIONARY_FLAGS[mode]).num_merged_items() == 0
    plan.destroy()


def test_header_is_plain_c_and_links_from_c(tmp_path):
    """include/dmm.h compiled as C99 with -pedantic -Werror; a C program plans configuration 1
    through the library (host calls only) and reads the accessors."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    exe = tmp_path / "abi_from_c"
    lib_dir = os.path.dirname(binding.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "native", "abi_from_c.c"), "-o", str(exe),
                    "-L", lib_dir, "-ldmm", "-Wl,-rpath," + lib_dir], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout
    assert "tasks 16 groups 8 items 8 merged 1 first 0:[0,64)x[0,128)x[0,128) tile 256" in out
    assert "both stationary flags: -1" in out
