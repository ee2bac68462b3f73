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
    for flags in (3, 7, 8, 16):
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
    L.dmm_plan_destroy(None)
