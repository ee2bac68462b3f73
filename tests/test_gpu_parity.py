"""GPU parity: the HIP path (through the C ABI) against the CPU oracle on the
same seeded inputs.

Bars (stated by the benchmark spec): task lists bit-exact (CPU tests); C within relative
Frobenius error 1e-5 for fp32 inputs and 2e-3 for bf16 inputs, the oracle run in
fp64 on the same (bf16-rounded) values.  The fp32 accumulation actually lands
around 1e-6, so an additional, much tighter per-element bound derived from the
arithmetic is checked too: |err| <= 4 K u32 * sum_k |a_ik b_kj| is implied by
|err| <= 4 K u32 * ||a_i|| ||b_j||, with u32 = 2^-24.
"""
import numpy as np
import pytest

import workloads
from oracle import matmul as omatmul
from oracle import planner as oplanner
from tests import helpers

torch = pytest.importorskip("torch")
pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-3}
U32 = 2.0 ** -24


def _device_problem(cfg, A, B, **kw):
    from paper_2510_08874_amd.tiles import DeviceProblem
    return DeviceProblem(cfg, A, B, **kw)


def _to_f64(X, cfg):
    return workloads.bf16_to_f32(X).astype(np.float64) if cfg["dtype"] == "bf16" else X.astype(np.float64)


def _check(C_gpu, C_ref, A64, B64, cfg, what=""):
    err = np.linalg.norm(C_gpu.astype(np.float64) - C_ref) / max(np.linalg.norm(C_ref), 1e-300)
    assert err <= TOL[cfg["dtype"]], f"{what}: relative Frobenius error {err:.3e}"
    # per-element bound from fp32 accumulation of exact products
    bound = 4.0 * A64.shape[1] * U32 * np.outer(np.linalg.norm(A64, axis=1), np.linalg.norm(B64, axis=0)) + 1e-30
    worst = np.max(np.abs(C_gpu.astype(np.float64) - C_ref) / bound)
    assert worst <= 1.0, f"{what}: element error {worst:.3f} x the fp32 accumulation bound"
    return err


def _run_full(cfg, ld_multiple=1):
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, ld_multiple=ld_multiple, c_fill=float("nan"))
    prob.execute()
    C_gpu = prob.c_global(0)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    C_ref = omatmul.matmul(A, B, bf16=(cfg["dtype"] == "bf16"))
    err = _check(C_gpu, C_ref, A64, B64, cfg, cfg["name"])
    prob.close()
    return err


# ---- element-by-element at sizes the oracle finishes in seconds ------------------

def test_cfg1_full():
    _run_full(workloads.config("cfg1"))


@pytest.mark.parametrize("name,dims,ldm", [
    ("cfg2", (768, 520, 640), 1),      # several macro-tiles, K not a multiple of the K step
    ("cfg3", (300, 333, 1100), 1),     # ragged tails in all three dimensions, odd leading dimensions
    ("cfg4", (1024, 1024, 1024), 8),   # replicated C: partial sums + replica sum
    ("cfg4", (515, 771, 1030), 1),     # same, ragged; share boundary floor(771/2) is odd
    ("cfg5", (1229, 997, 1100), 1),    # uneven cuts, 231-task structure, packed odd lds
    ("cfg5", (1229, 997, 1100), 8),    # same with leading dimensions padded to 8 elements
    ("cfg1", (260, 130, 515), 1),      # fp32 with ragged tails
])
def test_families_small(name, dims, ldm):
    cfg = workloads.scaled_config(name, *dims)
    _run_full(cfg, ld_multiple=ldm)


@pytest.mark.parametrize("seed", range(12))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_partitionings(seed, dtype):
    """Random grids, block-cyclic process grids, all replication divisors, empty tiles."""
    prob = helpers.random_problem(seed, max_dim=700, allow_empty=(seed % 2 == 1))
    cfg = dict(prob, name=f"random{seed}", dtype=dtype, dist=("normal", 1.0), seeds=(seed, seed + 500))
    _run_full(cfg)


# ---- the paper's own validation sweep (Section 5.2) ---------------------------------------------

def _family(kind, rows, cols, p_rep, c):
    """row block / column block / 2-D block over the ranks of one replica (p_rep of them)."""
    if kind == "row":
        return workloads.block_desc(rows, cols, p_rep, 1, replication=c)
    if kind == "col":
        return workloads.block_desc(rows, cols, 1, p_rep, replication=c)
    g = 2 if p_rep >= 4 else 1
    return workloads.block_desc(rows, cols, g, p_rep // g, replication=c)


@pytest.mark.parametrize("reps", [(1, 1, 1), (2, 2, 2), (4, 1, 2), (1, 8, 4), (8, 8, 8)])
def test_all_combinations_of_row_column_and_2d_blocks(reps):
    """Every combination of row block, column block and 2-D block for A, B and C (27 of them)
    under several replication triples, 8 ranks, sizes that split unevenly: all through one plan
    + execute each, element by element against the fp64 product."""
    p, M, K, N = 8, 141, 203, 167
    A, B = None, None
    worst = 0.0
    for ka in ("row", "col", "2d"):
        for kb in ("row", "col", "2d"):
            for kc in ("row", "col", "2d"):
                cfg = dict(name=f"{ka}-{kb}-{kc}/{reps}", M=M, K=K, N=N, nranks=p, dtype="bf16",
                           A=_family(ka, M, K, p // reps[0], reps[0]), B=_family(kb, K, N, p // reps[1], reps[1]),
                           C=_family(kc, M, N, p // reps[2], reps[2]), dist=("normal", 1.0), seeds=(31, 32))
                if A is None:
                    A, B = workloads.make_operands(cfg)
                    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
                    C_ref = omatmul.matmul(A, B, bf16=True)
                prob = _device_problem(cfg, A, B, c_fill=float("nan"))
                prob.execute()
                worst = max(worst, _check(prob.c_global(0), C_ref, A64, B64, cfg, cfg["name"]))
                prob.close()
    assert worst <= TOL["bf16"]


# ---- Stationary B and Stationary A plans through the same kernels -----------------------

@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("seed", range(8))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_random_partitionings_stationary_b_and_a(seed, dtype, mode):
    """Same random problems, ops attributed to the owners of B (A) tiles: other groups, other
    C replicas written, zero-filled remainders; C starts as NaN, so a region left out shows."""
    prob = helpers.random_problem(seed + 40, max_dim=700, allow_empty=(seed % 2 == 1))
    cfg = dict(prob, name=f"random{seed + 40}/S{mode}", dtype=dtype, dist=("normal", 1.0), seeds=(seed, seed + 500),
               stationary=mode)
    _run_full(cfg)


@pytest.mark.parametrize("mode", ["B", "A"])
@pytest.mark.parametrize("name,dims", [("cfg4", (515, 771, 1030)), ("cfg5", (1229, 997, 1100)), ("cfg3", (300, 333, 1100))])
def test_families_small_stationary_b_and_a(name, dims, mode):
    cfg = dict(workloads.scaled_config(name, *dims), stationary=mode)
    _run_full(cfg)


@pytest.mark.parametrize("mode", ["B", "A"])
def test_stationary_b_and_a_partials_per_replica(mode):
    """With DMM_NO_REDUCE every C replica holds exactly what the oracle's execution of the
    oracle's task list puts there (zeros included)."""
    from paper_2510_08874_amd import binding
    from oracle import execute as oexec
    A_d = dict(rows=300, cols=260, row_cuts=(0, 130, 300), col_cuts=(0, 100, 260), proc_rows=2, proc_cols=2, replication=2)
    B_d = dict(rows=260, cols=280, row_cuts=(0, 90, 260), col_cuts=(0, 150, 280), proc_rows=2, proc_cols=2, replication=2)
    C_d = dict(rows=300, cols=280, row_cuts=(0, 170, 300), col_cuts=(0, 280), proc_rows=2, proc_cols=1, replication=4)
    cfg = dict(name=f"partials/S{mode}", M=300, K=260, N=280, nranks=8, A=A_d, B=B_d, C=C_d, dtype="f32",
               dist=("normal", 1.0), seeds=(71, 72), stationary=mode)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    prob.execute(flags=binding.DMM_NO_REDUCE)
    Ad, Bd, Cd = helpers.dist(A_d), helpers.dist(B_d), helpers.dist(C_d)
    tasks = oplanner.plan(Ad, Bd, Cd, 8, stationary=mode)
    A64, B64 = A.astype(np.float64), B.astype(np.float64)
    c_tiles = oexec.execute_tasks(tasks, Ad, Bd, Cd, oexec.split_tiles(A64, Ad), oexec.split_tiles(B64, Bd))
    scale = np.linalg.norm(A64 @ B64)
    for rep in range(4):
        got = prob.c_global(rep).astype(np.float64)
        want = np.zeros((300, 280))
        for (r, ti, tj), tile in c_tiles.items():
            if r == rep:
                (r0, r1), (c0, c1) = Cd.tile_bounds((ti, tj))
                want[r0:r1, c0:c1] = tile
        assert np.isfinite(got).all()
        assert np.linalg.norm(got - want) / scale < 1e-5
        assert ((want == 0) <= (got == 0)).all()        # what nobody computes is an exact zero
    prob.close()


@pytest.mark.parametrize("dtype,dims,kcuts", [
    ("bf16", (300, 8192, 300), None),             # 4 macro-tiles x 256 K steps -> 4 runs each
    ("bf16", (515, 8200, 260), (0, 1000, 4100, 8200)),   # runs that start inside a segment, cross segments, end on a K tail
    ("f32", (260, 2100, 515), None),              # 6 macro-tiles x 132 steps -> 2 runs each
    ("bf16", (2048, 4096, 2048), None),           # 64 full macro-tiles, two runs each
    ("bf16", (70, 18000, 40), (0, 4444, 18000)),  # one small macro-tile, 8 runs
])
def test_k_split_of_the_last_round(dtype, dims, kcuts):
    """Few macro-tiles with long K: the library cuts them into runs of K steps that fill the
    idle CUs and adds the partial sums up in a fixed order.  Parity as everywhere else, bitwise
    identical from run to run, NaN-prefilled C fully overwritten."""
    M, K, N = dims
    kc = kcuts or (0, K)
    cfg = dict(name=f"ksplit-{dtype}-{M}x{K}x{N}", M=M, K=K, N=N, nranks=2, dtype=dtype,
               A=dict(rows=M, cols=K, row_cuts=(0, M), col_cuts=kc, proc_rows=1, proc_cols=min(2, len(kc) - 1), replication=1),
               B=dict(rows=K, cols=N, row_cuts=(0, K), col_cuts=(0, N), proc_rows=1, proc_cols=1, replication=2),
               C=dict(rows=M, cols=N, row_cuts=(0, M), col_cuts=(0, N), proc_rows=1, proc_cols=1, replication=1),
               dist=("normal", 1.0), seeds=(41, 42))
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    prob.execute()
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:    # (the sizes above are cut for 256 CUs)
        assert prob.plan.ran_k_split()
    first = prob.c_global(0)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    C_ref = omatmul.matmul(A, B, bf16=(dtype == "bf16"))
    _check(first, C_ref, A64, B64, cfg, cfg["name"])
    prob.execute()
    assert np.array_equal(first, prob.c_global(0))
    prob.close()


def test_one_plan_alternating_streams_and_output_sets():
    """The same plan run back to back on two streams into two different sets of C tiles (so the
    work table changes every call while the previous call may still be running): the library
    has to order its table uploads and its scratch buffer behind the earlier call itself."""
    from paper_2510_08874_amd.tiles import TileSet
    cfg = workloads.scaled_config("cfg4", 700, 8400, 520)      # long K (132 steps per share): the K-split path and its scratch too
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    other = TileSet(cfg["C"], torch.float32, "cuda", 1, fill=float("nan"))
    args = [prob.args, prob.plan.marshal(prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld, other.tensors, other.ld)]
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    for it in range(6):
        prob.plan.execute_marshalled(prob.dtype_code, args[it % 2], 0, streams[it % 2].cuda_stream)
    torch.cuda.synchronize()
    C_ref = omatmul.matmul(A, B, bf16=True)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    first = prob.C.gather(0)
    second = other.gather(0)
    _check(first, C_ref, A64, B64, cfg, "stream 0")
    assert np.array_equal(first, second)
    prob.close()


def test_work_table_grows_between_two_streams():
    """A plan whose work table outgrows its device buffer between two calls on different streams:
    the first call (partial sums only, a small table) may still be running when the second (with
    the replica sum's tables, past the buffer's 64 KB) makes the library take a larger buffer; the
    old one must not go back to the pool before the first call has finished with it."""
    from paper_2510_08874_amd import binding
    from paper_2510_08874_amd.tiles import TileSet
    cfg = workloads.scaled_config("cfg4", 4608, 2100, 4608)    # 5184 blocks of the replica sum: 83 KB of tables
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    other = TileSet(cfg["C"], torch.float32, "cuda", 1, fill=float("nan"))
    args2 = prob.plan.marshal(prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld, other.tensors, other.ld)
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    torch.cuda.synchronize()
    prob.plan.execute_marshalled(prob.dtype_code, prob.args, binding.DMM_NO_REDUCE, streams[0].cuda_stream)
    prob.plan.execute_marshalled(prob.dtype_code, args2, 0, streams[1].cuda_stream)
    torch.cuda.synchronize()
    partial = [prob.C.gather(r) for r in range(cfg["C"]["replication"])]
    total = other.gather(0)
    assert np.isfinite(total).all() and all(np.isfinite(x).all() for x in partial)
    assert np.array_equal(total, partial[0] + partial[1])       # fp32 a + b, as the replica sum computes it
    _check(total, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg, "grown table")
    assert np.array_equal(other.gather(1), partial[1])
    prob.close()


@pytest.mark.parametrize("name,dims,path", [("cfg4", (515, 771, 1030), "groups"), ("cfg4", (300, 16384, 300), "k-split"),
                                            ("bc128", (700, 333, 517), "merged")])
def test_repeated_execute_reuses_the_work_tables(name, dims, path):
    """A call with the inputs of the call before it (same tables of pointers and leading dimensions,
    same flags apart from DMM_TIMING) launches from the device tables that call left; any other call
    assembles its own.  Per-group macro-tiles, macro-tiles cut along K (their partial tiles share
    one scratch buffer across calls) and merged macro-tiles; results bitwise the same either way."""
    from paper_2510_08874_amd import binding
    from paper_2510_08874_amd.tiles import TileSet
    cfg = workloads.scaled_config(name, *dims)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    stream = torch.cuda.current_stream().cuda_stream
    c = cfg["C"]["replication"]
    base = 0 if path == "merged" else binding.DMM_NO_MERGE
    prob.execute(flags=base)
    assert not prob.plan.table_reused()
    assert prob.plan.ran_merged() == (path == "merged")
    if torch.cuda.get_device_properties(0).multi_processor_count == 256:
        assert prob.plan.ran_k_split() == (path == "k-split")
    first = [prob.c_global(r) for r in range(c)]
    _check(first[0], omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])
    for t in prob.C.tensors:
        if t is not None:
            t.fill_(float("nan"))
    prob.execute(flags=base | binding.DMM_TIMING)                # same inputs: the tables stay
    assert prob.plan.table_reused() and prob.plan.elapsed_ms()[0] > 0.0
    for r in range(c):
        assert np.array_equal(first[r], prob.c_global(r)), f"replica {r} differs on the reused tables"
    other = TileSet(cfg["C"], torch.float32, "cuda", 1, fill=float("nan"))
    args2 = prob.plan.marshal(prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld, other.tensors, other.ld)
    prob.plan.execute_marshalled(prob.dtype_code, args2, base, stream)   # other C tiles: new tables
    assert not prob.plan.table_reused()
    prob.plan.execute_marshalled(prob.dtype_code, args2, base, stream)
    assert prob.plan.table_reused()
    for r in range(c):
        assert np.array_equal(first[r], other.gather(r)), f"replica {r} differs in the second set of C tiles"
    prob.execute(flags=base)                                     # back to the first set: not the last call's inputs
    assert not prob.plan.table_reused()
    if c > 1:
        prob.execute(flags=base | binding.DMM_NO_REDUCE)         # other flags: new tables
        assert not prob.plan.table_reused()
        prob.execute(flags=base | binding.DMM_NO_REDUCE)
        assert prob.plan.table_reused()
        total = prob.c_global(0)
        for r in range(1, c):
            total = total + prob.c_global(r)                     # fp32 (p0 + p1) + ..., as the replica sum computes it
        assert np.array_equal(total, first[0])
    prob.close()


def test_iteration_offset_leaves_the_result_bitwise_unchanged():
    cfg = workloads.scaled_config("cfg5", 700, 900, 650)
    A, B = workloads.make_operands(cfg)
    outs = []
    for flag in (False, True):
        prob = _device_problem(dict(cfg, iteration_offset=flag), A, B, c_fill=float("nan"))
        prob.execute()
        outs.append(prob.c_global(0))
        prob.close()
    assert np.array_equal(outs[0], outs[1])


# ---- the MLP-shaped products of Section 5.2, four partitionings, reduced size ------------

@pytest.mark.parametrize("name", ["mlp1-column", "mlp1-inner", "mlp1-outer", "mlp1-2d", "mlp2-outer", "mlp2-2d"])
def test_mlp_partitionings_small(name):
    base = workloads.config(name)
    cfg = workloads.scaled_config(name, 520, base["K"] // 32 + 5, base["N"] // 32 + 3)
    _run_full(cfg)


# ---- full size, in the launch configuration the benchmark times -------------------

def _check_rows_streaming(prob, cfg, A, B, row_sets, what):
    """Rows of C against the oracle, a set of rows at a time (bounded host memory): the per-element
    bound on every set, the relative Frobenius error over all of them together."""
    B64 = _to_f64(B, cfg)
    bnorm = np.linalg.norm(B64, axis=0)
    num = den = 0.0
    for rows in row_sets:
        C_gpu = prob.C.gather_rows(rows, 0).astype(np.float64)
        assert np.isfinite(C_gpu).all(), f"{what}: rows {rows[0]}..{rows[-1]} hold non-finite values"
        C_ref = omatmul.matmul(A[rows], B, bf16=(cfg["dtype"] == "bf16"))
        diff = np.abs(C_gpu - C_ref)
        bound = 4.0 * cfg["K"] * U32 * np.outer(np.linalg.norm(_to_f64(A[rows], cfg), axis=1), bnorm) + 1e-30
        worst = float(np.max(diff / bound))
        assert worst <= 1.0, f"{what}: rows {rows[0]}..{rows[-1]}: element error {worst:.3f} x the fp32 accumulation bound"
        num += float(np.sum(diff * diff))
        den += float(np.sum(C_ref * C_ref))
    err = (num / max(den, 1e-300)) ** 0.5
    assert err <= TOL[cfg["dtype"]], f"{what}: relative Frobenius error {err:.3e}"
    return err


@pytest.mark.parametrize("name,ldm", [("cfg2", 1), ("cfg4", 1), ("cfg5", 1), ("cfg5", 8), ("cfg3", 1), ("bc128", 1), ("bc256", 1)])
def test_full_size_every_element(name, ldm):
    """The configurations at full size, as the benchmark launches them (cfg5 also with leading
    dimensions padded to a multiple of 8 elements; 8192^3 in 128 x 128 and 256 x 256 tiles dealt
    block-cyclically, which run the merged macro-tiles): every element of C against the oracle, in
    chunks of rows; and every element of every replica was written."""
    cfg = workloads.config(name)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    prob.execute()
    torch.cuda.synchronize()
    step = 2048
    sets = [np.arange(r, min(r + step, cfg["M"])) for r in range(0, cfg["M"], step)]
    _check_rows_streaming(prob, cfg, A, B, sets, f"{name} ld x{ldm}")
    if ldm == 1:                                            # (padding columns are never written: they keep the fill)
        for t in prob.C.tensors:
            if t is not None:
                assert not torch.isnan(t).any().item()
    prob.close()


# ---- exact cases ---------------------------------------------------------------------

@pytest.mark.parametrize("name,dims", [("cfg2", (512, 4096, 512)), ("cfg5", (700, 999, 300)), ("cfg4", (512, 2048, 512)),
                                       ("bc128", (640, 2048, 512))])
def test_all_ones_gives_exactly_k(name, dims):
    cfg = workloads.scaled_config(name, *dims)
    one = np.uint16(0x3F80)
    A = np.full((cfg["M"], cfg["K"]), one, dtype=np.uint16)
    B = np.full((cfg["K"], cfg["N"]), one, dtype=np.uint16)
    prob = _device_problem(cfg, A, B)
    prob.execute()
    C = prob.c_global(0)
    assert (C == np.float32(cfg["K"])).all()
    prob.close()


@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_identity_reproduces_b_exactly(dtype):
    cfg = dict(workloads.scaled_config("cfg5", 600, 600, 450), dtype=dtype)
    B = workloads.make_matrix(600, 450, ("normal", 1.0), 77)
    A = np.eye(600, dtype=np.float32)
    if dtype == "bf16":
        A, B = workloads.bf16_round(A), workloads.bf16_round(B)
        want = workloads.bf16_to_f32(B)
    else:
        want = B
    prob = _device_problem(cfg, A, B)
    prob.execute()
    assert np.array_equal(prob.c_global(0), want)
    prob.close()


def test_run_to_run_bitwise_identical():
    cfg = workloads.scaled_config("cfg5", 1229, 997, 1100)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B)
    prob.execute()
    first = prob.c_global(0)
    for _ in range(3):
        for t in prob.C.tensors:
            t.zero_()
        prob.execute()
        assert np.array_equal(prob.c_global(0), first)
    prob.close()


# ---- edges ----------------------------------------------------------------------------

def test_padding_of_c_is_never_written():
    cfg = workloads.scaled_config("cfg5", 523, 300, 517)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, ld_multiple=16, c_fill=-7.0)
    prob.execute()
    torch.cuda.synchronize()
    for idx, t in enumerate(prob.C.tensors):
        ti, tj = divmod(idx % (prob.C.gr * prob.C.gc), prob.C.gc)
        r0, r1, c0, c1 = prob.C.bounds(ti, tj)
        if t.shape[1] > c1 - c0:
            assert (t[:, c1 - c0:] == -7.0).all().item()
    prob.close()


@pytest.mark.parametrize("dims", [(1, 1, 1), (1, 7, 1), (3, 1, 2), (257, 65, 257), (256, 64, 256), (255, 63, 255)])
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_tiny_and_boundary_shapes(dims, dtype):
    M, K, N = dims
    cfg = dict(name="edge", M=M, K=K, N=N, dtype=dtype, nranks=1,
               A=workloads.block_desc(M, K, 1, 1), B=workloads.block_desc(K, N, 1, 1),
               C=workloads.block_desc(M, N, 1, 1), dist=("normal", 1.0), seeds=(5, 6))
    _run_full(cfg)


def test_empty_dimensions_are_noops():
    for M, K, N in [(0, 5, 4), (4, 5, 0)]:
        cfg = dict(name="empty", M=M, K=K, N=N, dtype="f32", nranks=1,
                   A=workloads.block_desc(M, K, 1, 1), B=workloads.block_desc(K, N, 1, 1),
                   C=workloads.block_desc(M, N, 1, 1), dist=("normal", 1.0), seeds=(5, 6))
        prob = _device_problem(cfg, None, None)
        assert prob.plan.num_tasks() == 0 and prob.plan.num_items() == 0
        prob.execute()
        prob.close()


def test_empty_inner_dimension_and_empty_shares_zero_fill():
    """K = 0 gives C = 0; with more C replicas than k values some replicas have
    an empty share and must still hold a defined (zero) partial sum."""
    cfg = dict(name="k0", M=40, K=0, N=30, dtype="f32", nranks=2,
               A=workloads.block_desc(40, 0, 2, 1), B=workloads.block_desc(0, 30, 1, 2),
               C=workloads.block_desc(40, 30, 1, 1, replication=2), dist=("normal", 1.0), seeds=(5, 6))
    prob = _device_problem(cfg, np.zeros((40, 0), np.float32), np.zeros((0, 30), np.float32), c_fill=float("nan"))
    prob.execute()
    assert (prob.c_global(0) == 0).all() and (prob.c_global(1) == 0).all()
    prob.close()
    cfg = dict(name="k1c4", M=33, K=1, N=20, dtype="bf16", nranks=4,
               A=workloads.block_desc(33, 1, 1, 1, replication=4), B=workloads.block_desc(1, 20, 1, 1, replication=4),
               C=workloads.block_desc(33, 20, 1, 1, replication=4), dist=("normal", 1.0), seeds=(8, 9))
    _run_full(cfg)


# ---- replica sum ----------------------------------------------------------------------

@pytest.mark.parametrize("c,origin,ldm,shape", [(2, 0, 4, (512, 384)), (2, 1, 1, (301, 203)), (3, 2, 4, (130, 260)),
                                                (4, 0, 1, (77, 1025)), (8, 3, 8, (64, 64))])
def test_reduce_replicas_exact(c, origin, ldm, shape):
    """Bit-exact against the oracle's fp32 left-to-right sum; other replicas untouched."""
    M, N = shape
    p = 2 * c
    cfg = dict(name="red", M=M, K=8, N=N, dtype="f32", nranks=p,
               A=workloads.block_desc(M, 8, 1, 1, replication=p), B=workloads.block_desc(8, N, 1, 1, replication=p),
               C=workloads.block_desc(M, N, 2, 1, replication=c), dist=("normal", 1.0), seeds=(1, 2))
    prob = _device_problem(cfg, None, None, ld_multiple=ldm)
    rng = np.random.default_rng(c * 100 + origin)
    parts = {}
    for rep in range(c):
        for ti in range(2):
            t = prob.C.tensors[prob.C.index(rep, ti, 0)]
            h = rng.standard_normal(tuple(t.shape)).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4))
            t.copy_(torch.from_numpy(h))
            parts[(rep, ti)] = h
    prob.reduce(origin)
    torch.cuda.synchronize()
    for ti in range(2):
        r0, r1, c0, c1 = prob.C.bounds(ti, 0)
        w = c1 - c0
        want = omatmul.reduce_replicas([parts[(rep, ti)][:, :w] for rep in range(c)])
        for rep in range(c):
            got = prob.C.tensors[prob.C.index(rep, ti, 0)].cpu().numpy()
            if rep == origin:
                assert np.array_equal(got[:, :w], want)
                assert np.array_equal(got[:, w:], parts[(rep, ti)][:, w:])     # padding untouched
            else:
                assert np.array_equal(got, parts[(rep, ti)])
    prob.close()


@pytest.mark.parametrize("origin,ldm", [(0, 1), (2, 8)])
def test_broadcast_replica_copies_the_origin_exactly(origin, ldm):
    """reduce + broadcast = the product in every replica (Table 1), bit for bit the origin's."""
    from oracle import execute as oexec
    cfg = workloads.scaled_config("cfg4", 333, 280, 517)
    cfg["C"] = dict(cfg["C"], replication=4)
    cfg["A"] = dict(cfg["A"], replication=1)
    cfg["B"] = dict(cfg["B"], replication=1)
    cfg["nranks"] = 64
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    from paper_2510_08874_amd import binding
    prob.execute(flags=binding.DMM_NO_REDUCE)
    before = [prob.c_global(r) for r in range(4)]
    prob.reduce(origin)
    prob.broadcast(origin)
    after = [prob.c_global(r) for r in range(4)]
    # oracle: same partials through the oracle's reduce (ascending replica order) and broadcast
    Cd = helpers.dist(cfg["C"])
    want = omatmul.reduce_replicas(before)
    tiles = {}
    gr, gc = Cd.grid_shape()
    for r in range(4):
        for ti in range(gr):
            for tj in range(gc):
                (r0, r1), (c0, c1) = Cd.tile_bounds((ti, tj))
                tiles[(r, ti, tj)] = (want if r == origin else before[r])[r0:r1, c0:c1]
    oexec.broadcast_replica(tiles, Cd, origin)
    for r in range(4):
        for ti in range(gr):
            for tj in range(gc):
                (r0, r1), (c0, c1) = Cd.tile_bounds((ti, tj))
                assert np.array_equal(after[r][r0:r1, c0:c1], tiles[(r, ti, tj)])
    prob.close()


def test_no_reduce_flag_leaves_partials():
    from paper_2510_08874_amd import DMM_NO_REDUCE
    cfg = workloads.scaled_config("cfg4", 512, 1024, 512)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B)
    prob.execute(flags=DMM_NO_REDUCE)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    for rep in range(2):
        ref = A64[:, 512 * rep:512 * (rep + 1)] @ B64[512 * rep:512 * (rep + 1), :]
        got = prob.c_global(rep)
        assert np.linalg.norm(got - ref) / np.linalg.norm(ref) < 1e-5
    prob.close()


# ---- bf16 C tiles (DMM_C_BF16) -------------------------------------------------------------

U16 = 2.0 ** -8          # half an ulp of bf16, relative: the most one rounding to nearest can move a value


def _check_bf16_out(C_gpu, C_ref, A64, B64, what):
    """A bf16 C element is the fp32 sum rounded to nearest: it may differ from the exact value by
    the fp32 accumulation bound plus half a bf16 ulp of the (bounded) sum.  Truncation instead of
    rounding, or rounding twice, breaks the element bound; the Frobenius bar is the stated one."""
    got = C_gpu.astype(np.float64)
    acc = 4.0 * A64.shape[1] * U32 * np.outer(np.linalg.norm(A64, axis=1), np.linalg.norm(B64, axis=0)) + 1e-30
    bound = acc + U16 * (np.abs(C_ref) + acc) * (1.0 + 1e-6) + 2.0 ** -133      # + half the smallest subnormal step
    worst = np.max(np.abs(got - C_ref) / bound)
    assert worst <= 1.0, f"{what}: element error {worst:.3f} x (accumulation bound + half a bf16 ulp)"
    err = np.linalg.norm(got - C_ref) / max(np.linalg.norm(C_ref), 1e-300)
    assert err <= TOL["bf16"], f"{what}: relative Frobenius error {err:.3e}"


@pytest.mark.parametrize("name,dims,ldm", [
    ("cfg2", (768, 520, 640), 1),
    ("cfg3", (300, 333, 1100), 1),     # odd leading dimensions: 2-byte aligned rows of C
    ("cfg5", (1229, 997, 1100), 1),
    ("cfg5", (1229, 997, 1100), 8),
    ("cfg1", (260, 130, 515), 1),      # fp32 operands, bf16 result
])
def test_bf16_c_tiles(name, dims, ldm):
    """C tiles in bf16: against the fp64 oracle within the stated bar and the element bound, bitwise
    equal to the fp32-C run of the same plan rounded to nearest even, padding columns untouched."""
    cfg = workloads.scaled_config(name, *dims)
    A, B = workloads.make_operands(cfg)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    C_ref = omatmul.matmul(A, B, bf16=(cfg["dtype"] == "bf16"))
    prob = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"), c_dtype="bf16")
    prob.execute()
    got = prob.c_global(0)
    _check_bf16_out(got, C_ref, A64, B64, cfg["name"])
    for t, ld, (ti, tj) in zip(prob.C.tensors, prob.C.ld, [(i, j) for i in range(prob.C.gr) for j in range(prob.C.gc)]):
        r0, r1, c0, c1 = prob.C.bounds(ti, tj)
        if t is not None and ld > c1 - c0:
            assert torch.isnan(t[:, c1 - c0:]).all(), "padding of a bf16 C tile was written"
    prob.close()
    wide = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    wide.execute()
    want = workloads.bf16_to_f32(workloads.bf16_round(wide.c_global(0)))
    wide.close()
    assert np.array_equal(got, want)


def test_bf16_c_tiles_k_split_and_zero_fill():
    """The two other writers of C honour the element type: the pass that adds up K-split runs, and zero fill."""
    M, K, N = 300, 8192, 300
    cfg = dict(name="ksplit-bf16out", M=M, K=K, N=N, nranks=1, dtype="bf16",
               A=workloads.block_desc(M, K, 1, 1), B=workloads.block_desc(K, N, 1, 1), C=workloads.block_desc(M, N, 1, 1),
               dist=("normal", 1.0), seeds=(41, 42))
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"), c_dtype="bf16")
    prob.execute()
    got = prob.c_global(0)
    _check_bf16_out(got, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg["name"])
    prob.execute()
    assert np.array_equal(got, prob.c_global(0))
    prob.close()
    cfg = dict(name="k0-bf16out", M=40, K=0, N=30, dtype="f32", nranks=2,
               A=workloads.block_desc(40, 0, 2, 1), B=workloads.block_desc(0, 30, 1, 2),
               C=workloads.block_desc(40, 30, 2, 1), dist=("normal", 1.0), seeds=(5, 6))
    prob = _device_problem(cfg, np.zeros((40, 0), np.float32), np.zeros((0, 30), np.float32), c_fill=float("nan"),
                           c_dtype="bf16")
    prob.execute()
    assert (prob.c_global(0) == 0).all()
    prob.close()


def test_bf16_c_tiles_need_an_unreplicated_c():
    from paper_2510_08874_amd import binding
    cfg = workloads.scaled_config("cfg4", 128, 128, 128)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B)
    with pytest.raises(binding.DmmError) as e:
        prob.execute(flags=binding.DMM_C_BF16)
    assert e.value.kind == "EINVAL"
    prob.close()


# ---- merged macro-tiles: tile grids much finer than 256 x 256 ---------------------------------

def _bc(dims, nb, dtype, reps=(1, 1, 1), p=8):
    M, K, N = dims
    pr, pc = 2, 4
    return dict(name=f"bc{nb}/{dtype}/{reps}@{M}x{K}x{N}", M=M, K=K, N=N, dtype=dtype, nranks=p,
                A=workloads.block_cyclic_desc(M, K, nb, nb, pr, pc, reps[0]),
                B=workloads.block_cyclic_desc(K, N, nb, nb, pr, pc, reps[1]),
                C=workloads.block_cyclic_desc(M, N, nb, nb, pr, pc, reps[2]),
                dist=("normal", 1.0), seeds=(71, 72))


@pytest.mark.parametrize("dims,nb,dtype,ldm,reps,p", [
    ((1536, 1024, 1280), 128, "bf16", 1, (1, 1, 1), 8),    # 2 x 2 tiles per macro-tile, everything aligned
    ((700, 333, 517), 96, "bf16", 1, (1, 1, 1), 8),        # macro-tiles start inside tiles; odd leading dimensions; K tails
    ((700, 333, 517), 96, "f32", 1, (1, 1, 1), 8),
    ((520, 200, 530), 40, "bf16", 8, (1, 1, 1), 8),        # seven pieces per axis
    ((300, 4100, 300), 24, "bf16", 1, (1, 1, 1), 8),       # 171 segments: too many to stage at once, run in three windows of 64
    ((200, 9000, 300), 40, "f32", 1, (1, 2, 2), 16),       # the same with two replicas (113 segments each) and the replica sum
    ((640, 900, 512), 64, "bf16", 1, (2, 2, 2), 16),       # replicated: every replica its share of k, then the replica sum
    ((640, 900, 512), 64, "f32", 4, (1, 2, 4), 32),        # C replicas read different replicas of B, all the one A
    ((515, 130, 260), 100, "bf16", 1, (1, 1, 1), 8),       # cuts at 100, 200: column pieces not at multiples of 8: tiles end there
    ((640, 900, 512), 64, "bf16", 1, (2, 1, 1), 16),       # A replicated, C not: the ranks of C read both replicas of A, tile by tile
    ((520, 600, 530), 40, "f32", 1, (1, 4, 2), 32),        # four replicas of B for two of C
    ((640, 900, 512), 64, "bf16", 1, (3, 1, 2), 24),       # three replicas of A for two of C: neither number divides the other
])
def test_merged_macro_tiles(dims, nb, dtype, ldm, reps, p):
    """Where the tiles are small against the macro-tile the library runs macro-tiles that span
    several tiles of A, B and C.  Parity with the oracle as everywhere, and bitwise the same C as
    the one-macro-tile-per-output-sub-tile path (same K-segments, same order of summation)."""
    from paper_2510_08874_amd import binding
    cfg = _bc(dims, nb, dtype, reps, p)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    assert prob.plan.num_merged_items() > 0
    prob.execute()
    assert prob.plan.ran_merged()
    merged_cut = prob.plan.ran_k_split()
    got = prob.c_global(0)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    C_ref = omatmul.matmul(A, B, bf16=(dtype == "bf16"))
    _check(got, C_ref, A64, B64, cfg, cfg["name"])
    parts = [prob.c_global(r) for r in range(1, reps[2])]
    for t, ld, (ti, tj) in zip(prob.C.tensors, prob.C.ld, [(i, j) for i in range(prob.C.gr) for j in range(prob.C.gc)]):
        r0, r1, c0, c1 = prob.C.bounds(ti, tj)
        if t is not None and ld > c1 - c0:
            assert torch.isnan(t[:, c1 - c0:]).all(), "padding of a C tile was written"
    prob.close()
    plain = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    plain.execute(flags=binding.DMM_NO_MERGE | binding.DMM_SEPARATE_REDUCE)
    assert not plain.plan.ran_merged()
    # The merged and the per-group work lists sum every C element over the same K-segments in the
    # same order, so they agree bit for bit, unless the library cut macro-tiles of one of the runs
    # along K (partial tiles are then added up separately); the library says whether it did.
    if not merged_cut and not plain.plan.ran_k_split():
        assert np.array_equal(got, plain.c_global(0))
        for r in range(1, reps[2]):
            assert np.array_equal(parts[r - 1], plain.c_global(r))
    else:
        _check(plain.c_global(0), C_ref, A64, B64, cfg, cfg["name"] + " per group")
    plain.close()


@pytest.mark.parametrize("seed", range(16))
@pytest.mark.parametrize("dtype", ["bf16", "f32"])
def test_merged_macro_tiles_random_partitionings(seed, dtype):
    """The merged kernel forced (DMM_MERGE_ALWAYS) onto random grids: uneven and empty tiles, odd
    leading dimensions, K tails in every segment, column cuts at any position, replication.  Plans
    that cannot have a merged list (empty shares of K) run the per-group path; either way parity, and bitwise the per-group result."""
    from paper_2510_08874_amd import binding
    prob = helpers.random_problem(seed + 300, max_dim=700, allow_empty=(seed % 2 == 1))
    cfg = dict(prob, name=f"random-merged{seed}", dtype=dtype, dist=("normal", 1.0), seeds=(seed, seed + 900),
               merge_always=True)
    A, B = workloads.make_operands(cfg)
    dev = _device_problem(cfg, A, B, c_fill=float("nan"))
    dev.execute()
    assert dev.plan.ran_merged() == (dev.plan.num_merged_items() > 0)
    merged_cut = dev.plan.ran_k_split()
    got = [dev.c_global(r) for r in range(cfg["C"]["replication"])]
    _check(got[0], omatmul.matmul(A, B, bf16=(dtype == "bf16")), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])
    dev.execute(flags=binding.DMM_NO_MERGE)
    if not merged_cut and not dev.plan.ran_k_split():
        for r in range(cfg["C"]["replication"]):
            assert np.array_equal(got[r], dev.c_global(r))
    dev.close()


@pytest.mark.parametrize("mode", ["B", "A"])
def test_merged_macro_tiles_stationary_b_and_a(mode):
    """Without replication the ops of a Stationary B (A) plan are the boxes of the Stationary C plan
    on other ranks, so its merged macro-tiles are the same and so is C, bit for bit."""
    cfg = _bc((700, 333, 517), 96, "bf16")
    A, B = workloads.make_operands(cfg)
    ref = _device_problem(cfg, A, B, c_fill=float("nan"))
    ref.execute()
    want = ref.c_global(0)
    ref.close()
    prob = _device_problem(dict(cfg, stationary=mode), A, B, c_fill=float("nan"))
    assert prob.plan.num_merged_items() > 0
    assert {t[0] for t in prob.plan.tasks()} == set(range(8))
    prob.execute()
    assert prob.plan.ran_merged()
    assert np.array_equal(want, prob.c_global(0))
    _check(want, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])
    prob.close()


@pytest.mark.parametrize("dims,nb,dtype,c_dtype", [
    ((300, 8192, 300), 64, "bf16", "f32"),       # 4 merged macro-tiles x 256 K steps -> 4 runs each, 5 x 5 pieces
    ((515, 8200, 260), 96, "bf16", "bf16"),      # macro-tiles that start inside tiles, K tail, bf16 C
    ((260, 2100, 515), 40, "f32", "f32"),        # fp32: 132 steps -> 2 runs each, seven pieces per axis
])
def test_merged_macro_tiles_k_split_of_the_last_round(dims, nb, dtype, c_dtype):
    """Few merged macro-tiles with long K are cut into runs like the per-group ones; the pass that
    adds the partial tiles up writes every piece to its own C tile.  Parity, rerun bitwise equal."""
    cfg = _bc(dims, nb, dtype)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"), c_dtype=c_dtype)
    assert 0 < prob.plan.num_merged_items() <= 8
    prob.execute()
    assert prob.plan.ran_merged()
    got = prob.c_global(0)
    A64, B64 = _to_f64(A, cfg), _to_f64(B, cfg)
    C_ref = omatmul.matmul(A, B, bf16=(dtype == "bf16"))
    if c_dtype == "bf16":
        _check_bf16_out(got, C_ref, A64, B64, cfg["name"])
    else:
        _check(got, C_ref, A64, B64, cfg, cfg["name"])
    prob.execute()
    assert np.array_equal(got, prob.c_global(0))
    prob.close()


def test_merged_macro_tiles_bf16_c_and_rerun():
    from paper_2510_08874_amd import binding
    cfg = _bc((700, 333, 517), 96, "bf16")
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"), c_dtype="bf16")
    assert prob.plan.num_merged_items() > 0
    prob.execute()
    got = prob.c_global(0)
    _check_bf16_out(got, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg["name"])
    prob.execute()
    assert np.array_equal(got, prob.c_global(0))
    prob.execute(flags=binding.DMM_NO_MERGE)
    assert np.array_equal(got, prob.c_global(0))
    prob.close()


def test_merged_macro_tiles_across_a_4gb_line():
    """The load slots of the merged kernel advance only the low half of a lane's address; a segment
    in which an address would carry into the high half has to take the step-by-step path.  All
    tiles of A and B are laid out back to back around a multiple of 2^32 inside one large buffer."""
    from paper_2510_08874_amd import binding
    cfg = _bc((300, 520, 300), 64, "bf16")
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B, c_fill=float("nan"))
    assert prob.plan.num_merged_items() > 0
    prob.execute()
    want = prob.c_global(0)
    big = torch.empty((1 << 32) + (64 << 20), dtype=torch.uint8, device="cuda")
    line = (big.data_ptr() + (1 << 32) - 1) // (1 << 32) * (1 << 32)       # the multiple of 2^32 inside it
    for ts in (prob.A, prob.B):                                             # first A around the line, then B
        kept = list(ts.tensors)
        pos = line - 150_000 - big.data_ptr()
        for i, t in enumerate(ts.tensors):
            if t is None:
                continue
            nbytes = t.numel() * 2
            view = big[pos:pos + nbytes].view(torch.bfloat16).view(t.shape)
            view.copy_(t)
            ts.tensors[i] = view
            pos += nbytes + 6                                               # keeps the tiles 2-byte aligned only
        assert big.data_ptr() + pos > line
        prob.args = prob.plan.marshal(prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld, prob.C.tensors, prob.C.ld)
        for t in prob.C.tensors:
            if t is not None:
                t.fill_(float("nan"))
        prob.execute()
        assert prob.plan.ran_merged()
        assert np.array_equal(want, prob.c_global(0))
        ts.tensors[:] = kept
    C_ref = omatmul.matmul(A, B, bf16=True)
    _check(want, C_ref, _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])
    prob.close()


# ---- fused replica sum (the default) against DMM_SEPARATE_REDUCE -----------------------------------------------------

def _fused_against_plain(cfg, A, B, ldm=1, must_fuse=True, launches=2):
    from paper_2510_08874_amd import binding
    c = cfg["C"]["replication"]
    plain = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    plain.execute(flags=binding.DMM_NO_MERGE | binding.DMM_SEPARATE_REDUCE)
    want = [plain.c_global(r) for r in range(c)]
    red_ms = None
    plain.execute(flags=binding.DMM_NO_MERGE | binding.DMM_SEPARATE_REDUCE | binding.DMM_TIMING)
    torch.cuda.synchronize()
    assert plain.plan.elapsed_ms()[1] >= 0.0            # the replica-sum kernel ran
    plain.close()
    fused = _device_problem(cfg, A, B, ld_multiple=ldm, c_fill=float("nan"))
    fused.execute(flags=binding.DMM_NO_MERGE | binding.DMM_TIMING)
    torch.cuda.synchronize()
    red_ms = fused.plan.elapsed_ms()[1]
    if must_fuse:
        assert red_ms < 0.0, "the replica-sum kernel ran although the sum was to be fused"
        assert fused.plan.ran_fused() == launches
        (ms0, fl0), (ms1, fl1) = fused.plan.gemm_launch_ms()      # the two launches, one by one
        if launches == 2:
            assert ms0 > 0.0 and ms1 > 0.0 and abs(ms0 + ms1 - fused.plan.elapsed_ms()[0]) < 1e-3
            assert fl0 + fl1 == 2.0 * cfg["M"] * cfg["K"] * cfg["N"] and fl0 > 0.0 and fl1 > 0.0
        else:
            assert ms0 < 0.0 and ms1 < 0.0 and fused.plan.elapsed_ms()[0] > 0.0
    else:
        assert fused.plan.ran_fused() in (0, 2)
    for r in range(c):
        assert np.array_equal(want[r], fused.c_global(r)), f"replica {r} differs"
    fused.close()
    return want[0]


@pytest.mark.parametrize("name,dims,ldm", [("cfg4", (1024, 1024, 1024), 8), ("cfg4", (515, 771, 1030), 1),
                                           ("mlp1-outer", (520, 1000, 300), 1)])
def test_fused_replica_sum_families(name, dims, ldm):
    """The replica sum folded into the epilogue of replica 0's macro-tiles: every replica ends up with
    bitwise the contents the GEMM + replica-sum kernel pair leaves (partials in replicas 1.., the
    sum in replica 0), and the sum is the product."""
    cfg = workloads.scaled_config(name, *dims)
    A, B = workloads.make_operands(cfg)
    C0 = _fused_against_plain(cfg, A, B, ldm)
    _check(C0, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])


@pytest.mark.parametrize("dims", [(4096, 512, 4096), (8192, 256, 8192)])
def test_fused_replica_sum_in_one_launch(dims):
    """Where every replica has the same macro-tiles, a whole number of rounds of them, one launch
    does everything: the work list is laid out so that the workgroup that stored a partial sum is
    the one that reads it back.  (2.5D on 4096 x 4096: 256 macro-tiles per replica, one round of a
    256-CU device each; on 8192 x 8192 four rounds each, where the XCDs alternate between two
    orders of their macro-tiles.)"""
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the work list is laid out for whole rounds per replica on 256 compute units")
    cfg = workloads.scaled_config("cfg4", *dims)
    A, B = workloads.make_operands(cfg)
    C0 = _fused_against_plain(cfg, A, B, launches=1)
    _check(C0, omatmul.matmul(A, B, bf16=True), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])


@pytest.mark.parametrize("c,dims,dtype", [(4, (4096, 1024, 8192), "bf16"), (3, (4096, 768, 4096), "f32")])
def test_fused_replica_sum_in_one_launch_of_several_replicas(c, dims, dtype):
    """More than two replicas of C (2.5D with c = 4 and c = 3): replica 0's macro-tiles add c - 1
    partial sums, ((own + p_1) + p_2) + ..., whose loads run as one stream of batches; every round of
    the work list is c - 1 rounds of other replicas' macro-tiles and one of replica 0's."""
    if torch.cuda.get_device_properties(0).multi_processor_count != 256:
        pytest.skip("the work list is laid out for whole rounds per replica on 256 compute units")
    M, K, N = dims
    g = 2
    cfg = dict(name=f"2.5d-c{c}-{dtype}@{M}x{K}x{N}", M=M, K=K, N=N, dtype=dtype, nranks=c * g * g,
               A=workloads.block_desc(M, K, g, g, replication=c), B=workloads.block_desc(K, N, g, g, replication=c),
               C=workloads.block_desc(M, N, g, g, replication=c), dist=("normal", 1.0), seeds=(81, 82))
    A, B = workloads.make_operands(cfg)
    C0 = _fused_against_plain(cfg, A, B, launches=1)
    _check(C0, omatmul.matmul(A, B, bf16=(dtype == "bf16")), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])


@pytest.mark.parametrize("seed", [2, 3, 4, 6, 8, 13, 15, 21, 24, 27])
@pytest.mark.parametrize("mode", ["C", "B", "A"])
def test_fused_replica_sum_random_partitionings(seed, mode):
    """Random grids with a replicated C (2 to 8 replicas), in all three data movement modes (with B
    or A in place some regions of a replica are zero fill): fused = unfused, bit for bit."""
    prob = helpers.random_problem(seed + 300, max_dim=700, allow_empty=(seed % 2 == 1))
    if prob["C"]["replication"] == 1:
        prob["C"] = dict(prob["C"], replication=prob["nranks"], proc_rows=1, proc_cols=1)
    cfg = dict(prob, name=f"random-fused{seed}/{mode}", dtype="bf16" if seed % 2 else "f32", dist=("normal", 1.0),
               seeds=(seed, seed + 900), stationary=mode)
    assert cfg["C"]["replication"] > 1, "the seeds above all draw at least two ranks"
    A, B = workloads.make_operands(cfg)
    C0 = _fused_against_plain(cfg, A, B, must_fuse=False)     # (tiny problems may be cut along K instead)
    _check(C0, omatmul.matmul(A, B, bf16=(cfg["dtype"] == "bf16")), _to_f64(A, cfg), _to_f64(B, cfg), cfg, cfg["name"])


# ---- error paths that reach the device entry points ---------------------------------

def test_execute_rejects_bad_arguments():
    from paper_2510_08874_amd import binding
    cfg = workloads.scaled_config("cfg1", 64, 64, 64)
    A, B = workloads.make_operands(cfg)
    prob = _device_problem(cfg, A, B)
    bad_ld = list(prob.A.ld)
    bad_ld[0] = 1
    with pytest.raises(binding.DmmError) as e:
        prob.plan.execute(binding.DMM_F32, prob.A.tensors, bad_ld, prob.B.tensors, prob.B.ld,
                          prob.C.tensors, prob.C.ld)
    assert e.value.kind == "ELD"
    # row pitches of 2^24 bytes and more are refused on the host, for every operand, before any launch
    for which in range(3):
        lds = [list(prob.A.ld), list(prob.B.ld), list(prob.C.ld)]
        lds[which][0] = (1 << 24) // 4
        with pytest.raises(binding.DmmError) as e:
            prob.plan.execute(binding.DMM_F32, prob.A.tensors, lds[0], prob.B.tensors, lds[1], prob.C.tensors, lds[2])
        assert e.value.kind == "ELD"
    with pytest.raises(binding.DmmError) as e:
        prob.plan.execute(binding.DMM_F32, [None] * len(prob.A.tensors), prob.A.ld, prob.B.tensors, prob.B.ld,
                          prob.C.tensors, prob.C.ld)
    assert e.value.kind == "EINVAL"
    with pytest.raises(binding.DmmError) as e:
        prob.plan.execute(7, prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld, prob.C.tensors, prob.C.ld)
    assert e.value.kind == "EINVAL"
    with pytest.raises(binding.DmmError):
        prob.plan.reduce_replicas(prob.C.tensors, prob.C.ld, origin=5)
    # a dmm_plan flag is not a dmm_execute flag (the two sets share no bit)
    for plan_flag in (binding.DMM_STATIONARY_B, binding.DMM_ITERATION_OFFSET, binding.DMM_MERGE_ALWAYS):
        with pytest.raises(binding.DmmError) as e:
            prob.plan.execute(binding.DMM_F32, prob.A.tensors, prob.A.ld, prob.B.tensors, prob.B.ld,
                              prob.C.tensors, prob.C.ld, flags=plan_flag)
        assert e.value.kind == "EINVAL"
    prob.close()


def test_mfma_rate_probe_reports_a_plausible_rate():
    """The measurement aid runs, rejects bad durations, and lands between 5 % and 100 % of the published peak."""
    from paper_2510_08874_amd import binding
    tf, mhz = binding.dmm_measure_mfma_rate(5.0, True)
    assert 125.0 < tf < 2600.0
    assert 300.0 < mhz < 2600.0
    # 32 cycles per MFMA per SIMD: TFLOP/s = CUs * 4 * 1024 flop/cycle * MHz
    import torch
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    assert abs(tf - cus * 4 * 1024 * mhz * 1e6 / 1e12) / tf < 0.05
    for bad in (0.0, -1.0, 5000.0):
        with pytest.raises(binding.DmmError) as e:
            binding.dmm_measure_mfma_rate(bad, True)
        assert e.value.kind == "EINVAL"
