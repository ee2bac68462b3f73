"""GPU test of the entry point for callers that cannot allocate: ``dmm_reduce_replicas_static``
against ``dmm_reduce_replicas`` through the C ABI, bit for bit, on two calls in a row, the second
with a smaller input (every call shares the library's one static device buffer, which keeps the
last call's contents)."""
import ctypes

import numpy as np
import pytest

import workloads

torch = pytest.importorskip("torch")
binding = pytest.importorskip("paper_2510_08874_amd.binding")

pytestmark = pytest.mark.gpu


def _problem(M, N, grid, c, ldm, seed):
    from paper_2510_08874_amd.tiles import DeviceProblem
    p = c * grid[0] * grid[1]
    cfg = dict(name="static-reduce", M=M, K=8, N=N, dtype="f32", nranks=p,
               A=workloads.block_desc(M, 8, 1, 1, replication=p), B=workloads.block_desc(8, N, 1, 1, replication=p),
               C=workloads.block_desc(M, N, grid[0], grid[1], replication=c), dist=("normal", 1.0), seeds=(1, 2))
    prob = DeviceProblem(cfg, None, None, ld_multiple=ldm)
    rng = np.random.default_rng(seed)
    start = []
    for t in prob.C.tensors:
        h = rng.standard_normal(tuple(t.shape)).astype(np.float32) * np.float32(10.0 ** rng.integers(-3, 4))
        t.copy_(torch.from_numpy(h))
        start.append(h)
    return prob, start


def _tables(prob):
    ct = (ctypes.c_void_p * len(prob.C.tensors))(*[int(t.data_ptr()) for t in prob.C.tensors])
    cl = (ctypes.c_int64 * len(prob.C.ld))(*prob.C.ld)
    return ct, cl


def _both_ways(M, N, grid, c, origin, ldm, seed):
    L = binding.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    prob, start = _problem(M, N, grid, c, ldm, seed)
    ct, cl = _tables(prob)
    # the existing entry point
    assert L.dmm_reduce_replicas(prob.plan.handle, ct, cl, origin, stream) == binding.DMM_OK
    torch.cuda.synchronize()
    want = [t.cpu().numpy().copy() for t in prob.C.tensors]
    # the same inputs again, through the entry point that allocates nothing
    for t, h in zip(prob.C.tensors, start):
        t.copy_(torch.from_numpy(h))
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]      # (what the driver has left: torch's own caching does not show here)
    assert L.dmm_reduce_replicas_static(prob.plan.handle, ct, cl, origin, stream) == binding.DMM_OK
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] >= free_before, "the call took device memory"
    got = [t.cpu().numpy() for t in prob.C.tensors]
    changed = 0
    for g, w, h in zip(got, want, start):
        assert np.array_equal(g, w)                 # sums, untouched replicas and padding alike
        changed += int(not np.array_equal(g, h))
    assert changed == grid[0] * grid[1]             # exactly the origin replica's tiles received a sum
    prob.close()


def test_static_replica_sum_matches_the_pooled_one_twice_in_a_row():
    torch.cuda.set_device(0)
    _both_ways(1000, 772, (2, 2), 3, origin=1, ldm=4, seed=5)      # float4 path, three replicas
    _both_ways(301, 203, (2, 1), 2, origin=0, ldm=1, seed=6)       # smaller, odd widths: the element path


def test_static_replica_sum_limits_and_errors():
    torch.cuda.set_device(0)
    L = binding.lib()
    stream = ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    # one replica: nothing to do
    prob, start = _problem(64, 64, (1, 1), 1, 1, 7)
    ct, cl = _tables(prob)
    assert L.dmm_reduce_replicas_static(prob.plan.handle, ct, cl, 0, stream) == binding.DMM_OK
    assert L.dmm_reduce_replicas_static(prob.plan.handle, ct, cl, 1, stream) == binding.DMM_EINVAL
    torch.cuda.synchronize()
    assert np.array_equal(prob.C.tensors[0].cpu().numpy(), start[0])
    prob.close()
    # tables beyond the static buffer: 16 bytes per 4096 elements of C -> more than 2^28 elements.
    # Only the descriptors are needed to be refused: the pointer table may name anything non-null.
    M = N = 1 << 15
    C = workloads.block_desc(M, N, 2, 2, replication=2)
    plan = binding.Plan(workloads.block_desc(M, 8, 1, 1, replication=8), workloads.block_desc(8, N, 1, 1, replication=8), C, 8)
    fake = (ctypes.c_void_p * 8)(*([0x1000] * 8))
    lds = (ctypes.c_int64 * 8)(*([N // 2] * 8))
    assert L.dmm_reduce_replicas_static(plan.handle, fake, lds, 0, stream) == binding.DMM_ELIMIT
    assert "static" in binding.dmm_strerror(binding.DMM_ELIMIT)
    plan.destroy()
