"""CPU oracle for the universal one-sided matmul hot path -- TEST INFRASTRUCTURE ONLY.

This package is the slow, plain statement of what the path computes:

* ``planner``  -- the distributed-matrix descriptor (Section 3, Table 1) and the
  Stationary-C op generation (Algorithm 1) with the replication rule of
  Section 4.1, written step by step in the paper's order, plus the plain
  stable-sort statement of the task grouping.
* ``matmul``   -- ``C = A B`` by its definition (Section 2.1): an fp64 i-k-j
  triple loop in C (``matmul.c``), and the fp32 left-to-right replica sum
  (``reduce_replicas``, Table 1).
* ``execute``  -- runs a task list tile by tile in fp64 (Section 4.2, steps
  1-4 of direct execution) so that the plan's meaning can be checked on the
  CPU without any GPU.

Nothing here is shared with, imported by, or imports the HIP library: only
``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may use it.  Every function is pinned by tests that run without a
GPU (brute-force coverage of the (i, k, j) iteration space, closed-form task
counts, textbook special cases, closed-form products); no part is
"parity unpinned".
"""
