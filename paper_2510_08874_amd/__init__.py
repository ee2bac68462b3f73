"""MI355X-native hot path of the universal one-sided matmul (arXiv 2510.08874):
slicing planner, grouping, grouped GEMM and replica sum live in ``libdmm.so``
(sources under ``csrc/``, C ABI in ``include/dmm.h``).  ``binding`` mirrors the
ABI; ``tiles`` allocates tile buffers with torch.  Nothing here computes."""
from .binding import (DMM_BF16, DMM_C_BF16, DMM_F32, DMM_ITERATION_OFFSET, DMM_NO_MERGE, DMM_NO_REDUCE, DMM_SEPARATE_REDUCE, DMM_STATIONARY_A, DMM_STATIONARY_B, DMM_TIMING, DmmError, Plan, dmm_execute, dmm_plan,  # noqa: F401
                      dmm_plan_destroy, dmm_reduce_replicas, dmm_strerror, dmm_version)
