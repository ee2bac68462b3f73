// Host-side doors to the grouped-GEMM kernels.  Every instantiation of the kernels is compiled
// in an object file of its own (gemm_instance.hip, once per value of DMM_INSTANCE), so that they
// compile side by side; the rest of the library reaches them through these functions only.
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "gemm_kernel.hpp"

namespace dmm {

// Per instantiation: allow the kernel its dynamic LDS on the current device; launch it.
#define DMM_DECLARE_GEMM(n)                                                                              \
  hipError_t gemm_allow_lds_##n();                                                                      \
  void gemm_launch_##n(unsigned grid, hipStream_t stream, const ItemDev *items, const SegDev *segs,     \
                       const RedSrc *red, int n_items);
DMM_DECLARE_GEMM(0)   // bf16
DMM_DECLARE_GEMM(1)   // fp32
DMM_DECLARE_GEMM(2)   // bf16, epilogue that can add other replicas' partial sums
DMM_DECLARE_GEMM(3)   // fp32, the same
#undef DMM_DECLARE_GEMM

#define DMM_DECLARE_COMP(n)                                                                              \
  hipError_t gemm_allow_lds_##n();                                                                      \
  void gemm_launch_##n(unsigned grid, hipStream_t stream, const CompItemDev *items, const PieceDev *a,  \
                       const PieceDev *b, const PieceDev *c, const int32_t *klen);
DMM_DECLARE_COMP(4)   // merged macro-tiles, bf16
DMM_DECLARE_COMP(5)   // merged macro-tiles, fp32
#undef DMM_DECLARE_COMP

// es = bytes per operand element (2 or 4); fuse = the instantiation whose epilogue can add partial sums
inline void launch_grouped_gemm(int es, bool fuse, unsigned grid, hipStream_t stream, const ItemDev *items,
                                const SegDev *segs, const RedSrc *red, int n_items) {
  if (es == 2 && !fuse) gemm_launch_0(grid, stream, items, segs, red, n_items);
  else if (es == 2) gemm_launch_2(grid, stream, items, segs, red, n_items);
  else if (!fuse) gemm_launch_1(grid, stream, items, segs, red, n_items);
  else gemm_launch_3(grid, stream, items, segs, red, n_items);
}

inline void launch_grouped_gemm_comp(int es, unsigned grid, hipStream_t stream, const CompItemDev *items,
                                     const PieceDev *a, const PieceDev *b, const PieceDev *c, const int32_t *klen) {
  if (es == 2) gemm_launch_4(grid, stream, items, a, b, c, klen);
  else gemm_launch_5(grid, stream, items, a, b, c, klen);
}

}  // namespace dmm
