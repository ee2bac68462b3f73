// One instantiation of the grouped-GEMM kernels (gemm_kernel.hpp) per object file: the build
// compiles this file once for each DMM_INSTANCE = 0 .. 5, side by side.
//   0, 1: per-group macro-tiles, bf16 / fp32 operands
//   2, 3: the same with the epilogue that can add other replicas' partial sums (fused replica sum)
//   4, 5: merged macro-tiles, bf16 / fp32 operands
#include "gemm_launch.hpp"

#ifndef DMM_INSTANCE
#error "compile with -DDMM_INSTANCE=0..5"
#endif

#define DMM_CAT2(a, b) a##b
#define DMM_CAT(a, b) DMM_CAT2(a, b)

namespace dmm {

#if DMM_INSTANCE < 4

constexpr int kES = (DMM_INSTANCE & 1) ? 4 : 2;
constexpr bool kFuse = DMM_INSTANCE >= 2;

hipError_t DMM_CAT(gemm_allow_lds_, DMM_INSTANCE)() {
  return hipFuncSetAttribute((const void *)grouped_gemm_kernel<kES, kFuse>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             LDS_BYTES);
}

void DMM_CAT(gemm_launch_, DMM_INSTANCE)(unsigned grid, hipStream_t stream, const ItemDev *items, const SegDev *segs,
                                         const RedSrc *red, int n_items) {
  hipLaunchKernelGGL((grouped_gemm_kernel<kES, kFuse>), dim3(grid), dim3(NT), LDS_BYTES, stream, items, segs, red, n_items);
}

#else

constexpr int kES = (DMM_INSTANCE & 1) ? 4 : 2;

hipError_t DMM_CAT(gemm_allow_lds_, DMM_INSTANCE)() {
  return hipFuncSetAttribute((const void *)grouped_gemm_comp_kernel<kES>, hipFuncAttributeMaxDynamicSharedMemorySize,
                             LDS_BYTES + DESC_LDS);
}

void DMM_CAT(gemm_launch_, DMM_INSTANCE)(unsigned grid, hipStream_t stream, const CompItemDev *items, const PieceDev *a,
                                         const PieceDev *b, const PieceDev *c, const int32_t *klen) {
  hipLaunchKernelGGL(grouped_gemm_comp_kernel<kES>, dim3(grid), dim3(NT), LDS_BYTES + DESC_LDS, stream, items, a, b, c, klen);
}

#endif

}  // namespace dmm
