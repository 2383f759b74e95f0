// gemm_bf16_wide for A m-major, B n-major
#include "gemm_dma.h"

hipError_t gemm_wide_launch_nn(int cfg, const GemmDev& p, int splits, hipStream_t s) {
  return cfg >= kFirstDmaCfg ? launch_dma_layout<false, false>(cfg, p, splits, s) : launch_wide_layout<false, false>(cfg, p, splits, s);
}

// the weight-gradient products of a layer in one launch: 256 x 128 x 64 tiles, one block per CU
hipError_t gemm_wide_group_launch_nn(const GemmGroupDev& g, hipStream_t s) { return launch_wide_group_one<false, false, 4, 2, 2, 2, 64, 2, 1>(g, s); }
