// gemm_bf16_wide for A k-major, B k-major
#include "gemm_dma.h"

hipError_t gemm_wide_launch_kk(int cfg, const GemmDev& p, int splits, hipStream_t s) {
  return cfg >= kFirstDmaCfg ? launch_dma_layout<true, true>(cfg, p, splits, s) : launch_wide_layout<true, true>(cfg, p, splits, s);
}
