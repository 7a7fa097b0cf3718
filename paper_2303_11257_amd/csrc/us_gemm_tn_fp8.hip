// GEMM family: grad_W product dW = X^T G: both operands K-strided (the reduction runs over tokens),
// cut into K slices with an ordered FP32 reduction when the output alone cannot fill the chip.
#include "us_gemm_dispatch.h"

namespace us {

hipError_t gemm_tn_fp8(const GemmProblem& p, hipStream_t st) {
  const int splits = p.workspace ? gemm_splits(p.M, p.N, p.K) : 1;
  if (splits <= 1) return launch_store<true, 0, 1, false, false>(p, st);
  const long k_per_split = gemm_k_per_split(p.K, splits);
  hipError_t e = launch_sized<true, 0, 1, false, false, EPI_PARTIAL, true>(p, splits, k_per_split, st);
  if (e != hipSuccess) return e;
  return launch_splitk_reduce((const float*)p.workspace, p.C, p.M * p.N, splits, p.scale, p.c_dt == US_F32, st);
}

}  // namespace us
