// GEMM family: grad_X product dX = G W^T: both operands K-contiguous.
#include "us_gemm_dispatch.h"

namespace us {

hipError_t gemm_nt_f16(const GemmProblem& p, hipStream_t st) {
  if (p.epi == US_EPI_GELU_GRAD && (table_path_ok<false>(p) || wide_table_path_ok(p))) {
    GemmProblem q = p;
    q.table = (char*)p.table + kGeluSlopeTableOffset;
    if (!p.tables_ready) {
      hipError_t e = launch_gelu_slope_table(q.table, p.epi_scale, st);
      if (e != hipSuccess) return e;
    }
    if (wide_table_path_ok(p)) return launch_one<true, CfgE192, false, 0, 0, true, true, EPI_GELU_GRAD_TAB, false>(q, 1, p.K, st);
    return launch_one<true, CfgD256, false, 0, 0, true, true, EPI_GELU_GRAD_TAB, false>(q, 1, p.K, st);
  }
  if (p.epi == US_EPI_GELU_GRAD) return launch_sized<false, 0, 0, true, true, EPI_GELU_GRAD, false>(p, 1, p.K, st);
  if (p.epi == US_EPI_RESIDUAL) return launch_sized<false, 0, 0, true, true, EPI_RESIDUAL, false>(p, 1, p.K, st);
  return launch_store<false, 0, 0, true, true>(p, st);
}

}  // namespace us
