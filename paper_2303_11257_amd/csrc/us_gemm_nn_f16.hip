// GEMM family: forward product Y = X W: activations K-contiguous, weights K-strided.
#include "us_gemm_dispatch.h"

namespace us {

hipError_t gemm_nn_f16(const GemmProblem& p, hipStream_t st) {
  if (p.epi == US_EPI_GELU && p.aux16 && !p.aux8 && (table_path_ok<false>(p) || wide_table_path_ok(p))) {
    GemmProblem q = p;
    q.table = (char*)p.table + kGeluHalfTableOffset;
    if (!p.tables_ready) {
      hipError_t e = launch_gelu_half_table(q.table, p.epi_scale, st);
      if (e != hipSuccess) return e;
    }
    if (wide_table_path_ok(p)) return launch_one<true, CfgE192, false, 0, 0, true, false, EPI_GELU_TAB16, false>(q, 1, p.K, st);
    return launch_one<true, CfgD256, false, 0, 0, true, false, EPI_GELU_TAB16, false>(q, 1, p.K, st);
  }
  if (p.epi == US_EPI_GELU) return launch_sized<false, 0, 0, true, false, EPI_GELU, false>(p, 1, p.K, st);
  if (p.epi == US_EPI_RESIDUAL) return launch_sized<false, 0, 0, true, false, EPI_RESIDUAL, false>(p, 1, p.K, st);
  return launch_store<false, 0, 0, true, false>(p, st);
}

}  // namespace us
