// Host-side selection of tile shape and epilogue for one (operand layout, operand type) family.
// Each family is instantiated in its own translation unit to keep compile times short.
#pragma once

#include "us_gemm_kernel.h"
#include "us_launch.h"

namespace us {

inline GemmArgs make_args(const GemmProblem& p, long k_per_split) {
  GemmArgs g;
  g.A = (const uint8_t*)p.A;
  g.B = (const uint8_t*)p.B;
  g.C = p.C;
  g.M = p.M; g.N = p.N; g.K = p.K;
  g.lda = p.lda; g.ldb = p.ldb; g.ldc = p.ldc;
  g.k_per_split = k_per_split;
  g.scale = p.scale;
  g.epi_scale = p.epi_scale;
  g.c_is_f32 = (p.c_dt == US_F32) ? 1 : 0;
  g.Zpre = (const _Float16*)p.Zpre;
  g.aux16 = (_Float16*)p.aux16;
  g.aux8 = (uint8_t*)p.aux8;
  g.partial = (float*)p.workspace;
  return g;
}

template <int BM, int BN, bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI>
hipError_t launch_one(const GemmArgs& g, int splits, hipStream_t st) {
  using T = GemmTile<BM, BN, FP8, A_KC, B_KC>;
  auto kern = gemm_kernel<BM, BN, 2, 2, FP8, FA, FB, A_KC, B_KC, EPI>;
  static bool configured = false;  // raising the dynamic-LDS limit is a per-function, once-only call
  if (!configured) {
    hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, T::LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  const long tiles = ((g.M + BM - 1) / BM) * ((g.N + BN - 1) / BN);
  dim3 grid((unsigned)tiles, (unsigned)splits, 1);
  kern<<<grid, kGemmThreads, T::LDS_BYTES, st>>>(g);
  return hipGetLastError();
}

// Large tiles once they fill the 256 CUs; small tiles for small problems.
inline bool use_big_tile(long M, long N, int splits) {
  const long big = ((M + 255) / 256) * ((N + 255) / 256) * splits;
  return big >= 192;
}

template <bool FP8, int FA, int FB, bool A_KC, bool B_KC, int EPI>
hipError_t launch_sized(const GemmProblem& p, int splits, long k_per_split, hipStream_t st) {
  GemmArgs g = make_args(p, k_per_split);
  if (use_big_tile(p.M, p.N, splits)) return launch_one<256, 256, FP8, FA, FB, A_KC, B_KC, EPI>(g, splits, st);
  return launch_one<128, 128, FP8, FA, FB, A_KC, B_KC, EPI>(g, splits, st);
}

hipError_t launch_splitk_reduce(const float* partial, void* out, long total, int splits, float scale, bool out_is_f32,
                                hipStream_t st);

// Families (defined one per translation unit).
hipError_t gemm_nn_f16(const GemmProblem& p, hipStream_t st);   // forward:  A K-contig, B K-strided
hipError_t gemm_nn_fp8(const GemmProblem& p, hipStream_t st);
hipError_t gemm_nt_f16(const GemmProblem& p, hipStream_t st);   // grad_X:   both K-contig
hipError_t gemm_nt_fp8(const GemmProblem& p, hipStream_t st);
hipError_t gemm_tn_f16(const GemmProblem& p, hipStream_t st);   // grad_W:   both K-strided, split-K
hipError_t gemm_tn_fp8(const GemmProblem& p, hipStream_t st);

}  // namespace us
